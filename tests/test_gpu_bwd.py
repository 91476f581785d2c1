"""GPU parity of swaa_attn_bwd (dQ, dK, dV) against the fp64 CPU oracle, through the C ABI.

The forward results the backward call consumes (out, lse) come from the library's own
forward call, as in training.

Tolerance (no figure is given for the backward pass; this one is derived from the arithmetic).
Every gradient element is a sum  x = c * sum_t a_t b_t  whose factor a_t (P for dV, dS for dQ
and dK) is rounded to bf16 before the product, accumulated in fp32, and rounded to bf16 at the
end.  With u = 2^-9 (half a bf16 step, relative) and rounding errors spread evenly over
[-u, u] (standard deviation u / sqrt 3):

    |error(x)|  <=  u |x|  +  4 * (u / sqrt 3) * rss(terms)          (four standard deviations)

and rss(terms) <= max|x| over the tensor for the elements that matter (an element is large
exactly when its terms align), so  error <= (1 + 4 / sqrt 3) u max|ref| = 6.5e-3 max|ref|; the
bar is MAX_REL = 8e-3.  One more channel reaches dQ and dK only: delta_i = <dO_i, O_i> is formed
from the forward's bf16 output, whose elements carry independent roundings of up to u |O_id|
(the forward divides by the sum of the ROUNDED P, so a row that sees a single key returns that
key's value row exactly and delta is exact there; the one-signed error of up to 2^-8 |delta| that
an earlier forward left in rows dominated by one key is gone).  So delta_i is off by about
(u / sqrt 3) * sqrt(sum_d dO_id^2 O_id^2), 0.013 for D = 128 and 0.009 for D = 64 with N(0,1)
data, dS_ij by P_ij times that, and dQ_i (dK_j) by scale * that * |P-weighted mean of k| (of q):
at four standard deviations and |k|, |q| <= 4.5 this is scale * 4.5 * 4 * 0.013 = 2e-2 for both
head dimensions, reached only by rows that put nearly all weight on one key with a large
component; rows that spread over many keys average it out.  Hence

    max-abs error  <=  8e-3 * max|ref| + abs,    abs = 2e-2 (dQ, dK), 2e-3 (dV)
    mean-abs error <=  4e-3 * mean|ref| + 1e-3

Measured over every case below: max-abs error <= 5.8e-3 max|ref| (dQ), 4.6e-3 (dK), 4.4e-3 (dV);
the absolute terms are never drawn upon by more than 1e-6 (they matter where the true gradient
is zero).
"""
import math

import numpy as np
import pytest
import torch

from oracle import swaa_attn_bwd_oracle
from paper_2512_10411_amd import binding
from paper_2512_10411_amd.inputs import f32_to_bf16_bits, make_qkv
from gpu_util import to_device

pytestmark = pytest.mark.gpu

MAX_REL = 8e-3
MAX_ABS = {"dq": 2e-2, "dk": 2e-2, "dv": 2e-3}
MEAN_REL, MEAN_ABS = 4e-3, 1e-3


def make_dout(shape, seed):
    rng = np.random.Generator(np.random.Philox(seed))
    return f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))


def assert_grad(name, got, ref, tag):
    g = got.float().cpu().numpy().astype(np.float64)
    assert g.shape == ref.shape and np.isfinite(g).all(), (tag, name)
    err = np.abs(g - ref)
    rmax, rmean = np.abs(ref).max(), np.abs(ref).mean()
    print(f"[grad] {tag} {name}: max-abs err {err.max():.3e} (max|ref| {rmax:.3e}), mean-abs err {err.mean():.3e} "
          f"(mean|ref| {rmean:.3e})", flush=True)
    assert err.max() <= MAX_REL * rmax + MAX_ABS[name], (tag, name, err.max(), rmax)
    assert err.mean() <= MEAN_REL * rmean + MEAN_ABS, (tag, name, err.mean(), rmean)


def check(B, Hq, Hkv, N, D, W, S, P, seed):
    tag = f"bwd B{B} Hq{Hq} Hkv{Hkv} N{N} D{D} W{W} S{S} P{P}"
    print(f"[case] {tag} seed {seed}", flush=True)
    scale = 1 / math.sqrt(D)
    q, k, v = make_qkv(B, Hq, Hkv, N, D, seed)
    dout = make_dout(q.shape, seed + 1)
    qd, kd, vd, dd = to_device(q), to_device(k), to_device(v), to_device(dout)
    n_prompt = N if P is None else P
    out, lse = binding.swaa_attn_fwd_fa_decode(qd, kd, vd, W, S, n_prompt, scale)
    dq, dk, dv = binding.swaa_attn_bwd(qd, kd, vd, out, lse, dd, W, S, n_prompt, scale)
    torch.cuda.synchronize()
    rq, rk, rv = swaa_attn_bwd_oracle(q, k, v, dout, W, S, scale, n_prompt=n_prompt)
    assert_grad("dq", dq, rq, tag)
    assert_grad("dk", dk, rk, tag)
    assert_grad("dv", dv, rv, tag)


@pytest.mark.parametrize("N", [1, 2, 63, 64, 65, 130, 300, 700])
@pytest.mark.parametrize("D", [64, 128])
def test_small_shapes_sweep_the_mask(N, D):
    seed = 9000 + N + D
    for W, S, P in ((1, 0, None), (7, 4, None), (64, 0, None), (65, 70, None), (N, 0, None), (50, 3, N // 2),
                    (200, 0, 0)):
        if W == 1 and S == 0:
            continue  # dK = dQ = 0 exactly: a relative bar has nothing to measure (covered below)
        check(1, 4, 1, N, D, W, S, P, seed)


def test_window_one_gives_zero_dq_dk_and_dv_equal_to_dout():
    B, Hq, Hkv, N, D = 1, 4, 2, 333, 128
    q, k, v = make_qkv(B, Hq, Hkv, N, D, seed=9100)
    dout = make_dout(q.shape, 9101)
    qd, kd, vd, dd = to_device(q), to_device(k), to_device(v), to_device(dout)
    out, lse = binding.swaa_attn_fwd(qd, kd, vd, 1, 0)
    dq, dk, dv = binding.swaa_attn_bwd(qd, kd, vd, out, lse, dd, 1, 0)
    torch.cuda.synchronize()
    # a row that sees one key has O = v exactly, so dP - delta vanishes up to the order of two
    # fp32 sums of 128 products of N(0,1) values: 1e-5 at most, times scale * |k| <= 0.4
    print(f"[grad] W=1: max |dq| {dq.float().abs().max().item():.3e}, max |dk| {dk.float().abs().max().item():.3e}",
          flush=True)
    assert dq.float().abs().max().item() <= 1e-4 and dk.float().abs().max().item() <= 1e-4
    want = dd.float().view(B, Hkv, 2, N, D).sum(dim=2)
    assert (dv.float() - want).abs().max().item() <= 2.0 ** -7 * want.abs().max().item()


@pytest.mark.parametrize("G", [1, 2, 3, 5, 8])
def test_gqa_group_sizes_and_batches(G):
    check(2, 2 * G, 2, 333, 128, 100, 3, None, seed=9200 + G)
    check(1, G, 1, 515, 64, 65, 10, 400, seed=9300 + G)


def test_run_to_run_determinism_and_errors():
    q, k, v = make_qkv(1, 8, 2, 1000, 128, seed=9400)
    qd, kd, vd = to_device(q), to_device(k), to_device(v)
    dd = to_device(make_dout(q.shape, 9401))
    out, lse = binding.swaa_attn_fwd(qd, kd, vd, 256, 4)
    a = binding.swaa_attn_bwd(qd, kd, vd, out, lse, dd, 256, 4)
    b = binding.swaa_attn_bwd(qd, kd, vd, out, lse, dd, 256, 4)
    torch.cuda.synchronize()
    assert all(torch.equal(x, y) for x, y in zip(a, b))
    with pytest.raises(binding.SwaaError) as e:
        binding.swaa_attn_bwd(qd, kd, vd, out, lse, dd, 256, 4, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == binding.SWAA_ERR_WORKSPACE
    with pytest.raises(binding.SwaaError):
        binding.swaa_attn_bwd(qd, kd, vd, out, lse, dd, 0, 4)


@pytest.mark.parametrize("shape", [(1, 8, 2, 4096 + 37, 128, 512, 4, None), (1, 16, 4, 8192, 128, 1024, 4, 8192 - 300),
                                   (2, 10, 2, 2048, 128, 2048, 0, None)])
def test_mid_size_every_element(shape):
    B, Hq, Hkv, N, D, W, S, P = shape
    check(B, Hq, Hkv, N, D, W, S, P, seed=9500 + N)


def test_benchmark_workload_at_full_size_two_kv_heads():
    """The launch configuration bench.py times (workload mid_bwd, all 32 heads), checked on
    every element of the first and the last KV head with their query heads: heads are
    independent, so the oracle runs on those slices only (about 20 s on the host)."""
    from paper_2512_10411_amd.inputs import WORKLOADS, make_workload

    w = WORKLOADS["mid_bwd"]
    q, k, v = make_workload(w)
    dout = make_dout(q.shape, w.seed + 1)
    qd, kd, vd, dd = to_device(q), to_device(k), to_device(v), to_device(dout)
    out, lse = binding.swaa_attn_fwd(qd, kd, vd, w.window, w.n_sink, w.scale)
    dq, dk, dv = binding.swaa_attn_bwd(qd, kd, vd, out, lse, dd, w.window, w.n_sink, None, w.scale)
    torch.cuda.synchronize()
    G = w.Hq // w.Hkv
    for kvh in (0, w.Hkv - 1):
        tag = f"mid_bwd full size, KV head {kvh}"
        print(f"[case] {tag}", flush=True)
        hs = slice(kvh * G, (kvh + 1) * G)
        rq, rk, rv = swaa_attn_bwd_oracle(np.ascontiguousarray(q[:, hs]), np.ascontiguousarray(k[:, kvh:kvh + 1]),
                                          np.ascontiguousarray(v[:, kvh:kvh + 1]), np.ascontiguousarray(dout[:, hs]),
                                          w.window, w.n_sink, w.scale)
        assert_grad("dq", dq[:, hs], rq, tag)
        assert_grad("dk", dk[:, kvh:kvh + 1], rk, tag)
        assert_grad("dv", dv[:, kvh:kvh + 1], rv, tag)
