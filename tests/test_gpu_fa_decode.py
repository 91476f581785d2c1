"""GPU parity of swaa_attn_fwd_fa_decode (window for prompt rows, full attention for
generated rows) against the fp64 CPU oracle, through the C ABI.  Same tolerances
as the prefill tests.
"""
import math

import numpy as np
import pytest
import torch

from oracle import swaa_attn_oracle
from paper_2512_10411_amd import binding
from paper_2512_10411_amd.inputs import (WORKLOADS, bf16_bits_to_f32, f32_to_bf16_bits, make_qkv,
                                         make_workload, sample_rows)
from gpu_util import assert_parity, to_device

pytestmark = pytest.mark.gpu


def run_gpu(q, k, v, W, S, P, scale):
    out, lse = binding.swaa_attn_fwd_fa_decode(to_device(q), to_device(k), to_device(v), W, S, P, scale)
    torch.cuda.synchronize()
    return out, lse


def check(B, Hq, Hkv, N, D, W, S, P, seed, rows=None):
    scale = 1.0 / math.sqrt(D)
    tag = f"B{B} Hq{Hq} Hkv{Hkv} N{N} D{D} W{W} S{S} P{P}"
    print(f"[case] {tag} seed {seed}", flush=True)
    q, k, v = make_qkv(B, Hq, Hkv, N, D, seed)
    out, lse = run_gpu(q, k, v, W, S, P, scale)
    ro, rl = swaa_attn_oracle(q, k, v, W, S, scale, rows=rows, n_prompt=P)
    assert_parity(out, lse, ro, rl, rows=rows, tag=tag)


@pytest.mark.parametrize("N", [1, 65, 130, 257, 700])
@pytest.mark.parametrize("D", [64, 128])
def test_small_shapes_sweep_prompt_length(N, D):
    # the prompt boundary inside a wave's rows, on wave, workgroup and tile boundaries, and at both ends
    seed = 5000 + N + D
    for W, S in ((1, 0), (7, 4), (64, 0), (200, 70)):
        for P in sorted({0, 1, 31, 32, 33, 64, 100, N // 2, N - 1, N, N + 5}):
            check(1, 4, 1, N, D, W, S, P, seed)


@pytest.mark.parametrize("G", [1, 2, 3, 5, 7, 8])
def test_gqa_group_sizes(G):
    check(2, 2 * G, 2, 333, 128, 100, 3, 250, seed=5200 + G)
    check(1, G, 1, 515, 64, 65, 10, 300, seed=5300 + G)


def test_prompt_length_at_or_past_n_equals_the_prefill_call_bit_for_bit():
    q, k, v = make_qkv(1, 6, 2, 1500, 128, seed=51)
    qd, kd, vd = to_device(q), to_device(k), to_device(v)
    o0, l0 = binding.swaa_attn_fwd(qd, kd, vd, 300, 4)
    for P in (1500, 1501, 2**31 - 1):
        o1, l1 = binding.swaa_attn_fwd_fa_decode(qd, kd, vd, 300, 4, P)
        torch.cuda.synchronize()
        assert torch.equal(o0, o1) and torch.equal(l0, l1)
    # no prompt rows at all: full causal attention, whatever the window
    of, lf = binding.swaa_attn_fwd(qd, kd, vd, 1500, 0)
    o2, l2 = binding.swaa_attn_fwd_fa_decode(qd, kd, vd, 300, 4, 0)
    torch.cuda.synchronize()
    assert torch.equal(of, o2) and torch.equal(lf, l2)
    with pytest.raises(binding.SwaaError):
        binding.swaa_attn_fwd_fa_decode(qd, kd, vd, 300, 4, -1)


def test_generated_rows_see_a_score_spike_deep_in_the_prompt():
    # the generated rows' reference comes from the first keys; a key far above it, outside
    # every prompt row's reach, must still come out right (and must not touch prompt rows)
    B, Hq, Hkv, N, D, W, S, P = 1, 4, 1, 3100, 128, 256, 4, 3000
    q, k, v = make_qkv(B, Hq, Hkv, N, D, seed=52)
    qf, kf = bf16_bits_to_f32(q), bf16_bits_to_f32(k)
    qf[..., 0] = 3.0
    kf[..., 0] = 0.0
    kf[:, :, 1500, 0] = 160.0
    q, k = f32_to_bf16_bits(qf), f32_to_bf16_bits(kf)
    scale = 1 / math.sqrt(D)
    out, lse = run_gpu(q, k, v, W, S, P, scale)
    ro, rl = swaa_attn_oracle(q, k, v, W, S, scale, n_prompt=P)
    assert_parity(out, lse, ro, rl, tag="spike seen by generated rows")


@pytest.mark.parametrize("P", [8192, 8192 - 37])
def test_long_prompt_with_generated_tail_sampled_rows(P):
    B, Hq, Hkv, N, D, W, S = 1, 10, 2, P + 300, 128, 1024, 4
    rows = sorted(set(sample_rows(N, W, S, count=160, seed=53).tolist())
                  | {P - 2, P - 1, P, P + 1, P + 31, P + 32, P + 63, P + 64, N - 1}
                  | set(range(P + 100, P + 140)))
    check(B, Hq, Hkv, N, D, W, S, P, seed=5400 + P, rows=np.array(rows, dtype=np.int32))


@pytest.mark.parametrize("name", ["mid_fa_decode", "long128k_fa_decode"])
def test_fa_decode_workloads_full_size_sampled_rows(name):
    # full-size launches exactly as the benchmark times them
    w = WORKLOADS[name]
    P = w.n_prompt
    print(f"[gen] {name} ...", flush=True)
    q, k, v = make_workload(w)
    rows = sorted(set(sample_rows(w.N, w.window, w.n_sink, count=128, seed=w.seed).tolist())
                  | {P - 1, P, P + 1, w.N - 1} | set(range(P + 200, P + 232)))
    rows = np.array(rows, dtype=np.int32)
    print(f"[gpu] {name}", flush=True)
    out, lse = run_gpu(q, k, v, w.window, w.n_sink, P, w.scale)
    assert torch.isfinite(lse).all()
    print(f"[oracle] {name}: {len(rows)} rows x {w.B * w.Hq} heads", flush=True)
    ro, rl = swaa_attn_oracle(q, k, v, w.window, w.n_sink, w.scale, rows=rows, n_prompt=P)
    assert_parity(out, lse, ro, rl, rows=rows, tag=name)


@pytest.mark.parametrize("D", [128, 64])
def test_prompt_lengths_of_their_own_per_sequence(D):
    # a batch as a serving engine sees it: every sequence has its own prompt length (FA Decode,
    # Sec. 3.1.1); fixed-length and packed calls, prompt lengths of 0, inside a row tile, and beyond
    # the sequence
    import math
    from oracle import swaa_decode_oracle
    Hq, Hkv, W, S = 8, 2, 64, 4
    # fixed-length batch
    B, N = 5, 700
    prompts = [0, 100, 333, 699, 5000]
    q, k, v = make_qkv(B, Hq, Hkv, N, D, seed=9700 + D)
    out, lse = binding.swaa_attn_fwd_ex(to_device(q), to_device(k), to_device(v), W, S, 17,   # (n_prompt itself is ignored)
                                        n_prompts=torch.tensor(prompts, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    for b in range(B):
        ro, rl = swaa_decode_oracle(q[b:b + 1], k[b:b + 1], v[b:b + 1], W, S, 1 / math.sqrt(D), n_prompt=prompts[b])
        assert_parity(out[b:b + 1], lse[b:b + 1], ro, rl, tag=f"per-sequence prompt length {prompts[b]} of {N} D{D}")
    # packed chunks: sequence b brings its newest nq[b] rows against nk[b] cached tokens
    nk = [300, 64, 1000, 130]
    nq = [300, 10, 400, 130]
    prompts = [250, 60, 650, 0]
    seqs = [make_qkv(1, Hq, Hkv, nk[i], D, 9750 + D + i, n_query=nq[i]) for i in range(len(nk))]
    q_pack = torch.cat([to_device(s[0])[0] for s in seqs], dim=1).contiguous()
    k_pack = torch.cat([to_device(s[1])[0] for s in seqs], dim=1).contiguous()
    v_pack = torch.cat([to_device(s[2])[0] for s in seqs], dim=1).contiguous()
    cu_q = torch.tensor(np.concatenate([[0], np.cumsum(nq)]), dtype=torch.int32, device="cuda")
    cu_k = torch.tensor(np.concatenate([[0], np.cumsum(nk)]), dtype=torch.int32, device="cuda")
    out, lse = binding.swaa_attn_fwd_ex(q_pack, k_pack, v_pack, W, S, None, cu_seqlens_q=cu_q, cu_seqlens_k=cu_k,
                                        max_seqlen_q=max(nq), max_seqlen_k=max(nk),
                                        n_prompts=torch.tensor(prompts, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    r0 = 0
    for b, (qs, ks, vs) in enumerate(seqs):
        ro, rl = swaa_decode_oracle(qs, ks, vs, W, S, 1 / math.sqrt(D), n_prompt=prompts[b])
        assert_parity(out[None, :, r0:r0 + nq[b]], lse[None, :, r0:r0 + nq[b]], ro, rl,
                      tag=f"packed, per-sequence prompt length {prompts[b]} of {nk[b]} D{D}")
        r0 += nq[b]
