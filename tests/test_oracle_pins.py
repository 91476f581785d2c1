"""Pins for the fp64 CPU oracle (CPU only).

The paper prints no numeric example of the attention computation and ships no
code, so the oracle is pinned to what the paper's prose and the mathematics
fix: the full-attention special case against a library routine (Sec. 4.1.2:
SWA equals full attention when the context fits the window), closed forms,
a literal boolean-mask brute force of the sentence in Sec. 3.2.1 (a token
attends to its local window AND the initial k tokens), locality (App. A: a
token's state is independent of tokens outside its window), and identities.
"""
import math

import numpy as np
import pytest
import torch

from oracle import swaa_attn_oracle, swaa_attn_oracle_numpy
from paper_2512_10411_amd.inputs import (bf16_bits_to_f32, f32_to_bf16_bits,
                                         make_qkv)


def f64(bits):
    return bf16_bits_to_f32(bits).astype(np.float64)


def dense_masked_attention(q, k, v, mask, scale):
    """Library route: torch float64 softmax over an explicit boolean mask [N,N]."""
    B, Hq, N, D = q.shape
    G = Hq // k.shape[1]
    qt = torch.from_numpy(f64(q))
    kt = torch.from_numpy(f64(k)).repeat_interleave(G, dim=1)
    vt = torch.from_numpy(f64(v)).repeat_interleave(G, dim=1)
    s = torch.matmul(qt, kt.transpose(-1, -2)) * scale
    s = s.masked_fill(~torch.from_numpy(mask), float("-inf"))
    lse = torch.logsumexp(s, dim=-1)
    o = torch.matmul(torch.softmax(s, dim=-1), vt)
    return o.numpy(), lse.numpy()


def brute_mask(N, W, S):
    """The sentence of Sec. 3.2.1, literally: causal, and (in the local window of
    W keys ending at the query, or among the first S tokens)."""
    M = np.zeros((N, N), dtype=bool)
    for i in range(N):
        for j in range(N):
            causal = j <= i
            in_window = (i - j) < W
            is_sink = j < S
            M[i, j] = causal and (in_window or is_sink)
    return M


def n_visible(i, W, S):
    return min(i + 1, W) + min(max(i - W + 1, 0), S)


# ---------------------------------------------------------------- P1
@pytest.mark.parametrize("W,S", [(64, 0), (64, 7), (1000, 3), (2**31 - 1, 0)])
def test_window_ge_n_is_full_causal_vs_sdpa(W, S):
    B, Hq, Hkv, N, D = 2, 4, 4, 64, 32
    q, k, v = make_qkv(B, Hq, Hkv, N, D, seed=11)
    scale = 1 / math.sqrt(D)
    o, lse = swaa_attn_oracle(q, k, v, W, S, scale)
    qt, kt, vt = (torch.from_numpy(f64(a)) for a in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, is_causal=True, scale=scale)
    assert np.abs(o - ref.numpy()).max() < 1e-12
    s = torch.matmul(qt, kt.transpose(-1, -2)) * scale
    s = s.masked_fill(~torch.tril(torch.ones(N, N, dtype=torch.bool)), float("-inf"))
    assert np.abs(lse - torch.logsumexp(s, -1).numpy()).max() < 1e-12


# ---------------------------------------------------------------- P2
def test_rows_below_window_equal_full_causal():
    q, k, v = make_qkv(1, 2, 1, 96, 16, seed=12)
    W = 40
    o_swa, l_swa = swaa_attn_oracle(q, k, v, W, 0, 0.25)
    o_full, l_full = swaa_attn_oracle(q, k, v, 96, 0, 0.25)
    assert np.array_equal(o_swa[:, :, :W], o_full[:, :, :W])
    assert np.array_equal(l_swa[:, :, :W], l_full[:, :, :W])
    assert not np.allclose(o_swa[:, :, W:], o_full[:, :, W:])


# ---------------------------------------------------------------- P3
def test_window_one_returns_own_value_row():
    q, k, v = make_qkv(1, 4, 2, 50, 32, seed=13)
    scale = 0.3
    o, lse = swaa_attn_oracle(q, k, v, 1, 0, scale)
    G = 2
    for h in range(4):
        assert np.array_equal(o[0, h], f64(v)[0, h // G])
        s_ii = scale * np.einsum("nd,nd->n", f64(q)[0, h], f64(k)[0, h // G])
        assert np.abs(lse[0, h] - s_ii).max() < 1e-13


# ---------------------------------------------------------------- P4
@pytest.mark.parametrize("N,W,S", [(40, 1, 0), (40, 5, 0), (40, 5, 3), (40, 5, 5), (40, 5, 9),
                                   (40, 16, 39), (40, 40, 4), (40, 64, 64), (37, 8, 1), (33, 2, 40)])
def test_zero_queries_give_mean_and_log_count(N, W, S):
    q, k, v = make_qkv(1, 2, 1, N, 8, seed=14)
    q[:] = 0
    o, lse = swaa_attn_oracle(q, k, v, W, S, 1.0)
    vf = f64(v)[0, 0]
    for i in range(N):
        vis = [j for j in range(i + 1) if i - j < W or j < S]
        assert len(vis) == n_visible(i, W, S)
        assert abs(lse[0, 0, i] - math.log(len(vis))) < 1e-13
        assert abs(lse[0, 1, i] - math.log(len(vis))) < 1e-13
        assert np.abs(o[0, 0, i] - vf[vis].mean(axis=0)).max() < 1e-13


# ---------------------------------------------------------------- P5
@pytest.mark.parametrize("N,G", [(7, 1), (20, 2), (33, 4)])
def test_brute_force_boolean_mask_all_w_s(N, G):
    Hkv, D = 2, 8
    q, k, v = make_qkv(1, Hkv * G, Hkv, N, D, seed=15 + N)
    for W in range(1, N + 3):
        for S in range(0, N + 3, 1 if N <= 20 else 3):
            o, lse = swaa_attn_oracle(q, k, v, W, S, 0.4)
            ro, rl = dense_masked_attention(q, k, v, brute_mask(N, W, S), 0.4)
            assert np.abs(o - ro).max() < 1e-12, (W, S)
            assert np.abs(lse - rl).max() < 1e-12, (W, S)


def test_numpy_route_agrees_with_c_route():
    q, k, v = make_qkv(2, 6, 3, 45, 16, seed=16)
    for W, S in [(1, 0), (7, 2), (16, 20), (100, 0)]:
        o1, l1 = swaa_attn_oracle(q, k, v, W, S, 0.21)
        o2, l2 = swaa_attn_oracle_numpy(q, k, v, W, S, 0.21)
        assert np.abs(o1 - o2).max() < 1e-13 and np.abs(l1 - l2).max() < 1e-13
    rows = [0, 3, 44, 17]
    o1, l1 = swaa_attn_oracle(q, k, v, 7, 2, 0.21, rows=rows)
    o2, l2 = swaa_attn_oracle(q, k, v, 7, 2, 0.21)
    assert np.array_equal(o1, o2[:, :, rows]) and np.array_equal(l1, l2[:, :, rows])


# ---------------------------------------------------------------- P6
def test_locality_nan_outside_visible_set_does_not_leak():
    N, W, S = 64, 8, 2
    q, k, v = make_qkv(1, 2, 1, N, 16, seed=17)
    o0, l0 = swaa_attn_oracle(q, k, v, W, S, 0.25)
    i = 40
    hidden = [j for j in range(N) if not (j <= i and (i - j < W or j < S))]
    k2, v2 = k.copy(), v.copy()
    k2[0, 0, hidden] = 0x7FC0  # bf16 NaN
    v2[0, 0, hidden] = 0x7FC0
    o1, l1 = swaa_attn_oracle(q, k2, v2, W, S, 0.25)
    assert np.array_equal(o1[:, :, i], o0[:, :, i]) and np.array_equal(l1[:, :, i], l0[:, :, i])
    # a sink row is seen by every later row; a non-sink row only inside the window
    v3 = v.copy()
    v3[0, 0, 1] = f32_to_bf16_bits(np.full(16, 3.0, np.float32))
    o3, _ = swaa_attn_oracle(q, k, v3, W, S, 0.25)
    changed = np.any(o3[0, 0] != o0[0, 0], axis=-1)
    assert changed[1:].all() and not changed[0]
    v4 = v.copy()
    v4[0, 0, 10] = f32_to_bf16_bits(np.full(16, 3.0, np.float32))
    o4, _ = swaa_attn_oracle(q, k, v4, W, S, 0.25)
    changed = np.any(o4[0, 0] != o0[0, 0], axis=-1)
    assert changed[10:10 + W].all() and not changed[:10].any() and not changed[10 + W:].any()


# ---------------------------------------------------------------- P7
@pytest.mark.parametrize("W,S", [(8, 3), (8, 12), (20, 1)])
def test_merge_of_band_and_sink_partials(W, S):
    N = 48
    q, k, v = make_qkv(1, 2, 2, N, 16, seed=18)
    o, lse = swaa_attn_oracle(q, k, v, W, S, 0.3)
    i_idx, j_idx = np.meshgrid(np.arange(N), np.arange(N), indexing="ij")
    band = (j_idx <= i_idx) & (i_idx - j_idx < W)
    sink_only = (j_idx < S) & (j_idx <= i_idx) & ~band
    ob, lb = dense_masked_attention(q, k, v, band, 0.3)
    for i in range(N):
        if sink_only[i].any():
            m = np.zeros((N, N), bool)
            m[:] = sink_only[i]
            os_, ls_ = dense_masked_attention(q, k, v, m, 0.3)
            l_tot = np.logaddexp(lb[:, :, i], ls_[:, :, i])
            o_tot = (np.exp(lb[:, :, i] - l_tot)[..., None] * ob[:, :, i]
                     + np.exp(ls_[:, :, i] - l_tot)[..., None] * os_[:, :, i])
        else:
            l_tot, o_tot = lb[:, :, i], ob[:, :, i]
        assert np.abs(lse[:, :, i] - l_tot).max() < 1e-12
        assert np.abs(o[:, :, i] - o_tot).max() < 1e-12


# ---------------------------------------------------------------- P8
def test_scale_placement_normalisation_and_convex_hull():
    N, W, S = 40, 9, 2
    q, k, v = make_qkv(1, 2, 1, N, 16, seed=19)
    o, lse = swaa_attn_oracle(q, k, v, W, S, 0.5)
    q2 = f32_to_bf16_bits(2.0 * bf16_bits_to_f32(q))
    o2, lse2 = swaa_attn_oracle(q2, k, v, W, S, 0.25)
    assert np.array_equal(o, o2) and np.array_equal(lse, lse2)
    vf = f64(v)[0, 0]
    assert np.array_equal(o[0, :, 0], np.stack([vf[0], vf[0]]))
    s00 = 0.5 * f64(q)[0, :, 0] @ f64(k)[0, 0, 0]
    assert np.abs(lse[0, :, 0] - s00).max() < 1e-14
    for i in range(N):
        vis = [j for j in range(i + 1) if i - j < W or j < S]
        lo, hi = vf[vis].min(axis=0), vf[vis].max(axis=0)
        assert (o[0, :, i] >= lo - 1e-12).all() and (o[0, :, i] <= hi + 1e-12).all()
    # constant value rows => output is that constant (probabilities sum to one)
    v1 = v.copy()
    v1[:] = f32_to_bf16_bits(np.float32(1.0).reshape(1))[0]
    o1, _ = swaa_attn_oracle(q, k, v1, W, S, 0.5)
    assert np.abs(o1 - 1.0).max() < 1e-14


# ---------------------------------------------------------------- P9
def test_gqa_equals_repeated_heads_and_batches_are_independent():
    B, Hq, Hkv, N, D = 3, 6, 2, 30, 8
    q, k, v = make_qkv(B, Hq, Hkv, N, D, seed=20)
    o, lse = swaa_attn_oracle(q, k, v, 7, 2, 0.35)
    kr, vr = np.repeat(k, 3, axis=1), np.repeat(v, 3, axis=1)
    o2, lse2 = swaa_attn_oracle(q, kr, vr, 7, 2, 0.35)
    assert np.array_equal(o, o2) and np.array_equal(lse, lse2)
    # the two KV heads hold different data, so a wrong head mapping would show
    kw, vw = np.repeat(k[:, ::-1], 3, axis=1), np.repeat(v[:, ::-1], 3, axis=1)
    o3, _ = swaa_attn_oracle(q, kw, vw, 7, 2, 0.35)
    assert not np.allclose(o, o3)
    perm = [2, 0, 1]
    o4, lse4 = swaa_attn_oracle(q[perm], k[perm], v[perm], 7, 2, 0.35)
    assert np.array_equal(o4, o[perm]) and np.array_equal(lse4, lse[perm])


# ---------------------------------------------------------------- P10
def test_planted_sink_is_reachable_only_with_sinks():
    N, D, W = 80, 16, 8
    q, k, v = make_qkv(1, 1, 1, N, D, seed=21)
    kf, qf = bf16_bits_to_f32(k), bf16_bits_to_f32(q)
    qf[..., 0] = 4.0                      # every query points along +e0
    kf[..., 0] = 0.0
    kf[0, 0, 1, 0] = 16.0                 # key 1 is strongly aligned with it
    q, k = f32_to_bf16_bits(qf), f32_to_bf16_bits(kf)
    o_sink, _ = swaa_attn_oracle(q, k, v, W, 2, 1.0)
    o_none, _ = swaa_attn_oracle(q, k, v, W, 0, 1.0)
    v1 = f64(v)[0, 0, 1]
    far = np.arange(1 + W, N)
    assert np.abs(o_sink[0, 0, far] - v1).max() < 1e-6
    assert np.abs(o_none[0, 0, far] - v1).max() > 0.1


def test_bad_arguments_are_rejected():
    q, k, v = make_qkv(1, 2, 1, 8, 4, seed=22)
    with pytest.raises(ValueError):
        swaa_attn_oracle(q, k, v, 0, 0, 1.0)
    with pytest.raises(ValueError):
        swaa_attn_oracle(q, k, v, 4, -1, 1.0)
    with pytest.raises(ValueError):
        swaa_attn_oracle(q, k, v, 4, 0, 1.0, rows=[8])
    with pytest.raises(ValueError):
        swaa_attn_oracle(q[:, :1], np.repeat(k, 2, 1), np.repeat(v, 2, 1), 4, 0, 1.0)


def test_bf16_rounding_helper_matches_torch():
    x = np.random.Generator(np.random.Philox(5)).standard_normal(4096, dtype=np.float32)
    x[:8] = [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40, -2.5]
    ours = f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)
    assert np.array_equal(bf16_bits_to_f32(ours), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_golden_record_of_tiny_workload_is_reproduced():
    """Regression record written by tests/golden/make_golden.py (oracle only)."""
    import os
    from paper_2512_10411_amd.inputs import WORKLOADS, make_workload
    path = os.path.join(os.path.dirname(__file__), "golden", "oracle_tiny_rows.txt")
    recs = [ln.split() for ln in open(path) if not ln.startswith("#")]
    w = WORKLOADS["tiny"]
    q, k, v = make_workload(w)
    rows = sorted({int(r[1]) for r in recs})
    out, lse = swaa_attn_oracle(q, k, v, w.window, w.n_sink, w.scale, rows=rows)
    for h, i, l, o0, o1, o31, o63 in recs:
        h, r = int(h), rows.index(int(i))
        got = [lse[0, h, r], out[0, h, r, 0], out[0, h, r, 1], out[0, h, r, 31], out[0, h, r, 63]]
        want = [float(x) for x in (l, o0, o1, o31, o63)]
        assert np.allclose(got, want, rtol=0, atol=1e-13)
