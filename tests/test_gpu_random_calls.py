"""Seeded random calls of every entry point against the fp64 CPU oracle (GPU).

Shapes, masks and layouts are drawn from a seeded generator, so every run tests the same
cases; the point is coverage of parameter combinations the hand-written cases do not list.
"""
import math

import numpy as np
import pytest
import torch

from oracle import swaa_attn_bwd_oracle, swaa_attn_oracle, swaa_decode_oracle
from paper_2512_10411_amd import binding
from paper_2512_10411_amd.inputs import f32_to_bf16_bits, make_qkv
from gpu_util import assert_parity, to_device

pytestmark = pytest.mark.gpu


def draw_mask(rng, n):
    W = int(rng.choice([1, 2, 31, 32, 33, 64, 100, 257, n, n + 3, 10**9]))
    S = int(rng.choice([0, 0, 1, 4, 33, 64, 100, n + 1]))
    P = rng.choice([None, 0, n // 3, n - 1, n]) if n > 1 else None
    return W, S, (None if P is None else int(P))


@pytest.mark.parametrize("seed", range(12))
def test_random_forward_calls(seed):
    rng = np.random.Generator(np.random.Philox(31000 + seed))
    D = int(rng.choice([64, 128]))
    Hkv = int(rng.integers(1, 4))
    G = int(rng.integers(1, 7))
    B = int(rng.integers(1, 3))
    Nk = int(rng.integers(1, 1400))
    chunk = bool(rng.integers(0, 2))
    Nq = int(rng.integers(1, Nk + 1)) if chunk else Nk
    W, S, P = draw_mask(rng, Nk)
    token_major = bool(rng.integers(0, 2))
    tag = f"random fwd seed {seed}: B{B} G{G} Hkv{Hkv} Nq{Nq} Nk{Nk} D{D} W{W} S{S} P{P} token_major={token_major}"
    print(f"[case] {tag}", flush=True)
    q, k, v = make_qkv(B, Hkv * G, Hkv, Nk, D, 32000 + seed, n_query=None if Nq == Nk else Nq)
    qd, kd, vd = to_device(q), to_device(k), to_device(v)
    if token_major:  # [B, N, H, D] memory order, passed as views
        qd, kd, vd = (t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for t in (qd, kd, vd))
    # (no scale above 1/sqrt(D): hotter softmaxes push |o| past 4, where the bf16 output's own
    # half-ulp is 1.6e-2 and the acceptance bar of 2e-2 is no longer the right yardstick)
    scale = float(rng.choice([1 / math.sqrt(D), 0.05, 0.02]))
    out, lse = binding.swaa_attn_fwd_ex(qd, kd, vd, W, S, P, scale)
    torch.cuda.synchronize()
    ro, rl = swaa_decode_oracle(q, k, v, W, S, scale, n_prompt=P)
    assert_parity(out.contiguous(), lse, ro, rl, tag=tag)


@pytest.mark.parametrize("seed", range(8))
def test_random_decode_calls(seed):
    rng = np.random.Generator(np.random.Philox(33000 + seed))
    Hkv, G, B = int(rng.integers(1, 4)), int(rng.integers(1, 9)), int(rng.integers(1, 4))
    Nq = int(rng.choice([1, 1, 2, 4, 9]))
    lens = [int(rng.integers(Nq, 4000)) for _ in range(B)]
    W = int(rng.choice([1, 64, 500, 10**9]))
    S = int(rng.choice([0, 4, 100]))
    page_size = int(rng.choice([0, 4, 16, 32, 256]))  # 0: contiguous cache
    tag = f"random decode seed {seed}: B{B} G{G} Hkv{Hkv} Nq{Nq} lens{lens} W{W} S{S} page{page_size}"
    print(f"[case] {tag}", flush=True)
    D, Hq = 128, Hkv * G
    host = [make_qkv(1, Hq, Hkv, n, D, 34000 + 10 * seed + i, n_query=Nq) for i, n in enumerate(lens)]
    qd = torch.cat([to_device(s[0]) for s in host], dim=0)
    seq_lens = torch.tensor(lens, dtype=torch.int32, device="cuda")
    max_len = max(lens)
    if page_size:
        pages_per_seq = -(-max_len // page_size)
        num_pages = B * pages_per_seq + 2
        order = rng.permutation(num_pages)
        kc = torch.zeros((num_pages, page_size, Hkv, D), dtype=torch.bfloat16, device="cuda")
        vc = torch.zeros_like(kc)
        table = np.zeros((B, pages_per_seq), dtype=np.int32)
        nxt = 0
        for b, (_, k, v) in enumerate(host):
            kt, vt = to_device(k)[0].permute(1, 0, 2), to_device(v)[0].permute(1, 0, 2)  # [n, Hkv, D]
            for pg in range(-(-lens[b] // page_size)):
                page = int(order[nxt]); nxt += 1
                table[b, pg] = page
                t0, t1 = pg * page_size, min(lens[b], (pg + 1) * page_size)
                kc[page, :t1 - t0], vc[page, :t1 - t0] = kt[t0:t1], vt[t0:t1]
        out, lse = binding.swaa_attn_decode_ex(qd, kc.permute(0, 2, 1, 3), vc.permute(0, 2, 1, 3), W, S,
                                               seq_lens=seq_lens, block_table=torch.from_numpy(table).cuda(),
                                               max_seqlen_k=max_len)
    else:
        kb = torch.zeros((B, Hkv, max_len, D), dtype=torch.bfloat16, device="cuda")
        vb = torch.zeros_like(kb)
        for b, (_, k, v) in enumerate(host):
            kb[b, :, :lens[b]], vb[b, :, :lens[b]] = to_device(k)[0], to_device(v)[0]
        out, lse = binding.swaa_attn_decode_ex(qd, kb, vb, W, S, seq_lens=seq_lens)
    torch.cuda.synchronize()
    for b, (qs, ks, vs) in enumerate(host):
        ro, rl = swaa_decode_oracle(qs, ks, vs, W, S, 1 / math.sqrt(D))
        assert_parity(out[b:b + 1], lse[b:b + 1], ro, rl, tag=f"{tag} / seq {b}")


@pytest.mark.parametrize("seed", range(6))
def test_random_backward_calls(seed):
    rng = np.random.Generator(np.random.Philox(35000 + seed))
    D = int(rng.choice([64, 128]))
    Hkv, G, B = int(rng.integers(1, 3)), int(rng.integers(1, 6)), int(rng.integers(1, 3))
    N = int(rng.integers(2, 900))
    W, S, P = draw_mask(rng, N)
    W = max(W, 2)  # W = 1 has zero dQ, dK: covered by its own test
    tag = f"random bwd seed {seed}: B{B} G{G} Hkv{Hkv} N{N} D{D} W{W} S{S} P{P}"
    print(f"[case] {tag}", flush=True)
    q, k, v = make_qkv(B, Hkv * G, Hkv, N, D, 36000 + seed)
    dout = f32_to_bf16_bits(np.random.Generator(np.random.Philox(37000 + seed)).standard_normal(q.shape, dtype=np.float32))
    qd, kd, vd, dd = to_device(q), to_device(k), to_device(v), to_device(dout)
    scale = 1 / math.sqrt(D)
    n_prompt = N if P is None else P
    out, lse = binding.swaa_attn_fwd_fa_decode(qd, kd, vd, W, S, n_prompt, scale)
    dq, dk, dv = binding.swaa_attn_bwd(qd, kd, vd, out, lse, dd, W, S, n_prompt, scale)
    torch.cuda.synchronize()
    rq, rk, rv = swaa_attn_bwd_oracle(q, k, v, dout, W, S, scale, n_prompt=n_prompt)
    from test_gpu_bwd import assert_grad
    assert_grad("dq", dq, rq, tag)
    assert_grad("dk", dk, rk, tag)
    assert_grad("dv", dv, rv, tag)


def _paged(host_kv, lens, ps, Hkv, D, dt, rng):
    """The sequences' keys and values as a paged cache (pages in random order, unused slots hold
    noise, unused table entries point outside the cache); returns (k_cache, v_cache, block_table)."""
    pages_of = [-(-n // ps) for n in lens]
    order = rng.permutation(sum(pages_of) + 2)
    kc = torch.randn((len(order), ps, Hkv, D), device="cuda").to(dt)
    vc = torch.randn((len(order), ps, Hkv, D), device="cuda").to(dt)
    table = np.full((len(lens), max(pages_of) + 1), 10**6, dtype=np.int32)
    nxt = 0
    for b, (kb, vb) in enumerate(host_kv):
        for pg in range(pages_of[b]):
            page = int(order[nxt]); nxt += 1
            table[b, pg] = page
            t0, t1 = pg * ps, min(lens[b], (pg + 1) * ps)
            kc[page, :t1 - t0] = kb[:, t0:t1].permute(1, 0, 2)
            vc[page, :t1 - t0] = vb[:, t0:t1].permute(1, 0, 2)
    return kc.permute(0, 2, 1, 3), vc.permute(0, 2, 1, 3), torch.from_numpy(table).cuda()


@pytest.mark.parametrize("seed", range(12))
def test_random_decode_batches_with_sequence_lengths(seed):
    # batches of up to 130 sequences with uniform, one-long-among-short and heavy-tailed lengths,
    # contiguous and paged, both formats; three calls must give the same bits (the split plan is
    # worked out on the device by every workgroup)
    from oracle import input_format
    from gpu_util import errors
    rng = np.random.Generator(np.random.Philox(61000 + seed))
    Hkv, G = int(rng.integers(1, 3)), int(rng.choice([1, 2, 4, 5, 8]))
    B, Nq = int(rng.choice([2, 3, 7, 16, 64, 65, 130])), int(rng.choice([1, 1, 1, 2, 5, 9, 17]))
    kind = seed % 3
    if kind == 0:
        lens = [int(x) for x in rng.integers(Nq, 400, size=B)]
    elif kind == 1:
        lens = [int(x) for x in rng.integers(Nq, 60, size=B)]
        lens[int(rng.integers(0, B))] = int(rng.integers(2000, 9000))
    else:
        lens = [int(min(6000, Nq + rng.pareto(1.0) * 50)) for _ in range(B)]
    W, S = int(rng.choice([1, 33, 100, 1000, 10**9, 10**9])), int(rng.choice([0, 4, 64, 100]))
    fmt = "fp16" if rng.integers(0, 4) == 0 else "bf16"
    dt = torch.float16 if fmt == "fp16" else torch.bfloat16
    paged, ps = bool(rng.integers(0, 2)), int(rng.choice([4, 16, 32, 48]))
    print(f"[case] seed {seed}: B{B} G{G} Hkv{Hkv} Nq{Nq} lengths {min(lens)}..{max(lens)} W{W} S{S} {fmt} paged {paged} ({ps})", flush=True)
    host = [make_qkv(1, Hkv * G, Hkv, n, 128, 62000 + 1000 * seed + i, n_query=Nq, fmt=fmt) for i, n in enumerate(lens)]
    q = torch.cat([to_device(h[0], fmt) for h in host], dim=0)
    dev_kv = [(to_device(h[1], fmt)[0], to_device(h[2], fmt)[0]) for h in host]
    sl = torch.tensor(lens, dtype=torch.int32, device="cuda")
    if paged:
        kc, vc, table = _paged(dev_kv, lens, ps, Hkv, 128, dt, rng)
        call = lambda: binding.swaa_attn_decode_ex(q, kc, vc, W, S, seq_lens=sl, block_table=table, max_seqlen_k=max(lens))
    else:
        kbuf = torch.randn((B, Hkv, max(lens), 128), device="cuda").to(dt)
        vbuf = torch.randn((B, Hkv, max(lens), 128), device="cuda").to(dt)
        for b, (kb, vb) in enumerate(dev_kv):
            kbuf[b, :, :lens[b]], vbuf[b, :, :lens[b]] = kb, vb
        call = lambda: binding.swaa_attn_decode_ex(q, kbuf, vbuf, W, S, seq_lens=sl)
    outs = [tuple(t.clone() for t in call()) for _ in range(3)]
    torch.cuda.synchronize()
    assert all(torch.equal(outs[0][0], o) and torch.equal(outs[0][1], l) for o, l in outs[1:])
    worst = [0.0, 0.0, 0.0]
    with input_format(fmt):
        for b, h in enumerate(host):
            ro, rl = swaa_decode_oracle(h[0], h[1], h[2], W, S, 1 / math.sqrt(128))
            worst = [max(a, c) for a, c in zip(worst, errors(outs[0][0][b:b + 1], outs[0][1][b:b + 1], ro, rl))]
    print(f"[parity] seed {seed}: O max-abs {worst[0]:.3e} mean-abs(max) {worst[1]:.3e} LSE {worst[2]:.3e}", flush=True)
    assert worst[0] <= 2e-2 and worst[1] <= 2e-3 and worst[2] <= 1e-3


@pytest.mark.parametrize("seed", range(12))
def test_random_packed_batches(seed):
    # packed prefill batches of up to 70 sequences with heavy-tailed lengths: plain prefills and
    # chunks against longer caches, sequences without new rows, contiguous and paged caches,
    # per-sequence prompt lengths, head dimensions 64 / 96 / 128; the compact work list (twice) and
    # the plain one must give the same bits
    from oracle import input_format
    from gpu_util import errors
    rng = np.random.Generator(np.random.Philox(71000 + seed))
    D, Hkv, G = int(rng.choice([128, 128, 128, 64, 96])), int(rng.integers(1, 3)), int(rng.choice([1, 2, 4, 5, 8]))
    B = int(rng.choice([1, 2, 5, 9, 64, 70]))
    nk = [int(min(3000, 1 + rng.pareto(1.0) * 40)) for _ in range(B)]
    if rng.integers(0, 2):
        nk[int(rng.integers(0, B))] = int(rng.integers(500, 3000))
    nq = [n if rng.integers(0, 2) else int(rng.integers(1, n + 1)) for n in nk]
    for i in range(B):
        if rng.integers(0, 8) == 0:
            nq[i] = 0   # no new rows
    if sum(nq) == 0:
        nq[0] = nk[0]
    W, S = int(rng.choice([1, 33, 100, 1000, 10**9])), int(rng.choice([0, 4, 64]))
    prompts = [int(rng.integers(0, n + 2)) for n in nk] if rng.integers(0, 2) else None
    fmt = "fp16" if rng.integers(0, 4) == 0 else "bf16"
    dt = torch.float16 if fmt == "fp16" else torch.bfloat16
    paged, ps = D == 128 and bool(rng.integers(0, 2)), int(rng.choice([16, 32, 48]))
    print(f"[case] seed {seed}: D{D} B{B} G{G} Hkv{Hkv} rows {sum(nq)} caches {min(nk)}..{max(nk)} W{W} S{S} {fmt} "
          f"paged {paged} ({ps}) prompts {prompts is not None}", flush=True)
    host = [make_qkv(1, Hkv * G, Hkv, nk[i], D, 72000 + 1000 * seed + i, n_query=max(nq[i], 1), fmt=fmt) for i in range(B)]
    q_pack = torch.cat([to_device(h[0], fmt)[0, :, :nq[i]] for i, h in enumerate(host)], dim=1).contiguous()
    args = dict(cu_seqlens_q=torch.tensor(np.concatenate([[0], np.cumsum(nq)]), dtype=torch.int32, device="cuda"),
                cu_seqlens_k=torch.tensor(np.concatenate([[0], np.cumsum(nk)]), dtype=torch.int32, device="cuda"),
                max_seqlen_q=max(max(nq), 1), max_seqlen_k=max(nk))
    if prompts is not None:
        args["n_prompts"] = torch.tensor(prompts, dtype=torch.int32, device="cuda")
    dev_kv = [(to_device(h[1], fmt)[0], to_device(h[2], fmt)[0]) for h in host]
    if paged:
        kk, vv, args["block_table"] = _paged(dev_kv, nk, ps, Hkv, D, dt, rng)
    else:
        kk = torch.cat([kv[0] for kv in dev_kv], dim=1).contiguous()
        vv = torch.cat([kv[1] for kv in dev_kv], dim=1).contiguous()
    outs = [tuple(t.clone() for t in binding.swaa_attn_fwd_ex(q_pack, kk, vv, W, S, None, total_rows_q=total, **args))
            for total in (None, None, 0)]
    torch.cuda.synchronize()
    assert all(torch.equal(outs[0][0], o) and torch.equal(outs[0][1], l) for o, l in outs[1:])
    worst, r0 = [0.0, 0.0, 0.0], 0
    with input_format(fmt):
        for b, h in enumerate(host):
            if nq[b] == 0:
                continue
            ro, rl = swaa_decode_oracle(h[0], h[1], h[2], W, S, 1 / math.sqrt(D), n_prompt=None if prompts is None else prompts[b])
            e = errors(outs[0][0][None, :, r0:r0 + nq[b]], outs[0][1][None, :, r0:r0 + nq[b]], ro, rl)
            worst = [max(a, c) for a, c in zip(worst, e)]
            r0 += nq[b]
    print(f"[parity] seed {seed}: O max-abs {worst[0]:.3e} mean-abs(max) {worst[1]:.3e} LSE {worst[2]:.3e}", flush=True)
    assert worst[0] <= 2e-2 and worst[1] <= 2e-3 and worst[2] <= 1e-3
