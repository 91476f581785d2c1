"""GPU parity of swaa_attn_fwd_ex: strided layouts, chunks of a longer prefill (the query
rows are the newest Nq of Nk tokens) and packed variable-length batches, against the fp64
CPU oracle, through the C ABI.  Same tolerances as the prefill tests.
"""
import math

import numpy as np
import pytest
import torch

from oracle import swaa_attn_oracle, swaa_decode_oracle
from paper_2512_10411_amd import binding
from paper_2512_10411_amd.inputs import make_qkv
from gpu_util import assert_parity, to_device

pytestmark = pytest.mark.gpu


def chunk_case(B, Hq, Hkv, Nq, Nk, D, W, S, P, seed):
    tag = f"chunk B{B} Hq{Hq} Hkv{Hkv} Nq{Nq} Nk{Nk} D{D} W{W} S{S} P{P}"
    print(f"[case] {tag} seed {seed}", flush=True)
    q, k, v = make_qkv(B, Hq, Hkv, Nk, D, seed, n_query=Nq)
    scale = 1 / math.sqrt(D)
    out, lse = binding.swaa_attn_fwd_ex(to_device(q), to_device(k), to_device(v), W, S, P, scale)
    torch.cuda.synchronize()
    ro, rl = swaa_decode_oracle(q, k, v, W, S, scale, n_prompt=P)
    assert_parity(out, lse, ro, rl, tag=tag)


@pytest.mark.parametrize("D", [64, 128])
def test_chunks_of_a_longer_prefill(D):
    # row tiles and key tiles out of phase (Nk - Nq not a multiple of 64), tiny and ragged chunks
    for Nq, Nk in ((1, 1), (1, 200), (5, 70), (64, 128), (64, 129), (100, 777), (300, 333), (257, 1500)):
        for W, S in ((1, 0), (50, 4), (64, 70), (Nk, 0)):
            for P in (None, Nk - Nq // 2):
                chunk_case(1, 4, 1, Nq, Nk, D, W, S, P, seed=8000 + Nq + Nk + D)
    chunk_case(2, 10, 2, 150, 900, D, 200, 3, None, seed=8100 + D)


def test_contiguous_arguments_equal_the_plain_call_bit_for_bit():
    q, k, v = make_qkv(2, 6, 2, 700, 128, seed=81)
    qd, kd, vd = to_device(q), to_device(k), to_device(v)
    o0, l0 = binding.swaa_attn_fwd_fa_decode(qd, kd, vd, 100, 4, 650)
    o1, l1 = binding.swaa_attn_fwd_ex(qd, kd, vd, 100, 4, 650)
    torch.cuda.synchronize()
    assert torch.equal(o0, o1) and torch.equal(l0, l1)


@pytest.mark.parametrize("D", [64, 128])
def test_token_major_layout_and_slices(D):
    # [B, N, H, D] tensors passed as permuted views; K and V as slices of one fused buffer
    B, Hq, Hkv, N, W, S = 2, 8, 2, 500, 120, 4
    q, k, v = make_qkv(B, Hq, Hkv, N, D, seed=82 + D)
    ro, rl = swaa_attn_oracle(q, k, v, W, S, 1 / math.sqrt(D))
    q_bnhd = to_device(q).permute(0, 2, 1, 3).contiguous()                      # memory order [B, N, Hq, D]
    kv = torch.stack([to_device(k), to_device(v)], dim=0).permute(1, 3, 0, 2, 4).contiguous()  # [B, N, 2, Hkv, D]
    k_view = kv[:, :, 0].permute(0, 2, 1, 3)   # [B, Hkv, N, D] view, row stride 2*Hkv*D
    v_view = kv[:, :, 1].permute(0, 2, 1, 3)
    out, lse = binding.swaa_attn_fwd_ex(q_bnhd.permute(0, 2, 1, 3), k_view, v_view, W, S)
    torch.cuda.synchronize()
    assert out.stride() == q_bnhd.permute(0, 2, 1, 3).stride()  # written in the caller's memory order
    assert_parity(out.contiguous(), lse, ro, rl, tag=f"token-major layout D{D}")
    # a window of heads and rows out of a larger allocation
    big = torch.zeros((B, Hq + 2, N + 16, D), dtype=torch.bfloat16, device="cuda")
    big[:, 1:1 + Hq, 8:8 + N] = to_device(q)
    out2, lse2 = binding.swaa_attn_fwd_ex(big[:, 1:1 + Hq, 8:8 + N], to_device(k), to_device(v), W, S)
    torch.cuda.synchronize()
    assert torch.equal(out2.contiguous(), out.contiguous()) and torch.equal(lse2, lse)


@pytest.mark.parametrize("D,chunked", [(128, False), (128, True), (64, True)])
def test_packed_variable_length_batch(D, chunked):
    Hq, Hkv, W, S = 8, 2, 100, 4
    lens_k = [1, 63, 64, 65, 300, 1000, 2, 517]
    lens_q = [max(1, n // 3) for n in lens_k] if chunked else list(lens_k)
    rng = np.random.Generator(np.random.Philox(83 + D))
    cu_q = np.concatenate([[0], np.cumsum(lens_q)]).astype(np.int32)
    cu_k = np.concatenate([[0], np.cumsum(lens_k)]).astype(np.int32)
    seqs = [make_qkv(1, Hq, Hkv, nk, D, int(rng.integers(1 << 30)), n_query=nq) for nq, nk in zip(lens_q, lens_k)]
    # packed token-major buffers [T, H, D]
    q_pack = torch.cat([to_device(s[0])[0].permute(1, 0, 2) for s in seqs], dim=0).contiguous()
    k_pack = torch.cat([to_device(s[1])[0].permute(1, 0, 2) for s in seqs], dim=0).contiguous()
    v_pack = torch.cat([to_device(s[2])[0].permute(1, 0, 2) for s in seqs], dim=0).contiguous()
    P = None if not chunked else 400
    out, lse = binding.swaa_attn_fwd_ex(
        q_pack.permute(1, 0, 2), k_pack.permute(1, 0, 2), v_pack.permute(1, 0, 2), W, S, P,
        cu_seqlens_q=torch.from_numpy(cu_q).cuda(), cu_seqlens_k=torch.from_numpy(cu_k).cuda(),
        max_seqlen_q=max(lens_q), max_seqlen_k=max(lens_k))
    torch.cuda.synchronize()
    assert out.shape == (Hq, int(cu_q[-1]), D) and lse.shape == (Hq, int(cu_q[-1]))
    for b, (qs, ks, vs) in enumerate(seqs):
        ro, rl = swaa_decode_oracle(qs, ks, vs, W, S, 1 / math.sqrt(D), n_prompt=P)
        o_b = out[:, cu_q[b]:cu_q[b + 1]].unsqueeze(0)
        l_b = lse[:, cu_q[b]:cu_q[b + 1]].unsqueeze(0)
        assert_parity(o_b, l_b, ro, rl, tag=f"packed seq {b}: Nq{lens_q[b]} Nk{lens_k[b]} D{D}")


def test_chunk_against_a_long_cache_full_size():
    # the benchmark's chunk workload, launched exactly as it is timed: one 2048-row chunk of a
    # 128k-token prefill, window 8192 + 4 sinks, Hq 32 / Hkv 8; every output row is compared
    from paper_2512_10411_amd.inputs import WORKLOADS, make_workload
    w = WORKLOADS["chunk2k_128k_swa"]
    print("[gen] chunk vs 128k cache ...", flush=True)
    q, k, v = make_workload(w)
    print("[gpu]", flush=True)
    out, lse = binding.swaa_attn_fwd_ex(to_device(q), to_device(k), to_device(v), w.window, w.n_sink, w.n_prompt,
                                        w.scale)
    torch.cuda.synchronize()
    print("[oracle]", flush=True)
    ro, rl = swaa_decode_oracle(q, k, v, w.window, w.n_sink, w.scale)
    assert_parity(out, lse, ro, rl, tag="2048-row chunk on a 128k cache")


def build_paged_cache(host_kv, lens, page_size, Hkv, D, rng):
    """Scatter each sequence's [1, Hkv, n, D] keys and values into pages in a random order;
    returns the cache views [num_pages, Hkv, page_size, D] and the block table."""
    B = len(lens)
    pages_per_seq = -(-max(lens) // page_size)
    num_pages = B * pages_per_seq + 3
    order = rng.permutation(num_pages)
    kc = torch.full((num_pages, page_size, Hkv, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros((num_pages, page_size, Hkv, D), dtype=torch.bfloat16, device="cuda")
    table = np.full((B, pages_per_seq), -7, dtype=np.int32)  # unused entries hold a bad page number
    nxt = 0
    for b, (k, v) in enumerate(host_kv):
        kt, vt = to_device(k)[0].permute(1, 0, 2), to_device(v)[0].permute(1, 0, 2)  # [n, Hkv, D]
        for pg in range(-(-lens[b] // page_size)):
            page = int(order[nxt]); nxt += 1
            table[b, pg] = page
            t0, t1 = pg * page_size, min(lens[b], (pg + 1) * page_size)
            kc[page, :t1 - t0], vc[page, :t1 - t0] = kt[t0:t1], vt[t0:t1]
            kc[page, t1 - t0:] = 0  # rows of a page past the sequence's end: finite, never visible
    return kc.permute(0, 2, 1, 3), vc.permute(0, 2, 1, 3), torch.from_numpy(table).cuda()


@pytest.mark.parametrize("page_size", [16, 32, 64, 256])
def test_chunked_prefill_over_a_paged_cache(page_size):
    # the query rows are the newest Nq of Nk cached tokens; pages in random order; cache lengths
    # on and off every alignment; whole prefills (Nq = Nk) as well
    rng = np.random.Generator(np.random.Philox(8800 + page_size))
    D, Hq, Hkv = 128, 8, 2
    for Nq, Nk, W, S, P in ((1, 1, 5, 0, None), (5, 70, 50, 4, None), (64, 129, 64, 70, None), (100, 777, 200, 4, None),
                            (300, 333, 1000, 0, None), (257, 1500, 300, 33, 1400), (700, 700, 128, 4, None),
                            (129, 2049, 2049, 0, None)):
        B = 2
        tag = f"paged prefill page{page_size} B{B} Nq{Nq} Nk{Nk} W{W} S{S} P{P}"
        print(f"[case] {tag}", flush=True)
        host = [make_qkv(1, Hq, Hkv, Nk, D, 8900 + 7 * i + Nk + page_size, n_query=Nq) for i in range(B)]
        kc, vc, table = build_paged_cache([(h[1], h[2]) for h in host], [Nk] * B, page_size, Hkv, D, rng)
        qd = torch.cat([to_device(h[0]) for h in host], dim=0)
        out, lse = binding.swaa_attn_fwd_ex(qd, kc, vc, W, S, P, block_table=table, max_seqlen_k=Nk)
        torch.cuda.synchronize()
        for b, (q, k, v) in enumerate(host):
            ro, rl = swaa_decode_oracle(q, k, v, W, S, 1 / math.sqrt(D), n_prompt=P)
            assert_parity(out[b:b + 1], lse[b:b + 1], ro, rl, tag=f"{tag} / seq {b}")


def test_packed_chunks_over_a_paged_cache_with_different_lengths():
    # packed query rows (cu_seqlens_q), cache lengths from cu_seqlens_k's differences, keys from the block table
    rng = np.random.Generator(np.random.Philox(8850))
    D, Hq, Hkv, page_size, W, S = 128, 4, 1, 32, 100, 4
    nq = [1, 63, 300, 64, 17]
    nk = [1, 500, 300, 1000, 77]
    host = [make_qkv(1, Hq, Hkv, nk[i], D, 8860 + i, n_query=nq[i]) for i in range(len(nq))]
    kc, vc, table = build_paged_cache([(h[1], h[2]) for h in host], nk, page_size, Hkv, D, rng)
    q_packed = torch.cat([to_device(h[0])[0] for h in host], dim=1)  # [Hq, sum nq, D]
    cu_q = torch.tensor(np.concatenate([[0], np.cumsum(nq)]), dtype=torch.int32, device="cuda")
    cu_k = torch.tensor(np.concatenate([[0], np.cumsum(nk)]), dtype=torch.int32, device="cuda")
    out, lse = binding.swaa_attn_fwd_ex(q_packed, kc, vc, W, S, None, cu_seqlens_q=cu_q, cu_seqlens_k=cu_k,
                                        max_seqlen_q=max(nq), max_seqlen_k=max(nk), block_table=table)
    torch.cuda.synchronize()
    r0 = 0
    for b, (q, k, v) in enumerate(host):
        ro, rl = swaa_decode_oracle(q, k, v, W, S, 1 / math.sqrt(D))
        assert_parity(out[None, :, r0:r0 + nq[b]], lse[None, :, r0:r0 + nq[b]], ro, rl, tag=f"packed paged seq {b}")
        r0 += nq[b]


@pytest.mark.parametrize("page_size", [16, 48, 256])
def test_paged_prefill_equals_the_contiguous_call_bit_for_bit(page_size):
    # long unmasked stretches of the band, where the paged kernel asks for its block-table
    # entries one step ahead: same arithmetic as the contiguous kernel, so the same bits
    B, Hq, Hkv, N, D = 2, 10, 2, 6144, 128
    gen = torch.Generator(device="cuda").manual_seed(8870 + page_size)
    q = torch.randn((B, Hq, N, D), device="cuda", dtype=torch.bfloat16, generator=gen)
    k = torch.randn((B, Hkv, N, D), device="cuda", dtype=torch.bfloat16, generator=gen)
    v = torch.randn((B, Hkv, N, D), device="cuda", dtype=torch.bfloat16, generator=gen)
    npg = N // page_size
    perm = torch.randperm(B * npg + 5, device="cuda", generator=gen)[:B * npg]
    table = perm.view(B, npg).to(torch.int32)
    kc = torch.full((B * npg + 5, Hkv, page_size, D), float("nan"), device="cuda", dtype=torch.bfloat16)
    vc = torch.zeros_like(kc)
    kc[perm] = k.view(B, Hkv, npg, page_size, D).permute(0, 2, 1, 3, 4).reshape(B * npg, Hkv, page_size, D)
    vc[perm] = v.view(B, Hkv, npg, page_size, D).permute(0, 2, 1, 3, 4).reshape(B * npg, Hkv, page_size, D)
    for W, S, P in ((1500, 4, None), (N, 0, None), (700, 100, 6000)):
        o1, l1 = binding.swaa_attn_fwd_ex(q, k, v, W, S, P)
        o2, l2 = binding.swaa_attn_fwd_ex(q, kc, vc, W, S, P, block_table=table, max_seqlen_k=N)
        torch.cuda.synchronize()
        assert torch.equal(o1, o2) and torch.equal(l1, l2), (page_size, W, S, P)


@pytest.mark.parametrize("D", [128, 64])
def test_packed_batch_of_many_sequences_of_very_different_lengths(D):
    # 150 sequences (three rounds of 64 in the work-list search), lengths from 1 to 3000 rows, some
    # of them chunks of longer caches; the compact work list against the launch of B x longest
    # sequence (same bits) and against the oracle
    Hq, Hkv, W, S, B = 10, 2, 200, 4, 150
    rng = np.random.Generator(np.random.Philox(8890 + D))
    lens_k = [int(x) for x in rng.integers(1, 120, size=B)]
    for i in (3, 70, 149):
        lens_k[i] = int(rng.integers(1500, 3000))
    lens_q = [n if rng.integers(0, 3) else max(1, n // 2) for n in lens_k]
    cu_q = np.concatenate([[0], np.cumsum(lens_q)]).astype(np.int32)
    cu_k = np.concatenate([[0], np.cumsum(lens_k)]).astype(np.int32)
    seqs = [make_qkv(1, Hq, Hkv, nk, D, int(rng.integers(1 << 30)), n_query=None if nq == nk else nq)
            for nq, nk in zip(lens_q, lens_k)]
    q_pack = torch.cat([to_device(s[0])[0].permute(1, 0, 2) for s in seqs], dim=0).contiguous()
    k_pack = torch.cat([to_device(s[1])[0].permute(1, 0, 2) for s in seqs], dim=0).contiguous()
    v_pack = torch.cat([to_device(s[2])[0].permute(1, 0, 2) for s in seqs], dim=0).contiguous()
    args = dict(cu_seqlens_q=torch.from_numpy(cu_q).cuda(), cu_seqlens_k=torch.from_numpy(cu_k).cuda(),
                max_seqlen_q=max(lens_q), max_seqlen_k=max(lens_k))
    out, lse = binding.swaa_attn_fwd_ex(q_pack.permute(1, 0, 2), k_pack.permute(1, 0, 2), v_pack.permute(1, 0, 2), W, S, None, **args)
    o0, l0 = binding.swaa_attn_fwd_ex(q_pack.permute(1, 0, 2), k_pack.permute(1, 0, 2), v_pack.permute(1, 0, 2), W, S, None,
                                      total_rows_q=0, **args)
    torch.cuda.synchronize()
    assert torch.equal(out, o0) and torch.equal(lse, l0)
    for b, (qs, ks, vs) in enumerate(seqs):
        ro, rl = swaa_decode_oracle(qs, ks, vs, W, S, 1 / math.sqrt(D))
        assert_parity(out[:, cu_q[b]:cu_q[b + 1]].unsqueeze(0), lse[:, cu_q[b]:cu_q[b + 1]].unsqueeze(0), ro, rl,
                      tag=f"packed, 150 sequences, seq {b}: Nq{lens_q[b]} Nk{lens_k[b]} D{D}")


@pytest.mark.parametrize("D", [128, 64])
def test_packed_batch_with_empty_sequences(D):
    # sequences without tokens, and sequences with cached keys but no new rows, between the others:
    # they take no work items and leave the neighbours' rows alone (both work lists)
    Hq, Hkv, W, S = 8, 2, 50, 4
    lens_k = [0, 5, 0, 0, 130, 40, 0, 257, 0]
    lens_q = [0, 5, 0, 0, 130, 0, 0, 100, 0]
    rng = np.random.Generator(np.random.Philox(8900 + D))
    cu_q = np.concatenate([[0], np.cumsum(lens_q)]).astype(np.int32)
    cu_k = np.concatenate([[0], np.cumsum(lens_k)]).astype(np.int32)
    seqs = [make_qkv(1, Hq, Hkv, max(nk, 1), D, int(rng.integers(1 << 30)), n_query=max(nq, 1)) for nq, nk in zip(lens_q, lens_k)]
    q_pack = torch.cat([to_device(s[0])[0, :, :nq] for s, nq in zip(seqs, lens_q)], dim=1).contiguous()   # [Hq, Tq, D]
    k_pack = torch.cat([to_device(s[1])[0, :, :nk] for s, nk in zip(seqs, lens_k)], dim=1).contiguous()
    v_pack = torch.cat([to_device(s[2])[0, :, :nk] for s, nk in zip(seqs, lens_k)], dim=1).contiguous()
    args = dict(cu_seqlens_q=torch.from_numpy(cu_q).cuda(), cu_seqlens_k=torch.from_numpy(cu_k).cuda(),
                max_seqlen_q=max(lens_q), max_seqlen_k=max(lens_k))
    for total in (None, 0):
        out = torch.full_like(q_pack, 7.0)
        lse = torch.full((Hq, q_pack.shape[1]), 7.0, dtype=torch.float32, device="cuda")
        binding.swaa_attn_fwd_ex(q_pack, k_pack, v_pack, W, S, None, out=out, lse=lse, total_rows_q=total, **args)
        torch.cuda.synchronize()
        for b, (qs, ks, vs) in enumerate(seqs):
            if lens_q[b] == 0:
                continue
            ro, rl = swaa_decode_oracle(qs, ks, vs, W, S, 1 / math.sqrt(D))
            assert_parity(out[:, cu_q[b]:cu_q[b + 1]].unsqueeze(0), lse[:, cu_q[b]:cu_q[b + 1]].unsqueeze(0), ro, rl,
                          tag=f"packed with empty sequences (rows stated: {total}), seq {b}")
