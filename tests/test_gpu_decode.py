"""GPU parity of swaa_attn_decode (the newest tokens against a KV cache; split keys,
merged by a second kernel) against the fp64 CPU oracle, through the C ABI.  Same
tolerances as the prefill tests.
"""
import math

import numpy as np
import pytest
import torch

from oracle import input_format, swaa_decode_oracle
from paper_2512_10411_amd import binding
from paper_2512_10411_amd.inputs import (WORKLOADS, bf16_bits_to_f32, f32_to_bf16_bits, make_qkv, make_workload,
                                          paged_cache)
from gpu_util import assert_parity, to_device

pytestmark = pytest.mark.gpu


def check(B, Hq, Hkv, Nq, Nk, W, S, seed, D=128):
    scale = 1.0 / math.sqrt(D)
    tag = f"decode B{B} Hq{Hq} Hkv{Hkv} Nq{Nq} Nk{Nk} W{W} S{S}"
    print(f"[case] {tag} seed {seed}", flush=True)
    q, k, v = make_qkv(B, Hq, Hkv, Nk, D, seed, n_query=Nq)
    out, lse = binding.swaa_attn_decode(to_device(q), to_device(k), to_device(v), W, S, scale)
    torch.cuda.synchronize()
    ro, rl = swaa_decode_oracle(q, k, v, W, S, scale)
    assert_parity(out, lse, ro, rl, tag=tag)


@pytest.mark.parametrize("Nk", [1, 31, 32, 33, 100, 129, 700, 3000])
def test_small_caches_sweep_rows_window_and_sinks(Nk):
    # one split and many, ragged last half, more query rows than one column tile holds
    seed = 7000 + Nk
    for Nq in (1, 2, 5, 8, 17):
        if Nq > Nk:
            continue
        for W, S in ((1, 0), (7, 4), (64, 0), (200, 70), (Nk, 0), (Nk + 9, 3)):
            check(1, 4, 1, Nq, Nk, W, S, seed)


@pytest.mark.parametrize("G", [1, 2, 3, 5, 8])
def test_gqa_group_sizes_and_batches(G):
    check(3, 2 * G, 2, 3, 1111, 300, 3, seed=7100 + G)
    check(2, G, 1, 1, 2050, 2050, 0, seed=7200 + G)


def test_score_spike_deep_in_the_cache():
    # the reference of a split follows its keys; a score tens of nats above the rest must merge correctly
    B, Hq, Hkv, Nq, Nk, D = 1, 4, 1, 2, 5000, 128
    q, k, v = make_qkv(B, Hq, Hkv, Nk, D, seed=73, n_query=Nq)
    qf, kf = bf16_bits_to_f32(q), bf16_bits_to_f32(k)
    qf[..., 0] = 3.0
    kf[..., 0] = 0.0
    kf[:, :, 3333, 0] = 160.0
    kf[:, :, 4000, 0] = -160.0
    q, k = f32_to_bf16_bits(qf), f32_to_bf16_bits(kf)
    scale = 1 / math.sqrt(D)
    for W, S in ((Nk, 0), (512, 4)):
        out, lse = binding.swaa_attn_decode(to_device(q), to_device(k), to_device(v), W, S, scale)
        torch.cuda.synchronize()
        ro, rl = swaa_decode_oracle(q, k, v, W, S, scale)
        assert_parity(out, lse, ro, rl, tag=f"decode spike W{W}")


def test_caller_workspace_stream_and_errors():
    B, Hq, Hkv, Nq, Nk, D, W, S = 2, 8, 2, 1, 4000, 128, 4000, 0
    q, k, v = make_qkv(B, Hq, Hkv, Nk, D, seed=74, n_query=Nq)
    qd, kd, vd = to_device(q), to_device(k), to_device(v)
    need = binding.swaa_attn_decode_workspace_bytes(B, Hq, Hkv, Nq, Nk, D, W, S)
    assert need > 0
    ws = torch.full((need,), 0xFF, dtype=torch.uint8, device="cuda")  # NaN bit patterns: stale reads would show
    out = torch.full_like(qd, 7.0)
    lse = torch.full((B, Hq, Nq), 7.0, dtype=torch.float32, device="cuda")
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    ro, rl = swaa_decode_oracle(q, k, v, W, S, 1 / math.sqrt(D))
    with torch.cuda.stream(s):
        for _ in range(2):  # the second call reuses the workspace the first one left
            o2, l2 = binding.swaa_attn_decode(qd, kd, vd, W, S, out=out, lse=lse, workspace=ws, stream=s)
    s.synchronize()
    assert o2.data_ptr() == out.data_ptr() and l2.data_ptr() == lse.data_ptr()
    assert_parity(out, lse, ro, rl, tag="decode, caller workspace on side stream")
    with pytest.raises(binding.SwaaError) as e:
        binding.swaa_attn_decode(qd, kd, vd, W, S, workspace=ws[:need - 16])
    assert e.value.status == binding.SWAA_ERR_WORKSPACE
    with pytest.raises(binding.SwaaError):
        binding.swaa_attn_decode(qd, kd, vd, 0, 0)
    with pytest.raises(binding.SwaaError):  # more query rows than cached tokens
        binding.swaa_attn_decode(torch.zeros((B, Hq, 200, D), dtype=torch.bfloat16, device="cuda"),
                                 kd[:, :, :100].contiguous(), vd[:, :, :100].contiguous(), 8, 0)


def test_decode_rows_equal_one_pass_fa_decode_rows():
    # the two entry points on the same sequence: rows >= n_prompt of the one-pass call against decode calls
    B, Hq, Hkv, N, D, W, S, P = 1, 8, 2, 3000, 128, 256, 4, 2990
    q, k, v = make_qkv(B, Hq, Hkv, N, D, seed=75)
    qd, kd, vd = to_device(q), to_device(k), to_device(v)
    o1, l1 = binding.swaa_attn_fwd_fa_decode(qd, kd, vd, W, S, P)
    o2, l2 = binding.swaa_attn_decode(qd[:, :, P:].contiguous(), kd, vd, N, 0)
    torch.cuda.synchronize()
    assert (o1[:, :, P:].float() - o2.float()).abs().max().item() <= 2e-2
    assert (l1[:, :, P:] - l2).abs().max().item() <= 1e-3


@pytest.mark.parametrize("name", ["decode128k_full", "decode128k_swa", "decode16k_b16", "decode16k_b16_paged",
                                  "decode128k_full_paged"])
def test_decode_workloads_full_size(name):
    # full-size launches exactly as the benchmark times them; every output row is compared
    w = WORKLOADS[name]
    print(f"[gen] {name} ...", flush=True)
    q, k, v = make_workload(w)
    print(f"[gpu] {name}", flush=True)
    if w.page_size:  # the same keys and values as a paged cache, as the benchmark hands them over
        kc, vc, table = paged_cache(to_device(k), to_device(v), w.page_size, w.seed + 31)
        out, lse = binding.swaa_attn_decode_ex(to_device(q), kc, vc, w.window, w.n_sink, w.scale, block_table=table,
                                               max_seqlen_k=w.N)
    else:
        out, lse = binding.swaa_attn_decode(to_device(q), to_device(k), to_device(v), w.window, w.n_sink, w.scale)
    torch.cuda.synchronize()
    print(f"[oracle] {name}", flush=True)
    ro, rl = swaa_decode_oracle(q, k, v, w.window, w.n_sink, w.scale)
    assert_parity(out, lse, ro, rl, tag=name)


def _paged_cache(seqs, page_size, Hkv, D, rng, extra_pages=3):
    """Scatter per-sequence K/V [1, Hkv, n, D] device tensors into a paged cache
    [num_pages, page_size, Hkv, D] under a random page order; returns (k_cache, v_cache, block_table)."""
    pages_of = [(-(-s[1].shape[2] // page_size)) for s in seqs]
    num_pages = sum(pages_of) + extra_pages
    order = rng.permutation(num_pages)
    kc = torch.randn((num_pages, page_size, Hkv, D), device="cuda").to(torch.bfloat16)  # unused slots hold noise
    vc = torch.randn((num_pages, page_size, Hkv, D), device="cuda").to(torch.bfloat16)
    table = np.full((len(seqs), max(pages_of) + 2), num_pages + 7, dtype=np.int32)   # unused entries: out of range
    nxt = 0
    for b, (_, k, v) in enumerate(seqs):
        n = k.shape[2]
        for pg in range(pages_of[b]):
            page = int(order[nxt]); nxt += 1
            table[b, pg] = page
            t0, t1 = pg * page_size, min(n, (pg + 1) * page_size)
            kc[page, :t1 - t0] = k[0, :, t0:t1].permute(1, 0, 2)
            vc[page, :t1 - t0] = v[0, :, t0:t1].permute(1, 0, 2)
    return kc, vc, torch.from_numpy(table).cuda()


@pytest.mark.parametrize("page_size,Nq", [(16, 1), (4, 3), (64, 1), (128, 2)])
def test_paged_cache_with_ragged_sequence_lengths(page_size, Nq):
    Hq, Hkv, D = 8, 2, 128
    lens = [1 + Nq, 31, 32, 33, 700, 2049, 129, 5000]
    rng = np.random.Generator(np.random.Philox(76 + page_size))
    host = [make_qkv(1, Hq, Hkv, n, D, int(rng.integers(1 << 30)), n_query=Nq) for n in lens]
    seqs = [tuple(to_device(a) for a in s) for s in host]
    kc, vc, table = _paged_cache(seqs, page_size, Hkv, D, rng)
    q = torch.cat([s[0] for s in seqs], dim=0)
    seq_lens = torch.tensor(lens, dtype=torch.int32, device="cuda")
    for W, S in ((10**9, 0), (512, 4)):
        out, lse = binding.swaa_attn_decode_ex(q, kc.permute(0, 2, 1, 3), vc.permute(0, 2, 1, 3), W, S,
                                               seq_lens=seq_lens, block_table=table, max_seqlen_k=max(lens))
        torch.cuda.synchronize()
        for b, (qs, ks, vs) in enumerate(host):
            ro, rl = swaa_decode_oracle(qs, ks, vs, W, S, 1 / math.sqrt(D))
            assert_parity(out[b:b + 1], lse[b:b + 1], ro, rl, tag=f"paged ps{page_size} seq {b} Nk{lens[b]} W{W}")


def test_contiguous_cache_with_sequence_lengths_and_strides():
    # a [B, max_len, Hkv, D] token-major cache buffer, each sequence filled up to its own length
    B, Hq, Hkv, Nq, D, max_len = 4, 8, 2, 1, 128, 3000
    lens = [3000, 17, 1500, 64]
    rng = np.random.Generator(np.random.Philox(77))
    host = [make_qkv(1, Hq, Hkv, n, D, int(rng.integers(1 << 30)), n_query=Nq) for n in lens]
    kbuf = torch.randn((B, max_len, Hkv, D), device="cuda").to(torch.bfloat16)
    vbuf = torch.randn((B, max_len, Hkv, D), device="cuda").to(torch.bfloat16)
    for b, (_, k, v) in enumerate(host):
        kbuf[b, :lens[b]] = to_device(k)[0].permute(1, 0, 2)
        vbuf[b, :lens[b]] = to_device(v)[0].permute(1, 0, 2)
    q = torch.cat([to_device(s[0]) for s in host], dim=0)
    out, lse = binding.swaa_attn_decode_ex(q, kbuf.permute(0, 2, 1, 3), vbuf.permute(0, 2, 1, 3), 10**9, 0,
                                           seq_lens=torch.tensor(lens, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    for b, (qs, ks, vs) in enumerate(host):
        ro, rl = swaa_decode_oracle(qs, ks, vs, 10**9, 0, 1 / math.sqrt(D))
        assert_parity(out[b:b + 1], lse[b:b + 1], ro, rl, tag=f"strided cache seq {b} Nk{lens[b]}")


def test_shorter_sequence_whose_band_straddles_one_more_half():
    # the splits are planned for the longest cache; a shorter one's window can touch one half more
    Hq, Hkv, D, W, S = 2, 1, 128, 500, 100
    lens = [2584, 1710, 1303]
    host = [make_qkv(1, Hq, Hkv, n, D, 7800 + i, n_query=1) for i, n in enumerate(lens)]
    kb = torch.zeros((3, Hkv, max(lens), D), dtype=torch.bfloat16, device="cuda")
    vb = torch.zeros_like(kb)
    for b, (_, k, v) in enumerate(host):
        kb[b, :, :lens[b]], vb[b, :, :lens[b]] = to_device(k)[0], to_device(v)[0]
    q = torch.cat([to_device(s[0]) for s in host], dim=0)
    out, lse = binding.swaa_attn_decode_ex(q, kb, vb, W, S, seq_lens=torch.tensor(lens, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    for b, (qs, ks, vs) in enumerate(host):
        ro, rl = swaa_decode_oracle(qs, ks, vs, W, S, 1 / math.sqrt(D))
        assert_parity(out[b:b + 1], lse[b:b + 1], ro, rl, tag=f"ragged windowed decode seq {b} Nk{lens[b]}")


@pytest.mark.parametrize("Nk", [250, 1024, 1030, 8192, 8200, 17000, 70000])
def test_one_pair_cut_into_many_splits(Nk):
    # one KV head, one token: the only pair has 2, 8, 9, 64, 65, 133 and 547 splits of four halves
    # (the merge kernel's strides of 4 x 8 splits with ragged ends); the workspace starts as noise
    # and is used twice
    B, Hq, Hkv, Nq, D = 1, 4, 1, 1, 128
    q, k, v = make_qkv(B, Hq, Hkv, Nk, D, seed=7900 + Nk % 97, n_query=Nq)
    qd, kd, vd = to_device(q), to_device(k), to_device(v)
    need = binding.swaa_attn_decode_workspace_bytes(B, Hq, Hkv, Nq, Nk, D, Nk, 0)
    ws = torch.randint(0, 256, (need,), dtype=torch.uint8, device="cuda")
    ro, rl = swaa_decode_oracle(q, k, v, Nk, 0, 1 / math.sqrt(D))
    for call in range(2):
        out, lse = binding.swaa_attn_decode(qd, kd, vd, Nk, 0, workspace=ws)
        torch.cuda.synchronize()
        assert_parity(out, lse, ro, rl, tag=f"many splits Nk{Nk} call {call}")


def test_replays_of_a_captured_decode_call():
    # both kernels of the call in a captured graph, replayed with new inputs each time, eager
    # work and synchronisation between the replays; every replay against the oracle and the eager call
    B, Hq, Hkv, Nq, Nk, D, W, S = 2, 8, 2, 1, 6000, 128, 2048, 4
    need = binding.swaa_attn_decode_workspace_bytes(B, Hq, Hkv, Nq, Nk, D, W, S)
    ws = torch.randint(0, 256, (need,), dtype=torch.uint8, device="cuda")
    host = [make_qkv(B, Hq, Hkv, Nk, D, seed=7950 + i, n_query=Nq) for i in range(3)]
    qd, kd, vd = (torch.empty_like(to_device(a)) for a in host[0])
    out = torch.empty_like(qd)
    lse = torch.empty((B, Hq, Nq), dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):  # warm-up outside the capture
        binding.swaa_attn_decode(qd.zero_(), kd.zero_(), vd.zero_(), W, S, out=out, lse=lse, workspace=ws, stream=side)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        binding.swaa_attn_decode(qd, kd, vd, W, S, out=out, lse=lse, workspace=ws, stream=torch.cuda.current_stream())
    for i, (q, k, v) in enumerate(host):
        qd.copy_(to_device(q)); kd.copy_(to_device(k)); vd.copy_(to_device(v))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ro, rl = swaa_decode_oracle(q, k, v, W, S, 1 / math.sqrt(D))
        assert_parity(out, lse, ro, rl, tag=f"captured decode, replay {i}")
        eo, el = binding.swaa_attn_decode(qd, kd, vd, W, S, workspace=ws)   # eager, same workspace
        torch.cuda.synchronize()
        assert torch.equal(eo, out) and torch.equal(el, lse)


@pytest.mark.parametrize("Nq,G", [(1, 4), (2, 4), (1, 8), (3, 5), (9, 4)])
def test_binary16_caches(Nq, G):
    # the paper serves in float16 (Sec. 4.1.1): q, k, v, out in binary16, one and several column
    # tiles, contiguous caches with sequence lengths and a paged cache
    Hkv, D = 2, 128
    Hq = Hkv * G
    lens = [Nq, 33, 700, 4100]
    rng = np.random.Generator(np.random.Philox(7970 + Nq + G))
    host = [make_qkv(1, Hq, Hkv, n, D, int(rng.integers(1 << 30)), n_query=Nq, fmt="fp16") for n in lens]
    q = torch.cat([to_device(s[0], "fp16") for s in host], dim=0)
    seq_lens = torch.tensor(lens, dtype=torch.int32, device="cuda")
    kb = torch.zeros((len(lens), Hkv, max(lens), D), dtype=torch.float16, device="cuda")
    vb = torch.zeros_like(kb)
    for b, (_, k, v) in enumerate(host):
        kb[b, :, :lens[b]], vb[b, :, :lens[b]] = to_device(k, "fp16")[0], to_device(v, "fp16")[0]
    page = 16
    pages = -(-max(lens) // page)
    order = rng.permutation(len(lens) * pages)
    kc = torch.zeros((len(lens) * pages, page, Hkv, D), dtype=torch.float16, device="cuda")
    vc = torch.zeros_like(kc)
    table = torch.from_numpy(order.reshape(len(lens), pages).astype(np.int32)).cuda()
    for b in range(len(lens)):
        kp = torch.zeros((pages * page, Hkv, D), dtype=torch.float16, device="cuda")
        vp = torch.zeros_like(kp)
        kp[:lens[b]], vp[:lens[b]] = kb[b, :, :lens[b]].permute(1, 0, 2), vb[b, :, :lens[b]].permute(1, 0, 2)
        kc[table[b].long()] = kp.view(pages, page, Hkv, D)
        vc[table[b].long()] = vp.view(pages, page, Hkv, D)
    for W, S in ((10**9, 0), (300, 4)):
        o1, l1 = binding.swaa_attn_decode_ex(q, kb, vb, W, S, seq_lens=seq_lens)
        o2, l2 = binding.swaa_attn_decode_ex(q, kc.permute(0, 2, 1, 3), vc.permute(0, 2, 1, 3), W, S, seq_lens=seq_lens,
                                             block_table=table, max_seqlen_k=max(lens))
        torch.cuda.synchronize()
        assert o1.dtype == torch.float16 and torch.equal(o1, o2) and torch.equal(l1, l2)
        for b, (qs, ks, vs) in enumerate(host):
            with input_format("fp16"):
                ro, rl = swaa_decode_oracle(qs, ks, vs, W, S, 1 / math.sqrt(D))
            assert_parity(o1[b:b + 1], l1[b:b + 1], ro, rl, tag=f"fp16 decode Nq{Nq} G{G} seq {b} Nk{lens[b]} W{W}")


def test_more_pairs_than_resident_workgroups():
    # 100 sequences x 8 KV heads = 800 (batch, KV head) pairs against 768 resident workgroups: the
    # plan cuts every pair into several short splits instead of one item per pair
    B, Hq, Hkv, Nq, D, max_len = 100, 16, 8, 1, 128, 640
    rng = np.random.Generator(np.random.Philox(7990))
    lens = [int(x) for x in rng.integers(1, max_len + 1, size=B)]
    lens[0], lens[1] = max_len, 1
    host = [make_qkv(1, Hq, Hkv, n, D, 7991 + i, n_query=Nq) for i, n in enumerate(lens)]
    kb = torch.zeros((B, Hkv, max_len, D), dtype=torch.bfloat16, device="cuda")
    vb = torch.zeros_like(kb)
    for b, (_, k, v) in enumerate(host):
        kb[b, :, :lens[b]], vb[b, :, :lens[b]] = to_device(k)[0], to_device(v)[0]
    q = torch.cat([to_device(s[0]) for s in host], dim=0)
    seq_lens = torch.tensor(lens, dtype=torch.int32, device="cuda")
    for W, S in ((10**9, 0), (100, 4)):
        out, lse = binding.swaa_attn_decode_ex(q, kb, vb, W, S, seq_lens=seq_lens)
        torch.cuda.synchronize()
        worst = [0.0, 0.0, 0.0]
        for b, (qs, ks, vs) in enumerate(host):
            ro, rl = swaa_decode_oracle(qs, ks, vs, W, S, 1 / math.sqrt(D))
            from gpu_util import errors
            e = errors(out[b:b + 1], lse[b:b + 1], ro, rl)
            worst = [max(a, c) for a, c in zip(worst, e)]
        print(f"[parity] 800 pairs W{W}: O max-abs {worst[0]:.3e} mean-abs(max) {worst[1]:.3e} LSE {worst[2]:.3e}", flush=True)
        assert worst[0] <= 2e-2 and worst[1] <= 2e-3 and worst[2] <= 1e-3


@pytest.mark.parametrize("Nq,paged", [(1, False), (1, True), (40, False)])
def test_one_long_sequence_among_short_ones(Nq, paged):
    # continuous batching: with sequence lengths the plan cuts for the longest cache into many short
    # splits and deals the items to the dies in turn; the short sequences' surplus items find no keys
    Hq, Hkv, D = 8, 2, 128
    lens = [40000] + [Nq + 37 * i for i in range(11)]
    rng = np.random.Generator(np.random.Philox(8100 + Nq))
    host = [make_qkv(1, Hq, Hkv, n, D, int(rng.integers(1 << 30)), n_query=Nq) for n in lens]
    seqs = [tuple(to_device(a) for a in s) for s in host]
    q = torch.cat([s[0] for s in seqs], dim=0)
    seq_lens = torch.tensor(lens, dtype=torch.int32, device="cuda")
    if paged:
        kc, vc, table = _paged_cache(seqs, 16, Hkv, D, rng)
        kb, vb, extra = kc.permute(0, 2, 1, 3), vc.permute(0, 2, 1, 3), dict(block_table=table, max_seqlen_k=max(lens))
    else:
        kb = torch.zeros((len(lens), Hkv, max(lens), D), dtype=torch.bfloat16, device="cuda")
        vb = torch.zeros_like(kb)
        for b, (_, k, v) in enumerate(seqs):
            kb[b, :, :lens[b]], vb[b, :, :lens[b]] = k[0], v[0]
        extra = {}
    for W, S in ((10**9, 0), (3000, 4)):
        out, lse = binding.swaa_attn_decode_ex(q, kb, vb, W, S, seq_lens=seq_lens, **extra)
        torch.cuda.synchronize()
        for b, (qs, ks, vs) in enumerate(host):
            ro, rl = swaa_decode_oracle(qs, ks, vs, W, S, 1 / math.sqrt(D))
            assert_parity(out[b:b + 1], lse[b:b + 1], ro, rl, tag=f"skewed batch Nq{Nq} paged{paged} seq {b} Nk{lens[b]} W{W}")


@pytest.mark.parametrize("B", [65, 256, 257])
def test_batches_around_the_limits_of_the_device_side_split_plan(B):
    # sequence lengths in the second round of 64 lanes, in the last lane of the last round, and one
    # sequence more than the device-side plan takes (then the splits are planned for the longest)
    Hq, Hkv, Nq, D, max_len = 2, 1, 1, 128, 900
    rng = np.random.Generator(np.random.Philox(8200 + B))
    lens = [int(x) for x in rng.integers(1, 200, size=B)]
    lens[B - 1], lens[B // 2], lens[0] = max_len, 777, 1
    host = [make_qkv(1, Hq, Hkv, n, D, 8300 + i, n_query=Nq) for i, n in enumerate(lens)]
    kb = torch.zeros((B, Hkv, max_len, D), dtype=torch.bfloat16, device="cuda")
    vb = torch.zeros_like(kb)
    for b, (_, k, v) in enumerate(host):
        kb[b, :, :lens[b]], vb[b, :, :lens[b]] = to_device(k)[0], to_device(v)[0]
    q = torch.cat([to_device(s[0]) for s in host], dim=0)
    out, lse = binding.swaa_attn_decode_ex(q, kb, vb, 10**9, 0, seq_lens=torch.tensor(lens, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    from gpu_util import errors
    worst = [0.0, 0.0, 0.0]
    for b, (qs, ks, vs) in enumerate(host):
        ro, rl = swaa_decode_oracle(qs, ks, vs, 10**9, 0, 1 / math.sqrt(D))
        worst = [max(a, c) for a, c in zip(worst, errors(out[b:b + 1], lse[b:b + 1], ro, rl))]
    print(f"[parity] B{B} ragged: O max-abs {worst[0]:.3e} mean-abs(max) {worst[1]:.3e} LSE {worst[2]:.3e}", flush=True)
    assert worst[0] <= 2e-2 and worst[1] <= 2e-3 and worst[2] <= 1e-3


@pytest.mark.parametrize("name", ["decode_skewed_b16", "decode_mixed_b32"])
def test_decode_workloads_with_sequence_lengths_full_size(name):
    # the benchmark's batches of sequences of very different lengths, launched as it launches them
    # (a [B, Hkv, longest, D] buffer filled up to each length, the rest left as allocated)
    w = WORKLOADS[name]
    print(f"[gen] {name} ...", flush=True)
    q, k, v = make_workload(w)   # k, v: the sequences' tokens back to back
    kd, vd = to_device(k), to_device(v)
    kbuf = torch.empty((w.B, w.Hkv, w.N, w.D), dtype=torch.bfloat16, device="cuda")
    vbuf = torch.empty_like(kbuf)
    t = 0
    for b, n in enumerate(w.seq_lens):
        kbuf[b, :, :n], vbuf[b, :, :n] = kd[0, :, t:t + n], vd[0, :, t:t + n]
        t += n
    print(f"[gpu] {name}", flush=True)
    out, lse = binding.swaa_attn_decode_ex(to_device(q), kbuf, vbuf, w.window, w.n_sink, w.scale,
                                           seq_lens=torch.tensor(w.seq_lens, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    print(f"[oracle] {name}", flush=True)
    t = 0
    for b, n in enumerate(w.seq_lens):
        ro, rl = swaa_decode_oracle(q[b:b + 1], k[:, :, t:t + n], v[:, :, t:t + n], w.window, w.n_sink, w.scale)
        assert_parity(out[b:b + 1], lse[b:b + 1], ro, rl, tag=f"{name} seq {b} ({n} tokens)")
        t += n
