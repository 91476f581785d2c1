"""Host-side checks of libswaa's C ABI: no GPU needed, nothing is launched."""
import ctypes
import os
import re

import pytest

from paper_2512_10411_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = binding.load_library()
    header = open(os.path.join(ROOT, "include", "swaa.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(swaa_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert binding.swaa_version() >= 100


def brute_pairs(N, W, S):
    return sum(1 for i in range(N) for j in range(i + 1) if (j > i - W) or (j < S))


@pytest.mark.parametrize("N", [1, 2, 7, 33])
def test_visible_pairs_matches_counting(N):
    for W in range(1, N + 3):
        for S in range(0, N + 3):
            assert binding.swaa_visible_pairs(N, W, S) == brute_pairs(N, W, S), (N, W, S)


def test_visible_pairs_of_benchmark_workloads():
    # per-head counts of the benchmark definition's workloads
    assert binding.swaa_visible_pairs(1024, 128, 4) == 126522
    assert binding.swaa_visible_pairs(16384, 2048, 4) == 31515642
    assert binding.swaa_visible_pairs(32768, 32768, 4) == 32768 * 32769 // 2
    assert binding.swaa_visible_pairs(131072, 8192, 4) == 1040683002
    with pytest.raises(binding.SwaaError):
        binding.swaa_visible_pairs(0, 1, 0)


def test_argument_errors_are_reported_before_any_launch():
    f = binding.swaa_attn_fwd_raw
    p = 4096  # a non-null, 16-byte aligned fake address; never dereferenced on these paths
    ok = dict(B=1, Hq=4, Hkv=2, N=128, D=128, window=16, n_sink=2, scale=0.1)

    def call(q=p, k=p, v=p, o=p, l=p, **kw):
        a = dict(ok, **kw)
        return f(q, k, v, o, l, a["B"], a["Hq"], a["Hkv"], a["N"], a["D"], a["window"], a["n_sink"], a["scale"], None)

    assert call(q=None) == binding.SWAA_ERR_NULL
    assert call(l=None) == binding.SWAA_ERR_NULL
    assert call(B=0) == binding.SWAA_ERR_SHAPE
    assert call(N=0) == binding.SWAA_ERR_SHAPE
    assert call(Hq=3) == binding.SWAA_ERR_SHAPE
    assert call(window=0) == binding.SWAA_ERR_SHAPE
    assert call(n_sink=-1) == binding.SWAA_ERR_SHAPE
    assert call(scale=0.0) == binding.SWAA_ERR_SHAPE
    assert call(scale=float("nan")) == binding.SWAA_ERR_SHAPE
    assert call(scale=float("inf")) == binding.SWAA_ERR_SHAPE
    assert call(D=80) == binding.SWAA_ERR_UNSUPPORTED
    assert call(D=288) == binding.SWAA_ERR_UNSUPPORTED
    assert call(k=p + 8) == binding.SWAA_ERR_ALIGN
    assert call(o=p + 2) == binding.SWAA_ERR_ALIGN
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert isinstance(binding.swaa_status_string(code), str) and binding.swaa_status_string(code)


def test_fa_decode_pair_count_and_argument_errors():
    def brute(N, W, S, P):
        return sum(1 for i in range(N) for j in range(i + 1) if i >= P or (j > i - W) or (j < S))

    for N in (1, 6, 19):
        for W in range(1, N + 2, 2):
            for S in range(0, N + 2, 3):
                for P in range(0, N + 3):
                    assert binding.swaa_visible_pairs_fa_decode(N, W, S, P) == brute(N, W, S, P), (N, W, S, P)
    assert binding.swaa_visible_pairs_fa_decode(500, 40, 3, 500) == binding.swaa_visible_pairs(500, 40, 3)
    with pytest.raises(binding.SwaaError):
        binding.swaa_visible_pairs_fa_decode(8, 4, 0, -1)

    p = 4096  # fake aligned address; never dereferenced on these paths
    f = binding.swaa_attn_fwd_fa_decode_raw
    assert f(p, p, p, p, p, 1, 4, 2, 128, 128, 16, 2, -1, 0.1, None) == binding.SWAA_ERR_SHAPE
    assert f(p, p, None, p, p, 1, 4, 2, 128, 128, 16, 2, 64, 0.1, None) == binding.SWAA_ERR_NULL
    assert f(p, p, p, p, p, 1, 4, 2, 128, 80, 16, 2, 64, 0.1, None) == binding.SWAA_ERR_UNSUPPORTED
    assert f(p, p, p, p + 4, p, 1, 4, 2, 128, 128, 16, 2, 64, 0.1, None) == binding.SWAA_ERR_ALIGN


def test_decode_workspace_size_and_argument_errors():
    ok = dict(B=1, Hq=32, Hkv=8, Nq=1, Nk=131072, D=128, window=131072, n_sink=4)

    def ws(**kw):
        a = dict(ok, **kw)
        return binding.load_library().swaa_attn_decode_workspace_bytes(
            a["B"], a["Hq"], a["Hkv"], a["Nq"], a["Nk"], a["D"], a["window"], a["n_sink"])

    full = ws()
    assert 0 < full < 64 << 20 and full % 16 == 0
    assert 0 < ws(window=8192) <= full       # fewer visited keys never need more
    assert ws(Nk=1, window=1) > 0
    assert ws(Nq=0) == binding.SWAA_ERR_SHAPE
    assert ws(Nq=9, Nk=8) == binding.SWAA_ERR_SHAPE
    assert ws(Hq=30) == binding.SWAA_ERR_SHAPE
    assert ws(window=0) == binding.SWAA_ERR_SHAPE
    assert ws(D=64) == binding.SWAA_ERR_UNSUPPORTED

    p = 4096  # fake aligned address; never dereferenced on these paths
    f = binding.swaa_attn_decode_raw

    def call(q=p, k=p, v=p, o=p, l=p, w=p, wb=None, scale=0.1, **kw):
        a = dict(ok, **kw)
        wb = ws(**kw) if wb is None else wb
        return f(q, k, v, o, l, a["B"], a["Hq"], a["Hkv"], a["Nq"], a["Nk"], a["D"], a["window"], a["n_sink"],
                 scale, w, wb, None)

    assert call(v=None) == binding.SWAA_ERR_NULL
    assert call(Nq=0, wb=1 << 30) == binding.SWAA_ERR_SHAPE
    assert call(scale=float("nan")) == binding.SWAA_ERR_SHAPE
    assert call(D=256, wb=1 << 30) == binding.SWAA_ERR_UNSUPPORTED
    assert call(q=p + 8) == binding.SWAA_ERR_ALIGN
    assert call(w=None) == binding.SWAA_ERR_WORKSPACE
    assert call(w=p + 4) == binding.SWAA_ERR_WORKSPACE
    assert call(wb=full - 1) == binding.SWAA_ERR_WORKSPACE


def test_general_forward_argument_errors():
    p = 4096  # fake aligned address; never dereferenced on these paths

    def args(**kw):
        a = binding.SwaaFwdArgs()
        Hq, Hkv, N, D = 4, 2, 128, 128
        for name, H in (("q", Hq), ("k", Hkv), ("v", Hkv), ("out", Hq)):
            setattr(a, name, binding.SwaaTensor(p, H * N * D, N * D, D))
        a.lse, a.lse_stride_b, a.lse_stride_h = p, Hq * N, N
        a.B, a.Hq, a.Hkv, a.D, a.Nq, a.Nk = 2, Hq, Hkv, D, N, N
        a.cu_seqlens_q = a.cu_seqlens_k = None
        a.window, a.n_sink, a.n_prompt, a.scale, a.stream = 16, 2, 2**31 - 1, 0.1, None
        for key, val in kw.items():
            if "." in key:
                t, f = key.split(".")
                setattr(getattr(a, t), f, val)
            else:
                setattr(a, key, val)
        return a

    call = lambda **kw: binding.swaa_attn_fwd_ex_raw(args(**kw))
    assert binding.load_library().swaa_attn_fwd_ex(None) == binding.SWAA_ERR_NULL
    assert call(lse=None) == binding.SWAA_ERR_NULL
    assert call(**{"v.ptr": None}) == binding.SWAA_ERR_NULL
    assert call(Nq=129) == binding.SWAA_ERR_SHAPE               # more query rows than tokens
    assert call(n_prompt=-1) == binding.SWAA_ERR_SHAPE
    assert call(**{"k.stride_n": 132}) == binding.SWAA_ERR_SHAPE  # rows would lose 16-byte alignment
    assert call(**{"q.stride_n": 64}) == binding.SWAA_ERR_SHAPE   # rows would overlap
    assert call(**{"out.stride_h": -128}) == binding.SWAA_ERR_SHAPE
    assert call(**{"q.stride_b": 0}) == binding.SWAA_ERR_SHAPE    # two batch entries on one address
    assert call(cu_seqlens_q=p) == binding.SWAA_ERR_NULL          # one offset array without the other
    assert call(cu_seqlens_q=p, cu_seqlens_k=p + 2) == binding.SWAA_ERR_ALIGN
    assert call(n_prompts=p + 2) == binding.SWAA_ERR_ALIGN
    assert call(D=80) == binding.SWAA_ERR_UNSUPPORTED
    assert call(dtype=7) == binding.SWAA_ERR_UNSUPPORTED
    assert call(**{"k.ptr": p + 8}) == binding.SWAA_ERR_ALIGN


def test_backward_argument_errors():
    assert binding.swaa_attn_bwd_workspace_bytes(2, 8, 2, 1000, 128, 100, 0) == 2 * 8 * 1000 * 4  # no sinks: delta only
    assert binding.swaa_attn_bwd_workspace_bytes(2, 8, 2, 1000, 128, 100, 4) > 2 * 8 * 1000 * 4
    assert binding.swaa_attn_bwd_workspace_bytes(1, 32, 8, 131072, 128, 8192, 1000) < 256 << 20
    with pytest.raises(binding.SwaaError):
        binding.swaa_attn_bwd_workspace_bytes(0, 8, 2, 1000, 128, 100, 0)
    p = 4096  # fake aligned address; never dereferenced on these paths
    f = binding.swaa_attn_bwd_raw
    ok = [p] * 9 + [1, 4, 2, 128, 128, 16, 2, 128, 0.1, p, 1 << 20, None]

    def call(**kw):
        a = list(ok)
        names = ["q", "k", "v", "out", "lse", "dout", "dq", "dk", "dv", "B", "Hq", "Hkv", "N", "D", "window", "n_sink",
                 "n_prompt", "scale", "ws", "wb", "stream"]
        for key, val in kw.items():
            a[names.index(key)] = val
        return f(*a)

    assert call(dout=None) == binding.SWAA_ERR_NULL
    assert call(dk=None) == binding.SWAA_ERR_NULL
    assert call(Hq=3) == binding.SWAA_ERR_SHAPE
    assert call(n_prompt=-1) == binding.SWAA_ERR_SHAPE
    assert call(scale=0.0) == binding.SWAA_ERR_SHAPE
    assert call(D=96) == binding.SWAA_ERR_UNSUPPORTED
    assert call(dq=p + 8) == binding.SWAA_ERR_ALIGN
    assert call(ws=None) == binding.SWAA_ERR_WORKSPACE
    assert call(wb=4 * 128 * 4 - 1) == binding.SWAA_ERR_WORKSPACE
    need = binding.swaa_attn_bwd_workspace_bytes(1, 4, 2, 128, 128, 16, 2, 128)
    assert call(wb=need - 1) == binding.SWAA_ERR_WORKSPACE


def test_general_decode_argument_errors():
    p = 4096  # fake aligned address; never dereferenced on these paths

    def args(**kw):
        a = binding.SwaaDecodeArgs()
        a.q = a.out = a.lse = p
        a.k = binding.SwaaTensor(p, 2 * 1024 * 128, 1024 * 128, 128)
        a.v = binding.SwaaTensor(p, 2 * 1024 * 128, 1024 * 128, 128)
        a.B, a.Hq, a.Hkv, a.Nq, a.Nk, a.D = 2, 8, 2, 1, 1024, 128
        a.window, a.n_sink, a.scale = 1024, 0, 0.1
        a.workspace, a.workspace_bytes = p, 1 << 30
        for key, val in kw.items():
            if "." in key:
                t, f = key.split(".")
                setattr(getattr(a, t), f, val)
            else:
                setattr(a, key, val)
        return a

    call = lambda **kw: binding.swaa_attn_decode_ex_raw(args(**kw))
    assert binding.load_library().swaa_attn_decode_ex(None) == binding.SWAA_ERR_NULL
    assert call(out=None) == binding.SWAA_ERR_NULL
    assert call(Nq=2000) == binding.SWAA_ERR_SHAPE
    assert call(**{"v.stride_n": 100}) == binding.SWAA_ERR_SHAPE
    assert call(block_table=p, page_size=6, num_pages=10, block_table_stride=512) == binding.SWAA_ERR_SHAPE
    assert call(block_table=p, page_size=16, num_pages=10, block_table_stride=8) == binding.SWAA_ERR_SHAPE  # 128 < Nk
    assert call(block_table=p, page_size=16, num_pages=0, block_table_stride=64) == binding.SWAA_ERR_SHAPE
    assert call(seq_lens=p + 2) == binding.SWAA_ERR_ALIGN
    assert call(D=64) == binding.SWAA_ERR_UNSUPPORTED
    assert call(workspace_bytes=16) == binding.SWAA_ERR_WORKSPACE
    assert call(dtype=7) == binding.SWAA_ERR_UNSUPPORTED

    # the workspace of the general call: without sequence lengths what the plain call needs; with
    # them the device-side split plan's bound, refused one byte short (checked before any launch)
    lib = binding.load_library()
    assert lib.swaa_attn_decode_ex_workspace_bytes(None) == binding.SWAA_ERR_NULL
    plain = binding.swaa_attn_decode_workspace_bytes(2, 8, 2, 1, 1024, 128, 1024, 0)
    assert binding.swaa_attn_decode_ex_workspace_bytes(args()) == plain
    ragged = binding.swaa_attn_decode_ex_workspace_bytes(args(seq_lens=p))
    assert 0 < ragged <= 2 * (1024 // 32 // 4) * 2 * (4 * 128 + 64) * 4 + 16   # B x ceil(halves / 4) units x Hkv items, B x 2 ints
    assert call(seq_lens=p, workspace_bytes=ragged - 1) == binding.SWAA_ERR_WORKSPACE
    with pytest.raises(binding.SwaaError):
        binding.swaa_attn_decode_ex_workspace_bytes(args(Nq=2000))
    # one sequence, and more sequences than the device-side plan takes: the plan for Nk
    for B in (1, 300):
        assert binding.swaa_attn_decode_ex_workspace_bytes(args(B=B, seq_lens=p)) == \
            binding.swaa_attn_decode_workspace_bytes(B, 8, 2, 1, 1024, 128, 1024, 0)
