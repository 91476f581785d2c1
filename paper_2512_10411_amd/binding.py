"""ctypes binding of libswaa.so: argument marshalling only.

Every step of the attention forward runs inside the HIP kernels; torch is
used for device memory and the stream handle.  There is no fallback: if the
library has not been built (python -m paper_2512_10411_amd.build), the first
call raises.
"""
from __future__ import annotations

import ctypes
import math
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libswaa.so")

SWAA_OK = 0
SWAA_ERR_NULL = -1
SWAA_ERR_SHAPE = -2
SWAA_ERR_UNSUPPORTED = -3
SWAA_ERR_ALIGN = -4
SWAA_ERR_LAUNCH = -5
SWAA_ERR_WORKSPACE = -6
SWAA_BF16 = 0
SWAA_F16 = 1

# every symbol include/swaa.h declares
EXPORTS = ("swaa_attn_fwd", "swaa_attn_fwd_fa_decode", "swaa_attn_fwd_ex", "swaa_visible_pairs",
           "swaa_visible_pairs_fa_decode",
           "swaa_attn_decode", "swaa_attn_decode_ex", "swaa_attn_decode_workspace_bytes", "swaa_attn_decode_ex_workspace_bytes", "swaa_attn_decode_static", "swaa_attn_bwd", "swaa_attn_bwd_workspace_bytes",
           "swaa_status_string", "swaa_version")

_lib = None


class SwaaTensor(ctypes.Structure):
    """swaa_tensor of include/swaa.h."""
    _fields_ = [("ptr", ctypes.c_void_p), ("stride_b", ctypes.c_longlong), ("stride_h", ctypes.c_longlong),
                ("stride_n", ctypes.c_longlong)]


class SwaaFwdArgs(ctypes.Structure):
    """swaa_fwd_args of include/swaa.h."""
    _fields_ = [("q", SwaaTensor), ("k", SwaaTensor), ("v", SwaaTensor), ("out", SwaaTensor),
                ("lse", ctypes.c_void_p), ("lse_stride_b", ctypes.c_longlong), ("lse_stride_h", ctypes.c_longlong),
                ("B", ctypes.c_int), ("Hq", ctypes.c_int), ("Hkv", ctypes.c_int), ("D", ctypes.c_int),
                ("Nq", ctypes.c_int), ("Nk", ctypes.c_int),
                ("cu_seqlens_q", ctypes.c_void_p), ("cu_seqlens_k", ctypes.c_void_p),
                ("window", ctypes.c_int), ("n_sink", ctypes.c_int), ("n_prompt", ctypes.c_int),
                ("scale", ctypes.c_float), ("stream", ctypes.c_void_p), ("dtype", ctypes.c_int),
                ("block_table", ctypes.c_void_p), ("block_table_stride", ctypes.c_int), ("page_size", ctypes.c_int),
                ("num_pages", ctypes.c_int), ("total_rows_q", ctypes.c_longlong), ("n_prompts", ctypes.c_void_p)]


class SwaaDecodeArgs(ctypes.Structure):
    """swaa_decode_args of include/swaa.h."""
    _fields_ = [("q", ctypes.c_void_p), ("out", ctypes.c_void_p), ("lse", ctypes.c_void_p),
                ("k", SwaaTensor), ("v", SwaaTensor),
                ("seq_lens", ctypes.c_void_p), ("block_table", ctypes.c_void_p),
                ("block_table_stride", ctypes.c_int), ("page_size", ctypes.c_int), ("num_pages", ctypes.c_int),
                ("B", ctypes.c_int), ("Hq", ctypes.c_int), ("Hkv", ctypes.c_int), ("Nq", ctypes.c_int),
                ("Nk", ctypes.c_int), ("D", ctypes.c_int), ("window", ctypes.c_int), ("n_sink", ctypes.c_int),
                ("scale", ctypes.c_float), ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_longlong),
                ("stream", ctypes.c_void_p), ("dtype", ctypes.c_int)]


class SwaaError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"libswaa: {message} (status {status})")
        self.status = status


def load_library() -> ctypes.CDLL:
    """Load libswaa.so.  A missing library is an error: nothing is built or substituted here."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2512_10411_amd.build` "
                           "(there is no CPU or PyTorch fallback for the attention kernels)")
    lib = ctypes.CDLL(LIB_PATH)
    lib.swaa_attn_fwd.restype = ctypes.c_int
    lib.swaa_attn_fwd.argtypes = [
        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
        ctypes.c_int, ctypes.c_int, ctypes.c_float, ctypes.c_void_p]
    lib.swaa_attn_fwd_fa_decode.restype = ctypes.c_int
    lib.swaa_attn_fwd_fa_decode.argtypes = [
        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
        ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_float, ctypes.c_void_p]
    lib.swaa_attn_fwd_ex.restype = ctypes.c_int
    lib.swaa_attn_fwd_ex.argtypes = [ctypes.POINTER(SwaaFwdArgs)]
    lib.swaa_visible_pairs.restype = ctypes.c_longlong
    lib.swaa_visible_pairs.argtypes = [ctypes.c_longlong] * 3
    lib.swaa_visible_pairs_fa_decode.restype = ctypes.c_longlong
    lib.swaa_visible_pairs_fa_decode.argtypes = [ctypes.c_longlong] * 4
    lib.swaa_attn_decode.restype = ctypes.c_int
    lib.swaa_attn_decode.argtypes = [
        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
        ctypes.c_int, ctypes.c_int, ctypes.c_float, ctypes.c_void_p, ctypes.c_longlong, ctypes.c_void_p]
    lib.swaa_attn_decode_static.restype = ctypes.c_int
    lib.swaa_attn_decode_static.argtypes = lib.swaa_attn_decode.argtypes[:14] + [ctypes.c_void_p]
    lib.swaa_attn_decode_ex.restype = ctypes.c_int
    lib.swaa_attn_decode_ex.argtypes = [ctypes.POINTER(SwaaDecodeArgs)]
    lib.swaa_attn_decode_workspace_bytes.restype = ctypes.c_longlong
    lib.swaa_attn_decode_workspace_bytes.argtypes = [ctypes.c_int] * 8
    lib.swaa_attn_decode_ex_workspace_bytes.restype = ctypes.c_longlong
    lib.swaa_attn_decode_ex_workspace_bytes.argtypes = [ctypes.POINTER(SwaaDecodeArgs)]
    lib.swaa_attn_bwd.restype = ctypes.c_int
    lib.swaa_attn_bwd.argtypes = [ctypes.c_void_p] * 9 + [ctypes.c_int] * 8 + [
        ctypes.c_float, ctypes.c_void_p, ctypes.c_longlong, ctypes.c_void_p]
    lib.swaa_attn_bwd_workspace_bytes.restype = ctypes.c_longlong
    lib.swaa_attn_bwd_workspace_bytes.argtypes = [ctypes.c_int] * 8
    lib.swaa_status_string.restype = ctypes.c_char_p
    lib.swaa_status_string.argtypes = [ctypes.c_int]
    lib.swaa_version.restype = ctypes.c_int
    lib.swaa_version.argtypes = []
    _lib = lib
    return lib


def swaa_status_string(status: int) -> str:
    return load_library().swaa_status_string(int(status)).decode()


def swaa_version() -> int:
    return int(load_library().swaa_version())


def swaa_visible_pairs(N: int, window: int, n_sink: int) -> int:
    """Visible (query, key) pairs per head; the benchmark counts 4*D flops each."""
    r = int(load_library().swaa_visible_pairs(int(N), int(window), int(n_sink)))
    if r < 0:
        raise SwaaError(SWAA_ERR_SHAPE, "invalid N / window / n_sink")
    return r


def swaa_visible_pairs_fa_decode(N: int, window: int, n_sink: int, n_prompt: int) -> int:
    """Visible pairs per head when rows >= n_prompt attend to every earlier key."""
    r = int(load_library().swaa_visible_pairs_fa_decode(int(N), int(window), int(n_sink), int(n_prompt)))
    if r < 0:
        raise SwaaError(SWAA_ERR_SHAPE, "invalid N / window / n_sink / n_prompt")
    return r


def swaa_attn_fwd_raw(q_ptr, k_ptr, v_ptr, out_ptr, lse_ptr, B, Hq, Hkv, N, D,
                      window, n_sink, scale, stream_ptr) -> int:
    """The C call itself, on raw addresses; returns the status code."""
    return int(load_library().swaa_attn_fwd(
        q_ptr, k_ptr, v_ptr, out_ptr, lse_ptr, B, Hq, Hkv, N, D, window, n_sink, scale, stream_ptr))


def swaa_attn_fwd_fa_decode_raw(q_ptr, k_ptr, v_ptr, out_ptr, lse_ptr, B, Hq, Hkv, N, D,
                                window, n_sink, n_prompt, scale, stream_ptr) -> int:
    """The C call itself, on raw addresses; returns the status code."""
    return int(load_library().swaa_attn_fwd_fa_decode(
        q_ptr, k_ptr, v_ptr, out_ptr, lse_ptr, B, Hq, Hkv, N, D, window, n_sink, n_prompt, scale, stream_ptr))


def swaa_attn_fwd(q, k, v, window: int, n_sink: int, scale: float | None = None,
                  out=None, lse=None, stream=None):
    """SWA + sink attention forward on the GPU.

    q: bf16 [B, Hq, N, D]; k, v: bf16 [B, Hkv, N, D]; all contiguous CUDA/HIP
    tensors on one device.  Returns (out bf16 [B, Hq, N, D], lse fp32 [B, Hq, N]).
    The call is asynchronous on `stream` (default: torch's current stream).
    """
    return _fwd(q, k, v, window, n_sink, None, scale, out, lse, stream)


def swaa_attn_fwd_fa_decode(q, k, v, window: int, n_sink: int, n_prompt: int, scale: float | None = None,
                            out=None, lse=None, stream=None):
    """As swaa_attn_fwd, with rows >= n_prompt (generated tokens) attending to every earlier key."""
    return _fwd(q, k, v, window, n_sink, int(n_prompt), scale, out, lse, stream)


def _fwd(q, k, v, window, n_sink, n_prompt, scale, out, lse, stream):
    import torch

    for name, t in (("q", q), ("k", k), ("v", v)):
        if t.dtype != torch.bfloat16:
            raise TypeError(f"{name} must be bfloat16")
        if not t.is_cuda:
            raise ValueError(f"{name} must live on the GPU")
        if not t.is_contiguous() or t.dim() != 4:
            raise ValueError(f"{name} must be a contiguous [B, H, N, D] tensor")
    B, Hq, N, D = q.shape
    if k.shape != v.shape or k.shape[0] != B or k.shape[2] != N or k.shape[3] != D:
        raise ValueError("k and v must be [B, Hkv, N, D] with q's B, N, D")
    if k.device != q.device or v.device != q.device:
        raise ValueError("q, k, v must be on the same device")
    Hkv = k.shape[1]
    if scale is None:
        scale = 1.0 / math.sqrt(D)
    with torch.cuda.device(q.device):
        if out is None:
            out = torch.empty_like(q)
        if lse is None:
            lse = torch.empty((B, Hq, N), dtype=torch.float32, device=q.device)
        if out.shape != q.shape or out.dtype != torch.bfloat16 or not out.is_contiguous():
            raise ValueError("out must be a contiguous bf16 tensor shaped like q")
        if lse.shape != (B, Hq, N) or lse.dtype != torch.float32 or not lse.is_contiguous():
            raise ValueError("lse must be a contiguous fp32 [B, Hq, N] tensor")
        if stream is None:
            stream = torch.cuda.current_stream(q.device)
        sptr = stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)
        ptrs = (q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), lse.data_ptr())
        if n_prompt is None:
            rc = swaa_attn_fwd_raw(*ptrs, B, Hq, Hkv, N, D, int(window), int(n_sink), float(scale), sptr)
        else:
            rc = swaa_attn_fwd_fa_decode_raw(*ptrs, B, Hq, Hkv, N, D, int(window), int(n_sink), n_prompt,
                                             float(scale), sptr)
    if rc != SWAA_OK:
        raise SwaaError(rc, swaa_status_string(rc))
    return out, lse


def swaa_attn_decode_workspace_bytes(B, Hq, Hkv, Nq, Nk, D, window, n_sink) -> int:
    """Bytes of device scratch swaa_attn_decode needs for this shape."""
    r = int(load_library().swaa_attn_decode_workspace_bytes(
        int(B), int(Hq), int(Hkv), int(Nq), int(Nk), int(D), int(window), int(n_sink)))
    if r < 0:
        raise SwaaError(r, swaa_status_string(r))
    return r


def swaa_attn_decode_raw(q_ptr, k_ptr, v_ptr, out_ptr, lse_ptr, B, Hq, Hkv, Nq, Nk, D,
                         window, n_sink, scale, ws_ptr, ws_bytes, stream_ptr) -> int:
    """The C call itself, on raw addresses; returns the status code."""
    return int(load_library().swaa_attn_decode(
        q_ptr, k_ptr, v_ptr, out_ptr, lse_ptr, B, Hq, Hkv, Nq, Nk, D, window, n_sink, scale,
        ws_ptr, ws_bytes, stream_ptr))


def swaa_attn_decode(q, k, v, window: int, n_sink: int, scale: float | None = None,
                     out=None, lse=None, workspace=None, stream=None):
    """Attention of the Nq newest tokens over a KV cache of Nk tokens, on the GPU.

    q: bf16 [B, Hq, Nq, D]; k, v: bf16 [B, Hkv, Nk, D] (the cache, the new tokens'
    own rows included); window >= Nk is full attention (FA Decode).  workspace: a
    uint8 tensor of at least swaa_attn_decode_workspace_bytes(...) bytes (allocated
    here with torch when None).  Returns (out bf16 [B, Hq, Nq, D], lse fp32 [B, Hq, Nq]).
    """
    import torch

    for name, t in (("q", q), ("k", k), ("v", v)):
        if t.dtype != torch.bfloat16:
            raise TypeError(f"{name} must be bfloat16")
        if not t.is_cuda:
            raise ValueError(f"{name} must live on the GPU")
        if not t.is_contiguous() or t.dim() != 4:
            raise ValueError(f"{name} must be a contiguous [B, H, N, D] tensor")
    B, Hq, Nq, D = q.shape
    if k.shape != v.shape or k.shape[0] != B or k.shape[3] != D:
        raise ValueError("k and v must be [B, Hkv, Nk, D] with q's B and D")
    if k.device != q.device or v.device != q.device:
        raise ValueError("q, k, v must be on the same device")
    Hkv, Nk = k.shape[1], k.shape[2]
    if scale is None:
        scale = 1.0 / math.sqrt(D)
    need = swaa_attn_decode_workspace_bytes(B, Hq, Hkv, Nq, Nk, D, window, n_sink)
    with torch.cuda.device(q.device):
        if out is None:
            out = torch.empty_like(q)
        if lse is None:
            lse = torch.empty((B, Hq, Nq), dtype=torch.float32, device=q.device)
        if workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
        if out.shape != q.shape or out.dtype != torch.bfloat16 or not out.is_contiguous():
            raise ValueError("out must be a contiguous bf16 tensor shaped like q")
        if lse.shape != (B, Hq, Nq) or lse.dtype != torch.float32 or not lse.is_contiguous():
            raise ValueError("lse must be a contiguous fp32 [B, Hq, Nq] tensor")
        if workspace.dtype != torch.uint8 or not workspace.is_cuda or not workspace.is_contiguous():
            raise ValueError("workspace must be a contiguous uint8 tensor on the GPU")
        if stream is None:
            stream = torch.cuda.current_stream(q.device)
        sptr = stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)
        rc = swaa_attn_decode_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), lse.data_ptr(),
                                  B, Hq, Hkv, Nq, Nk, D, int(window), int(n_sink), float(scale),
                                  workspace.data_ptr(), workspace.numel(), sptr)
    if rc != SWAA_OK:
        raise SwaaError(rc, swaa_status_string(rc))
    return out, lse


SWAA_DECODE_STATIC_SCRATCH_BYTES = 16 << 20  # include/swaa.h


def swaa_attn_decode_static_raw(q_ptr, k_ptr, v_ptr, out_ptr, lse_ptr, B, Hq, Hkv, Nq, Nk, D,
                                window, n_sink, scale, stream_ptr) -> int:
    """The C call itself, on raw addresses; returns the status code.  Allocates nothing."""
    return int(load_library().swaa_attn_decode_static(
        q_ptr, k_ptr, v_ptr, out_ptr, lse_ptr, B, Hq, Hkv, Nq, Nk, D, window, n_sink, scale, stream_ptr))


def swaa_attn_decode_static(q, k, v, out, lse, window: int, n_sink: int, scale: float | None = None, stream=None):
    """swaa_attn_decode on the library's own static scratch array: nothing is allocated,
    here or in the library, so `out` (bf16 [B, Hq, Nq, D]) and `lse` (fp32 [B, Hq, Nq]) are
    the caller's.  Calls that may overlap on one GPU must be serialised by the caller."""
    B, Hq, Nq, D = q.shape
    Hkv, Nk = k.shape[1], k.shape[2]
    if scale is None:
        scale = 1.0 / math.sqrt(D)
    for name, t in (("q", q), ("k", k), ("v", v), ("out", out), ("lse", lse)):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous GPU tensor")
    if stream is None:
        import torch
        stream = torch.cuda.current_stream(q.device)
    sptr = stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)
    rc = swaa_attn_decode_static_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), lse.data_ptr(),
                                     B, Hq, Hkv, Nq, Nk, D, int(window), int(n_sink), float(scale), sptr)
    if rc != SWAA_OK:
        raise SwaaError(rc, swaa_status_string(rc))
    return out, lse


def swaa_attn_fwd_ex_raw(args: SwaaFwdArgs) -> int:
    """The C call itself on a filled argument block; returns the status code."""
    return int(load_library().swaa_attn_fwd_ex(ctypes.byref(args)))


def swaa_attn_fwd_ex(q, k, v, window: int, n_sink: int, n_prompt: int | None = None, scale: float | None = None,
                     cu_seqlens_q=None, cu_seqlens_k=None, max_seqlen_q: int | None = None,
                     max_seqlen_k: int | None = None, out=None, lse=None, stream=None, block_table=None,
                     total_rows_q: int | None = None, n_prompts=None):
    """General forward: strided tensors, Nq <= Nk (the query rows are the newest Nq of Nk
    tokens), packed variable-length batches.

    Fixed-length batches: q [B, Hq, Nq, D] and k, v [B, Hkv, Nk, D] as *views* with any
    strides whose last dimension is contiguous (a [B, N, H, D] tensor is passed as
    ``t.permute(0, 2, 1, 3)``).  Packed batches: q [Hq, Tq, D], k, v [Hkv, Tk, D] views plus
    int32 device tensors cu_seqlens_q / cu_seqlens_k of B + 1 offsets and the largest
    sequence lengths.  Paged cache (head dimension 128): block_table int32 [B, pages_per_seq] on the
    GPU, k, v views [num_pages, Hkv, page_size, D], max_seqlen_k the (largest) number of cached tokens;
    with cu_seqlens the key offsets only give the cache lengths.  total_rows_q (packed batches): the
    rows of the packed q tensor, taken from q by default; 0 makes the launch as large as B times the
    longest sequence (slow for sequences of very different lengths).  n_prompts: int32 [B] GPU tensor of
    per-sequence prompt lengths, used in place of n_prompt.  bfloat16 or float16 tensors (all of
    one type).  out defaults to a new tensor with q's shape in q's memory order;
    lse is fp32 [B, Hq, Nq] ([Hq, Tq] when packed).  Returns (out, lse).
    """
    import torch

    packed = cu_seqlens_q is not None or cu_seqlens_k is not None
    nd = 3 if packed else 4
    if q.dtype not in (torch.bfloat16, torch.float16):
        raise TypeError("q must be bfloat16 or float16")
    for name, t in (("q", q), ("k", k), ("v", v)):
        want = 4 if (block_table is not None and name != "q") else nd  # (pages of a paged cache are 4-dimensional)
        if t.dtype != q.dtype or not t.is_cuda or t.dim() != want or t.stride(-1) != 1:
            raise ValueError(f"{name} must be a GPU tensor view of q's dtype with {want} dimensions and a contiguous "
                             "last one")
    D = q.shape[-1]
    Hq, Hkv = q.shape[-3], k.shape[-3]
    if scale is None:
        scale = 1.0 / math.sqrt(D)
    if packed:
        if cu_seqlens_q is None or cu_seqlens_k is None or max_seqlen_q is None or max_seqlen_k is None:
            raise ValueError("packed batches need cu_seqlens_q, cu_seqlens_k, max_seqlen_q and max_seqlen_k")
        for name, t in (("cu_seqlens_q", cu_seqlens_q), ("cu_seqlens_k", cu_seqlens_k)):
            if t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous() or t.dim() != 1:
                raise ValueError(f"{name} must be a contiguous int32 GPU vector")
        B = cu_seqlens_q.numel() - 1
        if cu_seqlens_k.numel() != B + 1:
            raise ValueError("cu_seqlens_q and cu_seqlens_k must have the same length")
        Nq, Nk = int(max_seqlen_q), int(max_seqlen_k)
        lse_shape = (Hq, q.shape[1])
    else:
        B, Nq, Nk = q.shape[0], q.shape[2], k.shape[2]
        lse_shape = (B, Hq, Nq)
    paged = block_table is not None
    if paged:
        if block_table.dtype != torch.int32 or not block_table.is_cuda or block_table.dim() != 2 \
                or block_table.stride(1) != 1 or block_table.shape[0] != B:
            raise ValueError("block_table must be an int32 [B, pages_per_seq] GPU tensor with contiguous rows")
        if max_seqlen_k is None or k.dim() != 4:
            raise ValueError("a paged cache needs max_seqlen_k and k, v views [num_pages, Hkv, page_size, D]")
        Nk = int(max_seqlen_k)
    with torch.cuda.device(q.device):
        if out is None:
            out = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
        if lse is None:
            lse = torch.empty(lse_shape, dtype=torch.float32, device=q.device)
        if out.shape != q.shape or out.dtype != q.dtype or out.stride(-1) != 1:
            raise ValueError("out must be a tensor view shaped and typed like q with a contiguous last dimension")
        if tuple(lse.shape) != lse_shape or lse.dtype != torch.float32 or not lse.is_contiguous():
            raise ValueError(f"lse must be a contiguous fp32 tensor of shape {lse_shape}")
        if stream is None:
            stream = torch.cuda.current_stream(q.device)

        def tensor(t):
            if t.dim() == 3:
                return SwaaTensor(t.data_ptr(), 0, t.stride(0), t.stride(1))
            return SwaaTensor(t.data_ptr(), t.stride(0), t.stride(1), t.stride(2))

        a = SwaaFwdArgs()
        a.q, a.k, a.v, a.out = tensor(q), tensor(k), tensor(v), tensor(out)
        a.lse = lse.data_ptr()
        a.lse_stride_b, a.lse_stride_h = (0, lse.stride(0)) if packed else (lse.stride(0), lse.stride(1))
        a.B, a.Hq, a.Hkv, a.D, a.Nq, a.Nk = B, Hq, Hkv, D, Nq, Nk
        a.cu_seqlens_q = cu_seqlens_q.data_ptr() if packed else None
        a.cu_seqlens_k = cu_seqlens_k.data_ptr() if packed else None
        a.window, a.n_sink = int(window), int(n_sink)
        a.n_prompt = 2**31 - 1 if n_prompt is None else int(n_prompt)
        a.scale = float(scale)
        a.stream = stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)
        a.dtype = SWAA_F16 if q.dtype == torch.float16 else SWAA_BF16
        a.block_table = block_table.data_ptr() if paged else None
        a.block_table_stride = block_table.stride(0) if paged else 0
        a.page_size = k.shape[2] if paged else 0
        a.num_pages = k.shape[0] if paged else 0
        a.total_rows_q = (q.shape[1] if packed else 0) if total_rows_q is None else int(total_rows_q)
        if n_prompts is not None:
            if n_prompts.dtype != torch.int32 or not n_prompts.is_cuda or not n_prompts.is_contiguous() \
                    or n_prompts.shape != (B,):
                raise ValueError("n_prompts must be a contiguous int32 [B] GPU tensor")
            a.n_prompts = n_prompts.data_ptr()
        rc = swaa_attn_fwd_ex_raw(a)
    if rc != SWAA_OK:
        raise SwaaError(rc, swaa_status_string(rc))
    return out, lse


def swaa_attn_bwd_workspace_bytes(B, Hq, Hkv, N, D, window, n_sink, n_prompt=None) -> int:
    """Bytes of device scratch swaa_attn_bwd needs for this shape and mask."""
    r = int(load_library().swaa_attn_bwd_workspace_bytes(
        int(B), int(Hq), int(Hkv), int(N), int(D), int(window), int(n_sink),
        2**31 - 1 if n_prompt is None else int(n_prompt)))
    if r < 0:
        raise SwaaError(r, swaa_status_string(r))
    return r


def swaa_attn_bwd_raw(q, k, v, out, lse, dout, dq, dk, dv, B, Hq, Hkv, N, D, window, n_sink, n_prompt, scale,
                      ws_ptr, ws_bytes, stream_ptr) -> int:
    """The C call itself, on raw addresses; returns the status code."""
    return int(load_library().swaa_attn_bwd(q, k, v, out, lse, dout, dq, dk, dv, B, Hq, Hkv, N, D, window, n_sink,
                                            n_prompt, scale, ws_ptr, ws_bytes, stream_ptr))


def swaa_attn_bwd(q, k, v, out, lse, dout, window: int, n_sink: int, n_prompt: int | None = None,
                  scale: float | None = None, workspace=None, stream=None):
    """Gradients (dq, dk, dv) of the forward call with the same mask arguments.

    q, out, dout: bf16 [B, Hq, N, D]; k, v: bf16 [B, Hkv, N, D]; lse: fp32 [B, Hq, N]; all
    contiguous GPU tensors (out and lse as the forward call returned them).
    """
    import torch

    for name, t in (("q", q), ("k", k), ("v", v), ("out", out), ("dout", dout)):
        if t.dtype != torch.bfloat16 or not t.is_cuda or not t.is_contiguous() or t.dim() != 4:
            raise ValueError(f"{name} must be a contiguous bf16 [B, H, N, D] GPU tensor")
    B, Hq, N, D = q.shape
    Hkv = k.shape[1]
    if k.shape != v.shape or k.shape != (B, Hkv, N, D) or out.shape != q.shape or dout.shape != q.shape:
        raise ValueError("shape mismatch between q, k, v, out and dout")
    if lse.shape != (B, Hq, N) or lse.dtype != torch.float32 or not lse.is_contiguous():
        raise ValueError("lse must be a contiguous fp32 [B, Hq, N] tensor")
    if scale is None:
        scale = 1.0 / math.sqrt(D)
    need = swaa_attn_bwd_workspace_bytes(B, Hq, Hkv, N, D, window, n_sink, n_prompt)
    with torch.cuda.device(q.device):
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        if workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
        if workspace.dtype != torch.uint8 or not workspace.is_cuda or not workspace.is_contiguous():
            raise ValueError("workspace must be a contiguous uint8 tensor on the GPU")
        if stream is None:
            stream = torch.cuda.current_stream(q.device)
        sptr = stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)
        rc = swaa_attn_bwd_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), lse.data_ptr(),
                               dout.data_ptr(), dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), B, Hq, Hkv, N, D,
                               int(window), int(n_sink), 2**31 - 1 if n_prompt is None else int(n_prompt),
                               float(scale), workspace.data_ptr(), workspace.numel(), sptr)
    if rc != SWAA_OK:
        raise SwaaError(rc, swaa_status_string(rc))
    return dq, dk, dv


def swaa_attn_decode_ex_workspace_bytes(args: SwaaDecodeArgs) -> int:
    """Bytes of workspace swaa_attn_decode_ex needs for this argument block (its shape fields
    and whether seq_lens is set); raises SwaaError on invalid shapes."""
    r = int(load_library().swaa_attn_decode_ex_workspace_bytes(ctypes.byref(args)))
    if r < 0:
        raise SwaaError(r, swaa_status_string(r))
    return r


def swaa_attn_decode_ex_raw(args: SwaaDecodeArgs) -> int:
    """The C call itself on a filled argument block; returns the status code."""
    return int(load_library().swaa_attn_decode_ex(ctypes.byref(args)))


def swaa_attn_decode_ex(q, k, v, window: int, n_sink: int, scale: float | None = None, seq_lens=None,
                        block_table=None, max_seqlen_k: int | None = None, out=None, lse=None, workspace=None,
                        stream=None):
    """Decode-shape attention on a strided or paged cache, with per-sequence cache lengths.

    q: bf16 or fp16 [B, Hq, Nq, D] contiguous (k, v in the same format; out takes it too).
    Contiguous cache: k, v views [B, Hkv, Nk, D] with any
    strides (last dimension contiguous).  Paged cache: block_table int32 [B, pages_per_seq] on
    the GPU and k, v views [num_pages, Hkv, page_size, D] (a [num_pages, page_size, Hkv, D]
    cache is passed as ``cache.permute(0, 2, 1, 3)``).  seq_lens: int32 [B] GPU tensor of cache
    lengths (the Nq newest tokens included) or None; max_seqlen_k: the largest of them (required
    with a paged cache).  Returns (out, lse).
    """
    import torch

    if q.dtype not in (torch.bfloat16, torch.float16) or not q.is_cuda or not q.is_contiguous() or q.dim() != 4:
        raise ValueError("q must be a contiguous bf16 or fp16 [B, Hq, Nq, D] GPU tensor")
    for name, t in (("k", k), ("v", v)) + ((("out", out),) if out is not None else ()):
        if t.dtype != q.dtype or not t.is_cuda or t.dim() != 4 or t.stride(-1) != 1:
            raise ValueError(f"{name} must be a GPU tensor view of q's format with 4 dimensions and a contiguous last one")
    B, Hq, Nq, D = q.shape
    Hkv = k.shape[1]
    paged = block_table is not None
    if paged:
        if max_seqlen_k is None:
            raise ValueError("a paged cache needs max_seqlen_k")
        if block_table.dtype != torch.int32 or not block_table.is_cuda or block_table.dim() != 2 \
                or block_table.stride(1) != 1 or block_table.shape[0] != B:
            raise ValueError("block_table must be an int32 [B, pages_per_seq] GPU tensor with contiguous rows")
        Nk = int(max_seqlen_k)
    else:
        Nk = k.shape[2] if max_seqlen_k is None else int(max_seqlen_k)
    if seq_lens is not None and (seq_lens.dtype != torch.int32 or not seq_lens.is_cuda or not seq_lens.is_contiguous()
                                 or seq_lens.shape != (B,)):
        raise ValueError("seq_lens must be a contiguous int32 [B] GPU tensor")
    if scale is None:
        scale = 1.0 / math.sqrt(D)
    with torch.cuda.device(q.device):
        if out is None:
            out = torch.empty_like(q)
        if lse is None:
            lse = torch.empty((B, Hq, Nq), dtype=torch.float32, device=q.device)
        if stream is None:
            stream = torch.cuda.current_stream(q.device)
        a = SwaaDecodeArgs()
        a.q, a.out, a.lse = q.data_ptr(), out.data_ptr(), lse.data_ptr()
        a.k = SwaaTensor(k.data_ptr(), k.stride(0), k.stride(1), k.stride(2))
        a.v = SwaaTensor(v.data_ptr(), v.stride(0), v.stride(1), v.stride(2))
        a.seq_lens = seq_lens.data_ptr() if seq_lens is not None else None
        a.block_table = block_table.data_ptr() if paged else None
        a.block_table_stride = block_table.stride(0) if paged else 0
        a.page_size = k.shape[2] if paged else 0
        a.num_pages = k.shape[0] if paged else 0
        a.B, a.Hq, a.Hkv, a.Nq, a.Nk, a.D = B, Hq, Hkv, Nq, Nk, D
        a.window, a.n_sink, a.scale = int(window), int(n_sink), float(scale)
        if workspace is None:
            need = swaa_attn_decode_ex_workspace_bytes(a)
            workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
        a.workspace, a.workspace_bytes = workspace.data_ptr(), workspace.numel()
        a.stream = stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)
        a.dtype = SWAA_F16 if q.dtype == torch.float16 else SWAA_BF16
        rc = swaa_attn_decode_ex_raw(a)
    if rc != SWAA_OK:
        raise SwaaError(rc, swaa_status_string(rc))
    return out, lse
