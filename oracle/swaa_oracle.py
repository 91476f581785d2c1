"""Python face of the fp64 CPU oracle.  TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Two independent routes to the same definition (paper Sec. 1, Sec. 3.2.1 /
Fig. 1b, Sec. 4.1.2):

* :func:`swaa_attn_oracle` -- calls ``swaa_oracle.c`` (plain C, fp64, OpenMP
  over rows) through ctypes; fast enough for the sampled rows of the largest
  configurations.
* :func:`swaa_attn_oracle_numpy` -- the same three lines of mathematics in
  numpy, one row at a time with an explicit list of visible keys; used for
  small cases and to cross-check the C build.

Both take ``n_prompt`` (FA Decode, paper Sec. 3.1.1 / Fig. 1a): rows at or
beyond it are generated tokens and see every earlier key; ``None`` means all
rows are prompt tokens.

:func:`swaa_decode_oracle` (and its numpy twin) is the decode shape: the Nq
newest tokens of a sequence against a cache of Nk keys and values.

Inputs are bf16 bit patterns held in ``uint16`` arrays of shape [B, H, N, D];
outputs are float64 and unrounded.  Parity status: pinned (see
``tests/test_oracle_pins.py``): full-causal special case against a library
softmax-attention, closed forms for W=1 and Q=0, brute-force boolean masks on
tiny inputs, locality, merge identity, GQA/batch identities; the FA Decode
mask and the decode shape in ``tests/test_oracle_pins_fa_decode.py`` and
``tests/test_oracle_pins_decode.py``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "swaa_oracle.c")
_LIB = os.path.join(_HERE, "libswaa_oracle.so")
_lib = None


def build_oracle(force: bool = False) -> str:
    """Compile ``swaa_oracle.c`` with gcc into ``libswaa_oracle.so`` (beside it)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_oracle())
        lib.swaa_oracle_rows.restype = ctypes.c_int
        lib.swaa_oracle_rows.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_long, ctypes.c_long, ctypes.c_double,
            ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        lib.swaa_oracle_rows_mixed.restype = ctypes.c_int
        lib.swaa_oracle_rows_mixed.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_long, ctypes.c_long, ctypes.c_long, ctypes.c_double,
            ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        lib.swaa_oracle_decode.restype = ctypes.c_int
        lib.swaa_oracle_decode.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_long, ctypes.c_long, ctypes.c_long, ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int]
        lib.swaa_oracle_bwd.restype = ctypes.c_int
        lib.swaa_oracle_bwd.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_long, ctypes.c_long, ctypes.c_long, ctypes.c_double,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        lib.swaa_oracle_set_format.restype = ctypes.c_int
        lib.swaa_oracle_set_format.argtypes = [ctypes.c_int]
        lib.swaa_oracle_decode_elems.restype = None
        lib.swaa_oracle_decode_elems.argtypes = [ctypes.c_void_p, ctypes.c_long, ctypes.c_void_p]
        lib.swaa_oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


class input_format:
    """``with input_format("fp16"):`` -- the uint16 inputs of the oracle calls inside are IEEE
    binary16 bit patterns instead of bfloat16 (a process-wide switch of the C oracle; the
    numpy routes read the same switch).  Not for concurrent use."""
    _current = "bf16"

    def __init__(self, fmt):
        if fmt not in ("bf16", "fp16"):
            raise ValueError("format must be 'bf16' or 'fp16'")
        self.fmt = fmt

    def __enter__(self):
        self.prev = input_format._current
        input_format._current = self.fmt
        _load().swaa_oracle_set_format(1 if self.fmt == "fp16" else 0)
        return self

    def __exit__(self, *exc):
        input_format._current = self.prev
        _load().swaa_oracle_set_format(1 if self.prev == "fp16" else 0)
        return False


def decode_elems(bits: np.ndarray) -> np.ndarray:
    """The C oracle's element decoder applied to an array of uint16 bit patterns."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, dtype=np.float64)
    _load().swaa_oracle_decode_elems(bits.ctypes.data, bits.size, out.ctypes.data)
    return out


def oracle_num_threads() -> int:
    """Threads the C oracle's OpenMP loop will use by default."""
    return int(_load().swaa_oracle_num_threads())


def _check(q, k, v):
    for name, a in (("q", q), ("k", k), ("v", v)):
        if not isinstance(a, np.ndarray) or a.dtype != np.uint16 or a.ndim != 4:
            raise TypeError(f"{name}: expected uint16 (bf16 bits) ndarray [B,H,N,D]")
    B, Hq, N, D = q.shape
    if k.shape != v.shape or k.shape[0] != B or k.shape[2] != N or k.shape[3] != D:
        raise ValueError("k/v shape mismatch")
    Hkv = k.shape[1]
    if Hq % Hkv:
        raise ValueError("Hq must be a multiple of Hkv")
    return B, Hq, Hkv, N, D


def swaa_attn_oracle(q, k, v, window, n_sink, scale, rows=None, n_threads=0, n_prompt=None):
    """fp64 SWA+sink attention via the C oracle.

    rows: optional 1-D int array of query rows to evaluate (same set for every
    (b, h)); None evaluates all N rows.  n_prompt: rows >= n_prompt attend to
    all earlier keys (None: no such rows).  Returns (out [B,Hq,R,D] float64,
    lse [B,Hq,R] float64).
    """
    B, Hq, Hkv, N, D = _check(q, k, v)
    q = np.ascontiguousarray(q)
    k = np.ascontiguousarray(k)
    v = np.ascontiguousarray(v)
    if rows is None:
        rows_arr, R, rows_p = None, N, None
    else:
        rows_arr = np.ascontiguousarray(np.asarray(rows, dtype=np.int32))
        R = int(rows_arr.shape[0])
        rows_p = rows_arr.ctypes.data
    out = np.empty((B, Hq, R, D), dtype=np.float64)
    lse = np.empty((B, Hq, R), dtype=np.float64)
    if n_prompt is None:
        rc = _load().swaa_oracle_rows(
            q.ctypes.data, k.ctypes.data, v.ctypes.data, B, Hq, Hkv, N, D,
            int(window), int(n_sink), float(scale), rows_p, R,
            out.ctypes.data, lse.ctypes.data, int(n_threads))
    else:
        rc = _load().swaa_oracle_rows_mixed(
            q.ctypes.data, k.ctypes.data, v.ctypes.data, B, Hq, Hkv, N, D,
            int(window), int(n_sink), int(n_prompt), float(scale), rows_p, R,
            out.ctypes.data, lse.ctypes.data, int(n_threads))
    if rc != 0:
        raise ValueError(f"swaa_oracle_rows failed with code {rc}")
    return out, lse


def _bf16_bits_to_f64(a: np.ndarray) -> np.ndarray:
    if input_format._current == "fp16":
        return np.ascontiguousarray(a).view(np.float16).astype(np.float64)
    return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def swaa_attn_oracle_numpy(q, k, v, window, n_sink, scale, rows=None, n_prompt=None):
    """The same definition in numpy, row by row (slow; small inputs only)."""
    B, Hq, Hkv, N, D = _check(q, k, v)
    W, S = int(window), int(n_sink)
    P = N if n_prompt is None else int(n_prompt)
    if W < 1 or S < 0 or P < 0:
        raise ValueError("window >= 1, n_sink >= 0 and n_prompt >= 0 required")
    G = Hq // Hkv
    qf, kf, vf = (_bf16_bits_to_f64(a) for a in (q, k, v))
    row_list = list(range(N)) if rows is None else [int(r) for r in rows]
    out = np.empty((B, Hq, len(row_list), D), dtype=np.float64)
    lse = np.empty((B, Hq, len(row_list)), dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            for r, i in enumerate(row_list):
                vis = [j for j in range(i + 1) if (i >= P) or (j > i - W) or (j < S)]
                s = scale * (kf[b, g, vis] @ qf[b, h, i])
                m = s.max()
                lse_i = m + np.log(np.exp(s - m).sum())
                p = np.exp(s - lse_i)
                out[b, h, r] = p @ vf[b, g, vis]
                lse[b, h, r] = lse_i
    return out, lse


def _check_decode(q, k, v):
    for name, a in (("q", q), ("k", k), ("v", v)):
        if not isinstance(a, np.ndarray) or a.dtype != np.uint16 or a.ndim != 4:
            raise TypeError(f"{name}: expected uint16 (bf16 bits) ndarray [B,H,N,D]")
    B, Hq, Nq, D = q.shape
    if k.shape != v.shape or k.shape[0] != B or k.shape[3] != D:
        raise ValueError("k/v shape mismatch")
    Hkv, Nk = k.shape[1], k.shape[2]
    if Hq % Hkv:
        raise ValueError("Hq must be a multiple of Hkv")
    if Nq > Nk:
        raise ValueError("the cache must hold the query tokens' own keys: Nq <= Nk")
    return B, Hq, Hkv, Nq, Nk, D


def swaa_decode_oracle(q, k, v, window, n_sink, scale, n_threads=0, n_prompt=None):
    """fp64 attention of the Nq newest tokens (q [B,Hq,Nq,D]) over a cache of Nk
    tokens (k, v [B,Hkv,Nk,D]) via the C oracle (paper Sec. 3.1.1).  Row r sits at
    position Nk - Nq + r; window >= Nk is full attention (FA Decode).  n_prompt:
    rows at positions >= n_prompt ignore the window (None: no such rows).  Returns
    (out [B,Hq,Nq,D] float64, lse [B,Hq,Nq] float64)."""
    B, Hq, Hkv, Nq, Nk, D = _check_decode(q, k, v)
    q, k, v = (np.ascontiguousarray(a) for a in (q, k, v))
    out = np.empty((B, Hq, Nq, D), dtype=np.float64)
    lse = np.empty((B, Hq, Nq), dtype=np.float64)
    rc = _load().swaa_oracle_decode(q.ctypes.data, k.ctypes.data, v.ctypes.data, B, Hq, Hkv, Nq, Nk, D,
                                    int(window), int(n_sink), Nk + 1 if n_prompt is None else int(n_prompt),
                                    float(scale), out.ctypes.data, lse.ctypes.data, int(n_threads))
    if rc != 0:
        raise ValueError(f"swaa_oracle_decode failed with code {rc}")
    return out, lse


def swaa_decode_oracle_numpy(q, k, v, window, n_sink, scale, n_prompt=None):
    """The same definition in numpy, row by row (slow; small inputs only)."""
    B, Hq, Hkv, Nq, Nk, D = _check_decode(q, k, v)
    W, S = int(window), int(n_sink)
    P = Nk + 1 if n_prompt is None else int(n_prompt)
    if W < 1 or S < 0 or P < 0:
        raise ValueError("window >= 1, n_sink >= 0 and n_prompt >= 0 required")
    G = Hq // Hkv
    qf, kf, vf = (_bf16_bits_to_f64(a) for a in (q, k, v))
    out = np.empty((B, Hq, Nq, D), dtype=np.float64)
    lse = np.empty((B, Hq, Nq), dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            for r in range(Nq):
                pos = Nk - Nq + r
                vis = [j for j in range(pos + 1) if (pos >= P) or (j > pos - W) or (j < S)]
                s = scale * (kf[b, g, vis] @ qf[b, h, r])
                m = s.max()
                lse_r = m + np.log(np.exp(s - m).sum())
                out[b, h, r] = np.exp(s - lse_r) @ vf[b, g, vis]
                lse[b, h, r] = lse_r
    return out, lse


def swaa_attn_bwd_oracle(q, k, v, dout, window, n_sink, scale, n_prompt=None, n_threads=0):
    """fp64 gradients of the one-pass forward (paper Sec. 3.2.2: fine-tuning trains through
    the mask) via the C oracle.  dout: uint16 bf16 bits [B,Hq,N,D].  Returns
    (dq [B,Hq,N,D], dk [B,Hkv,N,D], dv [B,Hkv,N,D]) float64."""
    B, Hq, Hkv, N, D = _check(q, k, v)
    if not isinstance(dout, np.ndarray) or dout.dtype != np.uint16 or dout.shape != q.shape:
        raise TypeError("dout: expected uint16 (bf16 bits) ndarray shaped like q")
    q, k, v, dout = (np.ascontiguousarray(a) for a in (q, k, v, dout))
    dq = np.empty((B, Hq, N, D), dtype=np.float64)
    dk = np.empty((B, Hkv, N, D), dtype=np.float64)
    dv = np.empty((B, Hkv, N, D), dtype=np.float64)
    rc = _load().swaa_oracle_bwd(q.ctypes.data, k.ctypes.data, v.ctypes.data, dout.ctypes.data, B, Hq, Hkv, N, D,
                                 int(window), int(n_sink), N if n_prompt is None else int(n_prompt), float(scale),
                                 dq.ctypes.data, dk.ctypes.data, dv.ctypes.data, int(n_threads))
    if rc != 0:
        raise ValueError(f"swaa_oracle_bwd failed with code {rc}")
    return dq, dk, dv
