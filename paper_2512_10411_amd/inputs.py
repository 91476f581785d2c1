"""Seeded synthetic inputs for SWA+sink prefill attention.

Data only: this module holds none of the method's arithmetic and is the one
piece that the tests, the benchmark, the GPU binding's callers and the CPU
oracle's callers share.  Values stand in for the long-context workloads the
paper evaluates on (16k-32k-token prompts, 128k-token prompts, windows of
2k/4k/8k or full attention: Sec. 4.1.2, Table 1, Table 5); the paper's own
efficiency experiment uses random inputs too (Sec. 4.2.2; its table is in App. D).

Tensors are returned as numpy uint16 arrays holding bf16 bit patterns in
[B, H, N, D] layout, drawn in the order q, k, v from a Philox stream.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even), return the uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    bits = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        bits[nan] = np.uint16(0x7FC0)
    return bits


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to float32 exactly."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass(frozen=True)
class Workload:
    """One attention-forward call: shapes, mask parameters, value recipe."""
    name: str
    B: int
    Hq: int
    Hkv: int
    N: int
    D: int
    window: int
    n_sink: int
    seed: int
    k_mult: float = 1.0   # k is multiplied by this (exact in bf16 for powers of two)
    n_prompt: int | None = None  # FA Decode runs: rows >= n_prompt are generated tokens
    n_query: int | None = None   # decode-shape and chunk runs: q holds only the n_query newest of the N tokens
    chunk: bool = False          # n_query rows are a chunk of a longer prefill (general forward), not a decode step
    backward: bool = False       # the timed call is the backward pass (the forward runs once, untimed)
    fmt: str = "bf16"            # element format of q, k, v, out: "bf16" or "fp16"
    recipe: str = "iid"          # "iid", or a structured score pattern laid over the draws (apply_recipe)
    page_size: int = 0           # > 0: k and v are handed over as a paged cache of such pages in a seeded random order
    packed_lens: tuple = ()      # a packed batch: sequences of these lengths back to back in one [H, sum, D] tensor (B = their number, N = the longest)
    seq_lens: tuple = ()         # a decode batch whose sequences hold this many cached tokens each (B = their number, N = the longest)

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.D)


_SEED0 = 2512104110

# The five configurations of the benchmark definition (seven runs: the third
# and fifth are run with an SWA window and again with window = N on the same
# tensors, modelling an SWA layer next to a full-attention layer).
WORKLOADS = {
    "tiny":        Workload("tiny",        1,  4, 1,   1024,  64,   128, 4, _SEED0 + 1),
    "mid":         Workload("mid",         1, 32, 8,  16384, 128,  2048, 4, _SEED0 + 2),
    "pair32k_swa": Workload("pair32k_swa", 1, 32, 8,  32768, 128,  4096, 4, _SEED0 + 3, 2.0),
    "pair32k_full": Workload("pair32k_full", 1, 32, 8, 32768, 128, 32768, 4, _SEED0 + 3, 2.0),
    "batched":     Workload("batched",     4, 40, 8,   8192, 128,  1024, 4, _SEED0 + 4),
    "long128k_swa": Workload("long128k_swa", 1, 32, 8, 131072, 128, 8192, 4, _SEED0 + 5),
    "long128k_full": Workload("long128k_full", 1, 32, 8, 131072, 128, 131072, 4, _SEED0 + 5),
    # FA Decode over a whole conversation in one pass (same tensors as the runs above):
    # the last 512 rows are generated tokens, the output length of the paper's
    # efficiency experiment (Sec. 4.2.2)
    "mid_fa_decode": Workload("mid_fa_decode", 1, 32, 8, 16384, 128, 2048, 4, _SEED0 + 2, 1.0, 16384 - 512),
    "long128k_fa_decode": Workload("long128k_fa_decode", 1, 32, 8, 131072, 128, 8192, 4, _SEED0 + 5, 1.0,
                                   131072 - 512),
    # decode steps of that experiment: one new token per sequence against a 128k-token cache,
    # with full attention (FA Decode) and on the window (decoding stays on SWA); and a batch of
    # 16 sequences of 16k tokens
    "decode128k_full": Workload("decode128k_full", 1, 32, 8, 131072, 128, 131072, 4, _SEED0 + 6, n_query=1),
    "decode128k_swa": Workload("decode128k_swa", 1, 32, 8, 131072, 128, 8192, 4, _SEED0 + 6, n_query=1),
    "decode16k_b16": Workload("decode16k_b16", 16, 32, 8, 16384, 128, 16384, 4, _SEED0 + 7, n_query=1),
    # the mid-size layer in binary16, the precision the paper serves in (Sec. 4.1.1); same draws
    # the serving engine's cache layout (Sec. 4.1.1: vLLM, whose default page holds 16 tokens)
    "decode16k_b16_paged": Workload("decode16k_b16_paged", 16, 32, 8, 16384, 128, 16384, 4, _SEED0 + 7, n_query=1,
                                    page_size=16),
    # continuous batching (Sec. 4.1.1: served with vLLM, batch size 64): one long sequence among
    # short ones, and a mix of lengths from 256 to 32k tokens
    "decode_skewed_b16": Workload("decode_skewed_b16", 16, 32, 8, 131072, 128, 131072, 4, _SEED0 + 8, n_query=1,
                                  seq_lens=(131072,) + (1024,) * 15),
    "decode_mixed_b32": Workload("decode_mixed_b32", 32, 32, 8, 32768, 128, 32768, 4, _SEED0 + 9, n_query=1,
                                 seq_lens=(32768, 16384, 8192, 4096, 2048, 1024, 512, 256) * 4),
    "decode128k_full_paged": Workload("decode128k_full_paged", 1, 32, 8, 131072, 128, 131072, 4, _SEED0 + 6, n_query=1,
                                      page_size=16),
    "mid_paged": Workload("mid_paged", 1, 32, 8, 16384, 128, 2048, 4, _SEED0 + 2, chunk=True, n_query=16384, page_size=16),
    "long128k_swa_paged": Workload("long128k_swa_paged", 1, 32, 8, 131072, 128, 8192, 4, _SEED0 + 5, chunk=True,
                                   n_query=131072, page_size=16),
    # prefill of a serving batch: prompts of different lengths packed into one tensor (cu_seqlens)
    "packed8_mixed": Workload("packed8_mixed", 8, 32, 8, 15909, 128, 1024, 4, _SEED0 + 9,
                              packed_lens=(12277, 10653, 12581, 8731, 11479, 11232, 9705, 15909)),
    "packed61_skewed": Workload("packed61_skewed", 61, 32, 8, 16000, 128, 1024, 4, _SEED0 + 10,
                                packed_lens=(16000, 113, 179, 227, 99, 52, 242, 367, 282, 348, 142, 344, 215, 91, 286, 372,
                                             198, 218, 55, 109, 166, 267, 334, 61, 274, 97, 109, 141, 195, 313, 162, 219,
                                             320, 210, 212, 335, 247, 387, 240, 399, 204, 301, 130, 179, 72, 79, 298, 97,
                                             126, 252, 317, 392, 233, 234, 195, 276, 97, 224, 369, 361, 231)),
    "mid_fp16": Workload("mid_fp16", 1, 32, 8, 16384, 128, 2048, 4, _SEED0 + 2, fmt="fp16"),
    # backward pass of the mid-size layer (fine-tuning under the window + sink mask)
    "mid_bwd": Workload("mid_bwd", 1, 32, 8, 16384, 128, 2048, 4, _SEED0 + 2, backward=True),
    # the last 2048-row chunk of a 128k-token prefill whose earlier keys and values are cached
    "chunk2k_128k_swa": Workload("chunk2k_128k_swa", 1, 32, 8, 131072, 128, 8192, 4, _SEED0 + 8, n_query=2048,
                                 chunk=True),
    # the mid-size layer with the paper's larger keep-first values (Table 1: k = 100, 1000; the
    # efficiency table of App. D has time to first token about 2 % higher at k = 100)
    "mid_s100": Workload("mid_s100", 1, 32, 8, 16384, 128, 2048, 100, _SEED0 + 2),
    "mid_s1000": Workload("mid_s1000", 1, 32, 8, 16384, 128, 2048, 1000, _SEED0 + 2),
    # the mid-size layer with attention-sink scores (Sec. 3.2.1): every query scores the first
    # tokens about 13 nats above the rest
    "mid_sinkheavy": Workload("mid_sinkheavy", 1, 32, 8, 16384, 128, 2048, 4, _SEED0 + 2, recipe="sink_heavy"),
    # and with isolated keys, one per 2048 positions deep inside the windows, that score about 42
    # nats above everything else: scores that outgrow a softmax reference taken from the first keys
    "mid_spike": Workload("mid_spike", 1, 32, 8, 16384, 128, 2048, 4, _SEED0 + 2, recipe="late_spike"),
    # the same with 80 nats: beyond what the pipelined kernel's fixed softmax reference covers, so
    # every workgroup takes its max-based second pass (the cost of that fallback)
    "mid_spike80": Workload("mid_spike80", 1, 32, 8, 16384, 128, 2048, 4, _SEED0 + 2, recipe="late_spike80"),
}


def apply_recipe(w: Workload, q: np.ndarray, k: np.ndarray):
    """Lay a structured score pattern over i.i.d. draws, in place (bit patterns of w.fmt).

    Component 0 of every query becomes 3 and that of every key 0, so that a key whose
    component 0 is set to c scores 3 c / sqrt(D) nats above the rest for every query.
      sink_heavy: the first n_sink keys get c = 48 (about 12.7 nats at D = 128);
      late_spike: keys 1500, 3548, 5596, ... (one per 2048 positions) get c = 160 (42 nats);
      late_spike80: the same keys get c = 304 (80 nats).
    """
    if w.recipe == "iid":
        return
    to_bits = f32_to_bf16_bits if w.fmt == "bf16" else f32_to_f16_bits
    bits = lambda x: to_bits(np.array([x], dtype=np.float32))[0]
    q[..., 0] = bits(3.0)
    k[..., 0] = bits(0.0)
    if w.recipe == "sink_heavy":
        k[:, :, :w.n_sink, 0] = bits(48.0)
    elif w.recipe == "late_spike":
        k[:, :, 1500::2048, 0] = bits(160.0)
    elif w.recipe == "late_spike80":
        k[:, :, 1500::2048, 0] = bits(304.0)
    else:
        raise ValueError(f"unknown recipe {w.recipe}")


def f32_to_f16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> IEEE binary16 bit patterns (round to nearest even), as uint16."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def f16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(bits, dtype=np.uint16).view(np.float16).astype(np.float32)


def make_qkv(B, Hq, Hkv, N, D, seed, k_mult=1.0, chunk_rows=1 << 22, n_query=None, fmt="bf16"):
    """i.i.d. N(0,1) q, k, v rounded to bf16; k scaled by k_mult before rounding.

    Generated in row chunks so that the float32 staging buffer stays small even
    for the 128k-token workloads.  n_query: q has only that many rows per head
    (decode shape), k and v keep N.  fmt: "bf16" or "fp16" (same draws, rounded to
    the other format).
    """
    to_bits = f32_to_bf16_bits if fmt == "bf16" else f32_to_f16_bits
    rng = np.random.Generator(np.random.Philox(int(seed)))

    def draw(H, mult, N=N):
        out = np.empty((B * H * N, D), dtype=np.uint16)
        for r0 in range(0, out.shape[0], chunk_rows):
            r1 = min(out.shape[0], r0 + chunk_rows)
            x = rng.standard_normal((r1 - r0, D), dtype=np.float32)
            if mult != 1.0:
                x *= np.float32(mult)
            out[r0:r1] = to_bits(x)
        return out.reshape(B, H, N, D)

    q = draw(Hq, 1.0) if n_query is None else draw(Hq, 1.0, int(n_query))
    k = draw(Hkv, k_mult)
    v = draw(Hkv, 1.0)
    return q, k, v


def make_workload(w: Workload):
    """q, k, v (uint16 bf16 bits) for a named workload."""
    if w.packed_lens:  # one [1, H, sum of the lengths, D] tensor each; the sequence boundaries are the caller's offsets
        return make_qkv(1, w.Hq, w.Hkv, sum(w.packed_lens), w.D, w.seed, w.k_mult, fmt=w.fmt)
    if w.seq_lens:  # q [B, Hq, n_query, D]; k, v [1, Hkv, sum of the lengths, D], the sequences' tokens back to back
        q, _, _ = make_qkv(w.B, w.Hq, 1, 1, w.D, w.seed, n_query=w.n_query, fmt=w.fmt)
        _, k, v = make_qkv(1, 1, w.Hkv, sum(w.seq_lens), w.D, w.seed + 1, w.k_mult, n_query=1, fmt=w.fmt)
        return q, k, v
    q, k, v = make_qkv(w.B, w.Hq, w.Hkv, w.N, w.D, w.seed, w.k_mult, n_query=w.n_query, fmt=w.fmt)
    apply_recipe(w, q, k)
    return q, k, v


def sample_rows(N, window, n_sink, count=256, seed=0, tile=64):
    """Query rows on which large runs are compared with the oracle.

    Always holds the rows where the mask changes shape (first rows, around the
    sink count, around the window length, the last row), rows around a few
    seeded tile boundaries, and seeded uniform rows up to `count` in total.
    Sorted, unique, all in [0, N).
    """
    W, S = int(window), int(n_sink)
    fixed = [0, 1, S - 1, S, S + 1, W - 2, W - 1, W, W + 1, W + S - 1, W + S, W + S + 1, N - 2, N - 1]
    rng = np.random.Generator(np.random.Philox(int(seed) + 977))
    n_tiles = max(1, N // tile)
    for t in rng.integers(1, n_tiles + 1, size=8):
        fixed += [int(t) * tile - 1, int(t) * tile, int(t) * tile + 1]
    rows = {r for r in fixed if 0 <= r < N}
    count = min(count, N)
    while len(rows) < count:
        for r in rng.integers(0, N, size=count - len(rows)):
            rows.add(int(r))
    return np.array(sorted(rows), dtype=np.int32)


def paged_cache(k, v, page_size: int, seed: int):
    """Rearranges device tensors k, v [B, Hkv, N, D] (N a multiple of page_size) into a paged cache:
    returns views (k_cache, v_cache) [num_pages, Hkv, page_size, D] and the int32 block table
    [B, N / page_size], pages in a seeded random order with a few unused pages in between."""
    import torch

    B, Hkv, N, D = k.shape
    assert N % page_size == 0
    npg = N // page_size
    num_pages = B * npg + 3
    order = np.random.Generator(np.random.Philox(seed)).permutation(num_pages)[:B * npg].astype(np.int64)
    perm = torch.from_numpy(order).to(k.device)
    caches = []
    for t in (k, v):
        c = torch.zeros((num_pages, Hkv, page_size, D), dtype=t.dtype, device=t.device)
        c[perm] = t.view(B, Hkv, npg, page_size, D).permute(0, 2, 1, 3, 4).reshape(B * npg, Hkv, page_size, D)
        caches.append(c)
    table = perm.view(B, npg).to(torch.int32)
    return caches[0], caches[1], table
