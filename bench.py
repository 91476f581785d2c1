#!/usr/bin/env python3
"""Benchmark of the SWA + sink prefill attention forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

One "step" is one call of swaa_attn_fwd (the whole hot path: tile schedule,
Q/K/V staging, QK^T, mask, online softmax, PV, epilogue) over one batch of
seeded synthetic bf16 inputs that are already resident in HBM.  The default
workload is the largest configuration of the benchmark definition, the 128k-token
prompt with an 8k window (long128k_swa: B=1, Hq=32, Hkv=8, N=131072, D=128,
W=8192, S=4; the prompt length of the paper's efficiency experiment, Sec. 4.2.2 /
App. D).  Prints ONE JSON line: effective TFLOP/s (4*D flops per visible
query-key pair per head), the MFMA roofline fraction of the kernel measured with
HIP events on the launch stream, for window < N also the same tensors timed with
window = N (linear_in_w: time ratio against visible-pair ratio, App. A: O(N W)),
and the fp64 CPU oracle timed on this machine's host cores on a bounded sample of
the same rows.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "SWA+sink prefill attention effective TFLOP/s and % bf16 MFMA peak, 1 MI355X"
BF16_MFMA_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak
HBM_PEAK_GBS = 8000.0           # MI355X HBM3E

# HBM bytes per launch (read + written) of the attention kernel, measured with two
# rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) scaled by a copy kernel of known size, and
# the summary under profiles/ each figure is taken from (calls made of several kernels: the
# sum over them).  roofline.traffic is NOT a reading of this run: traffic_source names the
# file (or "--traffic-bytes"); workloads without a summary report null.
MEASURED_TRAFFIC_BYTES = {
    "mid": (4.02e8, "profiles/swaa_fwd_pipelined_mid.txt"),
    "batched": (1.015e9, "profiles/swaa_fwd_pipelined_batched.txt"),
    "pair32k_swa": (1.083e9, "profiles/swaa_fwd_pipelined_pair32k_swa.txt"),
    "pair32k_full": (2.64e9, "profiles/swaa_fwd_pipelined_pair32k_full.txt"),
    "long128k_swa": (6.807e9, "profiles/swaa_fwd_pipelined_long128k_swa.txt"),
    "long128k_full": (2.669e11, "profiles/swaa_fwd_pipelined_long128k_full.txt"),
    "decode128k_full": (5.411e8, "profiles/swaa_decode_decode128k_full.txt"),
    "decode16k_b16": (1.079e9, "profiles/swaa_decode_decode16k_b16.txt"),
    "decode128k_swa": (3.665e7, "profiles/swaa_decode_decode128k_swa.txt"),
    "decode_skewed_b16": (6.081e8, "profiles/swaa_decode_decode_skewed_b16.txt"),
    "decode_mixed_b32": (1.078e9, "profiles/swaa_decode_decode_mixed_b32.txt"),
    "mid_bwd": (1.63e9, "profiles/swaa_bwd_mid_bwd.txt"),
}
MIN_WARMUP_S = 0.05  # the clocks settle only after some tens of ms of continuous work


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # The GPU's clocks take some tens of milliseconds of continuous work to settle after the
    # host-side input generation: whatever --warmup says, untimed launches go on until
    # MIN_WARMUP_S have passed (the JSON line reports how many ran).
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="long128k_swa")
    ap.add_argument("--no-linear-in-w", action="store_true",
                    help="skip the window = N launches on the same tensors (profiling runs)")
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="skip the oracle timing (profiling runs)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0,
                    help="target CPU time of the oracle sample")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="HBM bytes per launch from a separate rocprofv3 --pmc run, if known")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run one plain device-to-device copy of this many MiB after the warm-up: under "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE it is the kernel of known traffic that "
                         "the attention kernel's counters are scaled by")
    return ap.parse_args()


def decode_counts(w):
    """(visible pairs per launch, algorithmic HBM bytes per launch) of a decode-shape workload."""
    if w.seq_lens:  # one sequence at a time
        import dataclasses
        each = [decode_counts(dataclasses.replace(w, B=1, N=n, seq_lens=())) for n in w.seq_lens]
        return sum(e[0] for e in each), sum(e[1] for e in each)
    Nq, Nk = w.n_query, w.N
    W, S = min(w.window, Nk), min(w.n_sink, Nk)
    pairs = 0
    for r in range(Nq):
        pos = Nk - Nq + r
        pairs += min(pos + 1, W) + min(max(pos - W + 1, 0), S)
    band_lo = max(0, Nk - Nq - W + 1)
    keys = min(S, band_lo) + (Nk - band_lo)  # keys some query row sees: read once, K and V
    nbytes = w.B * w.Hkv * keys * 2 * w.D * 2 + w.B * w.Hq * Nq * (2 * w.D * 2 + 4)
    return pairs * w.B * w.Hq, nbytes


def cpu_baseline_decode(w, q, k, v):
    """Time the oracle as it stands on the whole decode-shape workload (it is small)."""
    from oracle import oracle_num_threads, swaa_decode_oracle
    t0 = time.perf_counter()
    if w.seq_lens:  # sequence by sequence (k, v hold their tokens back to back)
        t = 0
        for b, n in enumerate(w.seq_lens):
            swaa_decode_oracle(q[b:b + 1], k[:, :, t:t + n], v[:, :, t:t + n], w.window, w.n_sink, w.scale)
            t += n
    else:
        swaa_decode_oracle(q, k, v, w.window, w.n_sink, w.scale)
    dt = time.perf_counter() - t0
    pairs, _ = decode_counts(w)
    return {
        "value": 4.0 * w.D * pairs / dt / 1e12,
        "unit": "TFLOP/s",
        "cores": oracle_num_threads(),
        "kind": "oracle",
        "sample": f"the whole workload '{w.name}' once: all {w.B * w.Hq * w.n_query} query rows, {pairs} visible "
                  f"pairs in {dt:.2f} s; fp64, OpenMP over rows",
        "seconds": dt,
        "pairs_per_s": pairs / dt,
    }


def cpu_baseline_backward(w, q, k, v, dout, prefix=1024):
    """Time the oracle's backward as it stands on the first `prefix` tokens of every head."""
    import numpy as np
    from oracle import oracle_num_threads, swaa_attn_bwd_oracle
    from paper_2512_10411_amd.binding import swaa_visible_pairs
    n = min(prefix, w.N)
    cut = lambda a: np.ascontiguousarray(a[:, :, :n])
    t0 = time.perf_counter()
    swaa_attn_bwd_oracle(cut(q), cut(k), cut(v), cut(dout), w.window, w.n_sink, w.scale)
    dt = time.perf_counter() - t0
    pairs = swaa_visible_pairs(n, w.window, w.n_sink) * w.B * w.Hq
    return {
        "value": 10.0 * w.D * pairs / dt / 1e12,
        "unit": "TFLOP/s",
        "cores": oracle_num_threads(),
        "kind": "oracle",
        "sample": f"backward of the first {n} tokens of all {w.B * w.Hq} (batch, head) of workload '{w.name}': "
                  f"{pairs} visible pairs in {dt:.2f} s; fp64, OpenMP over rows",
        "seconds": dt,
        "pairs_per_s": pairs / dt,
    }


def cpu_baseline(w, q, k, v, target_s):
    """Time the oracle as it stands on a bounded sample of this workload's rows."""
    import numpy as np
    from oracle import oracle_num_threads, swaa_attn_oracle
    from paper_2512_10411_amd.binding import swaa_visible_pairs_fa_decode

    n_prompt = w.N if w.n_prompt is None else w.n_prompt

    def pairs_of(rows):
        r = np.asarray(rows, dtype=np.int64)
        vis = np.minimum(r + 1, min(w.window, w.N)) + np.clip(r - w.window + 1, 0, min(w.n_sink, w.N))
        vis = np.where(r >= n_prompt, r + 1, vis)
        return int(vis.sum()) * w.B * w.Hq

    rng = np.random.Generator(np.random.Philox(w.seed + 5))
    order = rng.permutation(w.N)
    pilot = np.sort(order[:8])
    t0 = time.perf_counter()
    swaa_attn_oracle(q, k, v, w.window, w.n_sink, w.scale, rows=pilot, n_prompt=n_prompt)
    t_pilot = max(time.perf_counter() - t0, 1e-4)
    rate = pairs_of(pilot) / t_pilot
    mean_pairs_per_row = swaa_visible_pairs_fa_decode(w.N, w.window, w.n_sink, n_prompt) * w.B * w.Hq / w.N
    n_rows = int(min(w.N, max(8, target_s * rate / mean_pairs_per_row)))
    rows = np.sort(order[:n_rows])
    t0 = time.perf_counter()
    swaa_attn_oracle(q, k, v, w.window, w.n_sink, w.scale, rows=rows, n_prompt=n_prompt)
    dt = time.perf_counter() - t0
    pairs = pairs_of(rows)
    return {
        "value": 4.0 * w.D * pairs / dt / 1e12,
        "unit": "TFLOP/s",
        "cores": oracle_num_threads(),
        "kind": "oracle",
        "sample": f"{n_rows} seeded random query rows x all {w.B * w.Hq} (batch, head) of workload "
                  f"'{w.name}': {pairs} visible pairs in {dt:.2f} s; fp64, OpenMP over rows",
        "seconds": dt,
        "pairs_per_s": pairs / dt,
    }


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); "
              f"--gpus {args.gpus} is not supported, use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2512_10411_amd import binding
    from paper_2512_10411_amd.inputs import WORKLOADS, make_workload

    if args.workload not in WORKLOADS:
        print(f"unknown workload {args.workload}; choose from {sorted(WORKLOADS)}", file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (there is no CPU fallback for the product path)", file=sys.stderr)
        return 2
    w = WORKLOADS[args.workload]
    binding.load_library()

    q, k, v = make_workload(w)

    def dev(bits):
        import numpy as np
        return torch.from_numpy(bits.view(np.int16)).view(torch.float16 if w.fmt == "fp16" else torch.bfloat16).cuda()

    qd, kd, vd = dev(q), dev(k), dev(v)
    out = torch.empty_like(qd)
    lse = torch.empty(qd.shape[:3], dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    n_prompt = w.N if w.n_prompt is None else w.n_prompt
    decode = w.n_query is not None and not w.chunk
    seq_lens = None
    if w.seq_lens:
        # a [B, Hkv, longest, D] cache buffer, each sequence filled up to its own length
        seq_lens = torch.tensor(w.seq_lens, dtype=torch.int32, device="cuda")
        kbuf = torch.empty((w.B, w.Hkv, w.N, w.D), dtype=kd.dtype, device="cuda")  # (rows past a sequence's length are never read)
        vbuf = torch.empty_like(kbuf)
        t = 0
        for b, n in enumerate(w.seq_lens):
            kbuf[b, :, :n], vbuf[b, :, :n] = kd[0, :, t:t + n], vd[0, :, t:t + n]
            t += n
        kd, vd = kbuf, vbuf
    if decode:
        # (the general call's size for the workloads that go through it: sequence lengths change the split plan)
        da = binding.SwaaDecodeArgs()
        da.B, da.Hq, da.Hkv, da.Nq, da.Nk, da.D, da.window, da.n_sink = w.B, w.Hq, w.Hkv, w.n_query, w.N, w.D, w.window, w.n_sink
        da.seq_lens = seq_lens.data_ptr() if seq_lens is not None else None
        ws = torch.empty(binding.swaa_attn_decode_ex_workspace_bytes(da), dtype=torch.uint8, device="cuda")

    if w.packed_lens:
        import numpy as np
        cu = torch.from_numpy(np.concatenate([[0], np.cumsum(w.packed_lens)]).astype(np.int32)).cuda()
        qd, kd, vd, out, lse = qd[0], kd[0], vd[0], out[0], lse[0]  # [H, T, D] / [H, T]

    if w.page_size:
        # the same keys and values as a paged cache (pages in a seeded random order)
        from paper_2512_10411_amd.inputs import paged_cache
        kd, vd, table = paged_cache(kd, vd, w.page_size, w.seed + 31)

    if w.backward:
        import numpy as np
        from paper_2512_10411_amd.inputs import f32_to_bf16_bits
        dout = f32_to_bf16_bits(np.random.Generator(np.random.Philox(w.seed + 9)).standard_normal(
            q.shape, dtype=np.float32))
        dd = dev(dout)
        binding.swaa_attn_fwd(qd, kd, vd, w.window, w.n_sink, w.scale, out=out, lse=lse, stream=stream)
        bws = torch.empty(binding.swaa_attn_bwd_workspace_bytes(w.B, w.Hq, w.Hkv, w.N, w.D, w.window, w.n_sink), dtype=torch.uint8, device="cuda")

    def step():
        if w.backward:
            binding.swaa_attn_bwd(qd, kd, vd, out, lse, dd, w.window, w.n_sink, None, w.scale, workspace=bws,
                                  stream=stream)
        elif w.packed_lens:
            binding.swaa_attn_fwd_ex(qd, kd, vd, w.window, w.n_sink, None, w.scale, cu_seqlens_q=cu, cu_seqlens_k=cu,
                                     max_seqlen_q=w.N, max_seqlen_k=w.N, out=out, lse=lse, stream=stream)
        elif decode and w.page_size:
            binding.swaa_attn_decode_ex(qd, kd, vd, w.window, w.n_sink, w.scale, block_table=table, max_seqlen_k=w.N,
                                        out=out, lse=lse, workspace=ws, stream=stream)
        elif decode and w.seq_lens:
            binding.swaa_attn_decode_ex(qd, kd, vd, w.window, w.n_sink, w.scale, seq_lens=seq_lens, out=out, lse=lse,
                                        workspace=ws, stream=stream)
        elif decode:
            binding.swaa_attn_decode(qd, kd, vd, w.window, w.n_sink, w.scale, out=out, lse=lse, workspace=ws,
                                     stream=stream)
        elif w.page_size:
            binding.swaa_attn_fwd_ex(qd, kd, vd, w.window, w.n_sink, w.n_prompt, w.scale, out=out, lse=lse,
                                     stream=stream, block_table=table, max_seqlen_k=w.N)
        elif w.chunk or w.fmt == "fp16":
            binding.swaa_attn_fwd_ex(qd, kd, vd, w.window, w.n_sink, w.n_prompt, w.scale, out=out, lse=lse,
                                     stream=stream)
        elif w.n_prompt is None:
            binding.swaa_attn_fwd(qd, kd, vd, w.window, w.n_sink, w.scale, out=out, lse=lse, stream=stream)
        else:
            binding.swaa_attn_fwd_fa_decode(qd, kd, vd, w.window, w.n_sink, n_prompt, w.scale, out=out, lse=lse,
                                            stream=stream)

    warmup_done = 0
    t_w = time.perf_counter()
    while warmup_done < args.warmup or time.perf_counter() - t_w < MIN_WARMUP_S:
        step()
        warmup_done += 1
        if warmup_done >= args.warmup:
            torch.cuda.synchronize()  # (only while topping up to the minimum time)
    torch.cuda.synchronize()
    if args.copy_probe_mib > 0:
        src = torch.ones(args.copy_probe_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)  # reads and writes copy_probe_mib MiB once
        torch.cuda.synchronize()
        del src, dst

    # K steps, wall clock bracketed by synchronisation on both sides.  One HIP event
    # pair on the launch stream brackets the same K launches: its elapsed time / K is
    # the kernel's average launch duration (nothing is recorded between launches, so
    # consecutive launches run back to back exactly as in the wall-clock figure).
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(args.steps):
        step()
    ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_avg_ms = ev0.elapsed_time(ev1) / args.steps
    ms_per_step = wall * 1e3 / args.steps

    if w.packed_lens:
        pairs = sum(binding.swaa_visible_pairs(n, w.window, w.n_sink) for n in w.packed_lens) * w.Hq
    elif decode or w.chunk:
        pairs, algo_bytes = decode_counts(w)
    else:
        pairs = binding.swaa_visible_pairs_fa_decode(w.N, w.window, w.n_sink, n_prompt) * w.B * w.Hq
    # forward: two products per visible pair; backward: five (the customary count; the
    # recomputation the two-kernel backward does on top of them is not credited)
    flops = (10.0 if w.backward else 4.0) * w.D * pairs
    value = flops / (ms_per_step * 1e-3) / 1e12
    achieved = flops / (kern_avg_ms * 1e-3) / 1e12
    if args.traffic_bytes is not None:
        traffic, traffic_source = args.traffic_bytes, "--traffic-bytes"
    else:
        traffic, traffic_source = MEASURED_TRAFFIC_BYTES.get(w.name, (None, None))

    # The same tensors with window = N (the full-attention layer next to this SWA layer):
    # the time ratio should follow the visible-pair ratio if the work is linear in N * W.
    linear_in_w = None
    plain_prefill = not (decode or w.chunk or w.backward or w.fmt == "fp16" or w.packed_lens) and w.n_prompt is None
    if plain_prefill and w.window < w.N and not args.no_linear_in_w:
        def full_step():
            binding.swaa_attn_fwd(qd, kd, vd, w.N, w.n_sink, w.scale, out=out, lse=lse, stream=stream)
        full_step()
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        full_step()
        e1.record(stream)
        torch.cuda.synchronize()
        t_one = e0.elapsed_time(e1)
        n_full = max(2, min(args.steps, int(300.0 / max(t_one, 1e-3))))  # about 0.3 s of launches
        e0.record(stream)
        for _ in range(n_full):
            full_step()
        e1.record(stream)
        torch.cuda.synchronize()
        t_full_ms = e0.elapsed_time(e1) / n_full
        pairs_full = binding.swaa_visible_pairs(w.N, w.N, w.n_sink) * w.B * w.Hq
        linear_in_w = {"t_swa_ms": kern_avg_ms, "t_full_ms": t_full_ms, "time_ratio": kern_avg_ms / t_full_ms,
                       "pair_ratio": pairs / pairs_full, "full_steps": n_full,
                       "full_tflops": 4.0 * w.D * pairs_full / (t_full_ms * 1e-3) / 1e12,
                       "full_frac": 4.0 * w.D * pairs_full / (t_full_ms * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS}
        # leave the SWA result in out / lse (nothing below reads them, but a reader of this file might)
        step()
        torch.cuda.synchronize()
    if decode:
        # few query rows against a long cache: the keys and values are read once and nothing is
        # reused, so HBM bandwidth bounds the call (split kernel + merge kernel, timed together)
        gbs = algo_bytes / (kern_avg_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                    "traffic": traffic, "traffic_source": traffic_source,
                    "kernel": "swaa_decode_split_kernel (+ swaa_decode_merge_kernel)",
                    "kernel_avg_ms": kern_avg_ms, "algorithmic_bytes": algo_bytes}
    else:
        # (the fp16 matrix peak equals the bf16 one)
        roofline = {"bound": "mfma", "achieved": achieved, "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / BF16_MFMA_PEAK_TFLOPS, "traffic": traffic, "traffic_source": traffic_source,
                    "kernel": (("swaa_bwd_dkv_dma_kernel + swaa_bwd_dq_pipelined_kernel + swaa_bwd_delta_kernel" if w.D == 128 else
                                f"swaa_bwd_dkv_kernel<{w.D}> + swaa_bwd_dq_kernel<{w.D}> + swaa_bwd_delta_kernel") if w.backward
                               else "swaa_fwd_pipelined_kernel" if w.D == 128
                               else f"swaa_fwd_kernel<{w.D}>"),
                    "kernel_avg_ms": kern_avg_ms}

    res = {
        "metric": METRIC,
        "value": value,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "warmup_launches": warmup_done,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16" if w.fmt == "fp16" else "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "N": w.N, "n_query": w.n_query or w.N,
                   "D": w.D,
                   "window": w.window, "n_sink": w.n_sink, "n_prompt": n_prompt, "seed": w.seed, "k_mult": w.k_mult,
                   "visible_pairs": pairs, "flops_per_step": flops,
                   "pct_bf16_mfma_peak": 100.0 * value / BF16_MFMA_PEAK_TFLOPS,
                   **({"packed_lens": list(w.packed_lens)} if w.packed_lens else {}),
                   **({"seq_lens": list(w.seq_lens)} if w.seq_lens else {})},
        "roofline": roofline,
    }
    if linear_in_w is not None:
        res["linear_in_w"] = linear_in_w
    if w.packed_lens:
        res["cpu_baseline"] = None  # (the oracle is timed on the fixed-length workloads)
    elif not args.no_cpu_baseline:
        from oracle import input_format
        with input_format(w.fmt):
            res["cpu_baseline"] = (cpu_baseline_backward(w, q, k, v, dout) if w.backward
                                   else cpu_baseline_decode(w, q, k, v) if decode or (w.chunk and w.n_query < w.N)
                                   else cpu_baseline(w, q, k, v, args.cpu_seconds))
        res["cpu_baseline"]["gpu_over_cpu"] = value / res["cpu_baseline"]["value"]
    print(json.dumps(res), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
