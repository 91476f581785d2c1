#!/usr/bin/env python3
"""Attention-only cost model of a stack of layers under the SWAA recipes.

    python -m paper_2512_10411_amd.layer_driver [--n 131072] [--gen 512] [--layers 36]

For every configuration of the paper's efficiency table (App. D, Table 5: window, keep
first k, FA Decode, fraction of full-attention layers) the script runs the attention calls
one request would make on one GPU -- per layer one prefill call over the n prompt tokens
(window W on a sliding-window layer, W >= n on a full-attention layer), then per generated
token and layer one decode call against the cache (full attention under FA Decode or on a
full-attention layer, the window otherwise) -- and reports the time per request spent in
attention and its ratio to the all-full-attention row.  Only attention is modelled: no
projections, MLP, sampling or scheduling, so the ratios bound what the recipes can gain,
they are not end-to-end numbers.  The tensors are synthetic (seeded N(0,1), bf16) and are
reused by all layers; head geometry Hq 32 / Hkv 8 / D 128 as in the mid-size benchmark.

Decode calls are timed at the cache length halfway through generation and multiplied by the
number of generated tokens (their cost is linear in the cache length).
"""
from __future__ import annotations

import argparse
import json
import sys


# (window, keep first, FA decode, one full-attention layer in every `fa_every` layers or 0)
TABLE = [
    ("Full", 0, False, 0),
    ("2k", 0, False, 0), ("2k", 100, False, 0), ("2k", 0, False, 2), ("2k", 0, True, 0), ("2k", 0, True, 2),
    ("2k", 0, True, 4),
    ("4k", 0, False, 0), ("4k", 100, False, 0), ("4k", 0, False, 2), ("4k", 0, True, 0), ("4k", 0, True, 2),
    ("4k", 0, True, 4),
]
WINDOWS = {"2k": 2048, "4k": 4096, "8k": 8192}


def time_calls(fn, reps):
    import torch
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / reps


def run(n, gen, layers, reps=5, seed=2512104190, Hq=32, Hkv=8, D=128, quiet=False):
    import torch
    from . import binding
    from .inputs import make_qkv

    q, k, v = make_qkv(1, Hq, Hkv, n + gen, D, seed)
    dev = lambda bits: torch.from_numpy(bits.view("int16")).view(torch.bfloat16).cuda()
    qd, kd, vd = dev(q), dev(k), dev(v)
    qp, kp, vp = (t[:, :, :n].contiguous() for t in (qd, kd, vd))  # the prompt
    n_mid = n + gen // 2                                            # cache length halfway through generation
    q1 = qd[:, :, n_mid - 1:n_mid].contiguous()
    kc, vc = (t[:, :, :n_mid].contiguous() for t in (kd, vd))
    out = torch.empty_like(qp)
    lse = torch.empty((1, Hq, n), dtype=torch.float32, device="cuda")
    o1 = torch.empty_like(q1)
    l1 = torch.empty((1, Hq, 1), dtype=torch.float32, device="cuda")
    ws = torch.empty(binding.swaa_attn_decode_workspace_bytes(1, Hq, Hkv, 1, n_mid, D, n_mid, 0), dtype=torch.uint8,
                     device="cuda")

    cache = {}

    def prefill_s(W, S):
        key = ("p", min(W, n), S if W < n else 0)
        if key not in cache:
            cache[key] = time_calls(lambda: binding.swaa_attn_fwd(qp, kp, vp, W, S, out=out, lse=lse), reps)
        return cache[key]

    def decode_s(W, S):
        key = ("d", min(W, n_mid), S if W < n_mid else 0)
        if key not in cache:
            cache[key] = time_calls(lambda: binding.swaa_attn_decode(q1, kc, vc, W, S, out=o1, lse=l1, workspace=ws),
                                    4 * reps)
        return cache[key]

    rows = []
    for wname, keep, fa_decode, fa_every in TABLE:
        W = WINDOWS.get(wname, 2**31 - 1)
        n_fa = layers // fa_every if fa_every else (layers if wname == "Full" else 0)
        n_swa = layers - n_fa
        prefill = n_swa * prefill_s(W, keep) + n_fa * prefill_s(2**31 - 1, 0)
        dec_swa = decode_s(2**31 - 1, 0) if fa_decode else decode_s(W, keep)
        decode_tok = n_swa * dec_swa + n_fa * decode_s(2**31 - 1, 0)
        rows.append({"window": wname, "keep_first": keep, "fa_decode": fa_decode,
                     "fa_layers": f"1/{fa_every}" if fa_every else ("all" if wname == "Full" else "none"),
                     "prefill_s": prefill, "decode_s_per_token": decode_tok, "request_s": prefill + gen * decode_tok})
    full = rows[0]["request_s"]
    for r in rows:
        r["speedup_vs_full"] = full / r["request_s"]
    if not quiet:
        print(f"attention-only time of one request: {n} prompt tokens, {gen} generated, {layers} layers, "
              f"Hq {Hq} / Hkv {Hkv} / D {D}, one MI355X")
        print(f"{'window':>6} {'keep':>5} {'FA decode':>9} {'FA layers':>9} {'prefill ms':>11} {'decode us/tok':>14} "
              f"{'request ms':>11} {'x vs full':>9}")
        for r in rows:
            print(f"{r['window']:>6} {r['keep_first']:>5} {str(r['fa_decode']):>9} {r['fa_layers']:>9} "
                  f"{r['prefill_s'] * 1e3:11.2f} {r['decode_s_per_token'] * 1e6:14.1f} {r['request_s'] * 1e3:11.2f} "
                  f"{r['speedup_vs_full']:9.2f}")
    return rows


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--n", type=int, default=131072, help="prompt length")
    ap.add_argument("--gen", type=int, default=512, help="generated tokens")
    ap.add_argument("--layers", type=int, default=36)
    ap.add_argument("--json", action="store_true", help="print the rows as one JSON line as well")
    args = ap.parse_args()
    rows = run(args.n, args.gen, args.layers)
    if args.json:
        print(json.dumps(rows))
    return 0


if __name__ == "__main__":
    sys.exit(main())
