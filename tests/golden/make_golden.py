#!/usr/bin/env python3
"""Writes the stored expected values of the large-model parity tests.

Calls only the CPU oracle and the seeded workload generators; nothing here
touches the HIP path.  For a workload (model shape, context length L0, window
k) it runs the oracle over the context, takes the model's greedy continuation
c[0..k] (c[0] is the model's token for position L0), and evaluates verify
windows: the uncorrupted window c[0..k) and corrupted ones.  Per window it
stores, for every row: the arg-max token, the top-2 margin, the eight largest
logits with their ids, and the logits at fixed sampled vocabulary ids.

Arithmetic: float32 numpy (the 8B-shape model in float64 would need more host
memory than the build machine has); weights are the bf16 values upcast.

    python tests/golden/make_golden.py 8b_k8_ctx2048 [--out tests/golden/8b_k8_ctx2048.json]
"""
import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import Decoder, argmax_lowest, top2_margin          # noqa: E402
from workload import SHAPES, WeightStore, prompt_tokens, corrupt_drafts   # noqa: E402

WORKLOADS = {
    # name: (shape, L0, k, seed, corruption probabilities of the extra windows)
    "8b_k8_ctx2048": ("8b", 2048, 8, 2, (0.1, 0.3, 0.6)),
    "8b_k16_ctx16384": ("8b", 16384, 16, 3, (0.3,)),
    "1b_k5_ctx512": ("1b", 512, 5, 1, (0.3,)),
}
# greedy-sequence workloads: name -> (shape, prompt length, tokens to generate, seed)
GREEDY = {
    "8b_greedy_p128_n256": ("8b", 128, 256, 4),
}
N_SAMPLED_IDS = 64


def log(msg):
    print(f"[golden {time.strftime('%H:%M:%S')}] {msg}", flush=True)


def sampled_ids(vocab, seed):
    g = np.random.Generator(np.random.Philox(key=[seed, 77]))
    return np.sort(g.choice(vocab, size=N_SAMPLED_IDS, replace=False)).astype(np.int64)


def describe_rows(logits, ids):
    rows = []
    for z in logits:
        top = np.argsort(-z, kind="stable")[:8]
        rows.append({"argmax": argmax_lowest(z), "margin": top2_margin(z),
                     "top_ids": [int(i) for i in top], "top_logits": [float(z[i]) for i in top],
                     "sampled_logits": [float(z[i]) for i in ids]})
    return rows


def greedy_sequence(name, out_path):
    """The verify model's plain greedy continuation of a prompt with the top-2
    margin at every position (the reference of the full decoding loops)."""
    shape_name, P, N, seed = GREEDY[name]
    shape = SHAPES[shape_name]
    store = WeightStore(shape, cache=False)
    dec = Decoder(shape, store, P + N + 1, dtype=np.float32, keep_weights=True)   # fp32 weights stay in memory
    dec.progress = log
    prompt = prompt_tokens(seed, P, shape.vocab)
    z = dec.rows(prompt, logits_from=P - 1)
    dec.progress = None
    toks, margins = [argmax_lowest(z[-1])], [top2_margin(z[-1])]
    for i in range(1, N):
        z = dec.step(toks[-1])
        toks.append(argmax_lowest(z))
        margins.append(top2_margin(z))
        if i % 16 == 0:
            log(f"  {i}/{N} tokens")
    doc = {"workload": name, "shape": shape_name, "prompt_len": P, "n_new": N, "seed": seed,
           "oracle_dtype": "float32", "prompt_sha256": hashlib.sha256(prompt.tobytes()).hexdigest(),
           "tokens": [int(t) for t in toks], "margins": margins}
    with open(out_path, "w") as f:
        json.dump(doc, f, indent=1)
    log(f"wrote {out_path}")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("workload", choices=sorted(WORKLOADS) + sorted(GREEDY))
    ap.add_argument("--out")
    ap.add_argument("--block", type=int, default=512, help="context rows per batched oracle pass")
    args = ap.parse_args()
    if args.workload in GREEDY:
        greedy_sequence(args.workload, args.out or os.path.join(os.path.dirname(os.path.abspath(__file__)),
                                                                args.workload + ".json"))
        return
    shape_name, L0, k, seed, ps = WORKLOADS[args.workload]
    shape = SHAPES[shape_name]
    out_path = args.out or os.path.join(os.path.dirname(os.path.abspath(__file__)), args.workload + ".json")

    store = WeightStore(shape, cache=True)
    dec = Decoder(shape, store, L0 + k + 1, dtype=np.float32, keep_weights=False)
    dec.progress = log
    prompt = prompt_tokens(seed, L0, shape.vocab)
    log(f"{args.workload}: oracle over the {L0}-token context, {args.block} rows per pass")
    last = None
    for s in range(0, L0, args.block):
        chunk = prompt[s:s + args.block]
        last = dec.rows(chunk, logits_from=len(chunk) - 1)
    dec.progress = None
    c = [argmax_lowest(last[-1])]
    margins_c = [top2_margin(last[-1])]
    log("greedy continuation, one token per step")
    for j in range(k):
        z = dec.step(c[-1])
        c.append(argmax_lowest(z))
        margins_c.append(top2_margin(z))
        log(f"  c[{j + 1}] = {c[-1]} (margin {margins_c[-1]:.4f})")
    ids = sampled_ids(shape.vocab, seed)
    windows = []
    drafts = [("clean", np.array(c[:k], dtype=np.int64))]
    for i, p in enumerate(ps):
        drafts.append((f"p={p}", corrupt_drafts(seed, 1000 + i, c[:k], p, shape.vocab).astype(np.int64)))
    for name, d in drafts:
        dec.rollback(L0)
        log(f"window {name}: {d.tolist()}")
        logits = dec.rows(d)
        g = [argmax_lowest(z) for z in logits]
        target = [c[0]] + g[:-1]
        n = 0
        while n < k and d[n] == target[n]:
            n += 1
        nxt = target[n] if n < k else g[k - 1]
        windows.append({"name": name, "draft": d.tolist(), "accept_len": n, "next_token": int(nxt),
                        "rows": describe_rows(logits, ids)})
    wq0 = store.bits("wq", 0)
    doc = {
        "workload": args.workload, "shape": shape_name, "ctx": L0, "k": k, "seed": seed,
        "oracle_dtype": "float32",
        "prompt_sha256": hashlib.sha256(prompt.tobytes()).hexdigest(),
        "wq0_sha256": hashlib.sha256(np.ascontiguousarray(wq0).tobytes()).hexdigest(),
        "continuation": [int(t) for t in c], "continuation_margins": margins_c,
        "sampled_ids": ids.tolist(), "windows": windows,
    }
    with open(out_path, "w") as f:
        json.dump(doc, f, indent=1)
    log(f"wrote {out_path}")


if __name__ == "__main__":
    main()
