#!/usr/bin/env python3
"""Benchmark of the verify pass on one MI355X.

A step is one whole verify pass (embedding, every decoder layer against the
key-value cache, LM head, arg-max, prefix acceptance, cache truncation) of the
8B-shape bf16 model, k=8 draft rows at context 2048, on seeded synthetic
weights and tokens.  Every round starts from the same context (the cache is
truncated back in O(1) by the call itself) with the greedy continuation
re-corrupted with probability p.

Prints one JSON line: latency, algorithmic HBM GB/s, accepted tokens/s, the
roofline of the dominant kernel (HIP events around each of its launches while
the same steps run a second time, so that the events' own cost stays out of
the reported latency) and the CPU oracle timed on the host cores as a baseline.
"""
import argparse
import json
import os
import sys
import time

# Kernel arguments in device memory instead of host memory: the first scalar load of every kernel
# then misses to HBM, not across PCIe.  Must be set before the HIP runtime initialises.
os.environ.setdefault("HIP_FORCE_DEV_KERNARG", "1")

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "verify-pass latency (ms) + HBM GB/s, 8B-shape bf16 k=8 ctx2048; accepted tok/s"
WORKLOADS = {
    # name: (shape, context, k, seed)
    "8b_bf16_k8_ctx2048": ("8b", 2048, 8, 2),
    "1b_bf16_k5_ctx512": ("1b", 512, 5, 1),
    "8b_bf16_k16_ctx16384": ("8b", 16384, 16, 3),
    "tiny_fp32_k4_ctx64": ("tiny_verify", 64, 4, 0),
}
HBM_PEAK_GBPS = 8000.0
# HBM bytes per launch of the timed stage (fetched + written), from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# recorded in profiles/ (counter readings scaled by the plain-copy calibration: 2.000 and 1.000 KiB per count).
MEASURED_TRAFFIC = {("8b_bf16_k8_ctx2048", "gateup"): 236_668_000}
TRAFFIC_SOURCE = "profiles/verify_pass_8b_bf16_k8_ctx2048.md: rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE per dispatch, " \
                 "scaled by the plain-copy calibration; a stored reading, not taken in this run"


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def _oracle_pass_times(sub, L0, k, draft, reps, rng, log_name):
    """Times of `reps` oracle passes (batched route, float32) of k rows at context L0 on a model of shape
    `sub`; the cache is filled with random values (its contents do not change the work)."""
    from oracle import Decoder
    from workload import WeightStore
    store = WeightStore(sub, cache=False)
    dec = Decoder(sub, store, L0 + k, dtype=np.float32, keep_weights=True)
    for l in range(sub.n_layers):
        dec.K[l][:, :L0, :] = rng.standard_normal((sub.n_kv_heads, L0, sub.head_dim), dtype=np.float32)
        dec.V[l][:, :L0, :] = rng.standard_normal((sub.n_kv_heads, L0, sub.head_dim), dtype=np.float32)
    dec.kv_len = L0
    t0 = time.perf_counter()
    dec.rows(draft)                      # generates and converts the weights; untimed
    log(f"cpu_baseline: {log_name}: weights ready after {time.perf_counter() - t0:.1f} s")
    times = []
    for _ in range(reps):
        dec.rollback(L0)
        t0 = time.perf_counter()
        dec.rows(draft)
        times.append(time.perf_counter() - t0)
    return times


def cpu_baseline(shape, L0, k, draft, full=True):
    """The oracle's verify pass (batched route, float32) timed on the host cores: the whole model, median of
    3 passes.  Beside it, the figure earlier runs reported: the pass over the first 1 and the first 3 layers
    (+ LM head), extrapolated linearly in the layer count.  With full=False only the extrapolation is made."""
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    rng = np.random.default_rng(0)
    times = {}
    for nl in (1, 3):
        t = _oracle_pass_times(shape.with_(n_layers=nl), L0, k, draft, 5, rng, f"{nl}-layer model")
        times[nl] = min(t)
        log(f"cpu_baseline: {nl}-layer oracle pass {times[nl] * 1e3:.1f} ms (best of {len(t)})")
    per_layer = (times[3] - times[1]) / 2.0
    extrapolated = times[1] + per_layer * (shape.n_layers - 1)
    measured, full_times = None, None
    if full:
        full_times = _oracle_pass_times(shape, L0, k, draft, 3, rng, f"{shape.n_layers}-layer model")
        measured = float(np.median(full_times))
        log(f"cpu_baseline: full oracle pass {measured * 1e3:.1f} ms (median of {len(full_times)}); "
            f"extrapolation from 1 and 3 layers {extrapolated * 1e3:.1f} ms")
    cpu_model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    cpu_model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    value = measured if measured is not None else extrapolated
    sample = (f"oracle batched k={k} pass at ctx {L0}, float32, all {shape.n_layers} layers + LM head of the same weights, "
              f"median of 3 passes; cache filled with random values" if measured is not None else
              f"oracle batched k={k} pass at ctx {L0}, float32, timed on the first 1 and 3 layers + LM head of the "
              f"same weights (best of 5), extrapolated linearly to {shape.n_layers} layers; cache filled with random values")
    return {"value": value * 1e3, "unit": "ms", "cores": int(cores), "host_cpus": os.cpu_count(), "cpu_model": cpu_model,
            "kind": "oracle", "sample": sample,
            "full_pass_ms": [round(t * 1e3, 2) for t in full_times] if full_times else None,
            "extrapolated_ms": round(extrapolated * 1e3, 2),
            "measured_ms": {"layers_1": times[1] * 1e3, "layers_3": times[3] * 1e3}}


def flag_accounting(workload, tol, conts):
    """Rows of the workload whose oracle top-2 margin is below the logit tolerance (such rows are left out of
    exact token comparison) and below twice it, from the stored oracle values of the parity tests; and whether
    the GPU's own greedy continuation agrees with the oracle's on every unflagged position."""
    name = {"8b_bf16_k8_ctx2048": "8b_k8_ctx2048", "8b_bf16_k16_ctx16384": "8b_k16_ctx16384"}.get(workload)
    path = os.path.join(ROOT, "tests", "golden", f"{name}.json") if name else None
    if not path or not os.path.exists(path):
        return None
    with open(path) as f:
        gold = json.load(f)
    cm = gold["continuation_margins"]
    rows = [r["margin"] for w in gold["windows"] for r in w["rows"]]
    n = min(len(conts), len(gold["continuation"]))
    agree = all(int(conts[i]) == gold["continuation"][i] for i in range(n) if cm[i] >= tol)
    # the GPU follows its own tokens: past a flagged position where it chose differently the paths part for good
    first_diff = next((i for i in range(n) if int(conts[i]) != gold["continuation"][i]), None)
    return {"tol": tol, "source": f"tests/golden/{name}.json (float32 oracle)",
            "greedy_path_positions": len(cm), "greedy_path_margin_lt_tol": sum(m < tol for m in cm),
            "greedy_path_margin_lt_2tol": sum(m < 2 * tol for m in cm),
            "window_rows": len(rows), "window_rows_margin_lt_tol": sum(m < tol for m in rows),
            "window_rows_margin_lt_2tol": sum(m < 2 * tol for m in rows),
            "windows": len(gold["windows"]),
            "windows_unflagged_to_accept_point": sum(bool(w.get("assertable")) for w in gold["windows"]),
            "gpu_greedy_path_compared": n, "gpu_greedy_path_first_difference": first_diff,
            "gpu_greedy_path_agrees_where_unflagged": bool(agree) if first_diff is None or cm[first_diff] < tol else False}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="8b_bf16_k8_ctx2048", choices=sorted(WORKLOADS))
    ap.add_argument("--p", type=float, default=0.3, help="draft corruption probability")
    ap.add_argument("--seqs", type=int, default=1,
                    help="independent sequences verified by every pass, each at the workload's context and k "
                         "(seqs * k <= 16); the default 1 is the headline workload")
    ap.add_argument("--time-stage", default="gateup", help="stage bracketed with HIP events ('none' to disable)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-baseline-extrapolated", action="store_true",
                    help="time the oracle on 1 and 3 layers only and extrapolate (saves the ~1 minute of the full pass)")
    ap.add_argument("--no-p-sweep", action="store_true", help="skip the extra rounds at p = 0.1 and 0.6")
    ap.add_argument("--loops", action="store_true",
                    help="instead of the verify-pass benchmark, time the three decoding strategies of the paper's "
                         "Table 1 (autoregressive, synchronous speculative, asynchronous) on one GPU: 8B-shape verify "
                         "model, 128-token prompt, 256 new tokens, with a random-weight 1B-shape draft model (nothing "
                         "it proposes is accepted) and with a copy of the verify model as draft (everything is)")
    ap.add_argument("--calibrate-chain", action="store_true",
                    help="run only chains of bare streaming kernels of the headline workload's stage sizes, each kernel "
                         "depending on the one before: the time per kernel that any implementation of a stage as one "
                         "kernel of a dependent chain has to beat (no arithmetic, no activations, no epilogue)")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="run only a plain copy kernel of this size 10 times (profiler byte-counter calibration)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    import paper_2410_17375_amd as A
    from paper_2410_17375_amd.harness import load_model
    from workload import SHAPES, prompt_tokens, corrupt_drafts

    if args.calibrate_copy:
        n = args.calibrate_copy << 20
        src = torch.ones(n, dtype=torch.uint8, device="cuda")
        dst = torch.empty(n, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        for _ in range(10):
            A.calibration_copy(dst.data_ptr(), src.data_ptr(), n)
        torch.cuda.synchronize()
        print(json.dumps({"calibration_copy_bytes_read": n, "calibration_copy_bytes_written": n, "launches": 10}))
        return

    if args.calibrate_chain:
        sh = SHAPES["8b"]
        e = sh.weight_elem_bytes
        sizes = {"qkv": sh.d_model * (sh.q_dim + 2 * sh.kv_dim) * e, "oproj": sh.q_dim * sh.d_model * e,
                 "gateup": 2 * sh.d_model * sh.d_ffn * e, "down": sh.d_model * sh.d_ffn * e,
                 "lmhead": sh.vocab * sh.d_model * e}
        buf = torch.ones(3 << 30, dtype=torch.uint8, device="cuda")
        scratch = torch.zeros(3072, dtype=torch.uint8, device="cuda")
        st = torch.cuda.Stream()
        res = {}
        with torch.cuda.stream(st):
            for name, nbytes in sizes.items():
                n = 40 if name == "lmhead" else 200
                best = None
                for _ in range(3):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(st)
                    A.calibration_chain(buf.data_ptr(), buf.numel(), nbytes, n, scratch.data_ptr(), st.cuda_stream)
                    e1.record(st)
                    e1.synchronize()
                    us = e0.elapsed_time(e1) * 1e3 / n
                    best = us if best is None else min(best, us)
                res[name] = {"bytes": int(nbytes), "us_per_kernel": round(best, 2),
                             "gbps": round(nbytes / best / 1e3, 1)}
        per_layer = sum(res[k]["us_per_kernel"] for k in ("qkv", "oproj", "gateup", "down"))
        print(json.dumps({"bare_streaming_chain": res, "projection_stages_per_layer_us": round(per_layer, 2),
                          "all_projection_stages_of_a_pass_ms": round((sh.n_layers * per_layer + res["lmhead"]["us_per_kernel"]) / 1e3, 4),
                          "note": "256 workgroups x 512 threads, 16 non-temporal 16-byte loads in flight per thread, "
                                  "kernels of one chain in one stream; attention, merge, embedding and acceptance "
                                  "kernels (2 x 32 + 2 launches) are not included"}))
        return

    if args.loops:
        sv, sd = SHAPES["8b"], SHAPES["1b_v128k"]
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        log("loading verify (8B shape), draft (1B shape) and twin models ...")
        v = load_model(sv, 512, stream=s1.cuda_stream)
        d = load_model(sd, 512, stream=s2.cuda_stream)
        twin = load_model(sv, 512, stream=s2.cuda_stream)
        prompt = prompt_tokens(4, 128, sv.vocab)
        res = {}
        ref, st = A.generate_greedy(v, prompt, 256)
        res["autoregressive"] = {"ms_per_token": st["wall_ms"] / 256}
        for name, dm in (("random_1b_draft", d), ("twin_draft", twin)):
            for kind, fn in (("sync", A.generate_sync), ("async", A.generate_async)):
                out, st = fn(dm, v, prompt, 256, 8)
                assert np.array_equal(out, ref), f"{kind}/{name}: output differs from the greedy sequence"
                res[f"{kind}_{name}"] = {"ms_per_token": st["wall_ms"] / 256, "rounds": st["rounds"],
                                         "rollbacks": st["rollbacks"], "draft_steps": st["draft_steps"],
                                         "accepted_per_round": st["accepted_total"] / max(st["rounds"], 1)}
        print(json.dumps({"loops": res, "n_new": 256, "prompt": 128, "k_max": 8, "identical_output": True}))
        return

    shape_name, L0, k, seed = WORKLOADS[args.workload]
    shape = SHAPES[shape_name]
    B = args.seqs
    if B < 1 or B * k > A.MAX_K:
        print(f"bench.py: --seqs {B} with k={k} does not fit the {A.MAX_K} rows of a pass", file=sys.stderr)
        sys.exit(2)
    stream = torch.cuda.Stream()
    t0 = time.perf_counter()
    log(f"loading {shape_name} ({shape.n_params_streamed() / 1e9:.2f} G weights) ...")
    model = load_model(shape, L0 + A.MAX_K, stream=stream.cuda_stream, progress=log, max_seqs=B)
    log(f"model loaded in {time.perf_counter() - t0:.1f} s")

    # sequence 0 is the headline sequence; further sequences get prompts of their own
    seq_ids = list(range(B))
    t0 = time.perf_counter()
    conts = []
    for sq in seq_ids:
        conts.append([model.seq_prefill(sq, prompt_tokens(seed + 1000 * sq, L0, shape.vocab))])
    log(f"{B} context(s) of {L0} tokens prefilled in {time.perf_counter() - t0:.2f} s")
    for _ in range(k - 1):
        for sq, t in zip(seq_ids, model.draft_step_batch(seq_ids)):
            conts[sq].append(int(t))
    for sq in seq_ids:
        model.seq_rollback(sq, L0)
    n_rounds = args.warmup + args.steps
    drafts = [[corrupt_drafts(seed + 1000 * sq, r, conts[sq], args.p, shape.vocab) for sq in seq_ids]
              for r in range(n_rounds)]
    ctx = [L0] * B

    def one_pass(r):
        if B == 1:
            return model.verify(L0, drafts[r][0])[0]
        return int(model.verify_batch(seq_ids, ctx, drafts[r])[0].sum())

    for r in range(args.warmup):
        one_pass(r)
    host_ms, dev_ms, accepts = [], [], []
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for r in range(args.warmup, n_rounds):
        t1 = time.perf_counter()
        n = one_pass(r)
        host_ms.append((time.perf_counter() - t1) * 1e3)
        dev_ms.append(model.last_pass_ms())
        accepts.append(n)
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t_begin
    ms_per_step = total_s * 1e3 / args.steps

    # the other corruption rates of the workload (the paper's accepted drafts per step sit between p = 0.1 and 0.3)
    by_p = {}
    # The same steps once more with HIP events around every launch of one stage (the roofline figure).  The
    # events cost ~4 us per bracketed launch, which is why they stay out of the region `value` is taken from.
    stage_stats, ms_per_step_events = None, None
    if args.time_stage != "none":
        model.set_option(A.OPT_TIME_STAGE, A.STAGES[args.time_stage])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for r in range(args.warmup, n_rounds):
            one_pass(r)
        torch.cuda.synchronize()
        ms_per_step_events = (time.perf_counter() - t1) * 1e3 / args.steps
        stage_stats = model.stage_time()
        model.set_option(A.OPT_TIME_STAGE, -1)
    for p_other in ((0.1, 0.6) if B == 1 and not args.no_p_sweep else ()):
        dr = [corrupt_drafts(seed, 100000 + r, conts[0], p_other, shape.vocab) for r in range(args.steps)]
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        acc = [model.verify(L0, d)[0] for d in dr]
        dt = time.perf_counter() - t1
        q = p_other * (1.0 - 1.0 / shape.vocab)
        by_p[str(p_other)] = {"ms_per_step": round(dt * 1e3 / args.steps, 4), "mean_accept_len": round(float(np.mean(acc)), 3),
                              "expected_mean_accept_len": round(sum((1 - q) ** j for j in range(1, k + 1)), 3),
                              "accepted_tok_per_s": round(sum(acc) / dt, 1),
                              "accept_hist": np.bincount(acc, minlength=k + 1).tolist()}

    bytes_pass = model.weight_bytes_per_pass() + B * (
        model.kv_bytes_per_pass(L0, k) + k * shape.d_model * shape.weight_elem_bytes
        + shape.n_layers * 2 * shape.kv_dim * shape.weight_elem_bytes * k)
    gbps = bytes_pass / (ms_per_step * 1e-3) / 1e9
    hist = np.bincount(accepts, minlength=B * k + 1).tolist()
    out = {
        "metric": METRIC, "value": round(ms_per_step, 4), "unit": "ms", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if shape.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "shape": shape_name, "ctx": L0, "k": k, "corruption_p": args.p,
                   "seed": seed, "seqs": B, "mode": "kernel_per_stage"},
        "latency_ms": {"host_median": round(float(np.median(host_ms)), 4),
                       "host_p10": round(float(np.percentile(host_ms, 10)), 4),
                       "host_p90": round(float(np.percentile(host_ms, 90)), 4),
                       "device_median": round(float(np.median(dev_ms)), 4)},
        "algorithmic_bytes_per_pass": int(bytes_pass),
        "hbm_gbps": round(gbps, 1), "hbm_frac_of_8TBps": round(gbps / HBM_PEAK_GBPS, 4),
        "accepted_tok_per_s": round(sum(accepts) / total_s, 1),
        "accept_hist": hist, "mean_accept_len": round(float(np.mean(accepts)), 3),
    }
    if by_p:
        out["other_corruption_rates"] = by_p
    if B == 1:
        flags = flag_accounting(args.workload, 3e-2 if shape.dtype == "bf16" else 1e-4, conts[0])
        if flags:
            out["flagged_rows"] = flags
    if args.time_stage != "none":
        ms, launches, b = stage_stats
        avg_ms = ms / max(launches, 1)
        ach = b / (avg_ms * 1e-3) / 1e9 if avg_ms > 0 else 0.0
        out["roofline"] = {"bound": "hbm", "kernel": args.time_stage, "achieved": round(ach, 1),
                           "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBPS, 4),
                           "traffic": MEASURED_TRAFFIC.get((args.workload, args.time_stage)) if B == 1 else None,
                           "traffic_source": TRAFFIC_SOURCE if B == 1 and (args.workload, args.time_stage) in MEASURED_TRAFFIC else None,
                           "avg_launch_ms": round(avg_ms, 5), "launches": int(launches),
                           "algorithmic_bytes_per_launch": int(b),
                           "ms_per_step_with_events": round(ms_per_step_events, 4)}
    if not args.no_cpu_baseline:
        try:
            out["cpu_baseline"] = cpu_baseline(shape, L0, k, drafts[0][0], full=not args.cpu_baseline_extrapolated)
            if B > 1:       # the oracle takes the sequences one after another
                out["cpu_baseline"]["value"] *= B
                out["cpu_baseline"]["sample"] += f"; times {B} sequences"

            out["cpu_baseline"]["accepted_tok_per_s"] = round(
                float(np.mean(accepts)) / (out["cpu_baseline"]["value"] * 1e-3), 2)
        except MemoryError as e:          # pragma: no cover
            out["cpu_baseline"] = {"value": None, "error": repr(e)}
    model.free()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
