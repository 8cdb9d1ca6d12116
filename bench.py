#!/usr/bin/env python3
"""Benchmark: generated tokens/s of early-exit decode with KV recomputation at the 7B shape
(threshold 0.8) against full-depth decode (threshold 1.0) on the same kernels, one MI355X.

A "step" is one ee_decode_step: the whole hot path (embedding, the layers up to the exit taken, exit
heads with the fused soft-max/decision, KV writes for the current and the deferred tokens) for one
batch.  Inputs are seeded and synthetic (workload/gen.py): the 7B-shaped model of the C3 workload,
a 1024-token uniform-random prompt, greedy decoding.  Weights and the KV cache are resident in HBM
before the timed region starts.

Prints ONE JSON line: the headline metric, `roofline` (the dominant decode kernel against HBM bandwidth),
`prefill` (the prompt phase, with its own `roofline` against the matrix-core peak), the threshold and
deferred-token-cap sweeps, and `cpu_baseline` (the CPU oracle timed on a bounded sample).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=240)
    ap.add_argument("--warmup", type=int, default=15)
    ap.add_argument("--workload", default="C3", choices=["C1", "C2", "C3", "C4", "C5"])
    ap.add_argument("--threshold", type=float, default=None,
                    help="exit threshold (default: 0.8 where the workload sweeps it, else the workload's own)")
    ap.add_argument("--max-pending", type=int, default=15)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--breakdown", action="store_true", help="also time every kernel family (extra passes, stderr)")
    ap.add_argument("--cpu-threads", type=int, default=0)
    ap.add_argument("--no-sweep", action="store_true", help="skip the threshold sweep of the workload")
    ap.add_argument("--refeed", action="store_true",
                    help="deferred tokens are fed again from the embedding (paper-literal) instead of resuming")
    ap.add_argument("--exit-structure", default="default", choices=["default", "no_norm", "tied", "mlp", "all", "layer"],
                    help="structure of the exits (Section 2): RMSNorm + own matrix (default), no norm, embeddings tied, "
                         "an MLP in front of each exit, all three, or a complete Transformer layer in each exit")
    ap.add_argument("--no-prefill-bench", action="store_true", help="skip the timing of the prompt phase")
    ap.add_argument("--prefill-only", action="store_true", help="time the prompt phase only and print its figures")
    ap.add_argument("--pmc-run", action="store_true",
                    help="short run for `rocprofv3 --pmc`: one 1-GiB device copy (counter calibration), then 12 decode steps")
    return ap.parse_args()


def generate(ee, gm, cache, prompts, tau, warmup, steps, shape, es, max_pending, profile_kernel=None, profile_every=1,
             pipeline=False, confidences=False):
    """Prefill every sequence, then (warmup + steps) decode steps over the whole batch; returns the timing of
    the last `steps` and the algorithmic-bytes model of exactly those steps.

    Bytes of one step (what the method itself must move): the weights of every layer some sequence runs, once;
    the heads that are evaluated (an exit head if some sequence tests it, the final head if some sequence
    reaches it), once each; per sequence K and V of its context in every layer it runs, K and V of its active
    rows written, one embedding row.  pipeline: the cache is in pipeline mode (nothing is deferred; the timed region
    ends when the fill stream has caught up).  confidences: also collect every evaluated head's confidence per step
    (one small host call per step, so not in the passes whose time is reported as the headline)."""
    import numpy as np
    import torch

    B = len(prompts)
    ids = list(range(B))
    d, F, V, L = shape.d_model, shape.d_ff, shape.vocab, shape.n_layers
    w_layer, w_head = (4 * d * d + 3 * d * F) * es, d * V * es
    # an exit with an MLP also streams that MLP; one with a layer of its own streams that layer, and its q|k|v matrix
    # even when the exit is not evaluated (every row that passes leaves its K and V there)
    w_exit = w_head + (3 * d * F * es if shape.exit_mlp else 0) + (w_layer if shape.exit_layer else 0)
    w_exit_kv_only = 3 * d * d * es if shape.exit_layer else 0
    seg_ends = list(shape.exit_layers) + [L]
    seg_of_layer = [next(k for k, se in enumerate(seg_ends) if l < se) for l in range(L)]
    seqs = ee.Sequences(L, pipeline=pipeline)
    confs = []
    fl = []  # host mirror of the fill watermarks, for the bytes model only
    for sq in ids:
        cache.reset(sq)
    for sq in ids:
        tok, ex, _ = ee.prefill(gm, cache, sq, prompts[sq], tau)
        seqs.start(sq, tok)
        fl.append([len(prompts[sq])] * len(seg_ends))
    exits, nbytes, forced = [], 0, 0
    prof = None
    t0 = None
    log = []  # (row offsets, exit layers) per step: the bytes model is worked out after the clock has stopped
    for i in range(warmup + steps):
        if i == warmup:
            torch.cuda.synchronize()
            if profile_kernel is not None:
                gm.profile_begin(profile_kernel, max_launches=steps * (shape.n_layers + 4) // profile_every + 64, every=profile_every)
            t0 = time.perf_counter()
        ro, tk, pm = seqs.rows(ids)
        nt, exl, _ = ee.decode_step(gm, cache, ids, ro, tk, pm, tau)
        seqs.update(ids, nt, exl)
        log.append((ro, exl))
        if confidences and i >= warmup:
            confs.append(gm.step_confidences(B))
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    if profile_kernel is not None:
        prof = gm.profile_end()
    for i, (ro, exl) in enumerate(log):
        deepest, heads = 0, set()
        for sq in ids:
            p, e = len(prompts[sq]) + i, int(exl[sq])
            if i >= warmup:
                was_forced = ro[sq + 1] - ro[sq] - 1 >= max_pending
                deepest = max(deepest, e)
                if not (tau >= 1.0 or was_forced):
                    heads |= {x for x in shape.exit_layers if x <= e}
                if e == L:
                    heads.add(L)
                rows = sum(p - fl[sq][seg_of_layer[l]] + 1 for l in range(e))
                nbytes += e * 2 * d * es * (p + 1) + rows * 2 * d * es + d * es
                exits.append(e)
                forced += int(was_forced)
            for k, se in enumerate(seg_ends):
                if se <= e:
                    fl[sq][k] = p + 1
        if i >= warmup:
            nbytes += deepest * w_layer + sum(w_head if h == L else w_exit for h in heads)
            nbytes += w_exit_kv_only * sum(1 for x in shape.exit_layers if x <= deepest and x not in heads)
    quant = None
    if confs:
        cf = np.stack(confs)  # [steps][B][n_exits+1]
        quant = {}
        for k, layer in enumerate(seg_ends):
            v = cf[:, :, k].ravel()
            v = v[v >= 0]
            if v.size:
                quant[str(layer)] = {"evaluated": int(v.size), "frac_ge_threshold": float(np.mean(v >= tau)),
                                     **{f"q{int(q * 100)}": float(np.quantile(v, q)) for q in (0.1, 0.5, 0.9, 0.99)},
                                     "max": float(v.max())}
    return dict(seconds=dt, exits=exits, bytes=nbytes, forced=forced, prof=prof, tokens=B * steps, confidences=quant)


PROFILE_EVERY = 8  # launches of the roofline kernel per timed one in the throughput pass
MFMA_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix-core rate


def prefill_bench(ee, gm, cache, prompt, shape, breakdown, traffic=None):
    """Times the prompt phase (GEMM path) on one prompt: plain ee_prefill, the scored variant (every head on
    every position), and the gate|up GEMM alone (HIP events on its dispatches).  Algorithmic flops: 2*P*params
    of the layers + causal attention; every activation operand is two bf16 terms, so the matrix cores issue
    twice that (except in the scored heads, which by default take the leading term of their input only)."""
    import torch

    P = len(prompt)
    d, F, V, L = shape.d_model, shape.d_ff, shape.vocab, shape.n_layers
    layer_flops = 2.0 * P * (4 * d * d + 3 * d * F) + 4.0 * d * P * (P + 1) / 2
    head_flops = 2.0 * P * d * V

    def run(scored, kernel=None):
        cache.reset(0)
        torch.cuda.synchronize()
        if kernel is not None:
            gm.profile_begin(kernel, max_launches=8 * L + 64)
        t0 = time.perf_counter()
        if scored:
            ee.prefill_scored(gm, cache, 0, prompt, 1.0)
        else:
            ee.prefill(gm, cache, 0, prompt, 1.0)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        return dt, (gm.profile_end() if kernel is not None else None)

    run(False)
    run(True)
    plain = min(run(False)[0] for _ in range(3))
    scored = min(run(True)[0] for _ in range(3))
    # (the clock moves with the load: the kernel's mean over one prompt phase is taken from the best of three passes)
    n_sw, ms_sw = min((run(False, ee.EE_K_SWIGLU)[1] for _ in range(3)), key=lambda r: r[1])
    _, (n_hd, ms_hd) = run(True, ee.EE_K_HEAD)
    sw_tflops = 2.0 * P * 2 * F * d / (ms_sw / max(n_sw, 1) * 1e-3) / 1e12
    # scored: the head GEMM dispatches are the first of each pair (GEMM, merge); the last launch is the final-head
    # decode kernel on the last row: time of the GEMMs alone = scored - plain, over n_exits + 1 heads
    n_heads = len(shape.exit_layers) + 1
    hd_tflops = n_heads * head_flops / max(scored - plain, 1e-9) / 1e12
    out = {
        "prompt_tokens": P, "ms": plain * 1e3, "prompt_tokens_per_s": P / plain,
        "algorithmic_tflops": (L * layer_flops + 2.0 * d * V) / plain / 1e12,
        "scored_ms": scored * 1e3, "scored_heads": n_heads,
        "scored_algorithmic_tflops": (L * layer_flops + n_heads * head_flops) / scored / 1e12,
        "head_gemm_algorithmic_tflops_from_difference": hd_tflops,
        "head_gemm_frac_of_mfma_peak": hd_tflops / MFMA_PEAK_TFLOPS,
        "scored_head_terms": int(gm.cfg.scored_head_terms) or 1,
        "roofline": {"bound": "mfma", "kernel": "pf_swiglu_kernel (gate|up GEMM over all prompt rows + SwiGLU)",
                     "achieved": sw_tflops, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": sw_tflops / MFMA_PEAK_TFLOPS,
                     "mfma_issue_tflops": 2 * sw_tflops, "mfma_issue_frac": 2 * sw_tflops / MFMA_PEAK_TFLOPS,
                     "launches": n_sw, "avg_us": ms_sw / max(n_sw, 1) * 1e3, "flops_per_launch": 2.0 * P * 2 * F * d,
                     "traffic": traffic},
    }
    if breakdown:
        for k, name in enumerate(ee.KERNEL_NAMES):
            _, (n, ms) = run(True, k)
            print(f"[bench] prefill {name:10s} launches {n:5d} avg {ms / max(n, 1) * 1e3:9.2f} us total {ms:8.2f} ms",
                  file=sys.stderr, flush=True)
    return out


def stored_traffic(key):
    """HBM bytes per launch measured with rocprofv3 counters (profiles/pmc_traffic.json), or None."""
    tpath = os.path.join(ROOT, "profiles", "pmc_traffic.json")
    if not os.path.exists(tpath):
        return None
    with open(tpath) as f:
        return json.load(f).get(key)


def cpu_baseline(shape, tensors_host, prompt, tau, max_pending, threads):
    """Times the CPU oracle (as it stands) on a bounded sample of the same workload."""
    from oracle import oracle as O
    from oracle.from_workload import config_of

    om = O.Model(config_of(shape))
    for (kind, idx), arr in tensors_host.items():
        om.set_tensor(kind, idx, arr)
    O.set_threads(threads)
    big = shape.d_model >= 2048
    n_prompt, n_new = (8, 80) if big else (len(prompt), 32)
    st = O.State(om, n_prompt + n_new + 1, max_pending)
    dg = st.prefill(prompt[:n_prompt])
    tok = dg[-1]["argmax"]
    for d in dg[:-1]:
        if tau < 1.0 and d["conf"] >= tau:
            tok = d["argmax"]
            break
    t0 = time.perf_counter()
    for _ in range(n_new):
        tok, _, _ = st.decode_step(tok, tau)
    dt = time.perf_counter() - t0
    return {"value": n_new / dt, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"same model and threshold; prompt cut to {n_prompt} tokens, {n_new} decode steps "
                      f"({dt:.1f} s of CPU work)"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2312_04916_amd as ee
    from workload import (CONFIGS, TABLE4_EXIT_HEAD_SCALE, TensorKind, model_tensor, model_tensor_list, prompt_lengths,
                          prompt_tokens, to_numpy)

    wl = CONFIGS[args.workload]
    shape = wl.shape
    if args.threshold is None:
        args.threshold = 0.8 if 0.8 in wl.thresholds else wl.thresholds[0]
    if args.exit_structure != "default":
        import dataclasses
        shape = dataclasses.replace(shape, exit_norm=args.exit_structure not in ("no_norm", "all"),
                                    tie_embeddings=args.exit_structure in ("tied", "all"),
                                    exit_mlp=args.exit_structure in ("mlp", "all"), exit_layer=args.exit_structure == "layer")
    es = 2 if shape.dtype == "bf16" else 4
    B = wl.batch
    lens = [wl.prompt_len[0]] * B if wl.prompt_len[0] == wl.prompt_len[1] else \
        prompt_lengths(B, wl.prompt_len[0], wl.prompt_len[1], wl.length_seed)
    n_prompt = lens[0] if B == 1 else f"{min(lens)}..{max(lens)}"
    max_pos = max(lens) + args.warmup + args.steps + 48
    t_setup = time.perf_counter()
    gm = ee.Model(ee.config_of_shape(shape, max_pos), max_rows=min(256, 16 * B + 48), max_seqs=B)
    keep_host = not args.no_cpu_baseline
    tensors_host = {}
    for kind, idx in model_tensor_list(shape):
        t = model_tensor(shape, kind, idx, wl.weight_seed, "cuda:0").contiguous()
        gm.set_tensor(int(kind), idx, t)
        if keep_host:
            tensors_host[(int(kind), idx)] = to_numpy(t)
        torch.cuda.synchronize()
        del t
    cache = ee.KvCache(gm, B, sum(lens) + B * (args.warmup + args.steps + 48), 64, args.max_pending)
    cache.set_refeed(args.refeed)
    prompts = [prompt_tokens(shape.vocab, lens[b], wl.prompt_seed + b).numpy() for b in range(B)]
    prompt = prompts[0]
    print(f"[bench] model {args.workload} ready in {time.perf_counter() - t_setup:.1f}s "
          f"({gm.weight_bytes / 1e9:.2f} GB weights)", file=sys.stderr, flush=True)

    if args.pmc_run:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0").normal_()
        b = torch.empty_like(a)
        torch.add(a, 1.0, out=b)  # plain elementwise kernel: reads 1 GiB, writes 1 GiB; what FETCH_SIZE / WRITE_SIZE
        torch.add(a, 1.0, out=b)  # report for it calibrates their unit (the float add kernel appears nowhere else)
        torch.cuda.synchronize()
        generate(ee, gm, cache, prompts, 1.0, 2, 10, shape, es, args.max_pending)
        print("[bench] pmc run done", file=sys.stderr)
        return
    prefill = None
    if shape.dtype == "bf16" and shape.d_model % 128 == 0 and not args.no_prefill_bench:
        prefill = prefill_bench(ee, gm, cache, prompts[0], shape, args.breakdown, stored_traffic(f"pf_swiglu_{args.workload}"))
        print(f"[bench] prefill {prefill['prompt_tokens']} tokens: {prefill['ms']:.2f} ms, "
              f"{prefill['algorithmic_tflops']:.0f} TFLOP/s algorithmic", file=sys.stderr, flush=True)
        if args.prefill_only:
            print(json.dumps({"prefill": prefill}), flush=True)
            return
    generate(ee, gm, cache, prompts, 1.0, 0, 40, shape, es, args.max_pending)  # untimed: clocks and caches warm
    full = generate(ee, gm, cache, prompts, 1.0, args.warmup, args.steps, shape, es, args.max_pending)
    # the timed pass: every 8th launch of the roofline kernel carries an event pair (an event pair costs a launch about
    # 5 us of queue time; on all 32 launches of a step that would take 5 % off the very throughput measured here)
    early = generate(ee, gm, cache, prompts, args.threshold, args.warmup, args.steps, shape, es, args.max_pending,
                     profile_kernel=ee.EE_K_SWIGLU, profile_every=PROFILE_EVERY)
    # the full-depth baseline once more after the timed pass; the faster of the two stands (the first decode pass after
    # the prompt-phase timing has been seen to run several percent slow on some boxes, which would flatter the speed-up)
    full2 = generate(ee, gm, cache, prompts, 1.0, args.warmup, args.steps, shape, es, args.max_pending)
    if full2["seconds"] < full["seconds"]:
        full = full2
    tps_full = full["tokens"] / full["seconds"]
    tps = early["tokens"] / early["seconds"]
    n_l, ms_l = early["prof"]
    w_swiglu = 2 * shape.d_ff * shape.d_model * es
    achieved = w_swiglu / (ms_l / n_l * 1e-3) / 1e9 if n_l else 0.0
    hist = {str(e): early["exits"].count(e) for e in sorted(set(early["exits"]))}
    ideal_speedup = full["bytes"] / early["bytes"]

    if args.breakdown:
        for k, name in enumerate(ee.KERNEL_NAMES):
            r = generate(ee, gm, cache, prompts, args.threshold, args.warmup, args.steps, shape, es, args.max_pending,
                         profile_kernel=k)
            n, ms = r["prof"]
            print(f"[bench] {name:10s} launches {n:6d} avg {ms / max(n, 1) * 1e3:8.2f} us total {ms:9.2f} ms "
                  f"of {r['seconds'] * 1e3:.1f} ms", file=sys.stderr, flush=True)

    sweep = {}
    if not args.no_sweep:
        for tau in wl.thresholds:
            if tau in (1.0, args.threshold):
                continue
            r = generate(ee, gm, cache, prompts, tau, args.warmup, args.steps, shape, es, args.max_pending)
            sweep[str(tau)] = {"tokens_per_s": r["tokens"] / r["seconds"], "speedup_vs_full_depth": full["seconds"] / r["seconds"],
                               "bytes_model_speedup": full["bytes"] / r["bytes"], "forced_full_steps": r["forced"],
                               "exit_histogram": {str(e): r["exits"].count(e) for e in sorted(set(r["exits"]))}}

    # confidence distribution at each head over the same steps as the headline (an untimed extra pass: one host call
    # per step), so that the reader sees what the exit mix is made of
    conf_quant = None
    if not args.no_sweep:
        conf_quant = generate(ee, gm, cache, prompts, args.threshold, args.warmup, args.steps, shape, es, args.max_pending,
                              confidences=True)["confidences"]
    # the smallest threshold tried at which early exit is measured faster than full depth
    first_win = None
    tried = sorted([(float(t), v["speedup_vs_full_depth"], v["bytes_model_speedup"]) for t, v in sweep.items()]
                   + [(args.threshold, tps / tps_full, ideal_speedup)])
    wins = [t for t in tried if t[1] > 1.0]
    if wins:
        t = max(wins, key=lambda x: x[0])
        first_win = {"largest_threshold_with_speedup_above_1": t[0], "speedup_vs_full_depth": t[1], "bytes_model_speedup": t[2]}

    # pipeline-based early exit on one GPU (second stream fills the KV of exited tokens) against KV recomputation,
    # same thresholds (the comparison of the paper's Appendix B.1, there across 4 pipeline stages)
    pipe_cmp = {}
    if not args.no_sweep and not args.refeed and args.max_pending >= 5:
        for tau in [t for t in (0.2, 0.4) if t in wl.thresholds]:
            cache.flush(list(range(B)))
            cache.set_pipeline(True)
            r = generate(ee, gm, cache, prompts, tau, args.warmup, args.steps, shape, es, args.max_pending, pipeline=True)
            cache.flush(list(range(B)))
            cache.set_pipeline(False)
            rec = sweep.get(str(tau))
            pipe_cmp[str(tau)] = {"pipeline_tokens_per_s": r["tokens"] / r["seconds"],
                                  "pipeline_speedup_vs_full_depth": full["seconds"] / r["seconds"],
                                  "kv_recomputation_tokens_per_s": rec["tokens_per_s"] if rec else None,
                                  "exit_histogram": {str(e): r["exits"].count(e) for e in sorted(set(r["exits"]))}}

    # cap on the deferred-token list (Appendix D.3) x how the deferred tokens are carried (resume / re-feed), at the
    # workload's lowest threshold: where carrying more rows stops being free
    pending_sweep = {}
    if not args.no_sweep and B == 1:
        # threshold 0: every token leaves at the first exit, the list always grows to the cap and is then cleared by
        # one forced full-depth step over cap + 1 rows (the cost of carrying rows in its purest form)
        for tau_s in (min(wl.thresholds), 0.0):
            res = {}
            for cap in (1, 3, 7, 15, 31, 63):
                for mode in ("resume", "refeed"):
                    pc = ee.KvCache(gm, B, sum(lens) + B * (args.warmup + args.steps + 48), 64, cap)
                    pc.set_refeed(mode == "refeed")
                    r = generate(ee, gm, pc, prompts, tau_s, args.warmup, args.steps, shape, es, cap)
                    res[f"{mode}_{cap}"] = {"tokens_per_s": r["tokens"] / r["seconds"], "forced_full_steps": r["forced"],
                                            "speedup_vs_full_depth": full["seconds"] / r["seconds"]}
                    pc.close()
            pending_sweep[f"threshold_{tau_s}"] = res

    # The seeded heads of the workload hardly ever reach the headline threshold (see head_confidences), so the run above
    # measures what the exit heads cost, not what exits save.  Second measurement at the same threshold with the exit
    # mix of the one generation the paper tabulates token by token (Table 4: 7 of 18 tokens leave at layer 8, 1 at
    # layer 16, 10 go to full depth): the same model with the two exit heads' std scaled (workload.TABLE4_EXIT_HEAD_SCALE).
    # Everything else, the final head and with it the full-depth baseline included, is unchanged.  Runs last: it
    # replaces the exit heads on the device.
    paper_mix = None
    if (not args.no_sweep and args.workload == "C3" and args.exit_structure == "default" and not shape.tie_embeddings
            and len(shape.exit_layers) == len(TABLE4_EXIT_HEAD_SCALE)):
        import dataclasses
        cal = dataclasses.replace(shape, exit_head_sigma=tuple(s * shape.head_sigma for s in TABLE4_EXIT_HEAD_SCALE))
        for i in range(len(shape.exit_layers)):
            t = model_tensor(cal, TensorKind.EXIT_HEAD, i, wl.weight_seed, "cuda:0").contiguous()
            gm.set_tensor(int(TensorKind.EXIT_HEAD), i, t)
            torch.cuda.synchronize()
            del t
        r = generate(ee, gm, cache, prompts, args.threshold, args.warmup, args.steps, shape, es, args.max_pending)
        n = len(r["exits"])
        paper_mix = {"exit_head_std_scale": list(TABLE4_EXIT_HEAD_SCALE), "threshold": args.threshold,
                     "tokens_per_s": r["tokens"] / r["seconds"], "speedup_vs_full_depth": full["seconds"] / r["seconds"],
                     "bytes_model_speedup": full["bytes"] / r["bytes"], "forced_full_steps": r["forced"],
                     "exit_histogram": {str(e): r["exits"].count(e) for e in sorted(set(r["exits"]))},
                     "exit_fractions": {str(e): r["exits"].count(e) / n for e in sorted(set(r["exits"]))},
                     "table4_fractions": {str(shape.exit_layers[0]): 7 / 18, str(shape.exit_layers[1]): 1 / 18,
                                          str(shape.n_layers): 10 / 18}}

    traffic = stored_traffic(f"swiglu_{args.workload}")

    # what a kernel that only reads gets out of this GPU's memory: the whole weight buffer in one launch, and launches
    # of the roofline kernel's own size back to back
    stream_all = gm.measure_stream_read(0, 3)
    stream_k = gm.measure_stream_read(w_swiglu, 50)

    out = {
        "metric": ("generated tokens/s at 7B early-exit decode (thr 0.8) vs full-depth; HBM GB/s" if args.workload == "C3"
                   else f"generated tokens/s, early-exit decode, workload {args.workload} ({wl.note})"),
        "value": tps, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": early["seconds"] / args.steps * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": f"{args.workload}: {wl.note}, batch {B}, prompt {n_prompt} random ids, greedy, "
                               f"threshold {args.threshold}, max_pending {args.max_pending}",
                   "threshold": args.threshold, "exit_layers": list(shape.exit_layers), "n_layers": shape.n_layers,
                   "exit_structure": args.exit_structure},
        "full_depth_tokens_per_s": tps_full, "full_depth_ms_per_step": full["seconds"] / args.steps * 1e3,
        "speedup_vs_full_depth": tps / tps_full, "bytes_model_speedup": ideal_speedup,
        "exit_histogram": hist, "forced_full_steps": early["forced"], "threshold_sweep": sweep,
        "head_confidences": conf_quant, "speedup_crossover": first_win, "pipeline_vs_kv_recomputation": pipe_cmp,
        "paper_exit_mix_at_threshold": paper_mix, "max_pending_sweep": pending_sweep, "deferred_tokens": "refeed" if args.refeed else "resume",
        "hbm_gbps": early["bytes"] / early["seconds"] / 1e9, "hbm_frac": early["bytes"] / early["seconds"] / 1e9 / HBM_PEAK_GBPS,
        "full_depth_hbm_gbps": full["bytes"] / full["seconds"] / 1e9,
        "full_depth_hbm_frac": full["bytes"] / full["seconds"] / 1e9 / HBM_PEAK_GBPS,
        "roofline": {"bound": "hbm", "kernel": "gemm_swiglu_kernel (gate|up projection + SwiGLU)",
                     "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "launches": n_l, "timed_every": PROFILE_EVERY, "avg_us": ms_l / max(n_l, 1) * 1e3, "bytes_per_launch": w_swiglu,
                     "traffic": traffic},
        "measured_stream_read": {"unit": "GB/s", "whole_weight_buffer": stream_all, "launches_of_roofline_kernel_size": stream_k,
                                 "roofline_kernel_frac_of_it": achieved / stream_k if stream_k > 0 else None,
                                 "full_depth_step_frac_of_whole_buffer_rate": full["bytes"] / full["seconds"] / 1e9 / stream_all if stream_all > 0 else None},
    }
    if prefill is not None:
        out["prefill"] = prefill
    if not args.no_cpu_baseline:
        threads = args.cpu_threads or min(16, os.cpu_count() or 1)
        cache.close()
        out["cpu_baseline"] = cpu_baseline(shape, tensors_host, prompt, args.threshold, args.max_pending, threads)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
