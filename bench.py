#!/usr/bin/env python3
"""Bench of the HSD hot path on one MI355X.

Workload: 1B-shaped early-exit hierarchy, bf16, batch 1 - 16 layers,
d 2048, 32 query / 8 KV heads x 64, FFN 8192, vocab 32000, drafters = exits after layers 2 and 6
sharing the final norm and head; prompt of 512 uniform-random ids, 256 generated tokens,
temperature 1.  Random-init weights (the paper's checkpoints and prompts are not available offline).

One step = one full generation of 256 tokens by HSD from the prefilled prompt (rewind + generate:
every draft pass, verify pass, softmax, accept/reject/resample kernel and the round driver), each
step along its own sample path (sampling seed + step index).
The (T_0, T_1) sweep {2,4,6} x {1,2,4}, the single-draft sweep and plain autoregressive decoding are
measured first (untimed part, eight sample paths per setting); the timed steps run the best HSD setting.

Prints ONE JSON line.  `value` = generated tokens per second of HSD with everything resident in HBM.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PROMPT, GEN, TEMPERATURE, SEED = 512, 256, 1.0, 20251019
EXITS = (2, 6, 16)
SWEEP_SEEDS = tuple(SEED + 100 + i for i in range(8))      # sample paths per setting of the sweeps
HBM_PEAK_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def gemm_site_bytes(shape, site, m):
    """Algorithmic bytes of one launch: the weight matrix once + activations in and out."""
    d, F, V = shape["d"], shape["ffn"], shape["vocab"]
    nq, nkv = shape["n_q"] * shape["hd"], shape["n_kv"] * shape["hd"]
    n, k, out_b = {"qkv": (nq + 2 * nkv, d, 4), "o": (d, nq, 4), "gateup": (2 * F, d, 1), "down": (d, F, 4),
                   "head": (V, d, 4)}[site]
    return n * k * 2 + m * k * 2 + m * n * out_b


def pass_bytes(shape, exit_layer, m, s_total, n_logit_rows):
    """Algorithmic bytes of one pass: weights of the layers run + head once, KV read and written,
    logits and probability rows."""
    d, F, V = shape["d"], shape["ffn"], shape["vocab"]
    nq, nkv = shape["n_q"] * shape["hd"], shape["n_kv"] * shape["hd"]
    layer_w = (d * (nq + 2 * nkv) + nq * d + 3 * d * F) * 2
    kv = exit_layer * (2 * s_total * nkv * 2 + 2 * m * nkv * 2)
    return exit_layer * layer_w + V * d * 2 + kv + n_logit_rows * V * 8


def layer_stack_microbench(hsd, inputs, torch, name, n_layers, ctx, rows_list):
    """Verify passes over `n_layers` layers of a larger model shape (weights drawn on the device: only the time is
    measured here), context `ctx` tokens: milliseconds and HBM fraction per pass, LM head excluded from neither."""
    shape = dict(inputs.SHAPES[name], n_layers=n_layers)
    d, F, V = shape["d"], shape["ffn"], shape["vocab"]
    nq, nkv = shape["n_q"] * shape["hd"], shape["n_kv"] * shape["hd"]
    model = hsd.Model(shape, hsd.BF16, ctx + 128, 64, inputs.ROPE_BASE, inputs.EPS)
    g = torch.Generator(device="cuda").manual_seed(1)
    rnd = lambda r, c, std: (torch.randn((r, c), device="cuda", generator=g) * std).to(torch.bfloat16)
    ones = torch.ones(d, device="cuda")
    for l in range(n_layers):
        model.load_layer_dev(l, {"norm1": ones, "norm2": ones, "wq": rnd(nq, d, d ** -0.5), "wk": rnd(nkv, d, d ** -0.5),
                                 "wv": rnd(nkv, d, d ** -0.5), "wo": rnd(d, nq, 0.1 * nq ** -0.5), "wg": rnd(F, d, d ** -0.5),
                                 "wu": rnd(F, d, d ** -0.5), "wd": rnd(d, F, 0.1 * F ** -0.5)})
    model.load_head_dev(rnd(V, d, 1.0), rnd(V, d, d ** -0.5), ones)
    tok = torch.randint(0, V, (ctx + 64,), device="cuda", dtype=torch.int32)
    for p0 in range(0, ctx, 64):
        model.model_pass(tok[p0:p0 + 64], p0, n_layers, 0)
    out = {}
    for m in rows_list:
        model.model_pass(tok[ctx:ctx + m], ctx, n_layers, m)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        iters = 20
        e0.record()
        for _ in range(iters):
            model.model_pass(tok[ctx:ctx + m], ctx, n_layers, m)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        b = pass_bytes(shape, n_layers, m, ctx + m, m)
        out["rows%d" % m] = {"ms": ms, "algorithmic_GB": b / 1e9, "hbm_frac": b / ms / 1e6 / HBM_PEAK_GBS}
    model.close()
    return out


def timed_generation(h, torch, n_prompt, n_gen, repeats):
    best = None
    for _ in range(repeats):
        h.rewind(n_prompt)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        out, st = h.generate(n_gen)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        if best is None or dt < best[0]:
            best = (dt, st)
    return best


def timed_sample_paths(h, torch, n_prompt, n_gen, seeds):
    """One generation per seed (the same prompt along different sample paths): total seconds, summed statistics.
    The acceptances of one path of 256 tokens scatter by several per cent, and any change of a kernel's summation
    order moves the path; the mean over paths is what a setting is worth."""
    total, acc = 0.0, None
    for seed in seeds:
        h.set_seed(seed)
        h.rewind(n_prompt)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        out, st = h.generate(n_gen)
        torch.cuda.synchronize()
        total += time.perf_counter() - t0
        if acc is None:
            acc = {"drafted": [0] * 8, "accepted": [0] * 8, "passes": [0] * 8, "rounds": 0}
        for i in range(8):
            acc["drafted"][i] += st.drafted[i]
            acc["accepted"][i] += st.accepted[i]
            acc["passes"][i] += st.passes[i]
        acc["rounds"] += st.rounds
    return total, acc


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="skip the sweeps; run HSD at T=(4,2) only")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py measures one GPU: this build has no multi-GPU path; run it with --gpus 1.")
        sys.exit(2)

    import torch
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    from paper_2510_19705_amd import hsd, inputs

    shape = inputs.SHAPES["1b"]
    t0 = time.time()
    weights = inputs.make_weights(shape, seed=SEED, bf16=True)
    prompt = inputs.make_prompt(shape["vocab"], PROMPT, seed=SEED + 1)
    log("weights generated in %.1f s" % (time.time() - t0))
    model = hsd.Model(shape, hsd.BF16, 1024, 64, inputs.ROPE_BASE, inputs.EPS, rows_copy_layers=EXITS[0])
    model.load(weights)
    log("model loaded (%.2f GB packed)" % (model.weights.numel() / 1e9))

    def make(levels, T):
        h = hsd.Hierarchy([(model, e) for e in levels], T, TEMPERATURE, SEED)
        h.prefill(prompt)
        return h

    results = {}

    def measure(name, levels, T, seeds=None):
        seeds = seeds or (SWEEP_SEEDS[:2] if args.no_sweep else SWEEP_SEEDS)     # --no-sweep: the short run for profilers
        h = make(levels, T)
        h.generate(GEN)                                   # warm-up
        dt, st = timed_sample_paths(h, torch, PROMPT, GEN, seeds)
        n = len(levels)
        results[name] = {"levels": list(levels), "T": list(T), "tokens_per_s": GEN * len(seeds) / dt, "sample_paths": len(seeds),
                         "acceptance": [st["accepted"][i] / max(1, st["drafted"][i]) for i in range(1, n)],
                         "passes": [st["passes"][i] for i in range(n)], "rounds": st["rounds"]}
        h.close()
        return results[name]

    # ---- untimed part: sweeps ---------------------------------------------------------------------
    ar = measure("autoregressive", (16,), ())
    log("autoregressive target: %.1f tok/s" % ar["tokens_per_s"])
    best_hsd, best_single = ("hsd_T4_2", None), (None, None)
    if args.no_sweep:
        r = measure("hsd_T4_2", EXITS, (4, 2))
        best_hsd = ("hsd_T4_2", r)
    else:
        for k1 in (2, 4, 6):
            for k2 in (1, 2, 4):
                name = "hsd_T%d_%d" % (k1, k2)
                r = measure(name, EXITS, (k1, k2))
                log("%s: %.1f tok/s acceptance %s" % (name, r["tokens_per_s"], ["%.2f" % a for a in r["acceptance"]]))
                if best_hsd[1] is None or r["tokens_per_s"] > best_hsd[1]["tokens_per_s"]:
                    best_hsd = (name, r)
        for e in EXITS[:-1]:
            for T in (1, 2, 3, 4, 6, 8):
                name = "single_exit%d_T%d" % (e, T)
                r = measure(name, (e, 16), (T,))
                log("%s: %.1f tok/s acceptance %.2f" % (name, r["tokens_per_s"], r["acceptance"][0]))
                if best_single[1] is None or r["tokens_per_s"] > best_single[1]["tokens_per_s"]:
                    best_single = (name, r)
    T_best = tuple(best_hsd[1]["T"])

    # ---- timed steps: HSD at the best setting ---------------------------------------------------
    # every step continues the prompt along its own sample path (seed + step), see timed_sample_paths
    h = make(EXITS, T_best)
    for i in range(args.warmup):
        h.set_seed(SEED + 1000 + i)
        h.rewind(PROMPT)
        h.generate(GEN)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        h.set_seed(SEED + i)
        h.rewind(PROMPT)
        h.generate(GEN)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    value = GEN * args.steps / elapsed
    h.set_seed(SEED)
    h.rewind(PROMPT)
    h.generate(GEN)                                            # the statistics below are those of the first path
    st = h.stats()

    # ---- per-pass HBM fraction (c_i of the latency model, measured at the M the level sees) --------
    passes = {}
    for lvl, e in enumerate(EXITS):
        m = 1 if lvl == 0 else min(int(round(st.pass_rows[lvl] / max(1, st.passes[lvl]))), T_best[0] + (T_best[1] if lvl == 2 else 0) + 1)
        m = max(1, m)
        ms = h.measure_pass(lvl, m, 50)
        b = pass_bytes(shape, e, m, h.sequence_length(), m)
        passes["exit%d" % e] = {"rows": m, "ms": ms, "algorithmic_GB": b / 1e9, "GBps": b / ms / 1e6,
                                "hbm_frac": b / ms / 1e6 / HBM_PEAK_GBS}

    # ---- roofline of the dominant kernel: one more step with per-site event brackets ------------
    h.rewind(PROMPT)
    model.profile_begin(60000)
    h.generate(GEN)
    sites = model.profile_end()
    bracket_us = sites.pop("empty_bracket_ms") * 1e3
    st2 = h.stats()
    gemm_sites = {k: v for k, v in sites.items() if k != "attn" and v[0] > 0}
    dom = max(gemm_sites, key=lambda k: gemm_sites[k][1])
    launches, total_ms = sites[dom]
    rows_avg = sum(st2.pass_rows[i] for i in range(3)) / max(1, sum(st2.passes[i] for i in range(3)))
    logit_rows_avg = (st2.passes[0] + st2.drafted[1] + st2.passes[1] + st2.drafted[2] + st2.passes[2]) / max(
        1, sum(st2.passes[i] for i in range(3)))
    m_avg = logit_rows_avg if dom == "head" else rows_avg
    bytes_per_launch = gemm_site_bytes(shape, dom, m_avg)
    raw_us = total_ms / launches * 1e3
    # The brackets rank the sites but inflate each launch by a few microseconds (two event packets), so the duration
    # that enters the roofline is measured separately: 320 launches of that site back to back between two events,
    # cycling through the 16 layers' weights (1 GB, more than the memory-side cache), at the row count of a target pass.
    m_dom = max(1, int(round(st2.pass_rows[2] / max(1, st2.passes[2]))))
    avg_us = model.measure_site(dom, m_dom, PROMPT, 320)
    bytes_per_launch = gemm_site_bytes(shape, dom, m_dom)
    achieved = bytes_per_launch / (avg_us * 1e-6) / 1e9
    # HBM bytes per launch measured with hardware counters (two rocprofv3 --pmc runs, see profiles/): not measurable
    # from inside this process, so the committed summary is quoted
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic_1b_layer_kernels_pmc.txt")
    if os.path.exists(tpath):
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch_%s:" % dom):
                traffic = int(line.split(":")[1])
    roofline = {"bound": "hbm", "kernel": "gemm_bf16_kernel (%s projection)" % dom, "achieved": achieved,
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                "avg_launch_us": avg_us, "rows": m_dom, "avg_launch_us_inside_event_brackets": raw_us,
                "empty_event_bracket_us": bracket_us, "launches_in_generation": launches, "bytes_per_launch": bytes_per_launch,
                "sites_ms": {k: round(v[1], 3) for k, v in sites.items()},
                "sites_launches": {k: v[0] for k, v in sites.items()}}
    # ---- the latency model on the measured quantities (Sec. 3.3, Sec. 4): which hierarchy does it pick? -------------
    selection = None
    if not args.no_sweep:
        cost = [passes["exit%d" % e]["ms"] for e in EXITS]
        a01 = results["hsd_T%d_%d" % T_best]["acceptance"][0]
        a02 = results["single_exit%d_T4" % EXITS[0]]["acceptance"][0]
        a12 = results["single_exit%d_T4" % EXITS[1]]["acceptance"][0]
        alpha = [[0, a01, a02], [0, 0, a12], [0, 0, 0]]
        lat, sigma, Tsel = hsd.select_hierarchy(cost, alpha, 8)
        slat, sdr, sT = hsd.best_single_draft(cost, alpha, 8)
        selection = {"cost_ms": cost, "alpha": {"0->1": a01, "0->2": a02, "1->2": a12},
                     "selected_levels": [EXITS[i] for i in sigma], "selected_T": Tsel,
                     "predicted_ms_per_token": lat, "predicted_tokens_per_s": 1e3 / lat,
                     "best_single_draft_predicted": {"exit": EXITS[sdr] if sdr >= 0 else None, "T": sT, "tokens_per_s": 1e3 / slat},
                     "hsd_T_best_predicted_tokens_per_s": 1e3 / hsd.expected_latency(cost, [a01, a12], list(T_best), True)}

    # ---- the four settings of the appendix on HSD's assumptions: real / coin-flip acceptances x measured / fixed costs ----
    cost_ms = [passes["exit%d" % e]["ms"] for e in EXITS]
    st_real = h.stats()                                         # of the profiled generation above (real rule)
    coin = [0.0] + [st_real.accepted[i] / max(1, st_real.tested[i]) for i in (1, 2)]
    h.set_ablation(coin, False)
    h.rewind(PROMPT)
    h.generate(GEN)                                             # warm-up
    dt_iid, st_iid = timed_generation(h, torch, PROMPT, GEN, 3)
    h.set_ablation(None, False)
    ablation = {"per_test_acceptance": coin[1:], "cost_ms_per_pass": cost_ms, "T": list(T_best),
                "ms_per_token": {"real_acceptance_real_cost": elapsed / args.steps / GEN * 1e3,
                                 "iid_acceptance_real_cost": dt_iid / GEN * 1e3,
                                 "real_acceptance_artificial_cost": hsd.stats_cost(st_real, cost_ms) / st_real.tokens,
                                 "iid_acceptance_artificial_cost": hsd.stats_cost(st_iid, cost_ms) / st_iid.tokens,
                                 "formula_exact_expectation": hsd.expected_latency(cost_ms, coin[1:], list(T_best), True),
                                 "formula_as_printed": hsd.expected_latency(cost_ms, coin[1:], list(T_best), False)}}

    # ---- calibration pass (Sec. 5.1) over the prompt + the tokens just generated: all-pairs acceptance rates of eight
    # candidate exits and their pass costs, the selection of Sec. 4 on them, and the selected hierarchy measured -------
    calibration = None
    if not args.no_sweep:
        h.rewind(PROMPT)
        gen_tokens, _ = h.generate(GEN)
        seq = torch.from_numpy(np.concatenate([prompt[:PROMPT], np.asarray(gen_tokens)]).astype(np.int32)).cuda()
        cand = [1, 2, 3, 4, 6, 8, 12, 16]
        alpha, cost = model.calibrate(cand, seq, PROMPT, TEMPERATURE, cost_rows=4)
        lat, sigma, Tsel = hsd.select_hierarchy(list(cost), alpha, 15)
        slat, sdr, sT = hsd.best_single_draft(list(cost), alpha, 15)
        tri = max(alpha[i, j] + alpha[j, k] - alpha[i, k] - 1 for i in range(len(cand)) for j in range(len(cand))
                  for k in range(len(cand)) if len({i, j, k}) == 3)
        calibration = {"exits": cand, "positions": GEN, "alpha": [[round(float(v), 4) for v in row] for row in alpha],
                       "cost_ms": [round(float(c), 4) for c in cost], "triangle_violation": float(tri),
                       "selected_levels": [cand[i] for i in sigma], "selected_T": list(Tsel),
                       "predicted_tokens_per_s": 1e3 / lat,
                       "best_single_draft_predicted": {"exit": cand[sdr] if sdr >= 0 else None, "T": sT, "tokens_per_s": 1e3 / slat}}
        try:
            if len(sigma) > 1:
                r = measure("calibrated_selection", [cand[i] for i in sigma], list(Tsel))
                calibration["measured_tokens_per_s"] = r["tokens_per_s"]
                calibration["measured_acceptance"] = r["acceptance"]
                log("calibrated selection %s T %s: predicted %.1f, measured %.1f tok/s" % (calibration["selected_levels"], Tsel,
                                                                                          1e3 / lat, r["tokens_per_s"]))
            if sdr >= 0 and [cand[sdr], 16] != calibration["selected_levels"]:
                r = measure("calibrated_single_draft", [cand[sdr], 16], [sT])
                calibration["best_single_draft_measured_tokens_per_s"] = r["tokens_per_s"]
        except hsd.HsdError as e:                 # e.g. a selection whose batches exceed the 64 rows of a pass
            calibration["error"] = str(e)

    # ---- verify passes of a larger shape: four layers of the 7B-shaped stack (32 x 128 heads, FFN 11008) ------------
    big = None if args.no_sweep else layer_stack_microbench(hsd, inputs, torch, "7b", 4, 4096, (1, 4, 8, 16))

    h.close()

    # ---- CPU baseline: the oracle on a bounded sample of the same workload ------------------------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import decoder, hsd as ohsd, specsample
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            threads = os.cpu_count()
        t0 = time.time()
        spec = decoder.Spec(shape["n_layers"], shape["d"], shape["n_q"], shape["n_kv"], shape["hd"], shape["ffn"],
                            shape["vocab"], inputs.ROPE_BASE, inputs.EPS)
        dec = decoder.Decoder(spec, weights, PROMPT + GEN + 32)
        log("oracle set up in %.1f s" % (time.time() - t0))
        levels = [decoder.Level(dec, e, TEMPERATURE) for e in EXITS]
        o = ohsd.HSD(levels, T_best, specsample.PhiloxChooser(SEED))
        n_p, n_g = PROMPT, 128
        o.levels[2].next_dists([int(t) for t in prompt[:n_p]], 1)      # prefill, untimed like the GPU's
        t0 = time.perf_counter()
        o.generate([int(t) for t in prompt[:n_p]], n_g)
        dt = time.perf_counter() - t0
        cpu = {"value": n_g / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
               "sample": "same 1B-shaped hierarchy and T, fp64 numpy oracle, prompt %d tokens (prefill untimed), first %d "
                         "generated tokens (%.1f s)" % (n_p, n_g, dt)}

    out = {
        "metric": "HSD tokens/sec at bs=1 vs best single-draft; verify-pass HBM GB/s / peak",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "1B-shaped early-exit hierarchy (16 layers, d 2048, 32q/8kv x 64, FFN 8192, vocab 32000), "
                               "exits 2/6/16, bf16, batch 1, prompt 512, generate 256, temperature 1",
                   "T": list(T_best), "global_batch": 1, "seq_len": PROMPT + GEN},
        "hsd": best_hsd[1], "best_single_draft": best_single[1], "autoregressive": ar,
        "hsd_vs_best_single_draft": (best_hsd[1]["tokens_per_s"] / best_single[1]["tokens_per_s"]) if best_single[1] else None,
        "hsd_vs_autoregressive": best_hsd[1]["tokens_per_s"] / ar["tokens_per_s"],
        "sweep": {k: round(v["tokens_per_s"], 1) for k, v in results.items()},
        "verify_pass": passes,
        "latency_model": selection,
        "calibration": calibration,
        "ablation": ablation,
        "verify_pass_7b_shaped_4_layers_ctx4096": big,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    model.close()


if __name__ == "__main__":
    main()
