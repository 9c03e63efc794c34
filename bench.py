#!/usr/bin/env python3
"""Bench of the HSD hot path on one MI355X.

Headline workload (the largest single-GPU configuration): a four-level hierarchy up to a 70B-shaped target, bf16,
batch 1, everything resident in HBM (161 GB of weights): candidates 1B-shaped (16 layers, d 2048, 32q/8kv x 64, FFN
8192), the 8B-shaped network (32 layers, d 4096, 32q/8kv x 128, FFN 14336) at its exit after layer 8 and at full
depth, target 80 layers, d 8192, 64q/8kv x 128, FFN 28672; vocabulary 128256; prompt of 8192 uniform-random ids, 256
generated tokens, temperature 1.  Random-init weights drawn on the device (the paper's checkpoints and prompts are not
available offline).  The hierarchy is the one the latency-optimal selection (Sec. 4) picks from acceptance rates and
pass costs measured on the prompt (Sec. 5.1).

One step = one full generation of 256 tokens by that hierarchy from the prefilled prompt (rewind + generate: every
draft pass, verify pass, softmax, accept / reject / resample kernel and the round driver), each step along its own
sample path (sampling seed + step index).  Before the timed steps, untimed: calibration, selection, one generation
each of plain decoding, every single draft, the full four-level hierarchy.  After them, as extra keys: per-pass HBM
fractions, the roofline of the dominant kernel, the headline's networks with drafters made close synthetically along
the chain 1B -> 8B -> 70B (where three levels beat every single draft, priced per pass), the 1B-shaped early-exit
configuration (its (T_0, T_1) sweep), the three-network configuration with synthetic drafters, verify passes of
7B- and 8B-shaped layer stacks, the many-row MFMA figure, and the CPU oracle's baseline.

Prints ONE JSON line.  `value` = generated tokens per second of the selected hierarchy.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

SEED, TEMPERATURE = 20251019, 1.0
HBM_PEAK_GBS = 8000.0
BIG = dict(models=["1b_v128k", "8b", "70b"], levels=[("1b_v128k", 16), ("8b", 8), ("8b", 32), ("70b", 80)], prompt=8192, gen=256,
           rows_copy={"1b_v128k": 16, "8b": 8, "70b": 0})
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_70b_layer_kernels_pmc.txt")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def generate_paths(h, torch, n_prompt, n_gen, seeds):
    """One generation per seed (the same prompt along different sample paths): total seconds, summed statistics."""
    total, acc = 0.0, {"drafted": [0] * 8, "accepted": [0] * 8, "tested": [0] * 8, "passes": [0] * 8, "pass_rows": [0] * 8, "rounds": 0}
    for seed in seeds:
        h.set_seed(seed)
        h.rewind(n_prompt)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        _, st = h.generate(n_gen)
        torch.cuda.synchronize()
        total += time.perf_counter() - t0
        for i in range(8):
            for k in ("drafted", "accepted", "tested", "passes", "pass_rows"):
                acc[k][i] += getattr(st, k)[i]
        acc["rounds"] += st.rounds
    return total, acc


def summarize(levels_named, T, n_gen, seeds, dt, st):
    n = len(levels_named)
    return {"levels": levels_named, "T": list(T), "tokens_per_s": n_gen * len(seeds) / dt, "sample_paths": len(seeds),
            "acceptance": [st["accepted"][i] / max(1, st["drafted"][i]) for i in range(1, n)],
            "per_test_acceptance": [st["accepted"][i] / max(1, st["tested"][i]) for i in range(1, n)],
            "passes": [st["passes"][i] for i in range(n)], "mean_pass_rows": [st["pass_rows"][i] / max(1, st["passes"][i]) for i in range(n)],
            "rounds": st["rounds"]}


# --------------------------------------------------------------------------------------------------------------------
# headline: the four-level configuration up to the 70B-shaped target
# --------------------------------------------------------------------------------------------------------------------
def big_configuration(args, torch, hsd, inputs, workloads):
    shp = workloads.shapes(inputs)
    prompt_len, gen = BIG["prompt"], BIG["gen"]
    max_seq = (prompt_len + gen + 128 + 63) // 64 * 64
    t0 = time.time()
    models = {}
    for i, name in enumerate(BIG["models"]):
        models[name] = workloads.random_model(hsd, inputs, torch, shp[name], SEED + i, max_seq, rows_copy_layers=BIG["rows_copy"][name])
        torch.cuda.synchronize()
        log("%s loaded (%.1f GB of weights) at %.0f s" % (name, models[name].weights.numel() / 1e9, time.time() - t0))
    levels = [(models[name], e) for name, e in BIG["levels"]]
    names = ["%s/exit%d" % ne for ne in BIG["levels"]]
    K = len(levels) - 1
    prompt = inputs.make_prompt(shp["70b"]["vocab"], prompt_len, seed=SEED + 100)
    tokens = torch.from_numpy(prompt.astype(np.int32)).cuda()

    # calibration pass (Sec. 5.1) over the prompt: all-pairs acceptance rates on its last 128 positions, pass costs at
    # four rows; it leaves every network's K/V of the whole prompt in place, which all hierarchies below share
    alpha, cost = hsd.calibrate_levels(levels, tokens, prompt_len - 128, TEMPERATURE, cost_rows=4)
    cost = [float(c) for c in cost]
    log("calibrated at %.0f s: cost ms %s\nalpha\n%s" % (time.time() - t0, np.round(cost, 3), np.round(alpha, 3)))
    lat, sigma, Tsel = hsd.select_hierarchy(cost, alpha, 15)
    slat, sdr, sT = hsd.best_single_draft(cost, alpha, 15)
    verify_pass = {}
    for (name, e), label, c in zip(BIG["levels"], names, cost):
        b = workloads.pass_bytes(shp[name], e, 4, prompt_len, 4)
        verify_pass[label] = {"rows": 4, "ms": c, "algorithmic_GB": b / 1e9, "GBps": b / c / 1e6, "hbm_frac": b / c / 1e6 / HBM_PEAK_GBS}

    results = {}

    def hierarchy(idx, T):
        h = hsd.Hierarchy([levels[i] for i in idx], T, TEMPERATURE, SEED)
        h.prefill_cached(prompt, prompt_len - 1)
        return h

    def measure(label, idx, T, seeds):
        h = hierarchy(idx, T)
        h.generate(16)                                          # warm-up
        dt, st = generate_paths(h, torch, prompt_len, gen, seeds)
        results[label] = summarize([names[i] for i in idx], T, gen, seeds, dt, st)
        log("%s: %.2f tok/s %s" % (label, results[label]["tokens_per_s"], {k: results[label][k] for k in ("levels", "T", "acceptance", "passes")}))
        h.close()
        return results[label]

    paths = [SEED, SEED + 1]                                   # the sample paths of the first two timed steps
    if not args.brief:
        measure("autoregressive", [K], [], paths)
        for i in range(K):
            _, _, Ti = hsd.best_single_draft([cost[i], cost[K]], [[1, alpha[i, K]], [alpha[i, K], 1]], 15)
            measure("single_draft_%s" % names[i], [i, K], [max(1, Ti)], paths)
        if list(sigma) != list(range(K + 1)):
            import itertools
            best = None
            for T in itertools.product(range(1, 7), repeat=K):
                l = hsd.expected_latency(cost, [alpha[i, i + 1] for i in range(K)], list(T), True)
                if best is None or l < best[0]:
                    best = (l, T)
            measure("full_hierarchy", list(range(K + 1)), list(best[1]), paths)

    # ---- timed steps: the selected hierarchy --------------------------------------------------------------------
    h = hierarchy(list(sigma), list(Tsel))
    for i in range(args.warmup):
        h.set_seed(SEED + 1000 + i)
        h.rewind(prompt_len)
        h.generate(gen)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(args.steps):
        h.set_seed(SEED + i)
        h.rewind(prompt_len)
        h.generate(gen)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t1
    value = gen * args.steps / elapsed
    dt, st = generate_paths(h, torch, prompt_len, gen, paths)
    results["selected"] = summarize([names[i] for i in sigma], Tsel, gen, paths, dt, st)      # on the paths the other settings ran
    log("selected %s T %s: %.2f tok/s over %d steps (predicted %.2f)" % ([names[i] for i in sigma], Tsel, value, args.steps, 1e3 / lat))

    # ---- per-pass HBM fraction at the pass sizes the selected hierarchy's levels saw ---------------------------------
    passes = {}
    for lvl, ci in enumerate(sigma):
        name, e = BIG["levels"][ci]
        m = max(1, min(int(round(st["pass_rows"][lvl] / max(1, st["passes"][lvl]))), 16))
        ms = h.measure_pass(lvl, m, 10 if ci == K else 30)
        b = workloads.pass_bytes(shp[name], e, m, h.sequence_length(), m)
        passes[names[ci]] = {"rows": m, "ms": ms, "algorithmic_GB": b / 1e9, "GBps": b / ms / 1e6, "hbm_frac": b / ms / 1e6 / HBM_PEAK_GBS}

    # ---- roofline of the dominant kernel ------------------------------------------------------------------------------
    # Which kernel dominates: per-site event brackets around every launch of a short generation of the selected hierarchy.
    target = models["70b"]
    h.rewind(prompt_len)
    target.profile_begin(20000)
    h.generate(32)
    sites = target.profile_end()
    bracket_us = sites.pop("empty_bracket_ms") * 1e3
    gemm_sites = {k: v for k, v in sites.items() if k != "attn" and v[0] > 0}
    dom = max(gemm_sites, key=lambda k: gemm_sites[k][1])
    m_dom = passes[names[K]]["rows"]
    # Its launch duration: 160 launches of that site back to back between two HIP events on the model's stream, cycling
    # through the 80 layers' weights (75 GB for gate/up, far beyond any cache), at the row count of a target pass.
    avg_us = target.measure_site(dom, m_dom, prompt_len, 160)
    bytes_per_launch = workloads.site_bytes(shp["70b"], dom, m_dom)
    achieved = bytes_per_launch / (avg_us * 1e-6) / 1e9
    kernel = target.site_kernel(dom, m_dom)
    # HBM bytes per launch from hardware counters (two rocprofv3 --pmc runs, summarised under profiles/): not
    # measurable from inside this process, so the committed summary is quoted, but only if it profiled the same kernel
    # instance at the same row count as the one just timed
    traffic, traffic_note = None, "no counter summary for this kernel"
    if os.path.exists(TRAFFIC_FILE):
        for line in open(TRAFFIC_FILE):
            if line.startswith("traffic_bytes_per_launch_%s:" % dom):
                fields = line.split()
                meta = line.split("kernel=")[1].rsplit(" rows=", 1)
                if meta[0].strip() == kernel and int(meta[1]) == m_dom:
                    traffic, traffic_note = int(fields[1]), "profiles/%s" % os.path.basename(TRAFFIC_FILE)
                else:
                    traffic_note = "STALE counter summary: it profiled %s at %s rows, this run timed %s at %d rows" % (
                        meta[0].strip(), meta[1].strip(), kernel, m_dom)
                    log("bench.py: " + traffic_note + " -> traffic is reported as null; re-run the counter profile")
    roofline = {"bound": "hbm", "kernel": "%s (%s projection of the 70B-shaped target)" % (kernel, dom), "achieved": achieved,
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_note,
                "avg_launch_us": avg_us, "rows": m_dom, "bytes_per_launch": bytes_per_launch,
                "scope": "ONE launch of the dominant kernel; whole verify passes are under verify_pass / verify_pass_selected",
                "empty_event_bracket_us": bracket_us,
                "sites_ms_in_32_tokens": {k: round(v[1], 3) for k, v in sites.items()},
                "sites_launches_in_32_tokens": {k: v[0] for k, v in sites.items()}}
    h.close()
    # ---- the same networks with synthetic closeness along the chain 1B -> 8B -> 70B ------------------------------------
    # Random-init networks of different shapes overlap by chance only (alpha ~ 0.48 above, whatever the pair), so the
    # calibrated selection can only ever be a single draft.  Trained model families are graded: a model is closest to
    # the next size up.  Stand-in: the 8B-shaped level takes the target's logits + noise of std 0.3, the 1B-shaped one
    # the 8B level's + noise of std 0.8 (hsd_hier_set_distilled), each still running (and being priced at) its own pass.
    chain = None
    if not args.brief:
        sub = [0, 2, K]
        d = workloads.distilled_study(hsd, [levels[i] for i in sub], [names[i] for i in sub], [cost[i] for i in sub], prompt,
                                      [0.8, 0.3], True, 128, TEMPERATURE, SEED, n_cached=prompt_len - 1)
        chain = {"workload": "the headline's 1B / 8B / 70B-shaped networks (same prompt, 128 tokens per run), drafters made close "
                             "synthetically: 8B level = the target's logits + Gaussian noise of std 0.3, 1B level = the 8B level's + "
                             "noise of std 0.8; every run priced with the calibrated cost per pass (the side passes that produce "
                             "the source logits make wall-clock meaningless)",
                 "cost_ms": d["cost_ms"], "alpha": d["alpha"], "selected": d["selected"],
                 "artificial_ms_per_token": {k: round(v["artificial_ms_per_token"], 4) for k, v in d["runs"].items()},
                 "per_test_acceptance": {k: v["per_test_acceptance"] for k, v in d["runs"].items()},
                 "selected_vs_best_single_draft": d["selected_vs_best_single_draft"]}
        log("chain-distilled study: selected %s T %s, %.3f x the best single draft" % (
            d["selected"]["levels"], d["selected"]["T"], d["selected_vs_best_single_draft"]))
    best_single = None
    for k, v in results.items():
        if k.startswith("single_draft_") and (best_single is None or v["tokens_per_s"] > best_single["tokens_per_s"]):
            best_single = v
    out = {"value": value, "ms_per_step": elapsed / args.steps * 1e3, "T": list(Tsel),
           "candidates": names, "alpha": [[round(float(v), 4) for v in row] for row in alpha], "cost_ms": cost,
           "selection": {"levels": [names[i] for i in sigma], "T": list(Tsel), "predicted_tokens_per_s": 1e3 / lat,
                         "best_single_draft_predicted": {"level": names[sdr] if sdr >= 0 else None, "T": sT, "tokens_per_s": 1e3 / slat}},
           "hsd": results["selected"], "best_single_draft": best_single, "autoregressive": results.get("autoregressive"),
           "full_hierarchy": results.get("full_hierarchy"),
           "runs": {k: round(v["tokens_per_s"], 2) for k, v in results.items()},
           "verify_pass": verify_pass, "verify_pass_selected": passes, "roofline": roofline, "acc_stats": st,
           "chain_distilled": chain}
    for m in models.values():
        m.close()
    del models, levels, h, tokens
    torch.cuda.empty_cache()
    return out


# --------------------------------------------------------------------------------------------------------------------
# extra: the 1B-shaped early-exit configuration (exits 2 / 6 / 16, prompt 512, 256 tokens), its sweeps and calibration
# --------------------------------------------------------------------------------------------------------------------
def small_configuration(args, torch, hsd, inputs, workloads):
    PROMPT, GEN, EXITS = 512, 256, (2, 6, 16)
    seeds = tuple(SEED + 100 + i for i in range(4))
    shape = inputs.SHAPES["1b"]
    weights = inputs.make_weights(shape, seed=SEED, bf16=True)
    prompt = inputs.make_prompt(shape["vocab"], PROMPT, seed=SEED + 1)
    model = hsd.Model(shape, hsd.BF16, 1024, 64, inputs.ROPE_BASE, inputs.EPS, rows_copy_layers=EXITS[0])
    model.load(weights)
    results = {}

    def measure(name, levels, T):
        h = hsd.Hierarchy([(model, e) for e in levels], T, TEMPERATURE, SEED)
        h.prefill(prompt)
        h.generate(GEN)                                   # warm-up
        dt, st = generate_paths(h, torch, PROMPT, GEN, seeds)
        results[name] = summarize(list(levels), T, GEN, seeds, dt, st)
        h.close()
        return results[name]

    ar = measure("autoregressive", (16,), ())
    best_hsd, best_single = None, None
    for k1 in (2, 4, 6):
        for k2 in (1, 2, 4):
            r = measure("hsd_T%d_%d" % (k1, k2), EXITS, (k1, k2))
            if best_hsd is None or r["tokens_per_s"] > best_hsd["tokens_per_s"]:
                best_hsd = r
    for e in EXITS[:-1]:
        for T in (2, 4, 6, 8):
            r = measure("single_exit%d_T%d" % (e, T), (e, 16), (T,))
            if best_single is None or r["tokens_per_s"] > best_single["tokens_per_s"]:
                best_single = r
    T_best = tuple(best_hsd["T"])
    h = hsd.Hierarchy([(model, e) for e in EXITS], T_best, TEMPERATURE, SEED)
    h.prefill(prompt)
    gen_tokens, st = h.generate(GEN)
    passes = {}
    for lvl, e in enumerate(EXITS):
        m = max(1, min(int(round(st.pass_rows[lvl] / max(1, st.passes[lvl]))), 16))
        ms = h.measure_pass(lvl, m, 50)
        b = workloads.pass_bytes(shape, e, m, h.sequence_length(), m)
        passes["exit%d" % e] = {"rows": m, "ms": ms, "algorithmic_GB": b / 1e9, "hbm_frac": b / ms / 1e6 / HBM_PEAK_GBS}
    # the appendix's four settings: real / coin-flip acceptances x measured / fixed cost per pass
    cost_ms = [passes["exit%d" % e]["ms"] for e in EXITS]
    dt_real, st_real = generate_paths(h, torch, PROMPT, GEN, [SEED])
    coin = [0.0] + [st_real["accepted"][i] / max(1, st_real["tested"][i]) for i in (1, 2)]
    h.set_ablation(coin, False)
    dt_iid, st_iid = generate_paths(h, torch, PROMPT, GEN, [SEED])
    h.set_ablation(None, False)
    art = lambda s: sum(s["passes"][i] * cost_ms[i] for i in range(3)) / GEN
    ablation = {"per_test_acceptance": coin[1:], "cost_ms_per_pass": cost_ms, "T": list(T_best),
                "ms_per_token": {"real_acceptance_real_cost": dt_real / GEN * 1e3, "iid_acceptance_real_cost": dt_iid / GEN * 1e3,
                                 "real_acceptance_artificial_cost": art(st_real), "iid_acceptance_artificial_cost": art(st_iid),
                                 "formula_exact_expectation": hsd.expected_latency(cost_ms, coin[1:], list(T_best), True),
                                 "formula_as_printed": hsd.expected_latency(cost_ms, coin[1:], list(T_best), False)}}
    # calibration over the prompt + the generated tokens: eight candidate exits, all pairs, the selection on them, measured
    seq = torch.from_numpy(np.concatenate([prompt[:PROMPT], np.asarray(gen_tokens)]).astype(np.int32)).cuda()
    cand = [1, 2, 3, 4, 6, 8, 12, 16]
    alpha, cost = model.calibrate(cand, seq, PROMPT, TEMPERATURE, cost_rows=4)
    lat, sigma, Tsel = hsd.select_hierarchy(list(cost), alpha, 15)
    calibration = {"exits": cand, "alpha_to_target": [round(float(v), 4) for v in alpha[:, -1]], "cost_ms": [round(float(c), 4) for c in cost],
                   "selected_levels": [cand[i] for i in sigma], "selected_T": list(Tsel), "predicted_tokens_per_s": 1e3 / lat}
    h.close()
    try:
        if len(sigma) > 1:
            calibration["measured_tokens_per_s"] = measure("calibrated_selection", [cand[i] for i in sigma], list(Tsel))["tokens_per_s"]
    except hsd.HsdError as e:                     # e.g. a selection whose batches exceed the 64 rows of a pass
        calibration["error"] = str(e)
    model.close()
    return {"workload": "1B-shaped early-exit hierarchy (16 layers, d 2048, 32q/8kv x 64, FFN 8192, vocab 32000), exits 2/6/16, bf16, "
                        "batch 1, prompt 512, generate 256, temperature 1; four sample paths per setting",
            "hsd": best_hsd, "best_single_draft": best_single, "autoregressive": ar,
            "hsd_vs_best_single_draft": best_hsd["tokens_per_s"] / best_single["tokens_per_s"],
            "hsd_vs_autoregressive": best_hsd["tokens_per_s"] / ar["tokens_per_s"],
            "sweep": {k: round(v["tokens_per_s"], 1) for k, v in results.items()}, "verify_pass": passes, "ablation": ablation,
            "calibration": calibration}, (shape, weights, prompt, EXITS, T_best)


def layer_stack_passes(torch, hsd, inputs, workloads, name, n_layers, ctx, rows_list):
    """Verify passes over `n_layers` layers of a larger model shape, context `ctx` tokens: milliseconds and HBM
    fraction per pass (embedding, layers and the LM head: everything a pass launches)."""
    shape = dict(inputs.SHAPES[name], n_layers=n_layers)
    model = workloads.random_model(hsd, inputs, torch, shape, 1, ctx + 128)
    tok = torch.randint(0, shape["vocab"], (ctx + 64,), device="cuda", dtype=torch.int32)
    for p0 in range(0, ctx, 64):
        model.model_pass(tok[p0:p0 + 64], p0, n_layers, 0)
    out = {}
    for m in rows_list:
        us = workloads._time(torch, lambda: model.model_pass(tok[ctx:ctx + m], ctx, n_layers, m), 20)
        b = workloads.pass_bytes(shape, n_layers, m, ctx + m, m)
        out["rows%d" % m] = {"ms": us / 1e3, "algorithmic_GB": b / 1e9, "hbm_frac": b / us / 1e3 / HBM_PEAK_GBS}
    model.close()
    return out


def cpu_baseline(inputs, workloads, big):
    """The oracle as it stands on the host cores, on a bounded sample of the headline workload: one fp64 oracle layer
    of each shape the selected hierarchy runs, at that level's pass size, plus an eighth of the LM head; a pass is
    priced as layers run x layer time + 8 x head-slice time, and the run as the sum over levels of passes x price."""
    from oracle import decoder
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count()
    shp = workloads.shapes(inputs)
    rng = np.random.default_rng(1)
    t_all = time.time()
    total_s, parts = 0.0, []
    st = big["acc_stats"]
    for lvl, label in enumerate(big["hsd"]["levels"]):
        name, e = label.split("/exit")
        e = int(e)
        s = dict(shp[name], n_layers=1)
        m = max(1, int(round(st["pass_rows"][lvl] / max(1, st["passes"][lvl]))))
        Vs = s["vocab"] // 8
        w = {"embed": rng.random((Vs, s["d"]), dtype=np.float32), "head": rng.random((Vs, s["d"]), dtype=np.float32) * 0.01,
             "norm_f": np.ones(s["d"], dtype=np.float32),
             "layers": [{k: (np.ones(sh, dtype=np.float32) if len(sh) == 1 else (rng.random(sh, dtype=np.float32) - 0.5) * (sh[1] ** -0.5))
                         for k, sh in inputs.LAYER_SHAPES(s).items()}]}
        spec = decoder.Spec(1, s["d"], s["n_q"], s["n_kv"], s["hd"], s["ffn"], Vs, inputs.ROPE_BASE, inputs.EPS)
        dec = decoder.Decoder(spec, w, 64 + m)
        toks = [int(t) for t in rng.integers(0, Vs, 32 + m)]
        dec.forward(toks[:32], 0, 1)                             # a short cached context (K/V is 2 % of a pass's bytes here)
        x = dec.embed[np.asarray(toks[32:], dtype=np.int64)]
        y = dec._layer(0, x, 32)                                 # untimed first call (page faults of the fresh arrays)
        reps = 0
        t0 = time.perf_counter()
        while reps < 3 or time.perf_counter() - t0 < 4.0:        # a few seconds per shape
            y = dec._layer(0, x, 32)
            reps += 1
        t_layer = (time.perf_counter() - t0) / reps
        reps = 0
        t0 = time.perf_counter()
        while reps < 3 or time.perf_counter() - t0 < 2.0:
            decoder.rmsnorm(y, dec.norm_f, spec.eps) @ dec.head.T
            reps += 1
        t_head = (time.perf_counter() - t0) / reps * 8
        per_pass = e * t_layer + t_head
        total_s += st["passes"][lvl] * per_pass
        parts.append("%s: %d rows, layer %.3f s, head %.3f s, pass %.2f s x %d passes" % (label, m, t_layer, t_head, per_pass, st["passes"][lvl]))
        del dec, w
    tokens = BIG["gen"] * big["hsd"]["sample_paths"]            # the pass counts are sums over that many generations
    return {"value": tokens / total_s, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": "EXTRAPOLATED from one fp64 numpy oracle layer per shape of the selected hierarchy at that level's pass size "
                      "(plus one eighth of the LM head): pass = layers run x layer time + 8 x head-slice time; run = sum over levels "
                      "of the GPU run's pass counts x pass; %s; %.0f s of CPU work" % ("; ".join(parts), time.time() - t_all)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--brief", action="store_true", help="the headline workload's timed steps and roofline only (profiler runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py measures one GPU: this build has no multi-GPU path; run it with --gpus 1.")
        sys.exit(2)

    import torch
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    from paper_2510_19705_amd import hsd, inputs, workloads

    t_start = time.time()
    big = big_configuration(args, torch, hsd, inputs, workloads)
    log("headline configuration done at %.0f s" % (time.time() - t_start))
    small = batched = distilled = stack7b = stack8b = mfma = cpu = None
    if not args.brief:
        small, _ = small_configuration(args, torch, hsd, inputs, workloads)
        batched = {"workload": "the same 1B-shaped early-exit hierarchy, T = (4, 1), over 1 / 4 / 8 sequences in lockstep (hsd_batch_*): own "
                               "prompt of 512 tokens and own sampling seed per sequence, 256 tokens each, temperature 1; tokens/s summed "
                               "over the sequences",
                   **workloads.batch_throughput(hsd, inputs, torch, dict(inputs.SHAPES["1b"]), (2, 6, 16), (4, 1), (1, 4, 8), 512, 256)}
        torch.cuda.empty_cache()
        log("1B-shaped configuration done at %.0f s" % (time.time() - t_start))
        torch.cuda.empty_cache()
        d = workloads.run_distilled("independent", [1.0, 0.5], gen=128)
        distilled = {"workload": "independent 125M / 1B / 7B-shaped networks, vocab 32000, prompt 1024, 128 tokens, drafters' logits = the "
                                 "target's + Gaussian noise of std 1.0 / 0.5; priced with the fixed cost per pass (the target's side "
                                 "passes make wall-clock meaningless)",
                     "cost_ms": d["cost_ms"], "alpha": d["alpha"], "selected": d["selected"],
                     "artificial_ms_per_token": {k: round(v["artificial_ms_per_token"], 4) for k, v in d["runs"].items()},
                     "per_test_acceptance": {k: v["per_test_acceptance"] for k, v in d["runs"].items()}}
        singles = [v for k, v in distilled["artificial_ms_per_token"].items() if k.startswith("single_draft_")]
        three = [d["runs"][k]["artificial_ms_per_token"] for k in ("selected", "full_hierarchy") if k in d["runs"] and len(d["runs"][k]["levels"]) == 3]
        distilled["three_levels_vs_best_single_draft"] = min(singles) / three[0] if singles and three else None
        log("distilled three-network configuration done at %.0f s" % (time.time() - t_start))
        torch.cuda.empty_cache()
        stack7b = layer_stack_passes(torch, hsd, inputs, workloads, "7b", 4, 4096, (1, 4, 8, 16))
        stack8b = layer_stack_passes(torch, hsd, inputs, workloads, "8b", 4, 8192, (1, 4, 8, 16))
        mm = workloads.many_rows_mfma(hsd, torch, dict(inputs.SHAPES["7b"]), (1024,))
        mfma = {"what": "the four projections of one 7B-shaped layer at 1024 rows (batch 64 x 16 drafted tokens) through hsd_gemm",
                "tflops": {k: round(v, 1) for k, v in mm[1024]["tflops"].items()}, "frac_of_2500_TFLOPs": mm[1024]["mfma_frac"]}
        torch.cuda.empty_cache()
        log("layer stacks done at %.0f s" % (time.time() - t_start))
    if not args.no_cpu_baseline and not args.brief:
        cpu = cpu_baseline(inputs, workloads, big)
        log("cpu baseline done at %.0f s" % (time.time() - t_start))

    hsd_tps = big["hsd"]["tokens_per_s"]
    out = {
        "metric": "HSD tokens/sec at bs=1 vs best single-draft; verify-pass HBM GB/s / peak",
        "value": big["value"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": big["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "4-level hierarchy up to a 70B-shaped target (80 layers, d 8192, 64q/8kv x 128, FFN 28672), candidates "
                               "1B-shaped, 8B-shaped exit 8, 8B-shaped; vocab 128256, bf16, batch 1, prompt 8192, generate 256, "
                               "temperature 1; hierarchy selected from measured acceptance rates and pass costs",
                   "T": big["T"], "global_batch": 1, "seq_len": BIG["prompt"] + BIG["gen"]},
        "candidates": big["candidates"], "alpha": big["alpha"], "cost_ms": big["cost_ms"], "selection": big["selection"],
        "hsd": big["hsd"], "best_single_draft": big["best_single_draft"], "autoregressive": big["autoregressive"],
        "full_hierarchy": big["full_hierarchy"], "runs_tokens_per_s": big["runs"],
        "hsd_vs_best_single_draft": hsd_tps / big["best_single_draft"]["tokens_per_s"] if big["best_single_draft"] else None,
        "hsd_vs_autoregressive": hsd_tps / big["autoregressive"]["tokens_per_s"] if big["autoregressive"] else None,
        "verify_pass": big["verify_pass"], "verify_pass_selected": big["verify_pass_selected"],
        "verify_pass_7b_shaped_4_layers_ctx4096": stack7b, "verify_pass_8b_shaped_4_layers_ctx8192": stack8b,
        "mfma_util": mfma,
        "config_5_networks_chain_distilled": big["chain_distilled"],
        "config_1b_early_exit": small, "config_1b_early_exit_batched": batched, "config_3_networks_distilled": distilled,
        "roofline": big["roofline"], "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
