"""Large-shape workloads of the HSD path on one MI355X, beyond what bench.py times: hierarchies of independent
networks, up to a 70B-shaped target (140 GB of bf16 weights resident in HBM).

    python -m paper_2510_19705_amd.workloads --config independent     # 125M / 1B / 7B-shaped, vocab 32000
    python -m paper_2510_19705_amd.workloads --config 70b             # 1B / 8B exit 8 / 8B / 70B-shaped, vocab 128256
    python -m paper_2510_19705_amd.workloads --config microbench      # one 7B-shaped layer: KV length x query tokens x batch
    python -m paper_2510_19705_amd.workloads --config projections     # its four projections alone, 1 to 1024 rows
    python -m paper_2510_19705_amd.workloads --config independent --distill   # drafters = target logits + noise (std 1.0 / 0.5)
    python -m paper_2510_19705_amd.workloads --config counters --shape 70b    # the workload of the hardware-counter runs
    python -m paper_2510_19705_amd.workloads --config launch-gap              # small models: kernel-busy share of a step, graph replay

Weights are drawn on the device (seeded normal, residual-writing matrices scaled by 0.1); prompts are uniform-random
ids.  For each workload: pass time and HBM fraction of every candidate (algorithmic bytes / time / 8 TB/s), pairwise
acceptance rates measured by teacher-forcing all candidates on the same positions (sum of min of the two
distributions, Sec. 2 / Sec. 5.1), the latency-optimal hierarchy for them (Sec. 4), and generated tokens per second
of that hierarchy, of the full hierarchy, of every single draft and of plain decoding of the target.  Prints one
JSON object.
"""
import argparse
import json
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = 2500.0      # dense bf16

CONFIGS = {
    # candidates (model name, exit layer) in ascending cost, the target last
    "independent": dict(models=["125m", "1b", "7b"], levels=[("125m", 12), ("1b", 16), ("7b", 32)], prompt=1024, gen=512),
    "70b": dict(models=["1b_v128k", "8b", "70b"], levels=[("1b_v128k", 16), ("8b", 8), ("8b", 32), ("70b", 80)], prompt=8192,
                gen=256),
    # a small stand-in with the same structure, for a quick check of this script
    "smoke": dict(models=["tiny_a", "tiny"], levels=[("tiny_a", 2), ("tiny", 4), ("tiny", 8)], prompt=64, gen=32),
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def pass_bytes(shape, exit_layer, m, s_total, n_logit_rows):
    """Algorithmic bytes of one pass: weights of the layers run + head once, KV read and written, logits and
    probability rows."""
    d, F, V = shape["d"], shape["ffn"], shape["vocab"]
    nq, nkv = shape["n_q"] * shape["hd"], shape["n_kv"] * shape["hd"]
    layer_w = (d * (nq + 2 * nkv) + nq * d + 3 * d * F) * 2
    kv = exit_layer * (2 * s_total * nkv * 2 + 2 * m * nkv * 2)
    return exit_layer * layer_w + V * d * 2 + kv + n_logit_rows * V * 8


def shapes(inputs):
    s = dict(inputs.SHAPES)
    s["1b_v128k"] = dict(s["1b"], vocab=128256)
    s["tiny_a"] = dict(n_layers=2, d=128, n_q=2, n_kv=1, hd=64, ffn=384, vocab=s["tiny"]["vocab"])
    return s


def random_model(hsd, inputs, torch, shape, seed, max_seq, max_rows=64, rows_copy_layers=0):
    """A bf16 model of `shape` with weights drawn on the device."""
    d, F, V = shape["d"], shape["ffn"], shape["vocab"]
    nq, nkv = shape["n_q"] * shape["hd"], shape["n_kv"] * shape["hd"]
    model = hsd.Model(shape, hsd.BF16, max_seq, max_rows, inputs.ROPE_BASE, inputs.EPS, rows_copy_layers=rows_copy_layers)
    g = torch.Generator(device="cuda").manual_seed(seed)
    rnd = lambda r, c, std: (torch.randn((r, c), device="cuda", generator=g) * std).to(torch.bfloat16)
    norm = lambda: 1 + 0.1 * torch.randn(d, device="cuda", generator=g)
    for l in range(shape["n_layers"]):
        model.load_layer_dev(l, {"norm1": norm(), "norm2": norm(), "wq": rnd(nq, d, d ** -0.5), "wk": rnd(nkv, d, d ** -0.5),
                                 "wv": rnd(nkv, d, d ** -0.5), "wo": rnd(d, nq, 0.1 * nq ** -0.5), "wg": rnd(F, d, d ** -0.5),
                                 "wu": rnd(F, d, d ** -0.5), "wd": rnd(d, F, 0.1 * F ** -0.5)})
        torch.cuda.synchronize()
    model.load_head_dev(rnd(V, d, 1.0), rnd(V, d, d ** -0.5), norm())
    torch.cuda.synchronize()
    return model


def measure_acceptance(hsd, torch, levels, tokens, n_ctx, chunk=16):
    """Teacher-forces every candidate over `tokens` (which also fills all KV caches) and returns alpha [n, n]: the
    mean over positions n_ctx.. of the overlap of the candidates' next-token distributions (temperature 1)."""
    n, n_tokens = len(levels), tokens.numel()
    sums = torch.zeros(n * (n - 1) // 2, dtype=torch.float64, device="cuda")
    deepest = {}
    for model, e in levels:
        deepest[id(model)] = (model, max(e, deepest.get(id(model), (model, 0))[1]))
    for pos in range(0, n_ctx, 64):                              # context-only positions: deepest exit of each network
        c = min(64, n_ctx - pos)
        for model, e in deepest.values():
            model.model_pass(tokens[pos:pos + c], pos, e, 0)
    for pos in range(n_ctx, n_tokens, chunk):
        c = min(chunk, n_tokens - pos)
        rows = []
        for model, e in levels:
            rows.append(hsd.softmax(model.model_pass(tokens[pos:pos + c], pos, e, c), 1.0))
        sums += hsd.overlap(torch.stack(rows)).sum(dim=1)
    alpha = np.ones((n, n))
    s = (sums / (n_tokens - n_ctx)).cpu().numpy()
    k = 0
    for i in range(n):
        for j in range(i + 1, n):
            alpha[i, j] = alpha[j, i] = s[k]
            k += 1
    return alpha


def run(config, seed=20251019, temperature=1.0):
    import torch
    assert torch.cuda.is_available(), "needs the GPU"
    from . import hsd, inputs
    cfg = CONFIGS[config]
    shp = shapes(inputs)
    prompt_len, gen = cfg["prompt"], cfg["gen"]
    max_seq = (prompt_len + gen + 128 + 63) // 64 * 64
    t0 = time.time()
    models = {}
    for i, name in enumerate(cfg["models"]):
        models[name] = random_model(hsd, inputs, torch, shp[name], seed + i, max_seq)
        log("%s loaded (%.1f GB of weights) at %.0f s" % (name, models[name].weights.numel() / 1e9, time.time() - t0))
    levels = [(models[name], e) for name, e in cfg["levels"]]
    names = ["%s/exit%d" % ne for ne in cfg["levels"]]
    V = shp[cfg["models"][0]]["vocab"]
    prompt = inputs.make_prompt(V, prompt_len, seed=seed + 100)
    tokens = torch.from_numpy(prompt.astype(np.int32)).cuda()

    n_score = min(128, prompt_len // 2)
    alpha = measure_acceptance(hsd, torch, levels, tokens, prompt_len - n_score)
    log("alpha\n", np.round(alpha, 3))

    # cost of a 4-token pass of every candidate at the end of the prompt, and its HBM fraction
    cost, passes = [], {}
    for (model, e), (name, _), label in zip(levels, cfg["levels"], names):
        m = 4
        tk = tokens[prompt_len - m:]
        model.model_pass(tk, prompt_len - m, e, m)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        iters = 5
        e0.record()
        for _ in range(iters):
            model.model_pass(tk, prompt_len - m, e, m)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / iters
        b = pass_bytes(shp[name], e, m, prompt_len, m)
        cost.append(ms)
        passes[label] = {"rows": m, "ms": ms, "algorithmic_GB": b / 1e9, "hbm_frac": b / ms / 1e6 / HBM_PEAK_GBS}
        log("%s: %.3f ms, %.1f%% of peak" % (label, ms, 100 * passes[label]["hbm_frac"]))

    lat, sigma, Tsel = hsd.select_hierarchy(cost, alpha, 15)
    results = {}

    def measure(label, idx, T):
        try:
            h = hsd.Hierarchy([levels[i] for i in idx], T, temperature, seed)
        except hsd.HsdError as err:
            results[label] = {"error": str(err)}
            return None
        h.prefill(prompt)
        h.generate(min(gen, 32))                                 # warm-up
        h.rewind(prompt_len)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        _, st = h.generate(gen)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t1
        n = len(idx)
        results[label] = {"levels": [names[i] for i in idx], "T": list(T), "tokens_per_s": gen / dt,
                          "acceptance": [st.accepted[i] / max(1, st.drafted[i]) for i in range(1, n)],
                          "passes": [st.passes[i] for i in range(n)]}
        log(label, results[label])
        h.close()
        return results[label]

    K = len(levels) - 1
    measure("autoregressive", [K], [])
    measure("selected", list(sigma), list(Tsel))
    for i in range(K):
        slat, _, sT = hsd.best_single_draft([cost[i], cost[K]], [[1, alpha[i, K]], [alpha[i, K], 1]], 15)
        measure("single_draft_%s" % names[i], [i, K], [sT])
    if list(sigma) != list(range(K + 1)):
        # the full hierarchy with the T the model picks when every level is forced in: search T in 1..8 by the formula
        best = None
        import itertools
        for T in itertools.product(range(1, 9), repeat=K):
            l = hsd.expected_latency(cost, [alpha[i, i + 1] for i in range(K)], list(T), True)
            if best is None or l < best[0]:
                best = (l, T)
        measure("full_hierarchy", list(range(K + 1)), list(best[1]))
    out = {"config": config, "candidates": names, "prompt": prompt_len, "generate": gen, "temperature": temperature,
           "alpha": [[round(float(v), 4) for v in row] for row in alpha], "cost_ms": cost, "verify_pass": passes,
           "selected": {"levels": [names[i] for i in sigma], "T": list(Tsel), "predicted_tokens_per_s": 1e3 / lat},
           "measured": results}
    for m in models.values():
        m.close()
    return out


def _time(torch, fn, iters):
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / iters                     # microseconds


def projections():
    """The four projections of one 7B-shaped layer (d 4096, 32 x 128 heads, FFN 11008), bf16, by row count: up to 64
    rows as the fused kernels of a pass (microseconds and TB/s of weights), 128 to 1024 rows as plain products through
    hsd_gemm (microseconds, TFLOP/s, fraction of the dense bf16 MFMA peak)."""
    import torch
    assert torch.cuda.is_available(), "needs the GPU"
    from . import hsd, inputs
    shape = dict(inputs.SHAPES["7b"], n_layers=4)
    d, F = shape["d"], shape["ffn"]
    n_q, n_kv, hd = shape["n_q"], shape["n_kv"], shape["hd"]
    model = random_model(hsd, inputs, torch, shape, 1, 256)
    tok = torch.randint(0, shape["vocab"], (128,), device="cuda", dtype=torch.int32)
    model.model_pass(tok[:64], 0, 4, 0)
    site_mb = {"qkv": (n_q + 2 * n_kv) * hd * d * 2 / 1e6, "o": n_q * hd * d * 2 / 1e6, "gateup": 2 * F * d * 2 / 1e6,
               "down": F * d * 2 / 1e6}
    gemm = {}
    for rows in (1, 2, 4, 8, 16, 32, 64):
        model.model_pass(tok[64:64 + rows], 64, 4, rows)
        us = {k: model.measure_site(k, rows, 64, 100) for k in site_mb}
        gemm[rows] = us
        log("rows %2d: " % rows + "  ".join("%s %.1f us (%.2f TB/s)" % (k, v, site_mb[k] / v) for k, v in us.items()))
    model.close()
    gemm_many = many_rows_mfma(hsd, torch, shape, (128, 256, 512, 1024))
    torch.cuda.empty_cache()
    site_nk = {"qkv": ((n_q + 2 * n_kv) * hd, d), "o": (d, n_q * hd), "gateup": (2 * F, d), "down": (d, F)}
    return {"shape": shape, "weight_MB": site_mb, "site_nk": site_nk, "projections_us_by_rows": gemm, "projections_many_rows": gemm_many}


def many_rows_mfma(hsd, torch, shape, rows_list):
    """Many-row cells (a batch of sequences times their drafted tokens): plain products y = x W^T through hsd_gemm at
    the four projection shapes of one layer (no fused epilogue at these row counts): microseconds, TFLOP/s and the
    fraction of the dense bf16 MFMA peak of the four together, by row count."""
    d, F = shape["d"], shape["ffn"]
    n_q, n_kv, hd = shape["n_q"], shape["n_kv"], shape["hd"]
    site_nk = {"qkv": ((n_q + 2 * n_kv) * hd, d), "o": (d, n_q * hd), "gateup": (2 * F, d), "down": (d, F)}
    packed = {k: hsd.pack_weight((torch.randn(n, kk, device="cuda") * kk ** -0.5).to(torch.bfloat16), hsd.BF16, 0)
              for k, (n, kk) in site_nk.items()}
    gemm_many = {}
    for rows in rows_list:
        us = {}
        for k, (n, kk) in site_nk.items():
            x = torch.randn(rows, kk, device="cuda").to(torch.bfloat16)
            ws = torch.zeros(hsd.lib.hsd_gemm_workspace_bytes(rows, n, kk), dtype=torch.uint8, device="cuda")
            us[k] = _time(torch, lambda: hsd.gemm(x, packed[k], n, hsd.BF16, ws), 20)
        flop = {k: 2.0 * rows * n * kk for k, (n, kk) in site_nk.items()}
        gemm_many[rows] = {"us": us, "tflops": {k: flop[k] / us[k] / 1e6 for k in us},
                           "mfma_frac": sum(flop.values()) / sum(us.values()) / 1e6 / MFMA_PEAK_TFLOPS}
        log("rows %4d: " % rows + "  ".join("%s %.1f us (%.0f TFLOP/s)" % (k, v, flop[k] / v / 1e6) for k, v in us.items()) +
            "  | MFMA fraction of the four: %.3f" % gemm_many[rows]["mfma_frac"])
    del packed
    return gemm_many


def microbench():
    """Isolated verify pass of ONE 7B-shaped layer (32 x 128 heads, MHA, d 4096, FFN 11008), bf16, random K/V and
    activations: k query tokens per sequence, cached length S, batch B.  Attention per layer at every cell whose K/V
    fits (one layer's K/V is B * S * 16 KiB); the four projections at B * k rows: up to 64 rows as the fused kernels
    of a pass, beyond (128 to 1024 rows, where the matrix cores and not the weight stream bound the time) as plain
    products through hsd_gemm, reported against the dense bf16 MFMA peak.  Also the sampler at vocab 128256 on random
    distributions."""
    import torch
    assert torch.cuda.is_available(), "needs the GPU"
    from . import hsd, inputs
    pr = projections()
    shape, site_mb, site_nk, gemm, gemm_many = pr["shape"], pr["weight_MB"], pr["site_nk"], pr["projections_us_by_rows"], pr["projections_many_rows"]
    n_q, n_kv, hd = shape["n_q"], shape["n_kv"], shape["hd"]
    cells = []
    for B in (1, 8, 64):
        for S in (4096, 16384, 32768):
            kv_bytes = 2 * S * n_kv * hd * 2 * B
            cache = hsd.KvLayer(B, S, n_kv, hd, hsd.BF16)
            cache.buf.view(torch.int16).random_(-16000, 16000)   # finite bf16 patterns
            ws = None
            for k in (1, 2, 4, 8, 16):
                q = torch.randn(B, k, n_q, hd, device="cuda").to(torch.bfloat16)
                pos0 = torch.full((B,), S - k, dtype=torch.int32, device="cuda")
                nb = hsd.lib.hsd_attention_workspace_bytes(B, k, n_q, n_kv, hd, S)
                if ws is None or ws.numel() < nb:
                    ws = torch.zeros(nb, dtype=torch.uint8, device="cuda")
                att_us = _time(torch, lambda: cache.attention(q, pos0, S, ws), 5 if kv_bytes > 4e9 else 20)
                rows = B * k
                cell = {"batch": B, "kv_len": S, "k": k, "kv_GB": kv_bytes / 1e9, "attention_us": att_us,
                        "attention_TBps": kv_bytes / att_us / 1e6}
                if rows in gemm:
                    g = sum(gemm[rows].values())
                    w_bytes = sum(site_mb.values()) * 1e6
                    cell.update({"projections_us": g, "layer_us": g + att_us,
                                 "layer_hbm_frac": (w_bytes + kv_bytes) / (g + att_us) / 1e3 / HBM_PEAK_GBS})
                elif rows in gemm_many:
                    g = sum(gemm_many[rows]["us"].values())
                    flop = 2.0 * rows * sum(n * kk for n, kk in site_nk.values()) + 4.0 * rows * S * n_q * hd
                    cell.update({"projections_us": g, "layer_us": g + att_us, "projections_mfma_frac": gemm_many[rows]["mfma_frac"],
                                 "layer_hbm_frac": (sum(site_mb.values()) * 1e6 + kv_bytes) / (g + att_us) / 1e3 / HBM_PEAK_GBS,
                                 "layer_mfma_frac": flop / (g + att_us) / 1e6 / MFMA_PEAK_TFLOPS})
                cells.append(cell)
                log(cell)
            del cache
            torch.cuda.empty_cache()
    # the same cells as ONE fused layer of the model (hsd_model_pass_batch: q/k/v + RoPE + KV append, attention,
    # o + residual, gate/up + SwiGLU, down + residual over the batch's rows), where batch x k fits the 64 rows of a pass
    # (a pass through three layers minus a pass through one, halved: the embedding kernel and the host's share of a
    # short pass drop out)
    fused = []
    three = dict(shape, n_layers=3)
    for B in (1, 8, 64):
        for S in (4096, 16384, 32768):
            pps = (S + 64) // 64
            model = random_model(hsd, inputs, torch, three, 3, B * pps * 64)
            model.set_batch(B, pps)
            for k in (1, 2, 4, 8, 16):
                if B * k > 64:
                    continue
                tk = torch.randint(0, three["vocab"], (B, k), device="cuda", dtype=torch.int32)
                iters = 10 if B * S > 500000 else 30
                t3 = _time(torch, lambda: model.model_pass_batch(tk, [S - k] * B, 3, with_logits=False), iters)
                t1 = _time(torch, lambda: model.model_pass_batch(tk, [S - k] * B, 1, with_logits=False), iters)
                us = (t3 - t1) / 2
                kv_bytes = 2 * S * n_kv * hd * 2 * B
                cell = {"batch": B, "kv_len": S, "k": k, "fused_layer_us": us, "three_layer_pass_us": t3, "one_layer_pass_us": t1,
                        "layer_hbm_frac": (sum(site_mb.values()) * 1e6 + kv_bytes) / us / 1e3 / HBM_PEAK_GBS}
                fused.append(cell)
                log(cell)
            model.close()
            del model
            torch.cuda.empty_cache()
    # sampler at the largest vocabulary (two launches: softmax, then accept / resample)
    sampler = []
    V = 128256
    for sigma in (1.0, 4.0):
        for t in (1, 4, 16):
            z = torch.randn(t + 1, V, device="cuda") * sigma
            p = hsd.softmax(z, 1.0)
            qd = hsd.softmax(z[:t] + torch.randn(t, V, device="cuda"), 1.0)
            x = torch.multinomial(qd, 1).to(torch.int32).flatten()
            xd = torch.cat([x, torch.zeros(1, dtype=torch.int32, device="cuda")])
            scratch = torch.zeros(hsd.lib.hsd_sampler_scratch_bytes(V), dtype=torch.uint8, device="cuda")
            res = torch.empty(2, dtype=torch.int32, device="cuda")
            pbuf = torch.empty_like(z)
            sm = torch.empty(max(256, hsd.lib.hsd_softmax_scratch_bytes(t + 1, V)), dtype=torch.uint8, device="cuda")

            def both():
                hsd._check(hsd.lib.hsd_softmax(z.data_ptr(), pbuf.data_ptr(), t + 1, V, 1.0, sm.data_ptr(), hsd._stream()))
                hsd._check(hsd.lib.hsd_accept_resample(pbuf.data_ptr(), qd.data_ptr(), xd.data_ptr(), t, V, 7, 1, 0, res.data_ptr(),
                                                       scratch.data_ptr(), hsd._stream()))
            sampler.append({"vocab": V, "sigma": sigma, "t": t, "softmax_plus_accept_us": _time(torch, both, 50)})
            log(sampler[-1])
    return {"config": "microbench", "projections_us_by_rows": gemm, "projections_many_rows": gemm_many, "weight_MB": site_mb,
            "cells": cells, "fused_layer_cells": fused, "sampler": sampler}


def site_bytes(shape, site, m, ctx=0):
    """Algorithmic bytes of one launch at a layer site: the weight matrix (or the K/V of the context) once +
    activations in and out."""
    d, F, V = shape["d"], shape["ffn"], shape["vocab"]
    nq, nkv = shape["n_q"] * shape["hd"], shape["n_kv"] * shape["hd"]
    if site == "attn":
        return 2 * (ctx + m) * nkv * 2 + 2 * m * nq * 2
    n, k, out_b = {"qkv": (nq + 2 * nkv, d, 2), "o": (d, nq, 10), "gateup": (2 * F, d, 1), "down": (d, F, 10),
                   "head": (V, d, 4)}[site]
    return n * k * 2 + m * k * 2 + m * n * out_b


REF_MIB = 256


def counters(shape_name, n_layers, rows, ctx):
    """Workload for hardware-counter runs (rocprofv3 --pmc FETCH_SIZE, then --pmc WRITE_SIZE, each with --kernel-trace):
    a plain element-wise kernel of known traffic (the scale reference: torch.add over REF_MIB MiB reads and writes that
    much), then ten verify passes of `rows` tokens through `n_layers` layers of the shape at context `ctx`, so that every
    kernel of a pass shows up with its per-dispatch counters.  Prints the manifest that profsum.py needs to label
    them: per site the kernel instance and the algorithmic bytes of a launch."""
    import torch
    assert torch.cuda.is_available(), "needs the GPU"
    from . import hsd, inputs
    shape = dict(shapes(inputs)[shape_name], n_layers=n_layers)
    model = random_model(hsd, inputs, torch, shape, 1, (ctx + 128 + 63) // 64 * 64)
    tok = torch.randint(0, shape["vocab"], (ctx + 64,), device="cuda", dtype=torch.int32)
    for p0 in range(0, ctx, 64):
        model.model_pass(tok[p0:p0 + min(64, ctx - p0)], p0, n_layers, 0)
    src = torch.ones(REF_MIB * (1 << 20) // 4, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(5):
        torch.add(src, 1.0, out=dst)
    torch.cuda.synchronize()
    for _ in range(10):
        model.model_pass(tok[ctx:ctx + rows], ctx, n_layers, rows)
    torch.cuda.synchronize()
    sites = {}
    for site in ("qkv", "o", "gateup", "down", "head"):
        sites[site] = {"kernel": model.site_kernel(site, rows), "algorithmic_bytes": site_bytes(shape, site, rows, ctx),
                       "launches": 10 * (1 if site == "head" else n_layers)}
    sites["attn"] = {"kernel": "attn_mfma_kernel<%d, 1>" % shape["hd"], "algorithmic_bytes": site_bytes(shape, "attn", rows, ctx),
                     "launches": 10 * n_layers}
    model.close()
    return {"config": "counters", "shape": shape_name, "shape_dims": shape, "layers": n_layers, "rows": rows, "ctx": ctx,
            "reference_kernel": "torch.add (vectorized_elementwise_kernel)", "reference_MiB_each_way": REF_MIB,
            "order_within_layer": ["qkv", "attn", "o", "gateup", "down"], "sites": sites}


def launch_gap(seed=20251019):
    """Where a generation step's time goes when the models are small (the 1B-shaped early-exit hierarchy, exits
    2 / 6 / 16, T = (4, 1), prompt 512, 256 tokens, temperature 1): wall-clock per generation; and, for two pass shapes,
    the same pass issued directly against a replay of the pass captured in a HIP graph (what a device-resident
    driver built from graphs could gain per pass), plus the host time one pass takes to enqueue.

    Run under `rocprofv3 --kernel-trace` the eight timed generations are bracketed by two launches of a kernel that
    nothing else here uses (the overlap kernel of the calibration), so that `profsum gap` can add up the kernel time
    inside the bracket: kernel-busy fraction of a generation, and the mean gap between launches."""
    import torch
    assert torch.cuda.is_available(), "needs the GPU"
    from . import hsd, inputs
    shape = inputs.SHAPES["1b"]
    prompt_len, gen, exits, T = 512, 256, (2, 6, 16), (4, 1)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):                                  # the models live on a stream a graph can capture
        model = random_model(hsd, inputs, torch, shape, seed, 1024, rows_copy_layers=exits[0])
        h = hsd.Hierarchy([(model, e) for e in exits], T, 1.0, seed)
        prompt = inputs.make_prompt(shape["vocab"], prompt_len, seed=seed + 1)
        h.prefill(prompt)
        h.generate(gen)
        marker_rows = torch.full((2, 1, 8), 0.125, device="cuda")
        seeds = [seed + 100 + i for i in range(8)]
        side.synchronize()
        hsd.overlap(marker_rows)
        t0 = time.perf_counter()
        for sd in seeds:
            h.set_seed(sd)
            h.rewind(prompt_len)
            h.generate(gen)
        side.synchronize()
        wall = (time.perf_counter() - t0) / len(seeds)
        hsd.overlap(marker_rows)
        side.synchronize()
        st = h.stats()
        out = {"config": "launch-gap", "workload": "1B-shaped early-exit hierarchy, exits 2/6/16, T (4, 1), prompt 512, 256 tokens",
               "generations_between_markers": len(seeds), "wall_ms_per_generation": wall * 1e3, "tokens_per_s": gen / wall,
               "passes_last_generation": [st.passes[i] for i in range(3)], "marker_kernel": "overlap_kernel", "graph_replay": {}}
        tok = torch.from_numpy(prompt.astype(np.int32)).cuda()
        for label, e, m in (("exit2_1row", 2, 1), ("exit6_5rows", 6, 5), ("exit16_6rows", 16, 6)):
            pos0 = prompt_len - m
            tk = tok[pos0:prompt_len].contiguous()
            fn = lambda: model.model_pass(tk, pos0, e, m)
            direct = _time_on(torch, side, fn, 50)
            t1 = time.perf_counter()
            for _ in range(50):
                fn()
            host_us = (time.perf_counter() - t1) / 50 * 1e6          # time to enqueue, nothing waited for
            side.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                ref = model.model_pass(tk, pos0, e, m)
            replay = _time_on(torch, side, g.replay, 50)
            same = bool(torch.equal(ref, fn()))                       # the replayed pass wrote the same logits
            out["graph_replay"][label] = {"direct_us": direct, "graph_replay_us": replay, "host_enqueue_us": host_us, "same_logits": same}
            log(label, out["graph_replay"][label])
        h.close()
        model.close()
    return out


def _time_on(torch, stream, fn, iters):
    fn()
    stream.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(iters):
        fn()
    e1.record(stream)
    stream.synchronize()
    return e0.elapsed_time(e1) * 1e3 / iters


def batch_throughput(hsd, inputs, torch, shape, exits, T, batches, prompt_len, gen, seed=20251019, temperature=1.0):
    """Generated tokens per second, summed over the sequences, of HSD over a batch of sequences in lockstep
    (hsd_batch_*): one early-exit hierarchy of one network, every sequence with its own prompt and sampling seed."""
    max_len = (prompt_len + gen + 128 + 63) // 64 * 64
    model = random_model(hsd, inputs, torch, shape, seed, max(batches) * max_len)
    out = {}
    for B in batches:
        prompts = [inputs.make_prompt(shape["vocab"], prompt_len, seed=seed + 200 + b) for b in range(B)]
        h = hsd.BatchHierarchy([(model, e) for e in exits], T, temperature, [seed + b for b in range(B)], max_len)
        h.prefill(prompts)
        h.generate(16)                                          # warm-up
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        _, st = h.generate(gen)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        n = len(exits)
        out["batch_%d" % B] = {"tokens_per_s": B * gen / dt, "per_sequence_tokens_per_s": gen / dt,
                               "passes": [st.passes[i] for i in range(n)],
                               "mean_pass_rows": [st.pass_rows[i] / max(1, st.passes[i]) for i in range(n)],
                               "acceptance": [st.accepted[i] / max(1, st.drafted[i]) for i in range(1, n)]}
        log("batch %d: %.0f tokens/s" % (B, out["batch_%d" % B]["tokens_per_s"]), out["batch_%d" % B])
        h.close()
    model.close()
    return out


def distilled_study(hsd, levels, names, cost, prompt, stds, chain, gen, temperature, seed, n_cached=None):
    """Hierarchies over candidates with synthetic closeness (hsd_hier_set_distilled), priced with the fixed cost per
    pass measured beforehand (the appendix's artificial-cost accounting: ms per token = sum of passes x cost / tokens;
    the side passes that produce the source logits make wall-clock meaningless).
    chain = False: every drafter's logits are the target's plus noise of std stds[i].
    chain = True: candidate i's logits are candidate i+1's plus noise of std stds[i] (the top drafter's: the target's),
    so neighbours are close and distant candidates less so; in a hierarchy that leaves candidates out, a level's
    noise towards the next level kept has the skipped steps' variances added.
    Acceptance rates are the per-test frequencies of the runs themselves.  n_cached: the networks already hold the K/V
    of that many prompt tokens (hsd_prefill_cached)."""
    import itertools
    K = len(levels) - 1
    assert len(stds) == K and len(cost) == K + 1
    results = {}

    def measure(label, idx, T):
        h = hsd.Hierarchy([levels[i] for i in idx], T, temperature, seed)
        top = len(idx) - 1
        for j in range(top - 1, -1, -1):                         # sources first: a chain is set from the top down
            if chain:
                h.set_distilled(j, j + 1, float(np.sqrt(sum(stds[i] ** 2 for i in range(idx[j], idx[j + 1])))))
            else:
                h.set_distilled(j, top, stds[idx[j]])
        if n_cached is None:
            h.prefill(prompt)
        else:
            h.prefill_cached(prompt, n_cached)
        _, st = h.generate(gen)
        n = len(idx)
        results[label] = {"levels": [names[i] for i in idx], "T": list(T),
                          "artificial_ms_per_token": hsd.stats_cost(st, [cost[i] for i in idx]) / st.tokens,
                          "per_test_acceptance": [st.accepted[i] / max(1, st.tested[i]) for i in range(1, n)],
                          "passes": [st.passes[i] for i in range(n)], "tokens": st.tokens}
        log(label, results[label])
        h.close()
        return results[label]

    measure("autoregressive", [K], [])
    alpha = np.eye(K + 1)
    for i in range(K):                                          # alpha_{i,K} from a single-draft run
        r = measure("probe_%s" % names[i], [i, K], [4])
        alpha[i, K] = alpha[K, i] = r["per_test_acceptance"][0]
    for i in range(K - 1):                                      # alpha_{i,i+1} from a three-level run
        r = measure("probe_%s_%s" % (names[i], names[i + 1]), [i, i + 1, K], [3, 2])
        alpha[i, i + 1] = alpha[i + 1, i] = r["per_test_acceptance"][0]
    for i in range(K + 1):                                      # pairs never measured: the triangle-inequality lower bound
        for j in range(i + 2, K):
            alpha[i, j] = alpha[j, i] = max(0.0, alpha[i, j - 1] + alpha[j - 1, j] - 1.0)
    log("alpha\n", np.round(alpha, 3))
    lat, sigma, Tsel = hsd.select_hierarchy(cost, alpha, 15)
    measure("selected", list(sigma), list(Tsel))
    for i in range(K):
        _, _, sT = hsd.best_single_draft([cost[i], cost[K]], [[1, alpha[i, K]], [alpha[i, K], 1]], 15)
        measure("single_draft_%s" % names[i], [i, K], [sT])
    if list(sigma) != list(range(K + 1)):
        best = None
        for T in itertools.product(range(1, 9), repeat=K):
            l = hsd.expected_latency(cost, [alpha[i, i + 1] for i in range(K)], list(T), True)
            if best is None or l < best[0]:
                best = (l, T)
        measure("full_hierarchy", list(range(K + 1)), list(best[1]))
    singles = [v["artificial_ms_per_token"] for k, v in results.items() if k.startswith("single_draft_")]
    return {"noise_std": list(stds), "noise": "each candidate = the next one up + noise" if chain else "each drafter = the target + noise",
            "candidates": names, "cost_ms": list(cost), "alpha": [[round(float(v), 4) for v in row] for row in alpha],
            "selected": {"levels": [names[i] for i in sigma], "T": list(Tsel), "predicted_ms_per_token": lat}, "runs": results,
            "selected_vs_best_single_draft": min(singles) / results["selected"]["artificial_ms_per_token"]}


def run_distilled(config, stds, seed=20251019, temperature=1.0, gen=None, chain=False):
    """distilled_study on the candidates of a configuration (which puts acceptance rates in the 0.5-0.9 range the
    paper works in); the fixed costs are 4-token passes at the end of the prompt."""
    import torch
    assert torch.cuda.is_available(), "needs the GPU"
    from . import hsd, inputs
    cfg = CONFIGS[config]
    shp = shapes(inputs)
    prompt_len = cfg["prompt"]
    gen = gen or cfg["gen"]
    max_seq = (prompt_len + gen + 128 + 63) // 64 * 64
    models = {name: random_model(hsd, inputs, torch, shp[name], seed + i, max_seq) for i, name in enumerate(cfg["models"])}
    levels = [(models[name], e) for name, e in cfg["levels"]]
    names = ["%s/exit%d" % ne for ne in cfg["levels"]]
    prompt = inputs.make_prompt(shp[cfg["models"][0]]["vocab"], prompt_len, seed=seed + 100)
    tokens = torch.from_numpy(prompt.astype(np.int32)).cuda()
    cost = []
    for (model, e) in levels:                                   # fixed cost: a 4-token pass at the end of the prompt
        for p0 in range(0, prompt_len, 64):
            model.model_pass(tokens[p0:p0 + min(64, prompt_len - p0)], p0, e, 0)
        tk = tokens[prompt_len - 4:]
        cost.append(_time(torch, lambda: model.model_pass(tk, prompt_len - 4, e, 4), 5) / 1e3)
    log("cost ms", cost)
    out = distilled_study(hsd, levels, names, cost, prompt, stds, chain, gen, temperature, seed)
    for m in models.values():
        m.close()
    out["config"] = config + (" (chain-distilled)" if chain else " (distilled)")
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", choices=sorted(CONFIGS) + ["microbench", "projections", "counters", "launch-gap"], default="independent")
    ap.add_argument("--shape", default="70b", help="counters: model shape")
    ap.add_argument("--layers", type=int, default=2, help="counters: layers of that shape")
    ap.add_argument("--rows", type=int, default=4, help="counters: tokens per verify pass")
    ap.add_argument("--ctx", type=int, default=8192, help="counters: cached positions")
    ap.add_argument("--distill", action="store_true", help="synthetic drafters: target logits + noise, fixed-cost accounting")
    ap.add_argument("--chain", action="store_true", help="with --distill: every candidate = the next one up + noise")
    ap.add_argument("--gen", type=int, default=0)
    args = ap.parse_args()
    if args.config == "microbench":
        out = microbench()
    elif args.config == "projections":
        out = projections()
    elif args.config == "launch-gap":
        out = launch_gap()
    elif args.config == "counters":
        out = counters(args.shape, args.layers, args.rows, args.ctx)
    elif args.distill:
        K = len(CONFIGS[args.config]["levels"]) - 1
        stds = ([0.8, 0.3, 0.3, 0.25] if args.chain else [1.0, 0.5, 0.35, 0.25])[:K] if K > 1 else [0.7]
        out = run_distilled(args.config, stds, gen=args.gen or None, chain=args.chain)
    else:
        out = run(args.config)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
