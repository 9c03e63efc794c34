// Calibration pass (Sec. 5.1, "Optimization and Results"): run the network over sample contexts, keep every candidate
// exit's output distribution at every position, and estimate the pairwise acceptance rates alpha_{i,j} as the mean
// over positions of sum_x min(p_i(x), p_j(x)) = 1 - TV(p_i, p_j) (Sec. 2); record each exit's pass cost.  The result
// feeds the hierarchy selection of Sec. 4 (hsd_select_hierarchy).
#include <algorithm>
#include <vector>

#include "common.h"
#include "model.h"

namespace {

// out[pair * stride + r] = sum_x min(P[i][r][x], P[j][r][x]) for pair = (i < j) in the order (0,1), (0,2), .., (1,2), ..
// grid (rows, pairs), 256 threads; fp64 partial sums in a fixed order, so the value does not depend on scheduling.
__global__ __launch_bounds__(256) void overlap_kernel(const float* __restrict__ P, int n, int R, int V, double* __restrict__ out,
                                                      size_t stride) {
    __shared__ double sh[4];
    const int r = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int i = 0, rest = blockIdx.y;                        // pair index -> (i, j)
    while (rest >= n - 1 - i) { rest -= n - 1 - i; ++i; }
    const int j = i + 1 + rest;
    const float* a = P + ((size_t)i * R + r) * V;
    const float* b = P + ((size_t)j * R + r) * V;
    double acc = 0.0;
    if ((V & 3) == 0 && (((uintptr_t)a | (uintptr_t)b) & 15) == 0) {
        for (int x = tid * 4; x < V; x += 1024) {
            const float4 u = *reinterpret_cast<const float4*>(a + x), w = *reinterpret_cast<const float4*>(b + x);
            acc += ((double)fminf(u.x, w.x) + (double)fminf(u.y, w.y)) + ((double)fminf(u.z, w.z) + (double)fminf(u.w, w.w));
        }
    } else {
        for (int x = tid; x < V; x += 256) acc += (double)fminf(a[x], b[x]);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (lane == 0) sh[wave] = acc;
    __syncthreads();
    if (tid == 0) out[(size_t)blockIdx.y * stride + r] = (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

int launch_overlap(const float* P, int n, int R, int V, double* out, size_t stride, hipStream_t s) {
    if (n < 2 || R < 1) return HSD_OK;
    overlap_kernel<<<dim3(R, n * (n - 1) / 2), 256, 0, s>>>(P, n, R, V, out, stride);
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

struct CalibLayout {
    size_t logits, probs, overlaps, softmax, total;
    int chunk, npairs, n_scored;
};

int calib_layout(const hsd_model* m, int n_exits, int n_tokens, int n_ctx, CalibLayout* L) {
    if (!m) HSD_FAIL(HSD_EINVAL, "calibrate: null model");
    if (n_exits < 1 || n_exits > m->desc.n_layers) HSD_FAIL(HSD_EINVAL, "calibrate: %d exits", n_exits);
    if (n_ctx < 0 || n_tokens <= n_ctx) HSD_FAIL(HSD_EINVAL, "calibrate: %d tokens of which %d are context only", n_tokens, n_ctx);
    if (n_tokens > m->desc.max_seq) HSD_FAIL(HSD_ECAPACITY, "calibrate: %d tokens exceed the KV capacity %d", n_tokens, m->desc.max_seq);
    L->chunk = m->desc.max_rows < 16 ? m->desc.max_rows : 16;
    L->npairs = n_exits * (n_exits - 1) / 2;
    L->n_scored = n_tokens - n_ctx;
    const size_t rows = (size_t)n_exits * L->chunk * m->desc.vocab * sizeof(float);
    size_t o = 0;
    L->logits = o;   o += align_up(rows, 256);
    L->probs = o;    o += align_up(rows, 256);
    L->overlaps = o; o += align_up((size_t)(L->npairs > 0 ? L->npairs : 1) * L->n_scored * sizeof(double), 256);
    L->softmax = o;  o += softmax_scratch_bytes(n_exits * L->chunk, m->desc.vocab);
    L->total = o;
    return HSD_OK;
}

}  // namespace

extern "C" int hsd_overlap(const float* rows_dev, int n_dists, int n_rows, int vocab, double* out_dev, void* stream) {
    if (!rows_dev || !out_dev) HSD_FAIL(HSD_EINVAL, "hsd_overlap: null pointer");
    if (n_dists < 2 || n_dists > 64 || n_rows < 1 || vocab < 1) HSD_FAIL(HSD_EINVAL, "hsd_overlap: n_dists=%d n_rows=%d vocab=%d", n_dists, n_rows, vocab);
    return launch_overlap(rows_dev, n_dists, n_rows, vocab, out_dev, (size_t)n_rows, (hipStream_t)stream);
}

extern "C" size_t hsd_calibrate_workspace_bytes(const hsd_model* m, int n_exits, int n_tokens, int n_ctx) {
    CalibLayout L;
    return calib_layout(m, n_exits, n_tokens, n_ctx, &L) ? 0 : L.total;
}

extern "C" int hsd_calibrate(hsd_model* m, const int* exits, int n_exits, const int32_t* tokens_dev, int n_tokens, int n_ctx,
                             float temperature, int cost_rows, void* workspace_dev, size_t workspace_bytes, double* alpha_out,
                             double* cost_ms_out) {
    CalibLayout L;
    if (int rc = calib_layout(m, n_exits, n_tokens, n_ctx, &L)) return rc;
    if (!exits || !tokens_dev || !workspace_dev || !alpha_out) HSD_FAIL(HSD_EINVAL, "hsd_calibrate: null pointer");
    if ((uintptr_t)workspace_dev & 255) HSD_FAIL(HSD_EINVAL, "hsd_calibrate: workspace must be 256-byte aligned");
    if (workspace_bytes < L.total) HSD_FAIL(HSD_ECAPACITY, "hsd_calibrate: workspace of %zu bytes, %zu needed", workspace_bytes, L.total);
    if (!(temperature >= 0.f)) HSD_FAIL(HSD_EINVAL, "hsd_calibrate: temperature %g", temperature);
    if (cost_ms_out && (cost_rows < 1 || cost_rows > L.chunk || cost_rows > n_tokens))
        HSD_FAIL(HSD_EINVAL, "hsd_calibrate: cost_rows=%d outside 1..%d", cost_rows, L.chunk < n_tokens ? L.chunk : n_tokens);
    const hsd_model_desc& d = m->desc;
    hipStream_t s = m->stream;
    char* wb = (char*)workspace_dev;
    float* logits = (float*)(wb + L.logits);
    float* probs = (float*)(wb + L.probs);
    double* overlaps = (double*)(wb + L.overlaps);

    // context-only positions through the deepest exit (model_pass_exits validates the list), then the scored positions
    // with every exit's rows
    for (int pos = 0; pos < n_ctx;) {
        const int c = std::min(d.max_rows, n_ctx - pos);
        if (int rc = model_pass_exits(m, tokens_dev + pos, pos, c, exits, n_exits, 0, nullptr)) return rc;
        pos += c;
    }
    for (int pos = n_ctx; pos < n_tokens;) {
        const int c = std::min(L.chunk, n_tokens - pos);
        if (int rc = model_pass_exits(m, tokens_dev + pos, pos, c, exits, n_exits, c, logits)) return rc;
        if (int rc = launch_softmax(logits, probs, n_exits * c, d.vocab, temperature, (float*)(wb + L.softmax), s)) return rc;
        if (int rc = launch_overlap(probs, n_exits, c, d.vocab, overlaps + (pos - n_ctx), (size_t)L.n_scored, s)) return rc;
        pos += c;
    }
    std::vector<double> host((size_t)L.npairs * L.n_scored);
    if (L.npairs > 0) {
        HSD_HIP(hipMemcpyAsync(host.data(), overlaps, host.size() * sizeof(double), hipMemcpyDeviceToHost, s));
    }
    HSD_HIP(hipStreamSynchronize(s));
    int pair = 0;
    for (int i = 0; i < n_exits; ++i) {
        alpha_out[i * n_exits + i] = 1.0;
        for (int j = i + 1; j < n_exits; ++j, ++pair) {
            double sum = 0.0;
            for (int t = 0; t < L.n_scored; ++t) sum += host[(size_t)pair * L.n_scored + t];
            alpha_out[i * n_exits + j] = alpha_out[j * n_exits + i] = sum / L.n_scored;
        }
    }
    if (!cost_ms_out) return HSD_OK;

    // cost of one pass of cost_rows tokens per exit (Sec. 3.2: c_i = time of a forward pass), at the end of the sequence
    hipEvent_t e0, e1;
    HSD_HIP(hipEventCreate(&e0));
    HSD_HIP(hipEventCreate(&e1));
    const int pos0 = n_tokens - cost_rows, iters = 10;
    int rc = HSD_OK;
    for (int i = 0; i < n_exits && !rc; ++i) {
        rc = model_pass(m, tokens_dev + pos0, pos0, cost_rows, exits[i], cost_rows, logits);            // warm-up
        if (!rc && hipEventRecord(e0, s) != hipSuccess) rc = HSD_EHIP;
        for (int k = 0; k < iters && !rc; ++k) rc = model_pass(m, tokens_dev + pos0, pos0, cost_rows, exits[i], cost_rows, logits);
        float ms = 0.f;
        if (!rc && (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                    hipEventElapsedTime(&ms, e0, e1) != hipSuccess)) {
            hsd_set_error("hsd_calibrate: event timing failed");
            rc = HSD_EHIP;
        }
        cost_ms_out[i] = (double)ms / iters;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return rc;
}

// ------------------------------------------------------------------------------------------------
// The same estimate over candidates that may be different networks (Sec. 3.2: models that share only the
// vocabulary; Sec. 5.1 records all candidates on the same contexts).
// ------------------------------------------------------------------------------------------------
namespace {

struct LevelsLayout {
    size_t logits, probs, overlaps, softmax, total;
    int chunk, npairs, n_scored, vocab;
};

int levels_layout(int n, const hsd_level* levels, int n_tokens, int n_ctx, LevelsLayout* L) {
    if (n < 1 || n > 64 || !levels) HSD_FAIL(HSD_EINVAL, "calibrate: %d candidates (1..64)", n);
    if (n_ctx < 0 || n_tokens <= n_ctx) HSD_FAIL(HSD_EINVAL, "calibrate: %d tokens of which %d are context only", n_tokens, n_ctx);
    L->chunk = 16;
    for (int i = 0; i < n; ++i) {
        const hsd_model* m = levels[i].model;
        if (!m) HSD_FAIL(HSD_EINVAL, "calibrate: candidate %d has no model", i);
        if (levels[i].exit_layer < 1 || levels[i].exit_layer > m->desc.n_layers)
            HSD_FAIL(HSD_EINVAL, "calibrate: candidate %d exit layer %d outside 1..%d", i, levels[i].exit_layer, m->desc.n_layers);
        if (m->desc.vocab != levels[0].model->desc.vocab)
            HSD_FAIL(HSD_EINVAL, "calibrate: candidate %d has vocabulary %d, candidate 0 has %d (all models must share one)", i,
                     m->desc.vocab, levels[0].model->desc.vocab);
        if (m->stream != levels[0].model->stream) HSD_FAIL(HSD_EINVAL, "calibrate: candidate %d's model was created on another stream", i);
        if (n_tokens > m->desc.max_seq) HSD_FAIL(HSD_ECAPACITY, "calibrate: %d tokens exceed the KV capacity %d of candidate %d", n_tokens, m->desc.max_seq, i);
        L->chunk = std::min(L->chunk, m->desc.max_rows);
        // candidates of one network must come in ascending exit order (they are scored in one pass of that network)
        for (int k = 0; k < i; ++k)
            if (levels[k].model == m && levels[k].exit_layer >= levels[i].exit_layer)
                HSD_FAIL(HSD_EINVAL, "calibrate: candidates %d and %d are exits %d and %d of one network: list them in ascending order", k, i,
                         levels[k].exit_layer, levels[i].exit_layer);
    }
    L->vocab = levels[0].model->desc.vocab;
    L->npairs = n * (n - 1) / 2;
    L->n_scored = n_tokens - n_ctx;
    const size_t rows = (size_t)n * L->chunk * L->vocab * sizeof(float);
    size_t o = 0;
    L->logits = o;   o += align_up(rows, 256);
    L->probs = o;    o += align_up(rows, 256);
    L->overlaps = o; o += align_up((size_t)(L->npairs > 0 ? L->npairs : 1) * L->n_scored * sizeof(double), 256);
    L->softmax = o;  o += softmax_scratch_bytes(n * L->chunk, L->vocab);
    L->total = o;
    return HSD_OK;
}

}  // namespace

extern "C" size_t hsd_calibrate_levels_workspace_bytes(int n, const hsd_level* levels, int n_tokens, int n_ctx) {
    LevelsLayout L;
    return levels_layout(n, levels, n_tokens, n_ctx, &L) ? 0 : L.total;
}

extern "C" int hsd_calibrate_levels(int n, const hsd_level* levels, const int32_t* tokens_dev, int n_tokens, int n_ctx,
                                    float temperature, int cost_rows, void* workspace_dev, size_t workspace_bytes,
                                    double* alpha_out, double* cost_ms_out) {
    LevelsLayout L;
    if (int rc = levels_layout(n, levels, n_tokens, n_ctx, &L)) return rc;
    if (!tokens_dev || !workspace_dev || !alpha_out) HSD_FAIL(HSD_EINVAL, "hsd_calibrate_levels: null pointer");
    if ((uintptr_t)workspace_dev & 255) HSD_FAIL(HSD_EINVAL, "hsd_calibrate_levels: workspace must be 256-byte aligned");
    if (workspace_bytes < L.total) HSD_FAIL(HSD_ECAPACITY, "hsd_calibrate_levels: workspace of %zu bytes, %zu needed", workspace_bytes, L.total);
    if (!(temperature >= 0.f)) HSD_FAIL(HSD_EINVAL, "hsd_calibrate_levels: temperature %g", temperature);
    if (cost_ms_out && (cost_rows < 1 || cost_rows > L.chunk || cost_rows > n_tokens))
        HSD_FAIL(HSD_EINVAL, "hsd_calibrate_levels: cost_rows=%d outside 1..%d", cost_rows, L.chunk < n_tokens ? L.chunk : n_tokens);
    hipStream_t s = levels[0].model->stream;
    char* wb = (char*)workspace_dev;
    float* logits = (float*)(wb + L.logits);
    float* probs = (float*)(wb + L.probs);
    double* overlaps = (double*)(wb + L.overlaps);

    // networks in order of first appearance, each with the ascending exits listed for it; slot[k] = candidate whose
    // rows sit k-th in the device buffers
    struct Net { hsd_model* m; std::vector<int> exits; std::vector<int> cand; };
    std::vector<Net> nets;
    for (int i = 0; i < n; ++i) {
        size_t k = 0;
        while (k < nets.size() && nets[k].m != levels[i].model) ++k;
        if (k == nets.size()) nets.push_back(Net{levels[i].model, {}, {}});
        nets[k].exits.push_back(levels[i].exit_layer);
        nets[k].cand.push_back(i);
    }
    std::vector<int> slot;
    for (const Net& nt : nets) slot.insert(slot.end(), nt.cand.begin(), nt.cand.end());
    for (const Net& nt : nets)
        if (nt.exits.size() > 1 && nt.m->desc.dtype == HSD_BF16 && nt.m->desc.ffn < nt.m->desc.d)
            HSD_FAIL(HSD_ECAPACITY, "hsd_calibrate_levels: several exits of one bf16 network need ffn >= d");

    for (const Net& nt : nets) {                         // context-only positions: every network through its deepest listed exit
        const int deepest = nt.exits.back();
        for (int pos = 0; pos < n_ctx;) {
            const int c = std::min(nt.m->desc.max_rows, n_ctx - pos);
            if (int rc = model_pass(nt.m, tokens_dev + pos, pos, c, deepest, 0, nullptr)) return rc;
            pos += c;
        }
    }
    for (int pos = n_ctx; pos < n_tokens;) {
        const int c = std::min(L.chunk, n_tokens - pos);
        size_t row0 = 0;
        for (const Net& nt : nets) {
            if (int rc = model_pass_exits(nt.m, tokens_dev + pos, pos, c, nt.exits.data(), (int)nt.exits.size(), c,
                                          logits + row0 * L.vocab))
                return rc;
            row0 += nt.exits.size() * c;
        }
        if (int rc = launch_softmax(logits, probs, n * c, L.vocab, temperature, (float*)(wb + L.softmax), s)) return rc;
        if (int rc = launch_overlap(probs, n, c, L.vocab, overlaps + (pos - n_ctx), (size_t)L.n_scored, s)) return rc;
        pos += c;
    }
    std::vector<double> host((size_t)L.npairs * L.n_scored);
    if (L.npairs > 0) HSD_HIP(hipMemcpyAsync(host.data(), overlaps, host.size() * sizeof(double), hipMemcpyDeviceToHost, s));
    HSD_HIP(hipStreamSynchronize(s));
    int pair = 0;
    for (int a = 0; a < n; ++a) {
        alpha_out[slot[a] * n + slot[a]] = 1.0;
        for (int b = a + 1; b < n; ++b, ++pair) {
            double sum = 0.0;
            for (int t = 0; t < L.n_scored; ++t) sum += host[(size_t)pair * L.n_scored + t];
            alpha_out[slot[a] * n + slot[b]] = alpha_out[slot[b] * n + slot[a]] = sum / L.n_scored;
        }
    }
    if (!cost_ms_out) return HSD_OK;

    hipEvent_t e0, e1;
    HSD_HIP(hipEventCreate(&e0));
    HSD_HIP(hipEventCreate(&e1));
    const int pos0 = n_tokens - cost_rows;
    int rc = HSD_OK;
    for (int i = 0; i < n && !rc; ++i) {
        hsd_model* m = levels[i].model;
        // enough repetitions for a stable mean: about 20 ms of passes, between 3 and 10
        rc = model_pass(m, tokens_dev + pos0, pos0, cost_rows, levels[i].exit_layer, cost_rows, logits);      // warm-up
        if (!rc && hipEventRecord(e0, s) != hipSuccess) rc = HSD_EHIP;
        const int iters = levels[i].exit_layer * (long long)m->desc.d * m->desc.ffn > (1ll << 32) ? 3 : 10;
        for (int k = 0; k < iters && !rc; ++k) rc = model_pass(m, tokens_dev + pos0, pos0, cost_rows, levels[i].exit_layer, cost_rows, logits);
        float ms = 0.f;
        if (!rc && (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                    hipEventElapsedTime(&ms, e0, e1) != hipSuccess)) {
            hsd_set_error("hsd_calibrate_levels: event timing failed");
            rc = HSD_EHIP;
        }
        cost_ms_out[i] = (double)ms / iters;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return rc;
}
