// HSD over a batch of sequences in lockstep (the paper decodes one sequence; Sec. 3.1's argument, that a load of
// the weights should serve as many tokens as possible, applies across sequences as well).  Every sequence runs
// Alg. 1 / Alg. 2 exactly as the single-sequence driver does, with its own sampling seed, Philox call counters,
// token buffer and cached lengths; what is shared is each forward pass: one pass of a level feeds the pending
// tokens of every sequence that is at that point of the recursion.  Sequences that need fewer rows than the widest
// one, or that sit out an iteration (an intermediate level that has already gathered its T tokens, a sequence that
// has finished), are padded with rows after their last token: causal attention keeps padding from touching real
// rows, its K/V lands beyond the sequence's valid length, and its logits are never read.
#include <algorithm>
#include <cstring>
#include <vector>

#include "model.h"

namespace {

struct BLevel {
    hsd_model* model;
    int exit_layer;
    int rows_cap;                 // distribution rows one HSD(level, .) call can produce, per sequence
    float* rows;                  // [B][rows_cap][V]
    std::vector<int> cached;      // per sequence: tokens whose K/V this level's layers hold
    std::vector<int> count;       // per sequence: tokens gathered by the current HSD(level, .) call
    std::vector<uint32_t> call;   // per sequence: Philox call index of the level
};

int most_tokens(const int* T, int level) {          // most tokens HSD(level, .) can return, level < K
    int b = T[0];
    for (int i = 1; i <= level; ++i) b += T[i];
    return b;
}

int rows_cap_of(int n_levels, const int* T, int level) {
    const int K = n_levels - 1;
    if (K == 0) return 1;
    if (level == 0) return T[0];
    if (level < K) return most_tokens(T, level);
    return most_tokens(T, K - 1) + 1;
}

struct BatchLayout {
    size_t tok, feed, logits, rows[HSD_MAX_LEVELS], result, sampler, calls, softmax, total;
    int V, pages_per_seq, pass_rows;
};

constexpr int MAILBOX_INTS = 68;      // per sequence: n, new token, up to 65 surviving tokens, sequence number

struct Starts {
    int v[HSD_MAX_PASS_ROWS];
};

// feed[b * m + i] = token start[b] + i of sequence b
__global__ void gather_tokens_kernel(const int32_t* __restrict__ tok, int max_len, Starts start, int batch, int m,
                                     int32_t* __restrict__ feed) {
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= batch * m) return;
    const int b = r / m, i = r % m;
    feed[r] = tok[(size_t)b * max_len + start.v[b] + i];
}

}  // namespace

struct hsd_batch {
    int B, K, V, max_len;
    BLevel lv[HSD_MAX_LEVELS];
    int T[HSD_MAX_LEVELS];
    float temperature;
    std::vector<uint64_t> seed;
    hipStream_t stream;
    int32_t* tok_dev;             // [B][max_len]
    int32_t* feed_dev;            // [rows of a pass]
    float* logits;                // [rows of a pass][V]
    int pass_rows;                // rows a pass may have: the smallest max_rows among the models
    int32_t* result_dev;          // [B][2]
    void* sampler_scratch;
    void* calls_scratch;          // [B] ticket / key pairs of the batched fused sampler
    float* softmax_scratch;
    int32_t* mailbox;             // pinned, [B][MAILBOX_INTS]
    int32_t* mailbox_dev;
    std::vector<std::vector<int32_t>> tok_host;
    std::vector<int> len;
    bool skip_target_rows;
    hsd_stats stats;
};

namespace {

int batch_layout(int n_levels, const hsd_level* levels, const int* T, int batch, int max_len, BatchLayout* L) {
    if (n_levels < 1 || n_levels > HSD_MAX_LEVELS) HSD_FAIL(HSD_EINVAL, "batch: %d levels outside 1..%d", n_levels, HSD_MAX_LEVELS);
    if (!levels || (n_levels > 1 && !T)) HSD_FAIL(HSD_EINVAL, "batch: null pointer");
    if (batch < 1 || batch > HSD_MAX_PASS_ROWS) HSD_FAIL(HSD_ECAPACITY, "batch: %d sequences outside 1..%d", batch, (int)HSD_MAX_PASS_ROWS);
    if (max_len < HSD_KV_PAGE || max_len % HSD_KV_PAGE != 0)
        HSD_FAIL(HSD_EINVAL, "batch: %d positions per sequence, must be a positive multiple of %d", max_len, (int)HSD_KV_PAGE);
    L->pass_rows = HSD_MAX_PASS_ROWS;
    for (int i = 0; i < n_levels; ++i) {
        if (!levels[i].model) HSD_FAIL(HSD_EINVAL, "batch: level %d has no model", i);
        const hsd_model_desc& d = levels[i].model->desc;
        if (levels[i].exit_layer < 1 || levels[i].exit_layer > d.n_layers)
            HSD_FAIL(HSD_EINVAL, "batch: level %d exit layer %d outside 1..%d", i, levels[i].exit_layer, d.n_layers);
        if (d.vocab != levels[0].model->desc.vocab) HSD_FAIL(HSD_EINVAL, "batch: level %d has another vocabulary", i);
        if ((long long)batch * max_len > d.max_seq)
            HSD_FAIL(HSD_ECAPACITY, "batch: %d sequences x %d positions exceed the %d KV positions of level %d's model", batch, max_len,
                     d.max_seq, i);
        L->pass_rows = std::min(L->pass_rows, d.max_rows);
    }
    for (int i = 0; i + 1 < n_levels; ++i)
        if (T[i] < 1) HSD_FAIL(HSD_EINVAL, "batch: T_%d = %d, must be >= 1", i, T[i]);
    // the widest pass: a Verify of the most drafts the level below can hand up, plus two pending tokens
    for (int i = 1; i < n_levels; ++i) {
        const int t = most_tokens(T, i - 1);
        if (t > 64 || (long long)batch * (t + 2) > L->pass_rows)
            HSD_FAIL(HSD_ECAPACITY, "batch: level %d may verify %d drafts per sequence; %d sequences x %d rows exceed the %d rows of a pass", i, t,
                     batch, t + 2, L->pass_rows);
    }
    if (batch * 2 > L->pass_rows) HSD_FAIL(HSD_ECAPACITY, "batch: %d sequences x 2 rows exceed the %d rows of a pass", batch, L->pass_rows);
    L->V = levels[0].model->desc.vocab;
    L->pages_per_seq = max_len / HSD_KV_PAGE;
    size_t o = 0;
    L->tok = o;    o += align_up((size_t)batch * max_len * 4, 256);
    L->feed = o;   o += align_up((size_t)L->pass_rows * 4, 256);
    L->logits = o; o += align_up((size_t)L->pass_rows * L->V * 4, 256);
    for (int i = 0; i < n_levels; ++i) {
        L->rows[i] = o;
        o += align_up((size_t)batch * rows_cap_of(n_levels, T, i) * L->V * 4, 256);
    }
    L->result = o;  o += align_up((size_t)batch * 2 * 4, 256);
    L->sampler = o; o += hsd_sampler_scratch_bytes(L->V);
    L->calls = o;   o += align_up((size_t)batch * 16, 256);
    L->softmax = o; o += softmax_scratch_bytes(L->pass_rows, L->V);
    L->total = o;
    return HSD_OK;
}

// What level idx may treat as cached for sequence b: its own count, or that of a deeper exit of the same network.
int effective_cached(const hsd_batch* h, int idx, int b) {
    int c = h->lv[idx].cached[b];
    for (int k = 0; k <= h->K; ++k)
        if (h->lv[k].model == h->lv[idx].model && h->lv[k].exit_layer >= h->lv[idx].exit_layer) c = std::max(c, h->lv[k].cached[b]);
    return c;
}

// One pass of level idx: sequence b feeds tokens [start[b], start[b] + m) (real ones up to its length, padding
// after); logits of all rows when asked.
int batch_pass(hsd_batch* h, int idx, const int* start, int m, bool with_logits, int real_rows) {
    BLevel& L = h->lv[idx];
    if ((long long)h->B * m > h->pass_rows) HSD_FAIL(HSD_ECAPACITY, "batch pass: %d sequences x %d rows exceed the %d rows of a pass", h->B, m, h->pass_rows);
    Starts st;
    for (int b = 0; b < h->B; ++b) {
        if (start[b] < 0 || start[b] + m > h->max_len)
            HSD_FAIL(HSD_ECAPACITY, "batch pass: sequence %d at positions %d..%d exceeds its %d positions", b, start[b], start[b] + m - 1, h->max_len);
        st.v[b] = start[b];
    }
    gather_tokens_kernel<<<1, HSD_MAX_PASS_ROWS, 0, h->stream>>>(h->tok_dev, h->max_len, st, h->B, m, h->feed_dev);
    HSD_LAUNCH_CHECK();
    if (int rc = hsd_model_pass_batch(L.model, h->feed_dev, start, m, L.exit_layer, with_logits ? 1 : 0, h->logits)) return rc;
    h->stats.passes[idx]++;
    h->stats.pass_rows[idx] += real_rows;
    return HSD_OK;
}

bool any(const std::vector<char>& a) {
    for (char c : a)
        if (c) return true;
    return false;
}

// Where a sequence that sits a pass out puts its padding: right after its tokens.
int idle_start(const hsd_batch* h, int b, int m) { return std::min(h->len[b], h->max_len - m); }

// One autoregressive step of level 0 for every active sequence (Alg. 1, base case): distribution row `row`,
// token appended on the device.
int draft_step(hsd_batch* h, int row, const std::vector<char>& active) {
    BLevel& L = h->lv[0];
    if (row >= L.rows_cap) HSD_FAIL(HSD_ECAPACITY, "batch draft: row %d beyond the level's %d rows", row, L.rows_cap);
    int start[HSD_MAX_PASS_ROWS], rows_of[HSD_MAX_PASS_ROWS], m = 1, real = 0;
    for (int b = 0; b < h->B; ++b) {
        rows_of[b] = 0;
        if (!active[b]) continue;
        if (h->len[b] + 1 > h->max_len) HSD_FAIL(HSD_ECAPACITY, "batch draft: sequence %d is full (%d positions)", b, h->max_len);
        start[b] = std::min(effective_cached(h, 0, b), h->len[b] - 1);
        rows_of[b] = h->len[b] - start[b];
        m = std::max(m, rows_of[b]);
        real += rows_of[b];
    }
    for (int b = 0; b < h->B; ++b)
        if (!active[b]) start[b] = idle_start(h, b, m);
    if (int rc = batch_pass(h, 0, start, m, true, real)) return rc;
    const bool fused = softmax_verify_supported(h->V);
    VerifyCall calls[HSD_MAX_PASS_ROWS];
    int n_calls = 0;
    for (int b = 0; b < h->B; ++b) {
        if (!active[b]) continue;
        const float* z = h->logits + ((size_t)b * m + rows_of[b] - 1) * h->V;
        float* p = L.rows + ((size_t)b * L.rows_cap + row) * h->V;
        int32_t* x = h->tok_dev + (size_t)b * h->max_len + h->len[b];
        if (fused) {
            calls[n_calls++] = VerifyCall{z, nullptr, x, p, h->result_dev + 2 * b, nullptr, h->seed[b], L.call[b]++, 0};
        } else {
            if (int rc = launch_softmax(z, p, 1, h->V, h->temperature, h->softmax_scratch, h->stream)) return rc;
            if (int rc = launch_accept_resample(p, nullptr, x, 0, h->V, h->seed[b], 0u, L.call[b]++, h->result_dev + 2 * b, h->sampler_scratch,
                                                -1.f, h->stream))
                return rc;
        }
        L.cached[b] = h->len[b];
        h->len[b] += 1;
    }
    if (n_calls)
        if (int rc = launch_softmax_verify_batch(calls, n_calls, h->V, h->temperature, 0u, h->calls_scratch, h->stream)) return rc;
    return HSD_OK;
}

// Verify (Alg. 2) at level idx for every active sequence: the last t_b tokens of sequence b are the drafts the level
// below has just produced (t_b = its count), with that level's rows as q.
int verify_step(hsd_batch* h, int idx, const std::vector<char>& active) {
    BLevel& L = h->lv[idx];
    const BLevel& D = h->lv[idx - 1];
    int start[HSD_MAX_PASS_ROWS], rows_of[HSD_MAX_PASS_ROWS], t_of[HSD_MAX_PASS_ROWS], m = 1, real = 0;
    for (int b = 0; b < h->B; ++b) {
        rows_of[b] = t_of[b] = 0;
        if (!active[b]) continue;
        const int t = D.count[b];
        if (t < 1 || h->len[b] - t < 1) HSD_FAIL(HSD_ESTATE, "batch verify: sequence %d has %d drafts in %d tokens", b, t, h->len[b]);
        if (L.count[b] + t + 1 > L.rows_cap) HSD_FAIL(HSD_ECAPACITY, "batch verify: level %d holds %d rows, %d more do not fit its %d", idx, L.count[b], t + 1, L.rows_cap);
        if (h->len[b] + 1 > h->max_len) HSD_FAIL(HSD_ECAPACITY, "batch verify: sequence %d is full (%d positions)", b, h->max_len);
        const int ctx_end = h->len[b] - t;
        start[b] = std::min(effective_cached(h, idx, b), ctx_end - 1);
        rows_of[b] = h->len[b] - start[b];
        t_of[b] = t;
        m = std::max(m, rows_of[b]);
        real += rows_of[b];
    }
    for (int b = 0; b < h->B; ++b)
        if (!active[b]) start[b] = idle_start(h, b, m);
    if (int rc = batch_pass(h, idx, start, m, true, real)) return rc;
    const bool fused = softmax_verify_supported(h->V);
    VerifyCall calls[HSD_MAX_PASS_ROWS];
    int n_calls = 0;
    for (int b = 0; b < h->B; ++b) {
        if (!active[b]) continue;
        const int t = t_of[b], ctx_end = h->len[b] - t;
        const float* z = h->logits + ((size_t)b * m + rows_of[b] - t - 1) * h->V;
        const float* q = D.rows + (size_t)b * D.rows_cap * h->V;
        float* p = L.rows + ((size_t)b * L.rows_cap + L.count[b]) * h->V;
        int32_t* x = h->tok_dev + (size_t)b * h->max_len + ctx_end;
        int32_t* box = h->mailbox_dev + (size_t)b * MAILBOX_INTS;
        if (fused) {
            // nobody verifies the target's tokens: inside hsd_batch_generate its rows need not be stored
            float* p_store = h->skip_target_rows && idx == h->K ? nullptr : p;
            calls[n_calls++] = VerifyCall{z, q, x, p_store, h->result_dev + 2 * b, box, h->seed[b], L.call[b]++, t};
        } else {
            if (int rc = launch_softmax(z, p, t + 1, h->V, h->temperature, h->softmax_scratch, h->stream)) return rc;
            if (int rc = launch_accept_resample(p, q, x, t, h->V, h->seed[b], (uint32_t)idx, L.call[b]++, h->result_dev + 2 * b,
                                                h->sampler_scratch, -1.f, h->stream))
                return rc;
            HSD_HIP(hipMemcpyAsync(h->mailbox + (size_t)b * MAILBOX_INTS, h->result_dev + 2 * b, 8, hipMemcpyDeviceToHost, h->stream));
            HSD_HIP(hipMemcpyAsync(h->mailbox + (size_t)b * MAILBOX_INTS + 2, x, (size_t)(t + 1) * 4, hipMemcpyDeviceToHost, h->stream));
        }
    }
    if (n_calls)
        if (int rc = launch_softmax_verify_batch(calls, n_calls, h->V, h->temperature, (uint32_t)idx, h->calls_scratch, h->stream)) return rc;
    HSD_HIP(hipStreamSynchronize(h->stream));           // one round trip per Verify of the whole batch
    for (int b = 0; b < h->B; ++b) {
        if (!active[b]) continue;
        const int t = t_of[b], ctx_end = h->len[b] - t;
        const int32_t* box = h->mailbox + (size_t)b * MAILBOX_INTS;
        const int n = box[0];
        if (n < 0 || n > t) HSD_FAIL(HSD_EHIP, "batch verify: device returned n=%d for t=%d (sequence %d)", n, t, b);
        for (int i = 0; i <= n; ++i) h->tok_host[b][ctx_end + i] = box[2 + i];
        h->len[b] = ctx_end + n + 1;
        const int valid = ctx_end + n;                  // accepted prefix: K/V beyond it belongs to rejected drafts
        L.cached[b] = valid;
        for (int j = 0; j < idx; ++j) {
            BLevel& J = h->lv[j];
            if (J.model == L.model && J.exit_layer <= L.exit_layer) J.cached[b] = valid;
            else J.cached[b] = std::min(J.cached[b], valid);
        }
        L.count[b] += n + 1;
        h->stats.drafted[idx] += t;
        h->stats.accepted[idx] += n;
        h->stats.tested[idx] += n + (n < t ? 1 : 0);
    }
    return HSD_OK;
}

// HSD(idx, context) of Alg. 1 for every active sequence, in lockstep: an intermediate level repeats
// (level below, Verify) while any of its sequences is still short of T_idx tokens; those that have them sit out.
int run_level(hsd_batch* h, int idx, const std::vector<char>& active) {
    BLevel& L = h->lv[idx];
    for (int b = 0; b < h->B; ++b)
        if (active[b]) L.count[b] = 0;
    if (idx == 0) {
        const int k = h->K == 0 ? 1 : h->T[0];
        for (int c = 0; c < k; ++c)
            if (int rc = draft_step(h, c, active)) return rc;
        for (int b = 0; b < h->B; ++b)
            if (active[b]) L.count[b] = k;
        return HSD_OK;
    }
    std::vector<char> cur = active;
    while (any(cur)) {
        if (int rc = run_level(h, idx - 1, cur)) return rc;
        if (int rc = verify_step(h, idx, cur)) return rc;
        if (idx == h->K) break;
        for (int b = 0; b < h->B; ++b)
            if (cur[b] && L.count[b] >= h->T[idx]) cur[b] = 0;
    }
    return HSD_OK;
}

// Brings tok_host up to date for positions [from[b], len[b]) (tokens level 0 wrote on the device).
int fetch_tokens(hsd_batch* h, const std::vector<int>& from) {
    for (int b = 0; b < h->B; ++b) {
        const int n = h->len[b] - from[b];
        if (n > 0)
            HSD_HIP(hipMemcpyAsync(h->tok_host[b].data() + from[b], h->tok_dev + (size_t)b * h->max_len + from[b], (size_t)n * 4,
                                   hipMemcpyDeviceToHost, h->stream));
    }
    HSD_HIP(hipStreamSynchronize(h->stream));
    return HSD_OK;
}

}  // namespace

extern "C" size_t hsd_batch_workspace_bytes(int n_levels, const hsd_level* levels, const int* T, int batch, int max_len) {
    BatchLayout L;
    return batch_layout(n_levels, levels, T, batch, max_len, &L) ? 0 : L.total;
}

extern "C" int hsd_batch_create(int n_levels, const hsd_level* levels, const int* T, int batch, int max_len, float temperature,
                                const uint64_t* seeds, void* workspace_dev, size_t workspace_bytes, void* stream, hsd_batch** out) {
    BatchLayout L;
    if (int rc = batch_layout(n_levels, levels, T, batch, max_len, &L)) return rc;
    if (!workspace_dev || !seeds || !out) HSD_FAIL(HSD_EINVAL, "hsd_batch_create: null pointer");
    if ((uintptr_t)workspace_dev & 255) HSD_FAIL(HSD_EINVAL, "hsd_batch_create: workspace must be 256-byte aligned");
    if (workspace_bytes < L.total) HSD_FAIL(HSD_ECAPACITY, "hsd_batch_create: workspace of %zu bytes, %zu needed", workspace_bytes, L.total);
    if (!(temperature >= 0.f)) HSD_FAIL(HSD_EINVAL, "hsd_batch_create: temperature %g", temperature);
    for (int i = 0; i < n_levels; ++i)
        if (levels[i].model->stream != (hipStream_t)stream) HSD_FAIL(HSD_EINVAL, "hsd_batch_create: level %d's model was created on another stream", i);
    // every network's KV pages are shared out among the sequences: sequence b owns pages [b * pages, (b + 1) * pages)
    std::vector<int32_t> table((size_t)batch * L.pages_per_seq);
    for (size_t i = 0; i < table.size(); ++i) table[i] = (int32_t)i;
    for (int i = 0; i < n_levels; ++i) {
        bool first = true;
        for (int k = 0; k < i; ++k) first = first && levels[k].model != levels[i].model;
        if (first)
            if (int rc = hsd_model_set_batch(levels[i].model, batch, L.pages_per_seq, table.data())) return rc;
    }
    hsd_batch* h = new hsd_batch();
    h->B = batch;
    h->K = n_levels - 1;
    h->V = L.V;
    h->max_len = max_len;
    h->temperature = temperature;
    h->seed.assign(seeds, seeds + batch);
    h->stream = (hipStream_t)stream;
    char* wb = (char*)workspace_dev;
    h->tok_dev = (int32_t*)(wb + L.tok);
    h->feed_dev = (int32_t*)(wb + L.feed);
    h->logits = (float*)(wb + L.logits);
    h->pass_rows = L.pass_rows;
    h->result_dev = (int32_t*)(wb + L.result);
    h->sampler_scratch = wb + L.sampler;
    h->calls_scratch = wb + L.calls;
    h->softmax_scratch = (float*)(wb + L.softmax);
    for (int i = 0; i < n_levels; ++i) {
        BLevel& B = h->lv[i];
        B.model = levels[i].model;
        B.exit_layer = levels[i].exit_layer;
        B.rows_cap = rows_cap_of(n_levels, T, i);
        B.rows = (float*)(wb + L.rows[i]);
        B.cached.assign(batch, 0);
        B.count.assign(batch, 0);
        B.call.assign(batch, 0u);
        if (i < h->K) h->T[i] = T[i];
    }
    h->tok_host.assign(batch, std::vector<int32_t>(max_len, 0));
    h->len.assign(batch, 0);
    h->skip_target_rows = false;
    memset(&h->stats, 0, sizeof(h->stats));
    h->mailbox = nullptr;
    h->mailbox_dev = nullptr;
    hipError_t e = hipHostMalloc((void**)&h->mailbox, (size_t)batch * MAILBOX_INTS * sizeof(int32_t), hipHostMallocMapped);
    if (e == hipSuccess) memset(h->mailbox, 0, (size_t)batch * MAILBOX_INTS * sizeof(int32_t));
    if (e == hipSuccess) e = hipHostGetDevicePointer((void**)&h->mailbox_dev, h->mailbox, 0);
    if (e == hipSuccess) e = hipMemsetAsync(h->sampler_scratch, 0, hsd_sampler_scratch_bytes(h->V), h->stream);
    if (e == hipSuccess) e = hipMemsetAsync(h->calls_scratch, 0, (size_t)batch * 16, h->stream);
    if (e == hipSuccess) e = hipMemsetAsync(h->tok_dev, 0, (size_t)batch * max_len * 4, h->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
    if (e != hipSuccess) {
        hsd_set_error("hsd_batch_create: %s", hipGetErrorString(e));
        if (h->mailbox) (void)hipHostFree(h->mailbox);
        delete h;
        return HSD_EHIP;
    }
    *out = h;
    return HSD_OK;
}

extern "C" void hsd_batch_destroy(hsd_batch* h) {
    if (!h) return;
    (void)hipStreamSynchronize(h->stream);
    if (h->mailbox) (void)hipHostFree(h->mailbox);
    delete h;
}

extern "C" int hsd_batch_prefill(hsd_batch* h, const int32_t* prompts, int stride, const int* lens) {
    if (!h || !prompts || !lens) HSD_FAIL(HSD_EINVAL, "hsd_batch_prefill: null pointer");
    int longest = 0;
    for (int b = 0; b < h->B; ++b) {
        if (lens[b] < 1 || lens[b] > stride || lens[b] >= h->max_len)
            HSD_FAIL(HSD_ECAPACITY, "hsd_batch_prefill: sequence %d has %d tokens (row stride %d, %d positions per sequence)", b, lens[b], stride, h->max_len);
        for (int i = 0; i < lens[b]; ++i) {
            const int32_t t = prompts[(size_t)b * stride + i];
            if (t < 0 || t >= h->V) HSD_FAIL(HSD_EINVAL, "hsd_batch_prefill: token %d of sequence %d outside the vocabulary of %d", t, b, h->V);
        }
        longest = std::max(longest, lens[b]);
    }
    const int m = h->pass_rows / h->B;                   // rows per sequence and pass
    if (longest - 1 > 0 && (longest - 1 + m - 1) / m * m > h->max_len)
        HSD_FAIL(HSD_ECAPACITY, "hsd_batch_prefill: prompts of up to %d tokens in passes of %d rows exceed %d positions per sequence", longest, m, h->max_len);
    HSD_HIP(hipStreamSynchronize(h->stream));
    for (int b = 0; b < h->B; ++b) {
        std::fill(h->tok_host[b].begin(), h->tok_host[b].end(), 0);
        std::copy(prompts + (size_t)b * stride, prompts + (size_t)b * stride + lens[b], h->tok_host[b].begin());
        HSD_HIP(hipMemcpyAsync(h->tok_dev + (size_t)b * h->max_len, h->tok_host[b].data(), (size_t)h->max_len * 4, hipMemcpyHostToDevice, h->stream));
    }
    HSD_HIP(hipStreamSynchronize(h->stream));
    memset(&h->stats, 0, sizeof(h->stats));
    // every network once, through its deepest exit in the hierarchy; all but the last token of each prompt
    for (int i = 0; i <= h->K; ++i) {
        bool deepest = true;
        for (int k = 0; k <= h->K; ++k)
            if (k != i && h->lv[k].model == h->lv[i].model &&
                (h->lv[k].exit_layer > h->lv[i].exit_layer || (h->lv[k].exit_layer == h->lv[i].exit_layer && k < i)))
                deepest = false;
        if (!deepest) continue;
        for (int pos = 0; pos < longest - 1; pos += m) {
            int start[HSD_MAX_PASS_ROWS], real = 0;
            for (int b = 0; b < h->B; ++b) {
                start[b] = pos;
                real += std::max(0, std::min(m, lens[b] - 1 - pos));
            }
            if (int rc = batch_pass(h, i, start, m, false, real)) return rc;
        }
    }
    HSD_HIP(hipStreamSynchronize(h->stream));
    memset(&h->stats, 0, sizeof(h->stats));
    for (int b = 0; b < h->B; ++b) {
        h->len[b] = lens[b];
        for (int i = 0; i <= h->K; ++i) {
            h->lv[i].cached[b] = lens[b] - 1;
            h->lv[i].count[b] = 0;
            h->lv[i].call[b] = 0;
        }
    }
    return HSD_OK;
}

extern "C" int hsd_batch_generate(hsd_batch* h, int n_tokens, int32_t* out, hsd_stats* stats) {
    if (!h || !out) HSD_FAIL(HSD_EINVAL, "hsd_batch_generate: null pointer");
    if (n_tokens < 0) HSD_FAIL(HSD_EINVAL, "hsd_batch_generate: n_tokens=%d", n_tokens);
    // room: the tokens asked for, what the last round may add beyond them, and the padding of the widest pass
    const int overshoot = h->K == 0 ? 1 : most_tokens(h->T, h->K - 1) + 1;
    const int widest = h->pass_rows / h->B;
    std::vector<int> base(h->len);
    for (int b = 0; b < h->B; ++b) {
        if (h->len[b] < 1) HSD_FAIL(HSD_ESTATE, "hsd_batch_generate: sequence %d is empty (call hsd_batch_prefill first)", b);
        if (h->len[b] + n_tokens + overshoot + widest > h->max_len)
            HSD_FAIL(HSD_ECAPACITY, "hsd_batch_generate: sequence %d: %d tokens + %d to generate (+ %d of slack) exceed %d positions", b, h->len[b],
                     n_tokens, overshoot + widest, h->max_len);
    }
    std::vector<char> active(h->B, 1);
    h->skip_target_rows = h->K > 0;
    for (;;) {
        int64_t before = 0, after = 0;
        for (int b = 0; b < h->B; ++b) {
            active[b] = h->len[b] - base[b] < n_tokens;
            before += h->len[b];
        }
        if (!any(active)) break;
        std::vector<int> from(h->len);
        const int rc = run_level(h, h->K, active);
        if (rc) {
            h->skip_target_rows = false;
            return rc;
        }
        if (h->K == 0)
            if (int rc2 = fetch_tokens(h, from)) return rc2;
        for (int b = 0; b < h->B; ++b) after += h->len[b];
        h->stats.rounds++;
        h->stats.tokens += after - before;
    }
    h->skip_target_rows = false;
    HSD_HIP(hipStreamSynchronize(h->stream));
    for (int b = 0; b < h->B; ++b)
        std::copy(h->tok_host[b].begin() + base[b], h->tok_host[b].begin() + base[b] + n_tokens, out + (size_t)b * n_tokens);
    if (stats) *stats = h->stats;
    return HSD_OK;
}

extern "C" int hsd_batch_sequence_length(const hsd_batch* h, int b) { return h && b >= 0 && b < h->B ? h->len[b] : -1; }
