// Host round driver: Alg. 1 (HSD recursion) and Alg. 2 (Verify) over device-resident state.
//
// One token buffer on the device holds the whole sequence (context, tokens collected by the
// intermediate levels, current drafts).  Draft steps and the verifier's pass + rejection kernel are
// enqueued without host round trips: the sampler writes each new token id straight into the buffer
// that the next pass embeds from.  The host only learns n (accepted count) and the corrected token
// once per Verify, which is the one round trip Alg. 1's control flow needs: the sampler kernel writes them into
// pinned host memory followed by a sequence number, and the host polls that number instead of waiting for the
// stream, so the next pass is queued while the kernel is still finishing.
//
// KV validity (the paper does not discuss caching): level i keeps cached_len_i = number of leading
// sequence tokens whose K/V for its layers is in the cache.  A pass of level i feeds every token
// from there on (pending context tokens + drafts).  A rejection at position r truncates the
// sequence to r, appends the corrected token and clamps cached_len of every level <= i to r, which
// is the caption of Fig. 1 read as a rule: a token belongs to a model's context only once a model
// above accepted it.  Levels that are exits of one network share its cache, so what a deeper exit
// has cached is cached for the shallower exits too.
#include <string.h>

#include <algorithm>
#include <chrono>
#include <vector>

#include "model.h"

struct LevelState {
    hsd_model* model;
    int exit_layer;
    int cached_len;
    float* rows;        // distribution rows of the tokens this level holds, [rows_cap, V]
    int rows_cap;
    int count;          // tokens collected by the current HSD(level, .) call
    uint32_t call;      // Philox call index: Verify calls (draft steps at level 0)
    int distill_src;    // >= 0: this level's logits are that level's logits plus noise (synthetic drafter), else -1
    float distill_std;
    // Hidden-state reuse: when the level above is a deeper exit of the same network, the residual rows after this level's
    // exit layer are kept by position (every pass of the network through that layer stores them), and the level above
    // resumes from them instead of recomputing the shallower layers.  Rows [hid_lo, hid_hi) match the current tokens.
    float* hidden;      // [max_seq, d] fp32, or null
    int hid_lo, hid_hi;
};

struct hsd_hier {
    int K;              // index of the target level
    LevelState lv[HSD_MAX_LEVELS];
    int T[HSD_MAX_LEVELS];
    float temperature;
    uint64_t seed;
    hipStream_t stream;
    int V, max_seq;
    int32_t* tok_dev;
    std::vector<int32_t> tok_host;
    int len;            // tokens currently in the sequence
    float* logits;
    int logit_rows_cap;
    int32_t* result_dev;
    void* sampler_scratch;
    float* softmax_scratch;
    int32_t* mailbox;   // pinned host memory: n, m, then up to 65 token ids
    int32_t* mailbox_dev;   // the same memory as the device addresses it
    int mailbox_seq;        // last sequence number handed to a sampler launch (the kernel stores it after its results)
    // The fused sampler leaves the token it emits embedded in level 0's model (EmbedNext): valid for a one-token pass
    // of that model at position pre_pos while the model's pass counter still reads pre_serial.
    hsd_model* pre_model;
    unsigned long long pre_serial;
    int pre_pos;
    float coin[HSD_MAX_LEVELS];   // >= 0: fixed acceptance probability at that level's Verify (ablation), < 0: Alg. 2
    bool exactly_T;               // intermediate levels hand up exactly T tokens (ablation)
    bool skip_target_rows;        // set while hsd_generate runs
    hsd_driver_tuning tuning;     // hsd_hier_set_tuning
    bool reuse_hidden;            // hsd_hier_set_reuse
    hsd_stats stats;
};

namespace {

int batch_max(const int* T, int level) {          // most tokens HSD(level, .) can return, level < K
    int b = T[0];
    for (int i = 1; i <= level; ++i) b += T[i];
    return b;
}

int rows_cap_of(int n_levels, const int* T, int level) {
    const int K = n_levels - 1;
    if (K == 0) return 1;
    if (level == 0) return T[0];
    if (level < K) return batch_max(T, level);
    return batch_max(T, K - 1) + 1;
}

struct HierLayout {
    size_t tok, logits, rows[HSD_MAX_LEVELS], hidden[HSD_MAX_LEVELS], result, sampler, softmax, total;
    int logit_rows, max_seq, V;
};

// The level above `i` is a deeper exit of the same network: level i keeps its hidden states for it.
bool keeps_hidden(int n_levels, const hsd_level* levels, int i) {
    return i + 1 < n_levels && levels[i + 1].model == levels[i].model && levels[i + 1].exit_layer > levels[i].exit_layer;
}

int hier_layout(int n_levels, const hsd_level* levels, const int* T, HierLayout* L) {
    if (n_levels < 1 || n_levels > HSD_MAX_LEVELS) HSD_FAIL(HSD_EINVAL, "hierarchy: %d levels outside 1..%d", n_levels, HSD_MAX_LEVELS);
    if (!levels || (n_levels > 1 && !T)) HSD_FAIL(HSD_EINVAL, "hierarchy: null pointer");
    for (int i = 0; i < n_levels; ++i) {
        if (!levels[i].model) HSD_FAIL(HSD_EINVAL, "hierarchy: level %d has no model", i);
        if (levels[i].exit_layer < 1 || levels[i].exit_layer > levels[i].model->desc.n_layers)
            HSD_FAIL(HSD_EINVAL, "hierarchy: level %d exit layer %d outside 1..%d", i, levels[i].exit_layer, levels[i].model->desc.n_layers);
        if (levels[i].model->desc.vocab != levels[0].model->desc.vocab)
            HSD_FAIL(HSD_EINVAL, "hierarchy: level %d has vocabulary %d, level 0 has %d (all models must share one)", i,
                     levels[i].model->desc.vocab, levels[0].model->desc.vocab);
    }
    for (int i = 0; i + 1 < n_levels; ++i)
        if (T[i] < 1) HSD_FAIL(HSD_EINVAL, "hierarchy: T_%d = %d, must be >= 1", i, T[i]);
    const int K = n_levels - 1;
    L->V = levels[0].model->desc.vocab;
    L->max_seq = levels[0].model->desc.max_seq;
    L->logit_rows = 1;
    for (int i = 0; i < n_levels; ++i) {
        L->max_seq = std::min(L->max_seq, levels[i].model->desc.max_seq);
        if (i > 0) {
            const int t = batch_max(T, i - 1);
            if (t + 1 > levels[i].model->desc.max_rows || t > 64)
                HSD_FAIL(HSD_ECAPACITY, "hierarchy: level %d may have to verify %d drafts in one pass; its model allows %d rows per pass", i, t,
                         levels[i].model->desc.max_rows);
            L->logit_rows = std::max(L->logit_rows, t + 1);
        }
    }
    (void)K;
    size_t o = 0;
    L->tok = o;    o += align_up((size_t)L->max_seq * 4, 256);
    L->logits = o; o += align_up((size_t)L->logit_rows * L->V * 4, 256);
    for (int i = 0; i < n_levels; ++i) {
        L->rows[i] = o;
        o += align_up((size_t)rows_cap_of(n_levels, T, i) * L->V * 4, 256);
    }
    for (int i = 0; i < n_levels; ++i) {
        L->hidden[i] = o;
        if (keeps_hidden(n_levels, levels, i)) o += align_up((size_t)L->max_seq * levels[i].model->desc.d * sizeof(float), 256);
    }
    L->result = o;  o += 256;
    L->sampler = o; o += hsd_sampler_scratch_bytes(L->V);
    L->softmax = o; o += softmax_scratch_bytes(L->logit_rows, L->V);
    L->total = o;
    return HSD_OK;
}

// What level idx may treat as cached: its own count, or that of a deeper exit of the same network.
int effective_cached(const hsd_hier* h, int idx) {
    int c = h->lv[idx].cached_len;
    for (int k = 0; k <= h->K; ++k)
        if (h->lv[k].model == h->lv[idx].model && h->lv[k].exit_layer >= h->lv[idx].exit_layer) c = std::max(c, h->lv[k].cached_len);
    return c;
}

// One pass of `model` over sequence tokens [pos, pos + rows) through `exit_layer` layers (from `from_layer`, resuming
// from kept hidden rows, if > 0).  Every level that keeps hidden states of this network at a layer the pass goes
// through gets the rows of this pass, and its interval of valid rows is extended.
int hier_pass(hsd_hier* h, hsd_model* model, int pos, int rows, int exit_layer, int n_logit_rows, float* logits, bool embedded,
              int from_layer = 0, const float* resume_rows = nullptr) {
    PassOpts o;
    o.from_layer = from_layer;
    o.resume_rows = resume_rows;
    int who[HSD_MAX_LEVELS];
    for (int j = 0; j < h->K && h->reuse_hidden; ++j) {
        LevelState& J = h->lv[j];
        if (!J.hidden || J.model != model || J.exit_layer <= from_layer || J.exit_layer > exit_layer) continue;
        bool dup = false;                                 // two levels may keep the same layer of one network: one copy each
        for (int t = 0; t < o.n_taps; ++t) dup = dup || o.tap_layer[t] == J.exit_layer;
        if (dup) continue;
        who[o.n_taps] = j;
        o.tap_layer[o.n_taps] = J.exit_layer;
        o.tap_rows[o.n_taps] = J.hidden + (size_t)pos * model->desc.d;
        ++o.n_taps;
    }
    const bool plain = o.n_taps == 0 && from_layer == 0;
    if (int rc = model_pass(model, h->tok_dev + pos, pos, rows, exit_layer, n_logit_rows, logits, embedded, plain ? nullptr : &o)) return rc;
    for (int t = 0; t < o.n_taps; ++t) {
        LevelState& J = h->lv[who[t]];
        if (J.hid_hi > J.hid_lo && pos >= J.hid_lo && pos <= J.hid_hi) J.hid_hi = std::max(J.hid_hi, pos + rows);
        else { J.hid_lo = pos; J.hid_hi = pos + rows; }
    }
    return HSD_OK;
}

// No kept hidden row beyond the first `valid` tokens matches the sequence any more.
void clamp_hidden(hsd_hier* h, int valid) {
    for (int j = 0; j <= h->K; ++j) {
        h->lv[j].hid_hi = std::min(h->lv[j].hid_hi, valid);
        if (h->lv[j].hid_hi <= h->lv[j].hid_lo) h->lv[j].hid_lo = h->lv[j].hid_hi = 0;
    }
}

// Feeds sequence tokens [start, len) through the level; logits of the last n_logit_rows.
int level_pass(hsd_hier* h, int idx, int start, int n_logit_rows) {
    LevelState& L = h->lv[idx];
    const int max_rows = L.model->desc.max_rows;
    int pos = start;
    while (h->len - pos > max_rows) {
        int chunk = std::min(max_rows, h->len - pos - n_logit_rows);      // keep the logit rows for the last chunk
        if (chunk < 1) HSD_FAIL(HSD_ECAPACITY, "pass: %d logit rows do not fit a pass of %d rows", n_logit_rows, max_rows);
        if (int rc = hier_pass(h, L.model, pos, chunk, L.exit_layer, 0, nullptr, false)) return rc;
        h->stats.passes[idx]++;
        h->stats.pass_rows[idx] += chunk;
        pos += chunk;
    }
    // Hidden-state reuse: the level below is a shallower exit of this network and has kept its residual rows for a
    // prefix [pos, r) of this pass: only the rows from r on go through the shallower layers (they are the tokens no
    // pass has seen yet: the newest draft, or the token a Verify has just emitted), then all rows resume above them.
    const LevelState* B = idx > 0 ? &h->lv[idx - 1] : nullptr;
    if (h->reuse_hidden && B && B->hidden && B->hid_lo <= pos && B->hid_hi > pos) {
        const int r = std::min(B->hid_hi, h->len);
        if (r < h->len) {
            const bool emb = h->pre_model == L.model && h->pre_serial == L.model->pass_serial && h->pre_pos == r && h->len - r == 1;
            if (int rc = hier_pass(h, L.model, r, h->len - r, B->exit_layer, 0, nullptr, emb)) return rc;
        }
        if (int rc = hier_pass(h, L.model, pos, h->len - pos, L.exit_layer, n_logit_rows, h->logits, false, B->exit_layer,
                               B->hidden + (size_t)pos * L.model->desc.d))
            return rc;
        h->stats.reused_rows[idx] += r - pos;
    } else {
        const bool embedded = h->pre_model == L.model && h->pre_serial == L.model->pass_serial && h->pre_pos == pos && h->len - pos == 1;
        if (int rc = hier_pass(h, L.model, pos, h->len - pos, L.exit_layer, n_logit_rows, h->logits, embedded)) return rc;
    }
    h->stats.passes[idx]++;
    h->stats.pass_rows[idx] += h->len - pos;
    if (L.distill_src < 0 || n_logit_rows == 0) return HSD_OK;
    // Synthetic drafter: the pass above is what the level costs; its distribution comes from the logits of the level its
    // chain of sources ends at (a real network), at the same contexts (a side pass that is not counted and does not move
    // that level's cached length; the K/V it writes are those of the current tokens), plus the noise of every synthetic
    // level of the chain from the top down to this one: a level whose source is synthetic too differs from it by its
    // own noise only.
    int chain[HSD_MAX_LEVELS], n_chain = 0, root = idx;
    while (h->lv[root].distill_src >= 0) {
        chain[n_chain++] = root;
        root = h->lv[root].distill_src;
    }
    const LevelState& S = h->lv[root];
    const int smax = S.model->desc.max_rows;
    int sp = std::max(0, std::min(effective_cached(h, root), h->len - n_logit_rows));
    while (h->len - sp > smax) {
        const int chunk = std::min(smax, h->len - sp - n_logit_rows);
        if (chunk < 1) HSD_FAIL(HSD_ECAPACITY, "pass: %d logit rows do not fit a pass of %d rows of the source level", n_logit_rows, smax);
        if (int rc = hier_pass(h, S.model, sp, chunk, S.exit_layer, 0, nullptr, false)) return rc;
        sp += chunk;
    }
    if (int rc = hier_pass(h, S.model, sp, h->len - sp, S.exit_layer, n_logit_rows, h->logits, false)) return rc;
    for (int c = n_chain - 1; c >= 0; --c)
        if (int rc = launch_add_noise(h->logits, n_logit_rows, h->V, h->seed, (uint32_t)chain[c], h->len - n_logit_rows,
                                      h->lv[chain[c]].distill_std, h->stream))
            return rc;
    return HSD_OK;
}

int check_room(const hsd_hier* h, int extra) {
    if (h->len + extra > h->max_seq) HSD_FAIL(HSD_ECAPACITY, "sequence of %d tokens + %d exceeds the KV capacity %d", h->len, extra, h->max_seq);
    return HSD_OK;
}

// One autoregressive step of level 0 (Alg. 1, base case): distribution row `row`, token appended on the device.
int draft_step(hsd_hier* h, int row) {
    LevelState& L = h->lv[0];
    if (h->len < 1) HSD_FAIL(HSD_ESTATE, "draft: empty sequence (call hsd_prefill first)");
    if (int rc = check_room(h, 1)) return rc;
    if (row >= L.rows_cap) HSD_FAIL(HSD_ECAPACITY, "draft: row %d beyond the level's %d rows", row, L.rows_cap);
    const int start = std::min(effective_cached(h, 0), h->len - 1);
    if (int rc = level_pass(h, 0, start, 1)) return rc;
    float* p = L.rows + (size_t)row * h->V;
    h->pre_model = nullptr;
    if (softmax_verify_supported(h->V, h->tuning.fused_sampler_max_v)) {
        const bool pre = h->tuning.preembed != 0;
        if (int rc = launch_softmax_verify(h->logits, nullptr, h->tok_dev + h->len, 0, h->V, h->temperature, h->seed, 0u, L.call++, p,
                                           h->result_dev, h->sampler_scratch, nullptr, pre ? embed_next_of(L.model) : EmbedNext{}, -1.f,
                                           0, h->stream))
            return rc;
        if (pre) {
            h->pre_model = L.model;
            h->pre_serial = L.model->pass_serial;
            h->pre_pos = h->len;
        }
    } else {
        if (int rc = launch_softmax(h->logits, p, 1, h->V, h->temperature, h->softmax_scratch, h->stream)) return rc;
        if (int rc = launch_accept_resample(p, nullptr, h->tok_dev + h->len, 0, h->V, h->seed, 0u, L.call++, h->result_dev,
                                            h->sampler_scratch, -1.f, h->stream))
            return rc;
    }
    L.cached_len = h->len;
    h->len += 1;
    return HSD_OK;
}

// Waits for the sampler kernel's sequence number in the pinned mailbox by polling it: the host learns n a few
// microseconds after the kernel wrote it, without the wake-up latency of a stream synchronisation, and queues the
// next pass while the kernel finishes.  Gives up after a while (returns false: the caller synchronises the stream).
bool wait_mailbox(hsd_hier* h) {
    if (!h->tuning.poll_mailbox) return false;
    volatile int32_t* slot = h->mailbox + MAILBOX_SEQ_SLOT;
    const auto t0 = std::chrono::steady_clock::now();
    for (unsigned spins = 0;; ++spins) {
        if (__atomic_load_n(slot, __ATOMIC_ACQUIRE) == h->mailbox_seq) return true;
        if ((spins & 1023) == 1023 && std::chrono::steady_clock::now() - t0 > std::chrono::milliseconds(200)) return false;
    }
}

// Verify (Alg. 2): the last t sequence tokens are drafts with rows q_dev.  Returns n+1 in *n_out.
int verify_step(hsd_hier* h, int idx, int t, const float* q_dev, int* n_out) {
    LevelState& L = h->lv[idx];
    if (t < 1) HSD_FAIL(HSD_EINVAL, "verify: t=%d", t);
    if (h->len - t < 1) HSD_FAIL(HSD_ESTATE, "verify: %d drafts but only %d tokens in the sequence", t, h->len);
    if (L.count + t + 1 > L.rows_cap) HSD_FAIL(HSD_ECAPACITY, "verify: level %d holds %d rows, %d more do not fit its %d", idx, L.count, t + 1, L.rows_cap);
    if (t + 1 > h->logit_rows_cap || t > 64) HSD_FAIL(HSD_ECAPACITY, "verify: %d drafts exceed the hierarchy's %d per pass", t, h->logit_rows_cap - 1);
    if (int rc = check_room(h, 1)) return rc;
    const int ctx_end = h->len - t;
    const int start = std::min(effective_cached(h, idx), ctx_end - 1);
    if (int rc = level_pass(h, idx, start, t + 1)) return rc;
    float* p = L.rows + (size_t)L.count * h->V;
    // Nobody verifies the target's tokens, so inside hsd_generate its rows p_1..p_{n+1} need not be stored (the
    // fused kernel keeps each row in registers); single calls (hsd_verify, hsd_run) always return them.
    float* p_store = h->skip_target_rows && idx == h->K && softmax_verify_supported(h->V, h->tuning.fused_sampler_max_v) ? nullptr : p;
    h->pre_model = nullptr;
    hsd_model* m0 = h->lv[0].model;
    bool pre = false, polled = false;
    if (softmax_verify_supported(h->V, h->tuning.fused_sampler_max_v)) {
        // one launch; the kernel writes n, m and the surviving tokens straight into the pinned mailbox, and leaves m
        // embedded in level 0's model, whose next draft pass is that one token
        pre = h->tuning.preembed != 0;
        if (int rc = launch_softmax_verify(h->logits, q_dev, h->tok_dev + ctx_end, t, h->V, h->temperature, h->seed, (uint32_t)idx,
                                           L.call++, p_store, h->result_dev, h->sampler_scratch, h->mailbox_dev,
                                           pre ? embed_next_of(m0) : EmbedNext{}, h->coin[idx], ++h->mailbox_seq, h->stream))
            return rc;
        polled = wait_mailbox(h);
    } else {
        if (int rc = launch_softmax(h->logits, p, t + 1, h->V, h->temperature, h->softmax_scratch, h->stream)) return rc;
        if (int rc = launch_accept_resample(p, q_dev, h->tok_dev + ctx_end, t, h->V, h->seed, (uint32_t)idx, L.call++, h->result_dev,
                                            h->sampler_scratch, h->coin[idx], h->stream))
            return rc;
        HSD_HIP(hipMemcpyAsync(h->mailbox, h->result_dev, 8, hipMemcpyDeviceToHost, h->stream));
        HSD_HIP(hipMemcpyAsync(h->mailbox + 2, h->tok_dev + ctx_end, (size_t)(t + 1) * 4, hipMemcpyDeviceToHost, h->stream));
    }
    if (!polled) HSD_HIP(hipStreamSynchronize(h->stream));
    const int n = h->mailbox[0];
    if (n < 0 || n > t) HSD_FAIL(HSD_EHIP, "verify: device returned n=%d for t=%d", n, t);
    for (int i = 0; i <= n; ++i) h->tok_host[ctx_end + i] = h->mailbox[2 + i];
    h->len = ctx_end + n + 1;
    if (pre) {
        h->pre_model = m0;
        h->pre_serial = m0->pass_serial;
        h->pre_pos = ctx_end + n;
    }
    const int valid = ctx_end + n;                 // accepted prefix: K/V beyond it belongs to rejected drafts
    L.cached_len = valid;
    for (int j = 0; j < idx; ++j) {
        LevelState& J = h->lv[j];
        if (J.model == L.model && J.exit_layer <= L.exit_layer) J.cached_len = valid;
        else J.cached_len = std::min(J.cached_len, valid);
    }
    clamp_hidden(h, valid);
    L.count += n + 1;
    h->stats.drafted[idx] += t;
    h->stats.accepted[idx] += n;
    h->stats.tested[idx] += n + (n < t ? 1 : 0);
    *n_out = n + 1;
    return HSD_OK;
}

// HSD(idx, context) of Alg. 1; returns the number of tokens appended in *count_out.
int run_level(hsd_hier* h, int idx, int* count_out) {
    LevelState& L = h->lv[idx];
    L.count = 0;
    if (idx == 0) {
        const int k = h->K == 0 ? 1 : h->T[0];
        for (int c = 0; c < k; ++c)
            if (int rc = draft_step(h, c)) return rc;
        L.count = k;
    } else if (idx == h->K) {
        int t = 0, n1 = 0;
        if (int rc = run_level(h, idx - 1, &t)) return rc;
        if (int rc = verify_step(h, idx, t, h->lv[idx - 1].rows, &n1)) return rc;
    } else {
        while (L.count < h->T[idx]) {
            int t = 0, n1 = 0;
            if (int rc = run_level(h, idx - 1, &t)) return rc;
            if (int rc = verify_step(h, idx, t, h->lv[idx - 1].rows, &n1)) return rc;
        }
        if (h->exactly_T && L.count > h->T[idx]) {
            // drop what was collected beyond T: the sequence ends earlier, and no level may count the dropped
            // positions as cached (their tokens are gone); the level's first T rows stay where they are
            h->len -= L.count - h->T[idx];
            L.count = h->T[idx];
            for (int j = 0; j <= h->K; ++j) h->lv[j].cached_len = std::min(h->lv[j].cached_len, h->len);
            clamp_hidden(h, h->len);
            h->pre_model = nullptr;
        }
    }
    *count_out = L.count;
    return HSD_OK;
}

// Brings tok_host up to date for positions [from, len) (tokens level 0 wrote on the device).
int fetch_tokens(hsd_hier* h, int from) {
    int pos = from;
    while (pos < h->len) {
        const int n = std::min(64, h->len - pos);
        HSD_HIP(hipMemcpyAsync(h->mailbox + 2, h->tok_dev + pos, (size_t)n * 4, hipMemcpyDeviceToHost, h->stream));
        HSD_HIP(hipStreamSynchronize(h->stream));
        for (int i = 0; i < n; ++i) h->tok_host[pos + i] = h->mailbox[2 + i];
        pos += n;
    }
    return HSD_OK;
}

void reset_counters(hsd_hier* h) {
    for (int i = 0; i <= h->K; ++i) {
        h->lv[i].call = 0;
        h->lv[i].count = 0;
    }
    memset(&h->stats, 0, sizeof(h->stats));
}

}  // namespace

extern "C" size_t hsd_hier_workspace_bytes(int n_levels, const hsd_level* levels, const int* T) {
    HierLayout L;
    return hier_layout(n_levels, levels, T, &L) ? 0 : L.total;
}

extern "C" int hsd_hier_create(int n_levels, const hsd_level* levels, const int* T, float temperature, uint64_t seed,
                               void* workspace_dev, size_t workspace_bytes, void* stream, hsd_hier** out) {
    HierLayout L;
    if (int rc = hier_layout(n_levels, levels, T, &L)) return rc;
    if (!workspace_dev || !out) HSD_FAIL(HSD_EINVAL, "hsd_hier_create: null pointer");
    if ((uintptr_t)workspace_dev & 255) HSD_FAIL(HSD_EINVAL, "hsd_hier_create: workspace must be 256-byte aligned");
    if (workspace_bytes < L.total) HSD_FAIL(HSD_ECAPACITY, "hsd_hier_create: workspace of %zu bytes, %zu needed", workspace_bytes, L.total);
    if (!(temperature >= 0.f)) HSD_FAIL(HSD_EINVAL, "hsd_hier_create: temperature %g", temperature);
    for (int i = 0; i < n_levels; ++i)
        if (levels[i].model->stream != (hipStream_t)stream) HSD_FAIL(HSD_EINVAL, "hsd_hier_create: level %d's model was created on another stream", i);
    hsd_hier* h = new hsd_hier();
    h->K = n_levels - 1;
    h->temperature = temperature;
    h->seed = seed;
    h->stream = (hipStream_t)stream;
    h->V = L.V;
    h->max_seq = L.max_seq;
    char* wb = (char*)workspace_dev;
    h->tok_dev = (int32_t*)(wb + L.tok);
    h->logits = (float*)(wb + L.logits);
    h->logit_rows_cap = L.logit_rows;
    h->result_dev = (int32_t*)(wb + L.result);
    h->sampler_scratch = wb + L.sampler;
    h->softmax_scratch = (float*)(wb + L.softmax);
    for (int i = 0; i < n_levels; ++i) {
        h->lv[i] = LevelState{levels[i].model, levels[i].exit_layer, 0, (float*)(wb + L.rows[i]), rows_cap_of(n_levels, T, i), 0, 0u, -1, 0.f,
                              keeps_hidden(n_levels, levels, i) ? (float*)(wb + L.hidden[i]) : nullptr, 0, 0};
        if (i < h->K) h->T[i] = T[i];
    }
    h->tok_host.assign(h->max_seq, 0);
    h->len = 0;
    h->mailbox = nullptr;
    h->mailbox_dev = nullptr;
    h->mailbox_seq = 0;
    h->pre_model = nullptr;
    h->exactly_T = false;
    h->skip_target_rows = false;
    h->tuning = default_driver_tuning();
    h->reuse_hidden = false;
    for (int i = 0; i < HSD_MAX_LEVELS; ++i) h->coin[i] = -1.f;
    reset_counters(h);
    hipError_t e = hipHostMalloc((void**)&h->mailbox, 68 * sizeof(int32_t), hipHostMallocMapped);
    if (e == hipSuccess) memset(h->mailbox, 0, 68 * sizeof(int32_t));
    if (e == hipSuccess) e = hipHostGetDevicePointer((void**)&h->mailbox_dev, h->mailbox, 0);
    if (e == hipSuccess) e = hipMemsetAsync(h->sampler_scratch, 0, hsd_sampler_scratch_bytes(h->V), h->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(h->stream);
    if (e != hipSuccess) {
        if (h->mailbox) (void)hipHostFree(h->mailbox);
        delete h;
        HSD_FAIL(HSD_EHIP, "hsd_hier_create: %s", hipGetErrorString(e));
    }
    *out = h;
    return HSD_OK;
}

extern "C" void hsd_hier_destroy(hsd_hier* h) {
    if (!h) return;
    if (h->mailbox) (void)hipHostFree(h->mailbox);
    delete h;
}

extern "C" int hsd_hier_set_distilled(hsd_hier* h, int level, int source_level, float noise_std) {
    if (!h) HSD_FAIL(HSD_EINVAL, "hsd_hier_set_distilled: null pointer");
    if (level < 0 || level >= h->K) HSD_FAIL(HSD_EINVAL, "hsd_hier_set_distilled: level %d outside 0..%d (the target is never synthetic)", level, h->K - 1);
    if (source_level < 0) {
        h->lv[level].distill_src = -1;
        return HSD_OK;
    }
    if (source_level <= level || source_level > h->K) HSD_FAIL(HSD_EINVAL, "hsd_hier_set_distilled: source level %d must lie in %d..%d", source_level, level + 1, h->K);
    if (!(noise_std >= 0.f)) HSD_FAIL(HSD_EINVAL, "hsd_hier_set_distilled: noise_std %g", noise_std);
    h->lv[level].distill_src = source_level;
    h->lv[level].distill_std = noise_std;
    return HSD_OK;
}

extern "C" int hsd_hier_set_tuning(hsd_hier* h, const hsd_driver_tuning* t) {
    if (!h) HSD_FAIL(HSD_EINVAL, "hsd_hier_set_tuning: null pointer");
    h->tuning = t ? *t : default_driver_tuning();
    h->pre_model = nullptr;
    return HSD_OK;
}

extern "C" int hsd_hier_set_reuse(hsd_hier* h, int on) {
    if (!h) HSD_FAIL(HSD_EINVAL, "hsd_hier_set_reuse: null pointer");
    h->reuse_hidden = on != 0;
    clamp_hidden(h, 0);             // rows are kept from the next pass on
    return HSD_OK;
}

extern "C" int hsd_hier_set_ablation(hsd_hier* h, const float* coin, int exactly_T) {
    if (!h) HSD_FAIL(HSD_EINVAL, "hsd_hier_set_ablation: null pointer");
    if (coin)
        for (int i = 1; i <= h->K; ++i)
            if (!(coin[i] <= 1.f)) HSD_FAIL(HSD_EINVAL, "hsd_hier_set_ablation: coin[%d] = %g above 1 (negative = real test)", i, coin[i]);
    for (int i = 0; i < HSD_MAX_LEVELS; ++i) h->coin[i] = coin && i >= 1 && i <= h->K ? coin[i] : -1.f;
    h->exactly_T = exactly_T != 0;
    return HSD_OK;
}

extern "C" double hsd_stats_cost(const hsd_stats* st, int n_levels, const double* cost) {
    if (!st || !cost || n_levels < 1 || n_levels > HSD_MAX_LEVELS) return -1.0;
    double c = 0.0;
    for (int i = 0; i < n_levels; ++i) c += (double)st->passes[i] * cost[i];
    return c;
}

static int prefill_from(hsd_hier* h, const int32_t* prompt, int n, int n_cached, const char* who) {
    if (!h || !prompt) HSD_FAIL(HSD_EINVAL, "%s: null pointer", who);
    if (n < 1 || n >= h->max_seq) HSD_FAIL(HSD_ECAPACITY, "%s: prompt of %d tokens, capacity %d", who, n, h->max_seq);
    if (n_cached < 0 || n_cached > n - 1) HSD_FAIL(HSD_EINVAL, "%s: %d cached tokens outside 0..%d", who, n_cached, n - 1);
    for (int i = 0; i < n; ++i)
        if (prompt[i] < 0 || prompt[i] >= h->V) HSD_FAIL(HSD_EINVAL, "%s: token %d at position %d outside the vocabulary of %d", who, prompt[i], i, h->V);
    std::copy(prompt, prompt + n, h->tok_host.begin());
    HSD_HIP(hipMemcpyAsync(h->tok_dev, h->tok_host.data(), (size_t)n * 4, hipMemcpyHostToDevice, h->stream));
    HSD_HIP(hipStreamSynchronize(h->stream));
    reset_counters(h);
    clamp_hidden(h, 0);
    // every network once, through its deepest exit in the hierarchy
    for (int i = 0; i <= h->K; ++i) {
        bool deepest = true;
        for (int k = 0; k <= h->K; ++k)
            if (k != i && h->lv[k].model == h->lv[i].model &&
                (h->lv[k].exit_layer > h->lv[i].exit_layer || (h->lv[k].exit_layer == h->lv[i].exit_layer && k < i)))
                deepest = false;
        if (!deepest || n < 2) continue;
        const int max_rows = h->lv[i].model->desc.max_rows;
        for (int pos = n_cached; pos < n - 1; pos += max_rows) {
            const int chunk = std::min(max_rows, n - 1 - pos);
            if (int rc = hier_pass(h, h->lv[i].model, pos, chunk, h->lv[i].exit_layer, 0, nullptr, false)) return rc;
        }
    }
    HSD_HIP(hipStreamSynchronize(h->stream));
    h->len = n;
    h->pre_model = nullptr;
    for (int i = 0; i <= h->K; ++i) h->lv[i].cached_len = n - 1;
    return HSD_OK;
}

extern "C" int hsd_prefill(hsd_hier* h, const int32_t* prompt, int n) { return prefill_from(h, prompt, n, 0, "hsd_prefill"); }

extern "C" int hsd_prefill_cached(hsd_hier* h, const int32_t* prompt, int n, int n_cached) {
    return prefill_from(h, prompt, n, n_cached, "hsd_prefill_cached");
}

extern "C" int hsd_hier_set_seed(hsd_hier* h, uint64_t seed) {
    if (!h) HSD_FAIL(HSD_EINVAL, "hsd_hier_set_seed: null pointer");
    h->seed = seed;
    return HSD_OK;
}

extern "C" int hsd_rewind(hsd_hier* h, int n) {
    if (!h) HSD_FAIL(HSD_EINVAL, "hsd_rewind: null pointer");
    if (n < 1 || n > h->len) HSD_FAIL(HSD_EINVAL, "hsd_rewind: %d outside 1..%d", n, h->len);
    HSD_HIP(hipStreamSynchronize(h->stream));
    HSD_HIP(hipMemcpyAsync(h->tok_dev, h->tok_host.data(), (size_t)n * 4, hipMemcpyHostToDevice, h->stream));
    HSD_HIP(hipStreamSynchronize(h->stream));
    h->len = n;
    h->pre_model = nullptr;
    for (int i = 0; i <= h->K; ++i) h->lv[i].cached_len = std::min(h->lv[i].cached_len, n - 1);
    clamp_hidden(h, n - 1);
    reset_counters(h);
    return HSD_OK;
}

extern "C" int hsd_draft(hsd_hier* h, int level, int k, int32_t* tokens_out, const float** probs_dev_out) {
    if (!h) HSD_FAIL(HSD_EINVAL, "hsd_draft: null pointer");
    if (level != 0) HSD_FAIL(HSD_EINVAL, "hsd_draft: level %d (only level 0 drafts autoregressively; higher levels produce tokens through hsd_run)", level);
    if (k < 1 || k > h->lv[0].rows_cap) HSD_FAIL(HSD_ECAPACITY, "hsd_draft: k=%d outside 1..%d (T_0)", k, h->lv[0].rows_cap);
    const int base = h->len;
    h->lv[0].count = 0;
    for (int c = 0; c < k; ++c)
        if (int rc = draft_step(h, c)) return rc;
    h->lv[0].count = k;
    if (int rc = fetch_tokens(h, base)) return rc;
    if (tokens_out) std::copy(h->tok_host.begin() + base, h->tok_host.begin() + base + k, tokens_out);
    if (probs_dev_out) *probs_dev_out = h->lv[0].rows;
    return HSD_OK;
}

extern "C" int hsd_verify(hsd_hier* h, int level, const int32_t* draft_tokens, const float* draft_probs_dev, int t, int append,
                          int32_t* tokens_out, int* n_out, const float** probs_dev_out) {
    if (!h || !draft_probs_dev || !n_out) HSD_FAIL(HSD_EINVAL, "hsd_verify: null pointer");
    if (level < 1 || level > h->K) HSD_FAIL(HSD_EINVAL, "hsd_verify: level %d outside 1..%d (level 0 only drafts)", level, h->K);
    if (t < 1) HSD_FAIL(HSD_EINVAL, "hsd_verify: t=%d", t);
    if (draft_tokens) {
        if (int rc = check_room(h, t + 1)) return rc;
        for (int i = 0; i < t; ++i)
            if (draft_tokens[i] < 0 || draft_tokens[i] >= h->V) HSD_FAIL(HSD_EINVAL, "hsd_verify: draft token %d outside the vocabulary of %d", draft_tokens[i], h->V);
        std::copy(draft_tokens, draft_tokens + t, h->tok_host.begin() + h->len);
        HSD_HIP(hipMemcpyAsync(h->tok_dev + h->len, h->tok_host.data() + h->len, (size_t)t * 4, hipMemcpyHostToDevice, h->stream));
        HSD_HIP(hipStreamSynchronize(h->stream));
        h->len += t;
    }
    LevelState& L = h->lv[level];
    if (!append) L.count = 0;
    const int row0 = L.count;
    const int ctx_end = h->len - t;
    int n1 = 0;
    if (int rc = verify_step(h, level, t, draft_probs_dev, &n1)) return rc;
    HSD_HIP(hipStreamSynchronize(h->stream));          // the driver itself only polls for n; a caller gets a finished stream
    if (tokens_out) std::copy(h->tok_host.begin() + ctx_end, h->tok_host.begin() + ctx_end + n1, tokens_out);
    *n_out = n1;
    if (probs_dev_out) *probs_dev_out = L.rows + (size_t)row0 * h->V;
    return HSD_OK;
}

extern "C" int hsd_run(hsd_hier* h, int level, int32_t* tokens_out, int cap, int* n_out, const float** probs_dev_out) {
    if (!h || !n_out) HSD_FAIL(HSD_EINVAL, "hsd_run: null pointer");
    if (level < 0 || level > h->K) HSD_FAIL(HSD_EINVAL, "hsd_run: level %d outside 0..%d", level, h->K);
    if (h->len < 1) HSD_FAIL(HSD_ESTATE, "hsd_run: empty sequence (call hsd_prefill first)");
    const int base = h->len;
    int count = 0;
    if (int rc = run_level(h, level, &count)) return rc;
    if (level == 0 || h->K == 0) {
        if (int rc = fetch_tokens(h, base)) return rc;
    } else {
        HSD_HIP(hipStreamSynchronize(h->stream));
    }
    if (level == h->K) {
        h->stats.rounds++;
        h->stats.tokens += count;
    }
    if (tokens_out) {
        if (cap < count) HSD_FAIL(HSD_ECAPACITY, "hsd_run: %d tokens produced, output holds %d", count, cap);
        std::copy(h->tok_host.begin() + base, h->tok_host.begin() + base + count, tokens_out);
    }
    *n_out = count;
    if (probs_dev_out) *probs_dev_out = h->lv[level].rows;
    return HSD_OK;
}

extern "C" int hsd_generate(hsd_hier* h, int n_tokens, int32_t* out, hsd_stats* stats) {
    if (!h || !out) HSD_FAIL(HSD_EINVAL, "hsd_generate: null pointer");
    if (n_tokens < 0) HSD_FAIL(HSD_EINVAL, "hsd_generate: n_tokens=%d", n_tokens);
    if (h->len < 1) HSD_FAIL(HSD_ESTATE, "hsd_generate: empty sequence (call hsd_prefill first)");
    const int base = h->len;
    h->skip_target_rows = h->K > 0;
    while (h->len - base < n_tokens) {
        const int before = h->len;
        int count = 0;
        const int rc0 = run_level(h, h->K, &count);
        if (rc0) {
            h->skip_target_rows = false;
            return rc0;
        }
        if (h->K == 0)
            if (int rc = fetch_tokens(h, before)) return rc;
        h->stats.rounds++;
        h->stats.tokens += count;
    }
    h->skip_target_rows = false;
    HSD_HIP(hipStreamSynchronize(h->stream));          // the rounds only polled for each Verify's result
    std::copy(h->tok_host.begin() + base, h->tok_host.begin() + base + n_tokens, out);
    if (stats) *stats = h->stats;
    return HSD_OK;
}

extern "C" int hsd_get_stats(const hsd_hier* h, hsd_stats* s) {
    if (!h || !s) HSD_FAIL(HSD_EINVAL, "hsd_get_stats: null pointer");
    *s = h->stats;
    return HSD_OK;
}

extern "C" int hsd_sequence_length(const hsd_hier* h) { return h ? h->len : HSD_EINVAL; }

extern "C" int hsd_measure_pass(hsd_hier* h, int level, int m, int iters, double* ms_out) {
    if (!h || !ms_out) HSD_FAIL(HSD_EINVAL, "hsd_measure_pass: null pointer");
    if (level < 0 || level > h->K) HSD_FAIL(HSD_EINVAL, "hsd_measure_pass: level %d outside 0..%d", level, h->K);
    LevelState& L = h->lv[level];
    if (m < 1 || m > L.model->desc.max_rows || m > h->len || m > h->logit_rows_cap)
        HSD_FAIL(HSD_EINVAL, "hsd_measure_pass: m=%d outside 1..min(%d, %d, %d)", m, L.model->desc.max_rows, h->len, h->logit_rows_cap);
    if (iters < 1) HSD_FAIL(HSD_EINVAL, "hsd_measure_pass: iters=%d", iters);
    hipEvent_t e0, e1;
    HSD_HIP(hipEventCreate(&e0));
    HSD_HIP(hipEventCreate(&e1));
    const int pos0 = h->len - m;
    int rc = model_pass(L.model, h->tok_dev + pos0, pos0, m, L.exit_layer, m, h->logits);       // warm-up
    if (!rc) rc = hipEventRecord(e0, h->stream) == hipSuccess ? HSD_OK : HSD_EHIP;
    for (int i = 0; i < iters && !rc; ++i) {
        rc = model_pass(L.model, h->tok_dev + pos0, pos0, m, L.exit_layer, m, h->logits);
    }
    float ms = 0.f;
    if (!rc && (hipEventRecord(e1, h->stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                hipEventElapsedTime(&ms, e0, e1) != hipSuccess)) {
        hsd_set_error("hsd_measure_pass: event timing failed");
        rc = HSD_EHIP;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc) return rc;
    *ms_out = (double)ms / iters;
    return HSD_OK;
}
