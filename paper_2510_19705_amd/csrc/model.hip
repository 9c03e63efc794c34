// hsd_model: weight packing, KV geometry and the assembly of one multi-token decoder pass
// (the verifier's parallel scoring of all prefixes in Alg. 2; with one row, a draft step of Alg. 1).
#include <string.h>

#include <algorithm>

#include "model.h"

static thread_local char g_err[512] = "";

void hsd_set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

extern "C" const char* hsd_last_error(void) { return g_err; }

static int check_desc(const hsd_model_desc* d) {
    if (!d) HSD_FAIL(HSD_EINVAL, "model: null descriptor");
    if (d->dtype != HSD_F32 && d->dtype != HSD_BF16) HSD_FAIL(HSD_EINVAL, "model: dtype %d", d->dtype);
    if (d->n_layers < 1 || d->d < 32 || d->d % 32 != 0) HSD_FAIL(HSD_EINVAL, "model: n_layers=%d d=%d (d must be a multiple of 32)", d->n_layers, d->d);
    if (d->n_q < 1 || d->n_kv < 1 || d->n_q % d->n_kv != 0) HSD_FAIL(HSD_EINVAL, "model: n_q=%d n_kv=%d", d->n_q, d->n_kv);
    if (d->hd % 32 != 0 || d->hd < 32 || d->hd > 256) HSD_FAIL(HSD_EINVAL, "model: head dim %d (multiple of 32, 32..256)", d->hd);
    if (d->ffn < 32 || d->ffn % 32 != 0) HSD_FAIL(HSD_EINVAL, "model: ffn=%d must be a multiple of 32", d->ffn);
    if (d->vocab < 2) HSD_FAIL(HSD_EINVAL, "model: vocab=%d", d->vocab);
    if (d->max_seq < HSD_KV_PAGE || d->max_seq % HSD_KV_PAGE != 0) HSD_FAIL(HSD_EINVAL, "model: max_seq=%d must be a positive multiple of %d", d->max_seq, HSD_KV_PAGE);
    if (d->max_rows < 1 || d->max_rows > HSD_MAX_PASS_ROWS) HSD_FAIL(HSD_EINVAL, "model: max_rows=%d outside 1..%d", d->max_rows, HSD_MAX_PASS_ROWS);
    if (!(d->eps > 0.f) || !(d->rope_base > 1.f)) HSD_FAIL(HSD_EINVAL, "model: eps=%g rope_base=%g", d->eps, d->rope_base);
    if (d->rows_copy_layers < 0 || d->rows_copy_layers > d->n_layers) HSD_FAIL(HSD_EINVAL, "model: rows_copy_layers=%d outside 0..%d", d->rows_copy_layers, d->n_layers);
    return HSD_OK;
}

namespace {

struct WeightLayout {
    size_t norm1, wqkv, wo, norm2, wgu, wd, layer_bytes, embed, head, norm_f, rows, rows_qkv, rows_o, rows_d, rows_layer_bytes, total;
};

WeightLayout weight_layout(const hsd_model_desc& d) {
    WeightLayout L;
    const int nqkv = (d.n_q + 2 * d.n_kv) * d.hd;
    size_t o = 0;
    L.norm1 = o; o += align_up((size_t)d.d * 4, 256);
    L.wqkv = o;  o += hsd_packed_bytes(nqkv, d.d, d.dtype);
    L.wo = o;    o += hsd_packed_bytes(d.d, d.n_q * d.hd, d.dtype);
    L.norm2 = o; o += align_up((size_t)d.d * 4, 256);
    L.wgu = o;   o += hsd_packed_bytes(2 * d.ffn, d.d, d.dtype);
    L.wd = o;    o += hsd_packed_bytes(d.d, d.ffn, d.dtype);
    L.layer_bytes = o;
    o = L.layer_bytes * d.n_layers;
    L.embed = o;  o += align_up((size_t)d.vocab * d.d * dtype_size(d.dtype), 256);
    L.head = o;   o += hsd_packed_bytes(d.vocab, d.d, d.dtype);
    L.norm_f = o; o += align_up((size_t)d.d * 4, 256);
    L.rows = o;
    size_t r = 0;
    L.rows_qkv = r; r += hsd_packed_bytes(nqkv, d.d, d.dtype);
    L.rows_o = r;   r += hsd_packed_bytes(d.d, d.n_q * d.hd, d.dtype);
    L.rows_d = r;   r += hsd_packed_bytes(d.d, d.ffn, d.dtype);
    L.rows_layer_bytes = r;
    o += r * (d.dtype == HSD_BF16 ? d.rows_copy_layers : 0);
    L.total = o;
    return L;
}

size_t part_elems_needed(const hsd_model_desc& d) {
    const int nqkv = (d.n_q + 2 * d.n_kv) * d.hd;
    if (d.dtype != HSD_BF16)   // the widest GEMM output that waits for its consumer (fused QKV or a residual update)
        return (size_t)d.max_rows * (nqkv > d.d ? nqkv : d.d);
    size_t need = 0;           // split-K partial tiles of the largest launch
    const int ms[3] = {16, 32, 64};
    for (int i = 0; i < 3; ++i) {
        const int m = ms[i] < d.max_rows ? ms[i] : d.max_rows;
        const size_t b[5] = {gemm_part_bytes(m, 2 * d.ffn, d.d, EPI_SWIGLU), gemm_part_bytes(m, d.vocab, d.d, EPI_STORE),
                             gemm_part_bytes(m, nqkv, d.d, EPI_ROPE), gemm_part_bytes(m, d.d, d.n_q * d.hd, EPI_RESID),
                             gemm_part_bytes(m, d.d, d.ffn, EPI_RESID)};
        for (int j = 0; j < 5; ++j)
            if (b[j] / 4 > need) need = b[j] / 4;
        // room for any layer projection cut in up to four K slices (tuning overrides of the plans)
        const int mt = m <= 16 ? 1 : (m <= 32 ? 2 : 4);
        const int widest = 2 * d.ffn > nqkv ? 2 * d.ffn : nqkv;
        const size_t four = (size_t)ceil_div(widest, 16) * 4 * mt * 256;
        if (four > need) need = four;
    }
    return need;
}

size_t ticket_count(const hsd_model_desc& d) {
    const int nqkv = (d.n_q + 2 * d.n_kv) * d.hd;
    int n = d.vocab;
    if (2 * d.ffn > n) n = 2 * d.ffn;
    if (nqkv > n) n = nqkv;
    if (d.d > n) n = d.d;
    return (size_t)ceil_div(n, 16);
}

struct ScratchLayout {
    size_t pages, batch_pages, batch_pos0, ss, tickets, x, xn, part, q, att, h, attn, total;
};

// The attention workspace must hold the partial states of any launch the model may make: one sequence of up to
// max_rows tokens, or a batch of sequences with batch * tokens <= max_rows.
size_t attn_ws_bytes_of(const hsd_model_desc& d) {
    size_t need = 0;
    for (int b = 1; b <= d.max_rows; ++b)
        need = std::max(need, attn_workspace_bytes(b, d.max_rows / b, d.n_q, d.n_kv, d.hd, d.max_seq));
    return need;
}

ScratchLayout scratch_layout(const hsd_model_desc& d) {
    ScratchLayout L;
    const size_t es = dtype_size(d.dtype);
    const int R = d.max_rows;
    size_t o = 0;
    L.pages = o; o += align_up((size_t)(d.max_seq / HSD_KV_PAGE) * 4, 256);
    L.batch_pages = o; o += align_up((size_t)(d.max_seq / HSD_KV_PAGE) * 4, 256);
    L.batch_pos0 = o; o += align_up((size_t)HSD_MAX_PASS_ROWS * 4, 256);
    L.ss = o;    o += align_up((size_t)2 * SS_SLOTS * HSD_MAX_PASS_ROWS * 8, 256);
    L.tickets = o; o += align_up(ticket_count(d) * 4, 256);
    L.x = o;     o += align_up((size_t)R * d.d * 4, 256);
    L.xn = o;    o += align_up((size_t)R * d.d * es, 256);
    L.part = o;  o += align_up(part_elems_needed(d) * 4, 256);
    L.q = o;     o += align_up((size_t)R * d.n_q * d.hd * es, 256);
    L.att = o;   o += align_up((size_t)R * d.n_q * d.hd * es, 256);
    L.h = o;     o += align_up((size_t)R * d.ffn * es, 256);
    L.attn = o;  o += attn_ws_bytes_of(d);
    L.total = o;
    return L;
}

size_t kv_layer_bytes(const hsd_model_desc& d) {
    return (size_t)(d.max_seq / HSD_KV_PAGE) * kv_page_elems(d.n_kv, d.hd) * dtype_size(d.dtype);
}

}  // namespace

extern "C" size_t hsd_model_weight_bytes(const hsd_model_desc* d) { return check_desc(d) ? 0 : weight_layout(*d).total; }
extern "C" size_t hsd_model_kv_bytes(const hsd_model_desc* d) { return check_desc(d) ? 0 : kv_layer_bytes(*d) * d->n_layers; }
extern "C" size_t hsd_model_scratch_bytes(const hsd_model_desc* d) { return check_desc(d) ? 0 : scratch_layout(*d).total; }

extern "C" int hsd_model_create(const hsd_model_desc* desc, void* weights_dev, void* kv_dev, void* scratch_dev, void* stream,
                                hsd_model** out) {
    if (int rc = check_desc(desc)) return rc;
    if (!weights_dev || !kv_dev || !scratch_dev || !out) HSD_FAIL(HSD_EINVAL, "hsd_model_create: null pointer");
    if (((uintptr_t)weights_dev | (uintptr_t)kv_dev | (uintptr_t)scratch_dev) & 255)
        HSD_FAIL(HSD_EINVAL, "hsd_model_create: device buffers must be 256-byte aligned");
    hsd_model* m = new hsd_model();
    m->desc = *desc;
    m->stream = (hipStream_t)stream;
    const WeightLayout W = weight_layout(*desc);
    char* wb = (char*)weights_dev;
    m->layers.resize(desc->n_layers);
    for (int l = 0; l < desc->n_layers; ++l) {
        char* lb = wb + W.layer_bytes * l;
        const bool copy = desc->dtype == HSD_BF16 && l < desc->rows_copy_layers;
        char* rb = wb + W.rows + W.rows_layer_bytes * l;
        m->layers[l] = LayerWeights{(float*)(lb + W.norm1), lb + W.wqkv, lb + W.wo, (float*)(lb + W.norm2), lb + W.wgu, lb + W.wd,
                                    copy ? rb + W.rows_qkv : nullptr, copy ? rb + W.rows_o : nullptr, copy ? rb + W.rows_d : nullptr};
    }
    m->embed = wb + W.embed;
    m->head = wb + W.head;
    m->norm_f = (float*)(wb + W.norm_f);
    m->kv = (char*)kv_dev;
    m->kv_layer_bytes = kv_layer_bytes(*desc);
    m->max_pages = desc->max_seq / HSD_KV_PAGE;
    const ScratchLayout S = scratch_layout(*desc);
    char* sb = (char*)scratch_dev;
    m->pages_dev = (int32_t*)(sb + S.pages);
    m->batch_pages_dev = (int32_t*)(sb + S.batch_pages);
    m->batch_pos0_dev = (int32_t*)(sb + S.batch_pos0);
    m->batch = 0;
    m->batch_pages_per_seq = 0;
    m->ss[0] = (unsigned long long*)(sb + S.ss);
    m->ss[1] = m->ss[0] + SS_SLOTS * HSD_MAX_PASS_ROWS;
    m->tickets = (int*)(sb + S.tickets);
    m->x = (float*)(sb + S.x);
    m->xn = sb + S.xn;
    m->part = (float*)(sb + S.part);
    m->q = sb + S.q;
    m->att = sb + S.att;
    m->h = sb + S.h;
    m->attn_ws = (float*)(sb + S.attn);
    m->part_elems = part_elems_needed(*desc);
    m->layer_loaded.assign(desc->n_layers, false);
    m->head_loaded = false;
    m->pass_serial = 0;
    m->tuning = default_kernel_tuning();
    m->prof_on = false;
    m->prof_used = 0;
    // Cache rows beyond the valid length are read (and masked) by the attention kernels: keep them finite.
    hipError_t e = hipMemsetAsync(kv_dev, 0, m->kv_layer_bytes * desc->n_layers, m->stream);
    if (e == hipSuccess) e = hipMemsetAsync(m->tickets, 0, ticket_count(*desc) * 4, m->stream);
    if (e == hipSuccess) e = hipMemsetAsync(m->attn_ws, 0, attn_ticket_bytes(), m->stream);
    // Padded rows of packed matrices must be zero.
    if (e == hipSuccess) e = hipMemsetAsync(m->head, 0, hsd_packed_bytes(desc->vocab, desc->d, desc->dtype), m->stream);
    std::vector<int32_t> ident(m->max_pages);
    for (int i = 0; i < m->max_pages; ++i) ident[i] = i;
    if (e == hipSuccess) e = hipMemcpyAsync(m->pages_dev, ident.data(), ident.size() * 4, hipMemcpyHostToDevice, m->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(m->stream);
    if (e != hipSuccess) {
        delete m;
        HSD_FAIL(HSD_EHIP, "hsd_model_create: %s", hipGetErrorString(e));
    }
    *out = m;
    return HSD_OK;
}

extern "C" void hsd_model_destroy(hsd_model* m) {
    if (!m) return;
    for (hipEvent_t e : m->prof_events) (void)hipEventDestroy(e);
    delete m;
}

extern "C" int hsd_profile_begin(hsd_model* m, int max_launches) {
    if (!m || max_launches < 1 || max_launches > (1 << 20)) HSD_FAIL(HSD_EINVAL, "hsd_profile_begin: bad arguments");
    while (m->prof_events.size() < (size_t)2 * max_launches) {
        hipEvent_t e;
        HSD_HIP(hipEventCreate(&e));
        m->prof_events.push_back(e);
    }
    m->prof_site.assign(max_launches, -1);
    m->prof_used = 0;
    m->prof_on = true;
    return HSD_OK;
}

extern "C" int hsd_profile_end(hsd_model* m, hsd_site_times* out) {
    if (!m || !out) HSD_FAIL(HSD_EINVAL, "hsd_profile_end: null pointer");
    if (!m->prof_on) HSD_FAIL(HSD_ESTATE, "hsd_profile_end: profiling was not started");
    m->prof_on = false;
    HSD_HIP(hipStreamSynchronize(m->stream));
    memset(out, 0, sizeof(*out));
    for (size_t i = 0; i < m->prof_used; ++i) {
        float ms = 0.f;
        HSD_HIP(hipEventElapsedTime(&ms, m->prof_events[2 * i], m->prof_events[2 * i + 1]));
        out->launches[m->prof_site[i]]++;
        out->ms[m->prof_site[i]] += ms;
    }
    // what a bracket costs by itself: pairs of events with nothing between them
    const int pairs = (int)(m->prof_events.size() / 2) < 64 ? (int)(m->prof_events.size() / 2) : 64;
    for (int i = 0; i < pairs; ++i) {
        HSD_HIP(hipEventRecord(m->prof_events[2 * i], m->stream));
        HSD_HIP(hipEventRecord(m->prof_events[2 * i + 1], m->stream));
    }
    HSD_HIP(hipStreamSynchronize(m->stream));
    double sum = 0.0;
    for (int i = 0; i < pairs; ++i) {
        float ms = 0.f;
        HSD_HIP(hipEventElapsedTime(&ms, m->prof_events[2 * i], m->prof_events[2 * i + 1]));
        sum += ms;
    }
    out->empty_bracket_ms = pairs ? sum / pairs : 0.0;
    return HSD_OK;
}

namespace {
// Brackets one launch with events when profiling is on.
struct SiteTimer {
    hsd_model* m;
    bool active;
    size_t slot;
    SiteTimer(hsd_model* m_, int site) : m(m_), active(false), slot(0) {
        if (m->prof_on && m->prof_used < m->prof_site.size()) {
            slot = m->prof_used++;
            m->prof_site[slot] = site;
            active = hipEventRecord(m->prof_events[2 * slot], m->stream) == hipSuccess;
        }
    }
    ~SiteTimer() {
        if (active) (void)hipEventRecord(m->prof_events[2 * slot + 1], m->stream);
    }
};
}  // namespace

extern "C" int hsd_model_set_pages(hsd_model* m, const int32_t* page_table, int n_pages) {
    if (!m || !page_table) HSD_FAIL(HSD_EINVAL, "hsd_model_set_pages: null pointer");
    if (n_pages != m->max_pages) HSD_FAIL(HSD_EINVAL, "hsd_model_set_pages: %d entries, model has %d pages", n_pages, m->max_pages);
    std::vector<char> seen(n_pages, 0);
    for (int i = 0; i < n_pages; ++i) {
        if (page_table[i] < 0 || page_table[i] >= n_pages || seen[page_table[i]])
            HSD_FAIL(HSD_EINVAL, "hsd_model_set_pages: entry %d (=%d) does not make a permutation", i, page_table[i]);
        seen[page_table[i]] = 1;
    }
    HSD_HIP(hipMemcpyAsync(m->pages_dev, page_table, (size_t)n_pages * 4, hipMemcpyHostToDevice, m->stream));
    HSD_HIP(hipStreamSynchronize(m->stream));
    return HSD_OK;
}

extern "C" int hsd_model_load_layer(hsd_model* m, int layer, const hsd_layer_weights* w) {
    if (!m || !w) HSD_FAIL(HSD_EINVAL, "hsd_model_load_layer: null pointer");
    if (layer < 0 || layer >= m->desc.n_layers) HSD_FAIL(HSD_EINVAL, "hsd_model_load_layer: layer %d outside 0..%d", layer, m->desc.n_layers - 1);
    if (!w->norm1_dev || !w->wq_dev || !w->wk_dev || !w->wv_dev || !w->wo_dev || !w->norm2_dev || !w->wg_dev || !w->wu_dev || !w->wd_dev)
        HSD_FAIL(HSD_EINVAL, "hsd_model_load_layer: null weight pointer");
    const hsd_model_desc& d = m->desc;
    const LayerWeights& L = m->layers[layer];
    hipStream_t s = m->stream;
    const int nq = d.n_q * d.hd, nkv = d.n_kv * d.hd;
    HSD_HIP(hipMemcpyAsync(L.norm1, w->norm1_dev, (size_t)d.d * 4, hipMemcpyDeviceToDevice, s));
    HSD_HIP(hipMemcpyAsync(L.norm2, w->norm2_dev, (size_t)d.d * 4, hipMemcpyDeviceToDevice, s));
    int rc;
    // bf16: MFMA tiles; q/k/v with each 16-dim block next to the block of its RoPE partners, gate/up interleaved
    const int qkv_mode = d.dtype == HSD_BF16 ? 3 : 0;
    if ((rc = launch_pack(w->wq_dev, L.wqkv, nq, d.d, d.dtype, 0, qkv_mode, d.hd, 0, s))) return rc;
    if ((rc = launch_pack(w->wk_dev, L.wqkv, nkv, d.d, d.dtype, nq, qkv_mode, d.hd, 0, s))) return rc;
    if ((rc = launch_pack(w->wv_dev, L.wqkv, nkv, d.d, d.dtype, nq + nkv, qkv_mode, d.hd, 0, s))) return rc;
    if ((rc = launch_pack(w->wo_dev, L.wo, d.d, nq, d.dtype, 0, 0, 0, 0, s))) return rc;
    if ((rc = launch_pack(w->wg_dev, L.wgu, d.ffn, d.d, d.dtype, 0, 1, 0, 0, s))) return rc;
    if ((rc = launch_pack(w->wu_dev, L.wgu, d.ffn, d.d, d.dtype, 0, 2, 0, 0, s))) return rc;
    if ((rc = launch_pack(w->wd_dev, L.wd, d.d, d.ffn, d.dtype, 0, 0, 0, 0, s))) return rc;
    if (L.wqkv_rows) {   // row-major copies, q/k/v with every dim directly followed by its RoPE partner
        if ((rc = launch_pack(w->wq_dev, L.wqkv_rows, nq, d.d, d.dtype, 0, 4, d.hd, 1, s))) return rc;
        if ((rc = launch_pack(w->wk_dev, L.wqkv_rows, nkv, d.d, d.dtype, nq, 4, d.hd, 1, s))) return rc;
        if ((rc = launch_pack(w->wv_dev, L.wqkv_rows, nkv, d.d, d.dtype, nq + nkv, 4, d.hd, 1, s))) return rc;
        if ((rc = launch_pack(w->wo_dev, L.wo_rows, d.d, nq, d.dtype, 0, 0, 0, 1, s))) return rc;
        if ((rc = launch_pack(w->wd_dev, L.wd_rows, d.d, d.ffn, d.dtype, 0, 0, 0, 1, s))) return rc;
    }
    HSD_HIP(hipStreamSynchronize(s));
    m->layer_loaded[layer] = true;
    return HSD_OK;
}

extern "C" int hsd_model_load_head(hsd_model* m, const void* embed_dev, const void* head_dev, const void* norm_f_dev) {
    if (!m || !embed_dev || !head_dev || !norm_f_dev) HSD_FAIL(HSD_EINVAL, "hsd_model_load_head: null pointer");
    const hsd_model_desc& d = m->desc;
    hipStream_t s = m->stream;
    HSD_HIP(hipMemcpyAsync(m->embed, embed_dev, (size_t)d.vocab * d.d * dtype_size(d.dtype), hipMemcpyDeviceToDevice, s));
    HSD_HIP(hipMemcpyAsync(m->norm_f, norm_f_dev, (size_t)d.d * 4, hipMemcpyDeviceToDevice, s));
    if (int rc = launch_pack(head_dev, m->head, d.vocab, d.d, d.dtype, 0, 0, 0, 0, s)) return rc;
    HSD_HIP(hipStreamSynchronize(s));
    m->head_loaded = true;
    return HSD_OK;
}

// A pass over a batch of sequences: `rows` = batch * m_seq tokens, row r = token r % m_seq of sequence r / m_seq at
// position pos0_dev[sequence] + r % m_seq; null for one sequence at pos0.
struct BatchGeom {
    int batch, m_seq, max_len;
};

static float* tap_after_layer(const PassOpts* o, int layer_count) {
    if (o)
        for (int i = 0; i < o->n_taps; ++i)
            if (o->tap_layer[i] == layer_count) return o->tap_rows[i];
    return nullptr;
}

// fp32 storage: plain kernels, one per step (the small correctness configuration).
static int pass_f32(hsd_model* m, const int32_t* tok, int pos0, int rows, const int* exits, int n_exits, int n_logit_rows,
                    float* logits, bool embedded, const BatchGeom* bg, const PassOpts* opts) {
    const hsd_model_desc& d = m->desc;
    hipStream_t s = m->stream;
    const int nq = d.n_q * d.hd, nqkv = (d.n_q + 2 * d.n_kv) * d.hd;
    const int exit_layer = exits[n_exits - 1];
    const size_t logit_stride = (size_t)n_logit_rows * d.vocab;
    int ei = 0;
    int rc;
    const int l0 = opts ? opts->from_layer : 0;
    if (l0 > 0) {       // resume above an exit another pass has reached: its residual rows are this pass's
        HSD_HIP(hipMemcpyAsync(m->x, opts->resume_rows, (size_t)rows * d.d * sizeof(float), hipMemcpyDeviceToDevice, s));
    } else if (!embedded && (rc = launch_embed(tok, m->embed, m->x, rows, d.d, d.vocab, d.dtype, nullptr, nullptr, nullptr, nullptr, s))) {
        return rc;
    }
    const float* pending = nullptr;     // output of the previous down projection, not yet added to x
    for (int l = l0; l < exit_layer; ++l) {
        const LayerWeights& L = m->layers[l];
        void* kv_layer = m->kv + m->kv_layer_bytes * l;
        if ((rc = launch_resid_rmsnorm(m->x, pending, 1, rows, 0, L.norm1, m->xn, rows, 0, d.d, d.eps, d.dtype, s))) return rc;
        {
            SiteTimer t(m, HSD_SITE_QKV);
            if ((rc = launch_gemm_f32((const float*)m->xn, (const float*)L.wqkv, m->part, rows, nqkv, d.d, false, s))) return rc;
        }
        if (bg) {
            if ((rc = launch_rope_kv(m->part, 1, rows, m->q, kv_layer, m->batch_pages_dev, 0, d.n_q, d.n_kv, d.hd, d.rope_base, d.dtype, s,
                                     m->batch_pos0_dev, bg->m_seq, m->batch_pages_per_seq))) return rc;
        } else if ((rc = launch_rope_kv(m->part, 1, rows, m->q, kv_layer, m->pages_dev, pos0, d.n_q, d.n_kv, d.hd, d.rope_base, d.dtype, s))) {
            return rc;
        }
        {
            SiteTimer t(m, HSD_SITE_ATTN);
            if (bg)
                rc = launch_attention(m->q, kv_layer, m->batch_pages_dev, m->batch_pages_per_seq, m->batch_pos0_dev, 0, bg->batch, bg->m_seq,
                                      bg->max_len, d.n_q, d.n_kv, d.hd, d.dtype, m->att, m->attn_ws, 0, s, m->tuning);
            else
                rc = launch_attention(m->q, kv_layer, m->pages_dev, m->max_pages, nullptr, pos0, 1, rows, pos0 + rows, d.n_q, d.n_kv,
                                      d.hd, d.dtype, m->att, m->attn_ws, 0, s, m->tuning);
            if (rc) return rc;
        }
        {
            SiteTimer t(m, HSD_SITE_O);
            if ((rc = launch_gemm_f32((const float*)m->att, (const float*)L.wo, m->part, rows, d.d, nq, false, s))) return rc;
        }
        if ((rc = launch_resid_rmsnorm(m->x, m->part, 1, rows, 0, L.norm2, m->xn, rows, 0, d.d, d.eps, d.dtype, s))) return rc;
        {
            SiteTimer t(m, HSD_SITE_GATEUP);
            if ((rc = launch_gemm_f32((const float*)m->xn, (const float*)L.wgu, (float*)m->h, rows, 2 * d.ffn, d.d, true, s))) return rc;
        }
        {
            SiteTimer t(m, HSD_SITE_DOWN);
            if ((rc = launch_gemm_f32((const float*)m->h, (const float*)L.wd, m->part, rows, d.d, d.ffn, false, s))) return rc;
        }
        pending = m->part;
        if (float* tap = tap_after_layer(opts, l + 1)) {
            // the residual rows after this layer are kept: the pending projection goes into x now (the same addition the
            // next step would make; the normalised rows it also writes are overwritten there)
            if ((rc = launch_resid_rmsnorm(m->x, pending, 1, rows, 0, m->norm_f, m->xn, rows, 0, d.d, d.eps, d.dtype, s))) return rc;
            pending = nullptr;
            HSD_HIP(hipMemcpyAsync(tap, m->x, (size_t)rows * d.d * sizeof(float), hipMemcpyDeviceToDevice, s));
        }
        if (l + 1 == exits[ei] && l + 1 < exit_layer) {
            // an exit on the way: the pending projection goes into x for every row (the deeper layers need them
            // all), the final norm of all rows into xn, the head reads the logit rows
            if (n_logit_rows > 0) {
                if ((rc = launch_resid_rmsnorm(m->x, pending, 1, rows, 0, m->norm_f, m->xn, rows, 0, d.d, d.eps, d.dtype, s))) return rc;
                pending = nullptr;
                SiteTimer t(m, HSD_SITE_HEAD);
                if ((rc = launch_gemm_f32((const float*)m->xn + (size_t)(rows - n_logit_rows) * d.d, (const float*)m->head,
                                          logits + ei * logit_stride, n_logit_rows, d.vocab, d.d, false, s))) return rc;
            }
            ++ei;
        }
    }
    if (n_logit_rows == 0) return HSD_OK;
    const int row0 = rows - n_logit_rows;
    if ((rc = launch_resid_rmsnorm(m->x, pending, 1, rows, row0, m->norm_f, m->xn, n_logit_rows, row0, d.d, d.eps, d.dtype, s))) return rc;
    SiteTimer t(m, HSD_SITE_HEAD);
    return launch_gemm_f32((const float*)m->xn, (const float*)m->head, logits + ei * logit_stride, n_logit_rows, d.vocab, d.d, false, s);
}

// bf16 storage: five launches per layer.  RoPE and the KV append live in the QKV epilogue, SwiGLU in the
// gate/up epilogue, the residual adds in the O and down projections.  Those two also prepare the next
// RMSNorm: they store bf16(x * w_norm) into m->xn and add the rows' sums of squares into m->ss[1]
// (second norm of the layer) or m->ss[0] (first norm of the next layer, or the final norm at the exit);
// the GEMM that consumes m->xn multiplies by 1/rms in its epilogue.
static int launch_site_bf16(hsd_model* m, int site, int l, int pos0, int rows, const float* next_norm_w, const BatchGeom* bg = nullptr,
                            float* tap = nullptr) {
    const hsd_model_desc& d = m->desc;
    hipStream_t s = m->stream;
    const int nq = d.n_q * d.hd, nqkv = (d.n_q + 2 * d.n_kv) * d.hd;
    const LayerWeights& L = m->layers[l];
    bf16_t* kv_layer = (bf16_t*)(m->kv + m->kv_layer_bytes * l);
    // one or two tokens: some projections stream their row-major copies
    const hsd_kernel_tuning& tn = m->tuning;
    // (two tokens: only matrices below 64 MB, 1B-shaped down 9.4 against 11.1 us; on the 7B / 8B-shaped down projections the
    // tile kernel is ahead, 19.9 / 23.3 against 23.1 / 25.3)
    const size_t site_bytes = site == HSD_SITE_DOWN ? (size_t)d.d * d.ffn * 2 : (size_t)d.d * nq * 2;
    const bool rowk = L.wqkv_rows && !bg && rows <= (site == HSD_SITE_QKV ? tn.gemv_max_m_qkv : (site == HSD_SITE_O ? tn.gemv_max_m_o : tn.gemv_max_m_down)) &&
                      (rows == 1 || site_bytes <= ((size_t)64 << 20));
    GemmArgs g = {};
    g.M = rows; g.part = m->part; g.part_bytes = m->part_elems * sizeof(float); g.tickets = m->tickets; g.eps = d.eps;
    switch (site) {
        case HSD_SITE_QKV:
            g.a = (const bf16_t*)m->xn; g.ss_in = m->ss[0]; g.ss_zero = m->ss[1];
            g.wp = (const bf16x8*)(rowk ? L.wqkv_rows : L.wqkv); g.N = nqkv; g.K = d.d;
            g.out_bf16 = (bf16_t*)m->q; g.kv_layer = kv_layer; g.pages = m->pages_dev;
            g.pos0 = pos0; g.n_q = d.n_q; g.n_kv = d.n_kv; g.hd = d.hd; g.rope_base = d.rope_base;
            if (bg) { g.pages = m->batch_pages_dev; g.pos0_arr = m->batch_pos0_dev; g.m_seq = bg->m_seq; g.max_pages = m->batch_pages_per_seq; }
            return rowk ? launch_gemv_bf16(g, EPI_ROPE, s) : launch_gemm_bf16(g, EPI_ROPE, gemm_plan(rows, nqkv, d.d, EPI_ROPE, tn), s);
        case HSD_SITE_ATTN:
            if (bg)
                return launch_attention(m->q, kv_layer, m->batch_pages_dev, m->batch_pages_per_seq, m->batch_pos0_dev, 0, bg->batch,
                                        bg->m_seq, bg->max_len, d.n_q, d.n_kv, d.hd, d.dtype, m->att, m->attn_ws, 0, s, m->tuning);
            return launch_attention(m->q, kv_layer, m->pages_dev, m->max_pages, nullptr, pos0, 1, rows, pos0 + rows, d.n_q, d.n_kv,
                                    d.hd, d.dtype, m->att, m->attn_ws, 0, s, m->tuning);
        case HSD_SITE_O:
            g.a = (const bf16_t*)m->att; g.wp = (const bf16x8*)(rowk ? L.wo_rows : L.wo); g.N = d.d; g.K = nq;
            g.out_f32 = m->x; g.ss_out = m->ss[1]; g.norm_w = L.norm2; g.out_bf16 = (bf16_t*)m->xn;
            return rowk ? launch_gemv_bf16(g, EPI_RESID, s) : launch_gemm_bf16(g, EPI_RESID, gemm_plan(rows, d.d, nq, EPI_RESID, tn), s);
        case HSD_SITE_GATEUP:
            g.a = (const bf16_t*)m->xn; g.ss_in = m->ss[1]; g.ss_zero = m->ss[0];
            g.wp = (const bf16x8*)L.wgu; g.N = 2 * d.ffn; g.K = d.d;
            g.out_bf16 = (bf16_t*)m->h;
            return launch_gemm_bf16(g, EPI_SWIGLU, gemm_plan(rows, 2 * d.ffn, d.d, EPI_SWIGLU, tn), s);
        case HSD_SITE_DOWN:
            g.a = (const bf16_t*)m->h; g.wp = (const bf16x8*)(rowk ? L.wd_rows : L.wd); g.N = d.d; g.K = d.ffn;
            g.out_f32 = m->x; g.ss_out = m->ss[0]; g.norm_w = next_norm_w; g.out_bf16 = (bf16_t*)m->xn; g.tap = tap;
            return rowk ? launch_gemv_bf16(g, EPI_RESID, s) : launch_gemm_bf16(g, EPI_RESID, gemm_plan(rows, d.d, d.ffn, EPI_RESID, tn), s);
        default:
            HSD_FAIL(HSD_EINVAL, "unknown site %d", site);
    }
}

static int launch_head_bf16(hsd_model* m, const void* xn, int rows, int n_logit_rows, float* logits) {
    const hsd_model_desc& d = m->desc;
    const int row0 = rows - n_logit_rows;
    GemmArgs g = {};
    g.part = m->part; g.part_bytes = m->part_elems * sizeof(float); g.tickets = m->tickets; g.eps = d.eps;
    g.M = n_logit_rows;
    g.a = (const bf16_t*)xn + (size_t)row0 * d.d; g.ss_in = m->ss[0] + row0;
    g.wp = (const bf16x8*)m->head; g.N = d.vocab; g.K = d.d;
    g.out_f32 = logits;
    return launch_gemm_bf16(g, EPI_STORE, gemm_plan(n_logit_rows, d.vocab, d.d, EPI_STORE, m->tuning), m->stream);
}

static int pass_bf16(hsd_model* m, const int32_t* tok, int pos0, int rows, const int* exits, int n_exits, int n_logit_rows,
                     float* logits, bool embedded, const BatchGeom* bg, const PassOpts* opts) {
    const hsd_model_desc& d = m->desc;
    const int exit_layer = exits[n_exits - 1];
    const size_t logit_stride = (size_t)n_logit_rows * d.vocab;
    int ei = 0;
    int rc;
    const int l0 = opts ? opts->from_layer : 0;
    if (l0 > 0) {       // resume above an exit another pass has reached, from the residual rows it kept there
        if ((rc = launch_resume_rows(opts->resume_rows, m->x, rows, d.d, m->ss[0], m->ss[1], m->layers[l0].norm1, m->xn, m->stream))) return rc;
    } else if (!embedded &&
               (rc = launch_embed(tok, m->embed, m->x, rows, d.d, d.vocab, d.dtype, m->ss[0], m->ss[1], m->layers[0].norm1, m->xn, m->stream))) {
        return rc;
    }
    for (int l = l0; l < exit_layer; ++l) {
        const float* next_norm = l + 1 == exit_layer ? m->norm_f : m->layers[l + 1].norm1;
        for (int site = HSD_SITE_QKV; site <= HSD_SITE_DOWN; ++site) {
            SiteTimer t(m, site);
            // the down projection's epilogue also stores the residual rows a deeper exit may resume from
            if ((rc = launch_site_bf16(m, site, l, pos0, rows, next_norm, bg, site == HSD_SITE_DOWN ? tap_after_layer(opts, l + 1) : nullptr))) return rc;
        }
        if (l + 1 == exits[ei] && l + 1 < exit_layer) {
            // an exit on the way: m->xn holds x scaled by the next layer's norm weights, the head needs the final
            // norm's (same sums of squares); m->h is free between the down projection and the next gate/up
            if (n_logit_rows > 0) {
                if ((rc = launch_scale_rows_bf16(m->x, m->norm_f, m->h, rows, d.d, m->stream))) return rc;
                SiteTimer t(m, HSD_SITE_HEAD);
                if ((rc = launch_head_bf16(m, m->h, rows, n_logit_rows, logits + ei * logit_stride))) return rc;
            }
            ++ei;
        }
    }
    if (n_logit_rows == 0) return HSD_OK;
    SiteTimer t(m, HSD_SITE_HEAD);
    return launch_head_bf16(m, m->xn, rows, n_logit_rows, logits + ei * logit_stride);
}

extern "C" int hsd_measure_site(hsd_model* m, int site, int rows, int pos0, int iters, double* us_out) {
    if (!m || !us_out) HSD_FAIL(HSD_EINVAL, "hsd_measure_site: null pointer");
    const hsd_model_desc& d = m->desc;
    if (d.dtype != HSD_BF16) HSD_FAIL(HSD_EINVAL, "hsd_measure_site: bf16 models only");
    if (site < HSD_SITE_QKV || site > HSD_SITE_DOWN || rows < 1 || rows > d.max_rows || iters < 1 || pos0 < 0 || pos0 + rows > d.max_seq)
        HSD_FAIL(HSD_EINVAL, "hsd_measure_site: bad arguments (sites: q/k/v, attention, o, gate/up, down)");
    for (int l = 0; l < d.n_layers; ++l)
        if (!m->layer_loaded[l]) HSD_FAIL(HSD_ESTATE, "hsd_measure_site: layer %d not loaded", l);
    hipEvent_t e0, e1;
    HSD_HIP(hipEventCreate(&e0));
    HSD_HIP(hipEventCreate(&e1));
    int rc = HSD_OK;
    ++m->pass_serial;                                    // the activation buffers are overwritten
    auto one = [&](int i) { return launch_site_bf16(m, site, i % d.n_layers, pos0, rows, m->norm_f); };
    for (int i = 0; i < d.n_layers && !rc; ++i) rc = one(i);                 // warm-up, one launch per layer
    if (!rc && hipEventRecord(e0, m->stream) != hipSuccess) rc = HSD_EHIP;
    for (int i = 0; i < iters && !rc; ++i) rc = one(i);
    float ms = 0.f;
    if (!rc && (hipEventRecord(e1, m->stream) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                hipEventElapsedTime(&ms, e0, e1) != hipSuccess)) {
        hsd_set_error("hsd_measure_site: event timing failed");
        rc = HSD_EHIP;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc) return rc;
    *us_out = (double)ms * 1e3 / iters;
    return HSD_OK;
}

extern "C" int hsd_site_kernel(const hsd_model* m, int site, int rows, char* name_out, int cap) {
    if (!m || !name_out || cap < 8) HSD_FAIL(HSD_EINVAL, "hsd_site_kernel: bad arguments");
    const hsd_model_desc& d = m->desc;
    if (d.dtype != HSD_BF16) HSD_FAIL(HSD_EINVAL, "hsd_site_kernel: bf16 models only");
    if (rows < 1 || rows > d.max_rows) HSD_FAIL(HSD_EINVAL, "hsd_site_kernel: rows=%d", rows);
    const int nq = d.n_q * d.hd, nqkv = (d.n_q + 2 * d.n_kv) * d.hd;
    int n = 0, k = 0, epi = 0;
    switch (site) {
        case HSD_SITE_QKV: n = nqkv; k = d.d; epi = EPI_ROPE; break;
        case HSD_SITE_O: n = d.d; k = nq; epi = EPI_RESID; break;
        case HSD_SITE_GATEUP: n = 2 * d.ffn; k = d.d; epi = EPI_SWIGLU; break;
        case HSD_SITE_DOWN: n = d.d; k = d.ffn; epi = EPI_RESID; break;
        case HSD_SITE_HEAD: n = d.vocab; k = d.d; epi = EPI_STORE; break;
        default: HSD_FAIL(HSD_EINVAL, "hsd_site_kernel: site %d is not a projection", site);
    }
    // layers without row-major copies (rows_copy_layers counts from the first layer): the tiled kernel
    gemm_kernel_name(rows, k, epi, gemm_plan(rows, n, k, epi, m->tuning), name_out, (size_t)cap);
    return HSD_OK;
}

// One pass: rows tokens at positions pos0.., layers [0, exit_layer), logits of the last n_logit_rows rows.
static int pass_checked(hsd_model* m, const int32_t* tok, int pos0, int rows, const int* exits, int n_exits, int n_logit_rows,
                        float* logits, bool embedded, const BatchGeom* bg = nullptr, const PassOpts* opts = nullptr);

// embedded: row 0 of the residual stream (and, bf16, of the normalised input and the sums of squares) already holds
// the one token of this pass, left there by the fused sampler (EmbedNext); only for rows == 1.
int model_pass(hsd_model* m, const int32_t* tok, int pos0, int rows, int exit_layer, int n_logit_rows, float* logits, bool embedded,
               const PassOpts* opts) {
    return pass_checked(m, tok, pos0, rows, &exit_layer, 1, n_logit_rows, logits, embedded && rows == 1, nullptr, opts);
}

int model_pass_exits(hsd_model* m, const int32_t* tok, int pos0, int rows, const int* exits, int n_exits, int n_logit_rows,
                     float* logits) {
    return pass_checked(m, tok, pos0, rows, exits, n_exits, n_logit_rows, logits, false);
}

EmbedNext embed_next_of(const hsd_model* m) {
    const hsd_model_desc& d = m->desc;
    const bool bf = d.dtype == HSD_BF16;
    return EmbedNext{m->embed, d.dtype, d.d, d.vocab, m->x, bf ? m->xn : nullptr, bf ? m->layers[0].norm1 : nullptr,
                     bf ? m->ss[0] : nullptr, bf ? m->ss[1] : nullptr};
}

static int pass_checked(hsd_model* m, const int32_t* tok, int pos0, int rows, const int* exits, int n_exits, int n_logit_rows,
                        float* logits, bool embedded, const BatchGeom* bg, const PassOpts* opts) {
    const hsd_model_desc& d = m->desc;
    if (!exits || n_exits < 1 || n_exits > d.n_layers) HSD_FAIL(HSD_EINVAL, "pass: %d exits", n_exits);
    for (int i = 0; i < n_exits; ++i)
        if (exits[i] < 1 || exits[i] > d.n_layers || (i > 0 && exits[i] <= exits[i - 1]))
            HSD_FAIL(HSD_EINVAL, "pass: exit layer %d (entry %d) outside 1..%d or not ascending", exits[i], i, d.n_layers);
    const int exit_layer = exits[n_exits - 1];
    if (n_exits > 1 && d.dtype == HSD_BF16 && d.ffn < d.d)
        HSD_FAIL(HSD_ECAPACITY, "pass: several exits need ffn >= d for the exit rows (ffn=%d d=%d)", d.ffn, d.d);
    if (rows < 1 || rows > d.max_rows) HSD_FAIL(HSD_ECAPACITY, "pass: %d rows, model allows 1..%d", rows, d.max_rows);
    if (!bg && (pos0 < 0 || pos0 + rows > d.max_seq)) HSD_FAIL(HSD_ECAPACITY, "pass: positions %d..%d exceed the KV capacity %d", pos0, pos0 + rows - 1, d.max_seq);
    if (n_logit_rows < 0 || n_logit_rows > rows) HSD_FAIL(HSD_EINVAL, "pass: %d logit rows of %d", n_logit_rows, rows);
    if (n_logit_rows > 0 && !logits) HSD_FAIL(HSD_EINVAL, "pass: logits buffer missing");
    if (!m->head_loaded) HSD_FAIL(HSD_ESTATE, "pass: embedding / head not loaded");
    for (int l = 0; l < exit_layer; ++l)
        if (!m->layer_loaded[l]) HSD_FAIL(HSD_ESTATE, "pass: layer %d not loaded", l);
    if (opts) {
        if (opts->from_layer < 0 || opts->from_layer >= exit_layer || (opts->from_layer > 0 && !opts->resume_rows))
            HSD_FAIL(HSD_EINVAL, "pass: resume layer %d outside 0..%d or without rows", opts->from_layer, exit_layer - 1);
        if (opts->n_taps < 0 || opts->n_taps > HSD_MAX_LEVELS) HSD_FAIL(HSD_EINVAL, "pass: %d taps", opts->n_taps);
        for (int i = 0; i < opts->n_taps; ++i)
            if (opts->tap_layer[i] <= opts->from_layer || opts->tap_layer[i] > exit_layer || !opts->tap_rows[i])
                HSD_FAIL(HSD_EINVAL, "pass: tap %d after layer %d outside %d..%d", i, opts->tap_layer[i], opts->from_layer + 1, exit_layer);
        if (opts->from_layer > 0 && embedded) HSD_FAIL(HSD_EINVAL, "pass: a resumed pass embeds nothing");
    }
    ++m->pass_serial;
    return d.dtype == HSD_BF16 ? pass_bf16(m, tok, pos0, rows, exits, n_exits, n_logit_rows, logits, embedded, bg, opts)
                               : pass_f32(m, tok, pos0, rows, exits, n_exits, n_logit_rows, logits, embedded, bg, opts);
}

extern "C" int hsd_model_set_tuning(hsd_model* m, const hsd_kernel_tuning* t) {
    if (!m) HSD_FAIL(HSD_EINVAL, "hsd_model_set_tuning: null pointer");
    m->tuning = t ? *t : default_kernel_tuning();
    return HSD_OK;
}

// ---- batch of sequences ------------------------------------------------------------------------------------------
extern "C" int hsd_model_set_batch(hsd_model* m, int batch, int pages_per_seq, const int32_t* page_table) {
    if (!m) HSD_FAIL(HSD_EINVAL, "hsd_model_set_batch: null pointer");
    if (batch == 0) {                                    // back to one sequence
        m->batch = 0;
        m->batch_pages_per_seq = 0;
        return HSD_OK;
    }
    if (!page_table) HSD_FAIL(HSD_EINVAL, "hsd_model_set_batch: null page table");
    if (batch < 1 || batch > m->desc.max_rows) HSD_FAIL(HSD_ECAPACITY, "hsd_model_set_batch: batch %d outside 1..%d (max_rows)", batch, m->desc.max_rows);
    if (pages_per_seq < 1 || (long long)batch * pages_per_seq > m->max_pages)
        HSD_FAIL(HSD_ECAPACITY, "hsd_model_set_batch: %d sequences x %d pages exceed the model's %d KV pages", batch, pages_per_seq, m->max_pages);
    std::vector<char> seen(m->max_pages, 0);
    for (int i = 0; i < batch * pages_per_seq; ++i) {
        if (page_table[i] < 0 || page_table[i] >= m->max_pages || seen[page_table[i]])
            HSD_FAIL(HSD_EINVAL, "hsd_model_set_batch: entry %d (=%d) is outside 0..%d or used twice", i, page_table[i], m->max_pages - 1);
        seen[page_table[i]] = 1;
    }
    HSD_HIP(hipMemcpyAsync(m->batch_pages_dev, page_table, (size_t)batch * pages_per_seq * 4, hipMemcpyHostToDevice, m->stream));
    HSD_HIP(hipStreamSynchronize(m->stream));
    m->batch = batch;
    m->batch_pages_per_seq = pages_per_seq;
    return HSD_OK;
}

extern "C" int hsd_model_pass_batch(hsd_model* m, const int32_t* tokens_dev, const int32_t* pos0, int tokens_per_seq, int exit_layer,
                                    int with_logits, float* logits_dev) {
    if (!m || !tokens_dev || !pos0) HSD_FAIL(HSD_EINVAL, "hsd_model_pass_batch: null pointer");
    if (m->batch < 1) HSD_FAIL(HSD_ESTATE, "hsd_model_pass_batch: no batch geometry (call hsd_model_set_batch first)");
    const int rows = m->batch * tokens_per_seq;
    if (tokens_per_seq < 1 || rows > m->desc.max_rows)
        HSD_FAIL(HSD_ECAPACITY, "hsd_model_pass_batch: %d sequences x %d tokens exceed the %d rows of a pass", m->batch, tokens_per_seq, m->desc.max_rows);
    const int cap = m->batch_pages_per_seq * HSD_KV_PAGE;
    int max_len = 0;
    for (int b = 0; b < m->batch; ++b) {
        if (pos0[b] < 0 || pos0[b] + tokens_per_seq > cap)
            HSD_FAIL(HSD_ECAPACITY, "hsd_model_pass_batch: sequence %d at positions %d..%d exceeds its %d cache positions", b, pos0[b],
                     pos0[b] + tokens_per_seq - 1, cap);
        max_len = std::max(max_len, pos0[b] + tokens_per_seq);
    }
    // pageable host memory: the runtime has staged the copy when the call returns, the caller's array is free again
    HSD_HIP(hipMemcpyAsync(m->batch_pos0_dev, pos0, (size_t)m->batch * 4, hipMemcpyHostToDevice, m->stream));
    const BatchGeom bg{m->batch, tokens_per_seq, max_len};
    return pass_checked(m, tokens_dev, 0, rows, &exit_layer, 1, with_logits ? rows : 0, logits_dev, false, &bg);
}

extern "C" int hsd_model_pass(hsd_model* m, const int32_t* tokens_dev, int pos0, int rows, int exit_layer, int n_logit_rows,
                              float* logits_dev) {
    if (!m || !tokens_dev) HSD_FAIL(HSD_EINVAL, "hsd_model_pass: null pointer");
    return model_pass(m, tokens_dev, pos0, rows, exit_layer, n_logit_rows, logits_dev);
}

extern "C" int hsd_model_pass_exits(hsd_model* m, const int32_t* tokens_dev, int pos0, int rows, const int* exits, int n_exits,
                                    int n_logit_rows, float* logits_dev) {
    if (!m || !tokens_dev) HSD_FAIL(HSD_EINVAL, "hsd_model_pass_exits: null pointer");
    return model_pass_exits(m, tokens_dev, pos0, rows, exits, n_exits, n_logit_rows, logits_dev);
}
