// Internal view of hsd_model shared by model.hip and hier.hip.
#pragma once
#include <vector>

#include "common.h"

struct LayerWeights {
    float* norm1;
    void* wqkv;   // packed [(n_q + 2 n_kv) hd, d]
    void* wo;     // packed [d, n_q hd]
    float* norm2;
    void* wgu;    // packed [2 ffn, d], gate / up tiles interleaved
    void* wd;     // packed [d, ffn]
    // bf16, first rows_copy_layers layers only: row-major copies for passes of one or two tokens
    void* wqkv_rows;   // [(n_q + 2 n_kv) hd, d], every dim followed by its RoPE partner
    void* wo_rows;     // [d, n_q hd]
    void* wd_rows;     // [d, ffn]
};

struct hsd_model {
    hsd_model_desc desc;
    hipStream_t stream;
    std::vector<LayerWeights> layers;
    void* embed;      // [vocab, d] row-major, dtype
    void* head;       // packed [vocab, d]
    float* norm_f;
    char* kv;         // [layer][page][kv head][K block | V block]
    size_t kv_layer_bytes;
    int max_pages;
    int32_t* pages_dev;
    // activation scratch
    float* x;         // residual stream [max_rows, d] fp32
    void* xn;         // input rows of the next normalising GEMM [max_rows, d] (bf16 path: x * w_norm, scaled by 1/rms later)
    float* part;      // fp32 path: GEMM outputs waiting to be added to the residual stream; bf16 path: split-K partial tiles
    int* tickets;     // bf16 path: arrival counters of the split-K column groups
    unsigned long long* ss[2];   // bf16 path: per-row sums of squares (fixed point) for the two norms of a layer
    void* q;          // [max_rows, n_q hd]
    void* att;        // [max_rows, n_q hd]
    void* h;          // [max_rows, ffn]
    float* attn_ws;
    size_t part_elems;
    std::vector<bool> layer_loaded;
    bool head_loaded;
    // batch of sequences (hsd_model_set_batch / hsd_model_pass_batch): the KV pages shared out among the sequences
    int32_t* batch_pages_dev;   // [batch][batch_pages_per_seq]
    int32_t* batch_pos0_dev;    // [batch]
    int batch, batch_pages_per_seq;
    hsd_kernel_tuning tuning;   // launch heuristics of this model's passes (hsd_model_set_tuning)
    unsigned long long pass_serial;   // counts passes: whoever left something in the activation buffers can tell if it is still there
    // optional per-site event timing (hsd_profile_begin / hsd_profile_end)
    bool prof_on;
    size_t prof_used;
    std::vector<hipEvent_t> prof_events;   // pairs
    std::vector<int> prof_site;
};

// Hidden-state reuse between exits of one network: a pass may start above layer `from_layer`, from the residual rows
// another pass kept there (`resume_rows` [rows, d] fp32), and may keep its own residual rows after given layers
// (`tap_rows[i]` [rows, d] receives them after layer `tap_layer[i]`, from_layer < tap_layer[i] <= exit layer).
struct PassOpts {
    int from_layer = 0;
    const float* resume_rows = nullptr;
    int n_taps = 0;
    int tap_layer[HSD_MAX_LEVELS] = {};
    float* tap_rows[HSD_MAX_LEVELS] = {};
};
int model_pass(hsd_model* m, const int32_t* tokens_dev, int pos0, int rows, int exit_layer, int n_logit_rows,
               float* logits_dev, bool embedded = false, const PassOpts* opts = nullptr);
// The same pass through the deepest of `exits` (ascending layer counts), with the last n_logit_rows rows' logits of
// every listed exit: logits_dev [n_exits][n_logit_rows][vocab].
int model_pass_exits(hsd_model* m, const int32_t* tokens_dev, int pos0, int rows, const int* exits, int n_exits,
                     int n_logit_rows, float* logits_dev);

// kernels_layer.hip
int launch_embed(const int32_t* tok, const void* E, float* x, int m, int d, int vocab, int dtype, unsigned long long* ss,
                 unsigned long long* ss_other, const float* norm_w, void* xn, hipStream_t s);
int launch_resume_rows(const float* rows, float* x, int m, int d, unsigned long long* ss, unsigned long long* ss_other,
                       const float* norm_w, void* xn, hipStream_t s);
int launch_resid_rmsnorm(float* x, const float* part, int ksplit, int part_rows, int part_row0, const float* w, void* xn,
                         int rows, int row0, int d, float eps, int dtype, hipStream_t s);
int launch_rope_kv(const float* part, int ksplit, int m, void* q, void* kv_layer, const int32_t* pages, int pos0, int n_q,
                   int n_kv, int hd, float rope_base, int dtype, hipStream_t s, const int32_t* pos0_arr = nullptr, int m_seq = 0,
                   int max_pages = 0);
size_t softmax_scratch_bytes(int rows, int vocab);
int launch_softmax(const float* z, float* p, int rows, int vocab, float temperature, float* scratch, hipStream_t s);
int launch_scale_rows_bf16(const float* x, const float* w, void* out, int rows, int d, hipStream_t s);
// kernels_attn.hip
size_t attn_workspace_bytes(int batch, int m, int n_q, int n_kv, int hd, int max_len);
size_t attn_ticket_bytes();   // leading bytes of an attention workspace that must be zero between launches
int launch_attention(const void* q, const void* kv_layer, const int32_t* pages, int max_pages, const int32_t* pos0_dev,
                     int pos0_all, int batch, int m, int max_len, int n_q, int n_kv, int hd, int dtype, void* att,
                     float* workspace, int force_simple, hipStream_t s, const hsd_kernel_tuning& t = default_kernel_tuning());
// kernels_sampler.hip
int launch_accept_resample(const float* p, const float* q, int32_t* x, int t, int vocab, uint64_t seed, uint32_t level,
                           uint32_t call, int32_t* result, void* scratch, float coin, hipStream_t s);
int launch_add_noise(float* z, int rows, int vocab, uint64_t seed, uint32_t level, int pos0, float std, hipStream_t s);
bool softmax_verify_supported(int vocab, int max_v = 1 << 30);   // max_v: the driver's own limit (a tuning setting)
// What the fused sampler needs to leave the emitted token embedded for a following one-token pass of `model`
// (row 0 of its residual stream, normalised input and sums of squares, exactly as the embedding kernel would):
// E == nullptr switches it off.
struct EmbedNext {
    const void* E;
    int dtype, d, vocab;
    float* x;
    void* xn;
    const float* norm_w;
    unsigned long long *ss, *ss_other;
};
EmbedNext embed_next_of(const hsd_model* m);
int launch_softmax_verify(const float* z, const float* q, int32_t* x, int t, int vocab, float temperature, uint64_t seed,
                          uint32_t level, uint32_t call, float* p_out, int32_t* result, void* scratch, int32_t* mailbox,
                          const EmbedNext& next, float coin, int mailbox_seq, hipStream_t s);
// Several independent calls of the fused sampler in one launch (the sequences of a batch at one level): call c uses
// the ticket / key pair at scratch + 16 c, which must be zero before the first launch (the kernel leaves it zero).
struct VerifyCall {
    const float* z;       // [t + 1, vocab] logits
    const float* q;       // [t, vocab] draft rows (unused for t == 0)
    int32_t* x;           // the t drafts; x[n] receives the emitted token
    float* p_out;         // [t + 1, vocab] or null
    int32_t* result;      // (n, token)
    int32_t* mailbox;     // pinned host memory or null
    uint64_t seed;
    uint32_t call;
    int t;
};
constexpr int VERIFY_CALLS_MAX = 16;
struct VerifyCalls {
    VerifyCall c[VERIFY_CALLS_MAX];
};
int launch_softmax_verify_batch(const VerifyCall* calls, int n_calls, int vocab, float temperature, uint32_t level, void* scratch,
                                hipStream_t s);
// With mailbox_seq != 0 the kernel ends its mailbox writes by storing mailbox_seq into this slot of the mailbox
// (which then must have MAILBOX_SEQ_SLOT + 1 entries), after a system-scope release: a host may poll it.
constexpr int MAILBOX_SEQ_SLOT = 67;
