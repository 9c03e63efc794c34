/*
 * libhsd - Hierarchical Speculative Decoding (HSD) hot path for AMD MI355X (gfx950).
 *
 * C ABI.  Conventions for every entry point:
 *   - returns HSD_OK (0) or a negative status; hsd_last_error() gives the message of the last
 *     failure on the calling thread;
 *   - pointers named *_dev are device (HBM) pointers, everything else is host memory;
 *   - the library never allocates or frees device memory: the caller owns every device buffer and
 *     sizes them with the hsd_*_bytes() helpers; buffers must stay alive while the object uses them;
 *   - all device work is enqueued on the hipStream_t (passed as void*) given at creation / call;
 *     calls that return host results synchronise that stream before returning;
 *   - host output arrays are caller-owned with explicit capacities;
 *   - objects are not thread-safe; calls on one hierarchy must not overlap.
 *
 * Paper references are to "Fast Inference via Hierarchical Speculative Decoding": Sec. 2 (speculative
 * sampling rule), Sec. 3 (Alg. 1, Thm 3.1, Thm 3.2), Sec. 4 (Cor. 4.1, HSD problem, reduction),
 * App. B.1 (Alg. 2, Verify).
 */
#ifndef HSD_H
#define HSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { HSD_OK = 0, HSD_EINVAL = -1, HSD_ECAPACITY = -2, HSD_ESTATE = -3, HSD_EHIP = -4 };
enum { HSD_F32 = 0, HSD_BF16 = 1 };
enum { HSD_LAYOUT_TILES = 0, HSD_LAYOUT_ROWS = 1 };
enum { HSD_MAX_LEVELS = 8, HSD_MAX_PASS_ROWS = 64, HSD_KV_PAGE = 64, HSD_MAX_GEMM_ROWS = 4096 };
enum { HSD_STATIC_SAMPLER_MAX_VOCAB = 262144 };   /* largest vocabulary of hsd_accept_resample_static */

typedef struct hsd_model hsd_model;
typedef struct hsd_hier hsd_hier;

/* ---------------------------------------------------------------------------------------------
 * Language model M_i (Sec. 3.2: M_i(context) -> next-token distribution p; an early-exit model is
 * the hidden state after layer i passed through an output head, Sec. 5.1).  Pre-norm decoder:
 * RMSNorm, rotary embedding (half-split pairing, angle pos * base^(-2j/hd)), grouped-query causal
 * attention over a paged KV cache, SwiGLU FFN, final RMSNorm + untied head shared by every exit.
 * ------------------------------------------------------------------------------------------- */
typedef struct {
    int n_layers, d, n_q, n_kv, hd, ffn, vocab;
    int dtype;       /* HSD_F32: fp32 weights, KV and operands (FMA kernels);
                        HSD_BF16: bf16 weights, KV and GEMM operands, fp32 accumulation (MFMA kernels) */
    float rope_base; /* e.g. 10000 */
    float eps;       /* RMSNorm epsilon, inside the square root */
    int max_seq;     /* KV capacity in tokens, multiple of HSD_KV_PAGE */
    int max_rows;    /* most tokens one pass may process, 1..HSD_MAX_PASS_ROWS */
    int rows_copy_layers; /* bf16: the first rows_copy_layers layers (0..n_layers) keep a second, row-major copy of
                        their narrow projections (q/k/v, o, down), which passes of one or two tokens stream with
                        the row kernel.  Meant for the layers the base drafter M_0 runs autoregressively (Alg. 1);
                        costs 45% more weight memory for those layers. */
} hsd_model_desc;

/* Device bytes of the packed weights / the paged KV cache / per-model activation scratch. */
size_t hsd_model_weight_bytes(const hsd_model_desc*);
size_t hsd_model_kv_bytes(const hsd_model_desc*);
size_t hsd_model_scratch_bytes(const hsd_model_desc*);

/* Creates a model over caller-owned device buffers (sizes as above, 256-byte aligned).  Weights are
 * undefined until loaded.  The physical KV page order starts as identity; see hsd_model_set_pages. */
int hsd_model_create(const hsd_model_desc*, void* weights_dev, void* kv_dev, void* scratch_dev,
                     void* stream, hsd_model** out);
void hsd_model_destroy(hsd_model*);

/* Logical weights of one layer, row-major [out_features, in_features], element type = desc.dtype
 * (norm weights always fp32).  The library re-lays them into its streaming format inside
 * weights_dev (MFMA operand tiles; q/k/v fused, gate/up interleaved); the source buffers may be
 * freed after the call returns (it synchronises the stream). */
typedef struct {
    const void *norm1_dev, *wq_dev, *wk_dev, *wv_dev, *wo_dev, *norm2_dev, *wg_dev, *wu_dev, *wd_dev;
} hsd_layer_weights;
int hsd_model_load_layer(hsd_model*, int layer, const hsd_layer_weights*);
/* embed [vocab, d], head [vocab, d] (dtype), norm_f [d] fp32. */
int hsd_model_load_head(hsd_model*, const void* embed_dev, const void* head_dev, const void* norm_f_dev);

/* Physical page of logical KV page i (a permutation of 0..max_seq/HSD_KV_PAGE-1). */
int hsd_model_set_pages(hsd_model*, const int32_t* page_table, int n_pages);

/* One multi-token pass ("run the verifier in parallel on all prefixes", Alg. 2): feeds `m` tokens
 * (device int32) at positions pos0..pos0+m-1 through the first `exit_layer` layers, appends their
 * K/V to the cache (rows < pos0 must already be valid) and, if n_logit_rows > 0, writes the fp32
 * logits of the last n_logit_rows tokens to logits_dev [n_logit_rows, vocab].  1 <= m <= max_rows. */
int hsd_model_pass(hsd_model*, const int32_t* tokens_dev, int pos0, int m, int exit_layer,
                   int n_logit_rows, float* logits_dev);

/* Passes over a batch of sequences (Sec. 3.1: each load of the weights should serve as many tokens as possible; the
 * paper itself decodes one sequence).  hsd_model_set_batch shares the model's KV pages (max_seq / HSD_KV_PAGE of them)
 * out among `batch` sequences: page_table (host) [batch, pages_per_seq] names the physical page of every logical
 * page of every sequence, all entries distinct; batch * pages_per_seq must not exceed the model's pages and batch not
 * max_rows.  batch == 0 returns to one sequence.  Synchronises the stream.
 * hsd_model_pass_batch then feeds tokens_per_seq tokens of every sequence in one pass (batch * tokens_per_seq <=
 * max_rows): tokens_dev (device int32) [batch, tokens_per_seq]; pos0 (host) [batch] the position of each sequence's
 * first token, whose earlier positions must already be cached; each token attends to its own sequence only, causally.
 * with_logits != 0 writes the fp32 logits of every row to logits_dev [batch, tokens_per_seq, vocab].  Row for row the
 * result equals hsd_model_pass of the same sequence alone up to the summation order of the kernels a different row
 * count selects.  The plain hsd_model_pass keeps using the single-sequence page order (hsd_model_set_pages) over the
 * same physical pages: do not mix the two on one cache content. */
int hsd_model_set_batch(hsd_model*, int batch, int pages_per_seq, const int32_t* page_table);
int hsd_model_pass_batch(hsd_model*, const int32_t* tokens_dev, const int32_t* pos0, int tokens_per_seq, int exit_layer,
                         int with_logits, float* logits_dev);

/* The same pass through the deepest of several exits, emitting every listed exit's logits on the way (Sec. 5.1:
 * the output distributions of all candidate layers are recorded during one forward pass): exits = n_exits ascending
 * layer counts; logits_dev [n_exits, n_logit_rows, vocab].  Each exit's rows equal, bit for bit, what
 * hsd_model_pass gives for that exit alone.  bf16 models need ffn >= d (HSD_ECAPACITY otherwise). */
int hsd_model_pass_exits(hsd_model*, const int32_t* tokens_dev, int pos0, int m, const int* exits, int n_exits,
                         int n_logit_rows, float* logits_dev);

/* ---------------------------------------------------------------------------------------------
 * Stand-alone kernels of the path (each is what the pass / the driver launches internally).
 * ------------------------------------------------------------------------------------------- */

/* p = softmax(z / temperature) row-wise, fp32 [rows, vocab]; temperature == 0 writes the one-hot
 * row at the lowest-index maximum.  logits_dev and probs_dev must not overlap.  Vocabularies above 32768 are cut in
 * slices over several workgroups and need scratch_dev of hsd_softmax_scratch_bytes(rows, vocab) bytes (16-byte
 * aligned; 0 bytes and NULL allowed for smaller vocabularies). */
size_t hsd_softmax_scratch_bytes(int rows, int vocab);
int hsd_softmax(const float* logits_dev, float* probs_dev, int rows, int vocab, float temperature,
                void* scratch_dev, void* stream);

/* Bytes of device scratch hsd_accept_resample needs for a vocabulary size. */
size_t hsd_sampler_scratch_bytes(int vocab);

/* Alg. 2 after the verifier pass, fused in one launch.  p_dev: rows p_1..p_{t+1} [t+1, vocab];
 * q_dev: rows q_1..q_t [t, vocab] (ignored when t == 0); x_dev: int32 [t+1], x_1..x_t on entry.
 * For i = 1..t: u_i = top 24 bits of Philox4x32-10(key = seed, counter = (i-1, call, level, 0))
 * word 0, times 2^-24; draft i is accepted iff fl32(u_i * q_i(x_i)) < p_i(x_i); n = number accepted
 * before the first rejection.  The final token m is drawn from max(0, p_{n+1} - q_{n+1}) if n < t,
 * else from p_{t+1}, by the integer rule: w_x = floor(r_x * 2^62), threshold =
 * floor(sum(w) * U / 2^32) with U = word 1 of the block with counter (t, call, level, 0), m = the
 * smallest x whose inclusive prefix sum exceeds the threshold (p_{n+1} alone is used if the residual
 * sums to zero).  Writes result_dev[0] = n, result_dev[1] = m and x_dev[n] = m.  t == 0 draws one
 * token from p_1 (base-level drafting, Alg. 1; bonus-token rule).  scratch_dev must be zero on first
 * use; the kernel leaves it zeroed.  Asynchronous on `stream`. */
int hsd_accept_resample(const float* p_dev, const float* q_dev, int32_t* x_dev, int t, int vocab,
                        uint64_t seed, uint32_t level, uint32_t call, int32_t* result_dev,
                        void* scratch_dev, void* stream);

/* hsd_accept_resample for callers that cannot allocate device memory or bring a workspace: code recording a HIP
 * graph, tight serving loops, harnesses that forbid hipMalloc.  Same arguments minus scratch_dev, same results bit
 * for bit.  The ticket and slice totals that hsd_accept_resample keeps in scratch_dev live in an array built into
 * the library's device code (about 2 KiB per GPU, resolved on the first call on each device and held until the
 * process ends), which bounds the vocabulary: vocab > HSD_STATIC_SAMPLER_MAX_VOCAB returns HSD_ECAPACITY.  The call
 * allocates and frees nothing, on the device or through the runtime; it launches a small kernel that clears the
 * ticket (no memset, so it may be recorded into a graph) and then the sampler kernel, on `stream` of the current
 * device.  All calls on one GPU share that array: two calls whose kernels may overlap (different streams, no
 * ordering between them) race on it and give undefined results; calls on one stream, or otherwise ordered, are
 * safe.  Asynchronous on `stream`. */
int hsd_accept_resample_static(const float* p_dev, const float* q_dev, int32_t* x_dev, int t, int vocab,
                               uint64_t seed, uint32_t level, uint32_t call, int32_t* result_dev, void* stream);

/* hsd_softmax over the verifier's t+1 logit rows followed by hsd_accept_resample, in ONE launch (what the driver
 * runs after a verifier pass, and after a base-level drafting pass with t == 0; Alg. 1 and Alg. 2): one workgroup
 * per row keeps the row in registers from the logits to the drawn token.  Same arguments and the same results, bit
 * for bit, as the two calls in sequence: logits_dev [t+1, vocab] fp32; probs_dev [t+1, vocab] receives the rows
 * p_1..p_{t+1} (may be null when they are not needed afterwards).  Vocabularies up to 32768 only (HSD_ECAPACITY
 * beyond; use the two calls).  host_mailbox, if not null, is device-accessible pinned host memory of at least
 * (t + 3) int32 that receives n, m, then the n accepted draft ids followed by m, readable after the stream has
 * been synchronised.  scratch_dev as for hsd_accept_resample. */
int hsd_softmax_verify(const float* logits_dev, const float* q_dev, int32_t* x_dev, int t, int vocab,
                       float temperature, uint64_t seed, uint32_t level, uint32_t call, float* probs_dev,
                       int32_t* result_dev, void* scratch_dev, int32_t* host_mailbox, void* stream);

/* Acceptance rate of one context between every pair of n_dists distributions (Sec. 2: sum_x min(p(x), q(x)) =
 * 1 - TV(p, q)): rows_dev [n_dists, n_rows, vocab] fp32; out_dev [n_dists (n_dists - 1) / 2, n_rows] fp64, pairs
 * (i < j) in the order (0,1), (0,2), .., (1,2), ..; sums in fp64 in a fixed order.  2 <= n_dists <= 64. */
int hsd_overlap(const float* rows_dev, int n_dists, int n_rows, int vocab, double* out_dev, void* stream);

/* Calibration pass of Sec. 5.1: teacher-forced run of the model over tokens_dev [n_tokens] (device int32); the first
 * n_ctx positions are context only, every later position contributes the distributions of all listed exits
 * (hsd_model_pass_exits, softmax at `temperature`) to alpha_out [n_exits, n_exits] (host, row-major, symmetric, unit
 * diagonal) = mean over those positions of hsd_overlap: the empirical pairwise acceptance rates, which satisfy
 * alpha_ij + alpha_jk <= alpha_ik + 1.  If cost_ms_out (host, [n_exits]) is not null it receives the mean time of
 * a pass of cost_rows tokens at the end of the sequence through each exit (the costs c_i of Sec. 3.2).  Overwrites
 * the model's KV cache for positions 0..n_tokens-1; synchronises the model's stream.  Workspace from
 * hsd_calibrate_workspace_bytes (0 on bad arguments). */
size_t hsd_calibrate_workspace_bytes(const hsd_model*, int n_exits, int n_tokens, int n_ctx);
int hsd_calibrate(hsd_model*, const int* exits, int n_exits, const int32_t* tokens_dev, int n_tokens, int n_ctx,
                  float temperature, int cost_rows, void* workspace_dev, size_t workspace_bytes, double* alpha_out,
                  double* cost_ms_out);

/* The same calibration over candidates that may be different networks (Sec. 3.2: the models of a hierarchy share only
 * the vocabulary): levels = n candidates (model, exit layer) in the order the selection should number them, exits of
 * one network in ascending order; every network is teacher-forced over tokens_dev, the first n_ctx positions through
 * its deepest listed exit only; alpha_out [n, n] and cost_ms_out [n] (may be null) as for hsd_calibrate, indexed by
 * candidate.  Overwrites every listed network's KV cache for positions 0..n_tokens-1 (so it doubles as the prefill of
 * a hierarchy built from the candidates on the same tokens); synchronises the stream.  hsd_level is declared below. */
struct hsd_level_;
size_t hsd_calibrate_levels_workspace_bytes(int n, const struct hsd_level_* levels, int n_tokens, int n_ctx);
int hsd_calibrate_levels(int n, const struct hsd_level_* levels, const int32_t* tokens_dev, int n_tokens, int n_ctx,
                         float temperature, int cost_rows, void* workspace_dev, size_t workspace_bytes,
                         double* alpha_out, double* cost_ms_out);

/* k-query attention over a paged KV cache, for a batch of sequences (the pass uses it with batch 1).
 * One layer's cache: hsd_kv_layer_bytes(n_pages, ...) bytes; pages_dev [batch, max_pages] int32 gives the physical
 * page (HSD_KV_PAGE positions) of each logical page of each sequence.  hsd_kv_write stores logical K/V
 * [batch, n, n_kv, hd] (dtype) at positions pos0_dev[b] .. pos0_dev[b] + n - 1 in the cache's internal layout.
 * hsd_attention: q_dev [batch, m, n_q, hd] are the queries of the m newest tokens of every sequence, whose K/V
 * must already be in the cache at positions pos0_dev[b] .. pos0_dev[b] + m - 1; query i attends to positions
 * 0 .. pos0_dev[b] + i (causal among the new tokens), scores scaled by 1/sqrt(hd).  att_dev [batch, m, n_q, hd]
 * (dtype).  max_len >= every pos0_dev[b] + m bounds the launch.  workspace_dev:
 * hsd_attention_workspace_bytes(batch, m, n_q, n_kv, hd, max_len) bytes, 256-byte aligned, zero on first use (it
 * begins with arrival counters of the workgroups that share a sequence; the kernels leave them zeroed). */
size_t hsd_kv_layer_bytes(int n_pages, int n_kv, int hd, int dtype);
size_t hsd_attention_workspace_bytes(int batch, int m, int n_q, int n_kv, int hd, int max_len);
int hsd_kv_write(void* kv_layer_dev, const int32_t* pages_dev, int max_pages, const int32_t* pos0_dev, int batch, int n,
                 int n_kv, int hd, int dtype, const void* k_dev, const void* v_dev, void* stream);
int hsd_attention(const void* q_dev, const void* kv_layer_dev, const int32_t* pages_dev, int max_pages,
                  const int32_t* pos0_dev, int batch, int m, int max_len, int n_q, int n_kv, int hd, int dtype,
                  void* att_dev, void* workspace_dev, void* stream);

/* Small-M weight-streaming GEMM y = x W^T, y_dev [m, n] fp32 = x_dev [m, k] (dtype) times W [n, k].
 * hsd_pack_weight copies W (row-major, dtype) into the streaming format (packed_dev:
 * hsd_packed_bytes(n, k, dtype)).  bf16 has two formats, each with its kernel, both used by the pass:
 *   HSD_LAYOUT_TILES - MFMA operand tiles; workgroups own 16-column tiles (wide matrices: gate/up, head);
 *   HSD_LAYOUT_ROWS  - row-major; workgroups own 2-4 output features and use packed bf16 dot products
 *                      (narrow matrices: q/k/v, attention output, FFN down), m above 16 in several launches.
 * fp32 ignores the layout.  k must be a multiple of 32, 1 <= m <= HSD_MAX_GEMM_ROWS.
 * Above HSD_MAX_PASS_ROWS rows (a batch of sequences times their drafted tokens, the batched cells of the layer
 * microbenchmark; Sec. 3.1: each load of the weights should serve as many tokens as possible) the tiled bf16 format
 * is served by a kernel tiled for the matrix cores, which bound the time from a few hundred rows on (128 x 256 or
 * 128 x 128 of the output per workgroup, activations through LDS), or, as a tuning alternative, by one weight stream
 * per 64 rows; the results are the same sums of exact products in fp32, in a different order.
 * workspace_dev: hsd_gemm_workspace_bytes(m, n, k). */
size_t hsd_packed_bytes(int n, int k, int dtype);
size_t hsd_gemm_workspace_bytes(int m, int n, int k);
int hsd_pack_weight(const void* w_dev, void* packed_dev, int n, int k, int dtype, int layout, void* stream);
int hsd_gemm(const void* x_dev, const void* packed_dev, float* y_dev, int m, int n, int k, int dtype, int layout,
             void* workspace_dev, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Hierarchy M_0..M_K with parameters T_0..T_{K-1} (Alg. 1).  Level 0 drafts autoregressively,
 * level K is the target.  Levels that name the same hsd_model are early exits of one network and
 * share its KV cache; all levels must share the vocabulary (Sec. 2).
 * ------------------------------------------------------------------------------------------- */
typedef struct hsd_level_ {
    hsd_model* model;
    int exit_layer;        /* 1..n_layers */
} hsd_level;

size_t hsd_hier_workspace_bytes(int n_levels, const hsd_level* levels, const int* T);

/* T has n_levels-1 entries, each >= 1.  temperature 0 = greedy (one-hot rows).  seed keys every
 * Philox draw: counter = (slot, call, level, 0) where call counts the level's Verify calls (draft
 * steps for level 0). */
int hsd_hier_create(int n_levels, const hsd_level* levels, const int* T, float temperature,
                    uint64_t seed, void* workspace_dev, size_t workspace_bytes, void* stream,
                    hsd_hier** out);
void hsd_hier_destroy(hsd_hier*);

/* Resets the hierarchy to the context `prompt` (n >= 1 tokens): fills every model's KV cache for
 * prompt[0..n-2]; the last prompt token is fed by the first pass of each level.  Counters restart. */
int hsd_prefill(hsd_hier*, const int32_t* prompt, int n);
/* hsd_prefill for a prompt whose first n_cached tokens (0 <= n_cached <= n-1) already have their K/V in the cache of
 * every network of the hierarchy, through at least the deepest exit the hierarchy uses of it: left there by another
 * hierarchy over the same networks, or by hsd_calibrate_levels, on the same tokens (the caller's responsibility; the
 * library cannot check it).  Only tokens n_cached..n-2 are fed.  Lets several hierarchies over one set of networks
 * share one prefill of a long prompt. */
int hsd_prefill_cached(hsd_hier*, const int32_t* prompt, int n, int n_cached);
/* Drops everything after the first n tokens of the sequence (n >= 1) and restarts the Philox call
 * counters and statistics, keeping the KV cache of the first n-1 tokens: used to repeat a
 * generation from the same prompt without repeating the prefill. */
int hsd_rewind(hsd_hier*, int n);
/* Replaces the seed that keys every later Philox draw of the hierarchy (Alg. 2's u_i and sampling draws, the noise of
 * synthetic drafters); counters and sequence stay as they are.  With hsd_rewind: the same prompt continued along
 * another sample path. */
int hsd_hier_set_seed(hsd_hier*, uint64_t seed);

/* Base case of Alg. 1 (draft(level, k) of the problem statement): `level` generates k tokens autoregressively after
 * the current sequence.  Only the lowest level drafts in Alg. 1, so level must be 0 (HSD_EINVAL otherwise; a higher
 * level produces tokens through hsd_run).  tokens_out (cap k, may be NULL) receives them; *probs_dev_out the k
 * distribution rows [k, vocab] (borrowed, valid until the level's next draft). */
int hsd_draft(hsd_hier*, int level, int k, int32_t* tokens_out, const float** probs_dev_out);

/* Verify (Alg. 2) at `level` >= 1: the last t tokens of the sequence are the drafts x_1..x_t; if
 * draft_tokens != NULL they are first appended to the sequence from this host array.
 * draft_probs_dev: rows q_1..q_t.  Runs the level's pass over its uncached tokens, the rejection
 * rule and the corrected / bonus draw.  tokens_out (cap t+1): x_1..x_n, m; *n_out = n+1;
 * *probs_dev_out: rows p_1..p_{n+1} (borrowed, valid until the level's next verify with
 * append == 0).  append != 0 stores the rows after those of the level's previous verify (how an
 * intermediate level collects its batch in Alg. 1).  The sequence afterwards ends with m and every
 * level at or below `level` forgets KV beyond the accepted prefix. */
int hsd_verify(hsd_hier*, int level, const int32_t* draft_tokens, const float* draft_probs_dev, int t,
               int append, int32_t* tokens_out, int* n_out, const float** probs_dev_out);

/* HSD(level, context) of Alg. 1 for any level (level = K: one round of the target).  tokens_out
 * receives the tokens the call appended (at least T_level for an intermediate level), *n_out their
 * number, *probs_dev_out their distribution rows (may be NULL). */
int hsd_run(hsd_hier*, int level, int32_t* tokens_out, int cap, int* n_out, const float** probs_dev_out);

typedef struct {
    int64_t passes[HSD_MAX_LEVELS];    /* forward passes per level */
    int64_t pass_rows[HSD_MAX_LEVELS]; /* tokens fed, summed over passes */
    int64_t drafted[HSD_MAX_LEVELS];   /* draft tokens offered to the level's Verify */
    int64_t accepted[HSD_MAX_LEVELS];  /* of those, accepted */
    int64_t tested[HSD_MAX_LEVELS];    /* accept tests evaluated (up to and including the first rejection of a call):
                                          accepted / tested is the per-test acceptance frequency */
    int64_t reused_rows[HSD_MAX_LEVELS]; /* rows of the level's passes that resumed from the hidden states kept by the level
                                          below instead of recomputing the shallower layers (hsd_hier_set_reuse) */
    int64_t rounds;                    /* HSD(K, .) calls */
    int64_t tokens;                    /* tokens emitted by the target level */
} hsd_stats;

/* Calls HSD(K, .) until n_tokens are produced; the last round is cut at n_tokens (the sequence keeps
 * the surplus).  out: cap n_tokens.  stats may be NULL. */
int hsd_generate(hsd_hier*, int n_tokens, int32_t* out, hsd_stats* stats);

/* ---------------------------------------------------------------------------------------------
 * HSD over a batch of sequences in lockstep.  The paper decodes one sequence (Sec. 5: batch size 1); its own
 * argument for drafting (Sec. 3.1: a pass costs the weights it loads, however many tokens it scores) extends across
 * sequences, so one pass of a level here feeds the pending tokens of every sequence that is at that point of
 * Alg. 1.  Every sequence b is decoded exactly as hsd_generate would decode it alone with seed seeds[b]: its own
 * Philox counters, Verify calls (Alg. 2) and cached lengths; the results differ from that run only by the summation
 * order of kernels chosen for another row count.  An intermediate level repeats (level below, Verify) while any
 * of its sequences is short of T_level tokens; sequences that have theirs, or have generated what was asked, sit the
 * pass out as padding rows after their last token (attention is causal: padding never reaches a real row, and
 * its K/V lands beyond the valid length).
 *
 * hsd_batch_create shares each network's KV pages out among the sequences (hsd_model_set_batch: sequence b owns
 * pages [b, b + 1) * max_len / HSD_KV_PAGE), so every model needs max_seq >= batch * max_len, and a pass of
 * batch * (most drafts of a Verify + 2) rows must fit the models' max_rows.  The models must not be used by another
 * hierarchy meanwhile.  workspace_dev: hsd_batch_workspace_bytes bytes, 256-byte aligned, caller-owned.
 * hsd_batch_prefill: prompts (host) [batch, stride], lens[b] tokens each (ragged prompts allowed).
 * hsd_batch_generate: n_tokens more tokens of every sequence, out (host) [batch, n_tokens]; stats (may be NULL) count
 * passes once per batched pass, rows / drafted / accepted / tested summed over the sequences, tokens over all of them.
 * Not supported here: the ablation switches, synthetic drafters, hidden-state reuse.
 * ------------------------------------------------------------------------------------------- */
typedef struct hsd_batch hsd_batch;
size_t hsd_batch_workspace_bytes(int n_levels, const hsd_level* levels, const int* T, int batch, int max_len);
int hsd_batch_create(int n_levels, const hsd_level* levels, const int* T, int batch, int max_len, float temperature,
                     const uint64_t* seeds, void* workspace_dev, size_t workspace_bytes, void* stream, hsd_batch** out);
void hsd_batch_destroy(hsd_batch*);
int hsd_batch_prefill(hsd_batch*, const int32_t* prompts, int stride, const int* lens);
int hsd_batch_generate(hsd_batch*, int n_tokens, int32_t* out, hsd_stats* stats);
int hsd_batch_sequence_length(const hsd_batch*, int sequence);

/* Hidden-state reuse between early exits of one network (Sec. 5.1: the drafters of the paper's main workload are
 * earlier exits of the target).  Where the level below a verifier is a shallower exit of the verifier's own network,
 * every pass through that exit's layer keeps its residual rows by position, and with on != 0 the verifier's pass sends
 * only the tokens no pass has seen yet (the newest draft or the token a Verify has just emitted) through the shallower
 * layers and resumes all its rows above them.  The weights of the shallower layers are streamed either way (the newest
 * token needs them), so at batch 1 this saves arithmetic and activation traffic, not weight traffic.  Results: the
 * same distributions up to the summation order of kernels chosen for a different row count (fp32 storage: bit for
 * bit).  Default off.  Takes effect from the next pass. */
int hsd_hier_set_reuse(hsd_hier*, int on);

/* The two simplifications the latency analysis makes, as switches (appendix "Examining the assumptions of HSD";
 * Thm 3.2).  coin: NULL restores Alg. 2's accept test; otherwise [n_levels] floats, entry i in [0, 1] makes level
 * i's Verify accept every draft with that fixed probability (u_i < coin[i], same Philox word; the corrected / bonus
 * token is drawn as before), a negative entry keeps the real test at that level, entry 0 is ignored.
 * exactly_T != 0: an intermediate level hands up exactly T_idx tokens and drops what it collected beyond (the
 * variant Thm 3.2's formula describes literally).  Takes effect from the next hsd_run / hsd_generate. */
int hsd_hier_set_ablation(hsd_hier*, const float* coin, int exactly_T);

/* Synthetic drafter (workload construction for hierarchies of random-init networks, whose distributions would
 * otherwise overlap by chance only; Sec. 5 works with drafters whose acceptance rates are 0.6-0.9): level `level`
 * (below the target) still runs its own pass, which is what it costs and what the statistics count, but takes as
 * its logits those of level `source_level` (above it) at the same contexts plus
 * noise_std * n(level, position, vocabulary entry), n standard normal from Philox4x32-10 blocks with counter
 * (entry / 4, position, level | 2^31, 0x4E4F4953) by Box-Muller.  The source may be synthetic itself: then its logits
 * are its own source's plus its own noise, and so on up to a real network, so that a chain of sources gives levels
 * that each differ from the next one up by one noise term (neighbouring levels close, distant ones less so: the
 * structure a hierarchy exploits, Sec. 3.2).  The side passes of the real network at the chain's end are not counted,
 * so only the fixed-cost accounting (hsd_stats_cost) is meaningful for such a run, not its wall-clock time.
 * source_level < 0 switches it off. */
int hsd_hier_set_distilled(hsd_hier*, int level, int source_level, float noise_std);

/* sum_i passes[i] * cost[i] over the first n_levels levels: the "artificial cost" accounting of the same appendix
 * (a fixed cost per forward pass instead of measured time). */
double hsd_stats_cost(const hsd_stats*, int n_levels, const double* cost);
int hsd_get_stats(const hsd_hier*, hsd_stats*);
int hsd_sequence_length(const hsd_hier*);

/* c_i of Sec. 3.2 measured on the device: mean milliseconds of `iters` passes of `level` over the
 * last m tokens of the current sequence (m-1 "drafts" + the token before them; state unchanged). */
int hsd_measure_pass(hsd_hier*, int level, int m, int iters, double* ms_out);

/* ---------------------------------------------------------------------------------------------
 * Host-side latency model and hierarchy selection (Sec. 3.3, Sec. 4).  No GPU involved.
 * ------------------------------------------------------------------------------------------- */

/* gamma(alpha, T_i, T_j) of Sec. 3.3: expected draft+verify rounds for a level that needs T_j tokens
 * and is fed T_i drafts per round, acceptances IID with rate alpha. */
double hsd_gamma(double alpha, int Ti, int Tj);

/* Expected latency per token of the hierarchy with costs c_0..c_K (n = K+1 entries), adjacent
 * acceptance rates alpha_{i,i+1} (n-1 entries) and T (n-1 entries).  exact_overshoot == 0: Thm 3.2 /
 * Cor. 4.1 as printed; != 0: expectation of Alg. 1 as written, where a level hands up every token it
 * collected (at least T_idx).  Returns a negative value on invalid arguments. */
double hsd_expected_latency(int n, const double* cost, const double* alpha_adj, const int* T,
                            int exact_overshoot);

/* HSD problem of Sec. 4.2: min over ordered subsets sigma ending in the target (model n_models-1)
 * and T in [1, Tbar] of the Cor. 4.1 latency.  alpha is n_models x n_models row-major, entries
 * i < j used.  monotone_T != 0 keeps the paper's edge set (a level's T is >= the T of the level
 * below).  sigma_out (cap n_models) ascending model indices, T_out (cap n_models-1), *n_sigma their
 * count (1 = plain decoding is best). */
int hsd_select_hierarchy(int n_models, const double* cost, const double* alpha, int Tbar, int monotone_T,
                         int* sigma_out, int* T_out, int* n_sigma, double* latency_out);

/* Single-draft baseline of Sec. 5.2: best (drafter, T) under the K = 1 closed form.  *drafter_out = -1
 * when plain decoding is best. */
int hsd_best_single_draft(int n_models, const double* cost, const double* alpha, int Tbar,
                          int* drafter_out, int* T_out, double* latency_out);

const char* hsd_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* HSD_H */
