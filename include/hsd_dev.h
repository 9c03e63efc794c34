/*
 * libhsd - development instruments: per-site timing for roofline accounting, and the launch heuristics of the
 * kernels as per-object settings for tuning sweeps.  Nothing here is needed to run the method; see hsd.h for the
 * interface (draft, verify, the round driver, selection).  Conventions as in hsd.h.
 */
#ifndef HSD_DEV_H
#define HSD_DEV_H

#include "hsd.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-site device timing of a model's passes, for roofline accounting.  Between begin and end every
 * launch at the sites below is bracketed by two events on the model's stream (up to max_launches
 * launches, later ones are not timed; the brackets add a little host and device overhead, so throughput
 * is measured without them).  end synchronises the stream and returns launches and total
 * milliseconds per site (raw: subtract launches * empty_bracket_ms for the kernels alone). */
enum { HSD_SITE_QKV = 0, HSD_SITE_ATTN = 1, HSD_SITE_O = 2, HSD_SITE_GATEUP = 3, HSD_SITE_DOWN = 4, HSD_SITE_HEAD = 5,
       HSD_N_SITES = 6 };
typedef struct {
    int64_t launches[HSD_N_SITES];
    double ms[HSD_N_SITES];
    double empty_bracket_ms; /* mean time between the two events of a bracket with nothing inside, measured by
                                hsd_profile_end on the same stream: what a bracket adds to the launch it times */
} hsd_site_times;
int hsd_profile_begin(hsd_model*, int max_launches);
int hsd_profile_end(hsd_model*, hsd_site_times* out);
/* Mean duration, in microseconds, of one launch of a layer site (bf16 models; HSD_SITE_QKV .. HSD_SITE_DOWN) in the
 * configuration a pass of `rows` tokens at position pos0 uses: `iters` launches
 * back to back between two events on the model's stream, cycling through the layers so that every launch streams
 * different weights.  Inputs are whatever the last pass left in the activation buffers; the residual stream and the KV
 * rows at pos0.. are overwritten, so run a pass before trusting the model's state again. */
int hsd_measure_site(hsd_model*, int site, int rows, int pos0, int iters, double* us_out);

/* Name of the kernel instance (as a profiler prints it, e.g. "gemm_bf16_kernel<2, 1, 2, true>") that a pass of
 * `rows` tokens launches at a projection site (HSD_SITE_QKV, _O, _GATEUP, _DOWN, _HEAD) of a bf16 model, in layers
 * without row-major copies: lets a measurement be matched with a profile of the same kernel. */
int hsd_site_kernel(const hsd_model*, int site, int rows, char* name_out, int cap);

/* ---------------------------------------------------------------------------------------------
 * Launch heuristics as settings of one model / one hierarchy / one stand-alone call (never process-wide).
 * hsd_kernel_tuning_default / hsd_driver_tuning_default fill in the library's own choices; a field left at its
 * default keeps the heuristic.
 * ------------------------------------------------------------------------------------------- */
typedef struct {
    int gemm_nt[4];          /* per epilogue kind (0 store, 1 residual, 2 SwiGLU, 3 RoPE: 2 or 4 only): 16-column tiles
                                per workgroup of the tiled GEMM, 0 = heuristic */
    int gemm_ksplit[4];      /* per epilogue kind: workgroups along K (partial tiles exchanged through memory), 0 = heuristic */
    int gemm_deep;           /* 1 / -1: twice / once the loads per batch whatever K; 0 = by K */
    int gemm_interleave[4];  /* per epilogue kind: 2, 4 or 8: groups of that many waves of a workgroup take the 32-wide
                                k-steps of their part of K round-robin (8: the workgroup's requests of a round are one
                                contiguous run per tile); -1 or 1: each wave takes a contiguous slice of K; 0 = heuristic */
    int gemv_max_m_qkv, gemv_max_m_o, gemv_max_m_down;   /* most tokens of a pass that a projection with a row-major copy
                                serves with the row kernel (defaults 0, 1, 2) */
    int halves_max_groups;   /* residual / RoPE projections of at most this many column groups get two workgroups per
                                group in passes of few rows, each owning half of the columns of its tiles (default 128;
                                0 switches the scheme off) */
    int attn_qt1_rows;       /* most query rows per KV head for which every workgroup of the MFMA attention takes one
                                16-row query tile; above it, two (default: always one) */
    int attn_steps_per_wave; /* > 0: K/V steps per wave the attention plans for when it splits a sequence (default 0:
                                about attn_target_wgs workgroups) */
    int attn_target_wgs;     /* workgroups a split attention launch aims for (default 256) */
    int attn_fused_merge;    /* 0: the splits of a sequence are always merged by a second launch (default 1: by the last
                                workgroup to arrive when there are very few rows) */
    int wide_min_rows;       /* hsd_gemm above HSD_MAX_PASS_ROWS rows: fewest rows served by the kernel tiled for the matrix
                                cores, fewer stream the weights once per 64 rows (default 0: every such call) */
    int wide_cols;           /* 128 or 256 columns per workgroup of that kernel (default 0: 256 unless that leaves half
                                the CUs idle) */
} hsd_kernel_tuning;

typedef struct {
    int fused_sampler_max_v; /* largest vocabulary the driver hands to the fused softmax + verify launch (default and
                                limit 32768); smaller values send small vocabularies down the two-launch path */
    int preembed;            /* 0: the fused sampler does not embed the token it emits for the one-token pass that
                                follows (default 1; same results either way) */
    int poll_mailbox;        /* 0: the driver synchronises the stream after each Verify instead of polling the sampler's
                                sequence number in pinned host memory (default 1; same results either way) */
} hsd_driver_tuning;

void hsd_kernel_tuning_default(hsd_kernel_tuning*);
void hsd_driver_tuning_default(hsd_driver_tuning*);
/* Settings of every later pass of the model / every later call on the hierarchy (NULL restores the defaults). */
int hsd_model_set_tuning(hsd_model*, const hsd_kernel_tuning*);
int hsd_hier_set_tuning(hsd_hier*, const hsd_driver_tuning*);
/* hsd_gemm / hsd_attention (hsd.h) under the given settings. */
int hsd_gemm_tuned(const void* x_dev, const void* packed_dev, float* y_dev, int m, int n, int k, int dtype, int layout,
                   void* workspace_dev, void* stream, const hsd_kernel_tuning*);
int hsd_attention_tuned(const void* q_dev, const void* kv_layer_dev, const int32_t* pages_dev, int max_pages,
                        const int32_t* pos0_dev, int batch, int m, int max_len, int n_q, int n_kv, int hd, int dtype,
                        void* att_dev, void* workspace_dev, void* stream, const hsd_kernel_tuning*);

#ifdef __cplusplus
}
#endif
#endif /* HSD_DEV_H */
