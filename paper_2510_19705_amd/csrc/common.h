// Shared declarations of libhsd's translation units (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>

#include "../../include/hsd_dev.h"

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;

void hsd_set_error(const char* fmt, ...);

#define HSD_FAIL(code, ...)            \
    do {                               \
        hsd_set_error(__VA_ARGS__);    \
        return (code);                 \
    } while (0)

#define HSD_HIP(expr)                                                                           \
    do {                                                                                        \
        hipError_t e_ = (expr);                                                                 \
        if (e_ != hipSuccess) HSD_FAIL(HSD_EHIP, "%s: %s", #expr, hipGetErrorString(e_));       \
    } while (0)

#define HSD_LAUNCH_CHECK()                                                                      \
    do {                                                                                        \
        hipError_t e_ = hipGetLastError();                                                      \
        if (e_ != hipSuccess) HSD_FAIL(HSD_EHIP, "kernel launch: %s", hipGetErrorString(e_));   \
    } while (0)

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
static inline size_t dtype_size(int dtype) { return dtype == HSD_BF16 ? 2 : 4; }

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// ---- KV cache geometry (kernels_attn.hip, kernels_layer.hip) ---------------------------------
// Per layer, per physical page, per KV head: a K block then a V block of HSD_KV_PAGE * hd elements.
// fp32: natural [pos][hd].  bf16: MFMA operand tiles, see kv_k_index / kv_v_index.
__host__ __device__ __forceinline__ size_t kv_block_elems(int hd) { return (size_t)HSD_KV_PAGE * hd; }
__host__ __device__ __forceinline__ size_t kv_page_elems(int n_kv, int hd) { return 2 * n_kv * kv_block_elems(hd); }

// K element (pos in page, d) of a bf16 block: tiles of 16 positions x 32 dims, 512 elements each, in
// the lane order of the 16x16x32 MFMA A operand: lane = pos%16 + 16*((d%32)/8), element d%8.
__host__ __device__ __forceinline__ int kv_k_index(int pos, int d, int hd) {
    int tile = (pos >> 4) * (hd >> 5) + (d >> 5);
    int lane = (pos & 15) + 16 * ((d & 31) >> 3);
    return tile * 512 + lane * 8 + (d & 7);
}
// V element (pos in page, d): tiles of 32 positions x 16 dims in the lane order of the A operand of
// O^T += V^T P^T, with the position order that matches the accumulator layout of S^T = K Q^T:
// within a 32-block, position q = 16*half + 4*g + r sits in lane group g, element r + 4*half.
__host__ __device__ __forceinline__ int kv_v_index(int pos, int d, int hd) {
    int tile = (pos >> 5) * (hd >> 4) + (d >> 4);
    int q = pos & 31, half = q >> 4, g = (q & 15) >> 2, r = q & 3;
    int lane = (d & 15) + 16 * g;
    return tile * 512 + lane * 8 + r + 4 * half;
}

// ---- Packed weight geometry (kernels_gemm.hip) ------------------------------------------------
// W [n, k] bf16 -> tiles of 16 rows x 32 columns in the lane order of the 16x16x32 MFMA B operand,
// tile (nt, kt) at ((nt * k/32) + kt) * 512, lane = n%16 + 16*((k%32)/8), element k%8.  Rows are
// padded to a multiple of 16 with zeros.  fp32 weights stay row-major.
__host__ __device__ __forceinline__ size_t packed_index(int n, int k, int K) {
    size_t tile = (size_t)(n >> 4) * (K >> 5) + (k >> 5);
    int lane = (n & 15) + 16 * ((k & 31) >> 3);
    return tile * 512 + lane * 8 + (k & 7);
}

// ---- GEMM launch interface (kernels_gemm.hip) ---------------------------------------------------
enum { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_ROPE = 3 };   // epilogue
enum { SS_SLOTS = 16 };   // accumulators per row for the sums of squares (spreads the atomics)

struct GemmArgs {
    const bf16_t* a;                    // activations [M, K]
    const bf16x8* wp;                   // W [N, K]: MFMA tiles (launch_gemm_bf16) or row-major (launch_gemv_bf16)
    int M, N, K;
    float* part;                        // split-K partial tiles (ksplit > 1)
    size_t part_bytes;                  // capacity of `part`: a plan that needs more runs unsplit
    int* tickets;                       // one arrival counter per column group, zero between launches
    int rotate;                         // set by the launcher: every workgroup walks its k-steps from its own offset (with interleave)
    int interleave;                     // set by the launcher from the plan: waves take the k-steps round-robin instead of contiguous slices
    int halves;                         // set by the launcher from the plan: workgroup b owns columns 8 (b & 1) .. + 8 of the tiles of group b >> 1
    // consumers of a normalised input: rows of `a` are x * w_norm, the 1/rms factor is applied in the epilogue
    const unsigned long long* ss_in;    // [SS_SLOTS][HSD_MAX_PASS_ROWS]: per row, sum of squares of x times 2^24, spread over the
                                        // slots; null: no scaling (EPI_STORE only)
    unsigned long long* ss_zero;        // accumulator the next producer will add into (cleared here), or null
    float eps;
    // outputs
    float* out_f32;                     // EPI_STORE: y [M, N]; EPI_RESID: residual rows [M, N], updated in place
    float* tap;                         // EPI_RESID: if not null, the new residual rows are also stored here [M, N] (hidden states
                                        // kept for a deeper exit of the same network to resume from)
    unsigned long long* ss_out;         // EPI_RESID: per row, += sum of squares of the new residual times 2^24
    const float* norm_w;                // EPI_RESID: weight of the norm that reads the new residual
    bf16_t* out_bf16;                   // EPI_RESID: bf16(new residual * norm_w) [M, N] (or null); EPI_SWIGLU: h [M, N/2];
                                        // EPI_ROPE: q [M, n_q, hd]
    bf16_t* kv_layer;                   // EPI_ROPE: this layer's KV pages
    const int32_t* pages;
    int pos0, n_q, n_kv, hd;
    float rope_base;
    // EPI_ROPE over a batch of sequences: row ml is token ml % m_seq of sequence ml / m_seq, at position
    // pos0_arr[sequence] + ml % m_seq, with the sequence's page table at pages + sequence * max_pages.
    // pos0_arr == null: one sequence, row ml at position pos0 + ml.
    const int32_t* pos0_arr;
    int m_seq, max_pages;
};

// position and page table of row ml under the geometry above
__device__ __forceinline__ int gemm_row_position(const GemmArgs& g, int ml, const int32_t** ptab) {
    if (!g.pos0_arr) {
        *ptab = g.pages;
        return g.pos0 + ml;
    }
    const int b = ml / g.m_seq;
    *ptab = g.pages + (size_t)b * g.max_pages;
    return g.pos0_arr[b] + ml % g.m_seq;
}

struct GemmPlan {
    int nt;       // 16-column tiles per workgroup
    int ksplit;   // workgroups along K per column group
    int waves;    // waves per workgroup; they split the workgroup's K slice
    int halves;   // 1: two workgroups per column group, each owning 8 of the 16 columns of its tiles (ksplit = 1 only)
    int deep;     // 1 / -1: the deeper / shallower load batches whatever K; 0: by K
    int interleave;   // 2, 4, 8: groups of that many waves take the k-steps of the group's run round-robin; 0, 1: contiguous slices
};
const hsd_kernel_tuning& default_kernel_tuning();
const hsd_driver_tuning& default_driver_tuning();
GemmPlan gemm_plan(int m, int n, int k, int epi, const hsd_kernel_tuning& t = default_kernel_tuning());
size_t gemm_part_bytes(int m, int n, int k, int epi);
int launch_gemm_bf16(const GemmArgs& g, int epi, const GemmPlan& p, hipStream_t s);   // W in MFMA tiles
void gemm_kernel_name(int m, int k, int epi, const GemmPlan& p, char* out, size_t cap);
int launch_gemv_bf16(const GemmArgs& g, int epi, hipStream_t s);   // row-major W: EPI_STORE, EPI_RESID, EPI_ROPE
// more than 64 rows, W in MFMA tiles, plain store (kernels_gemm_wide.hip)
int launch_gemm_wide_bf16(const bf16_t* a, const bf16x8* wp, float* out, int m, int n, int k, int wide_cols, hipStream_t s);
int launch_gemm_f32(const float* x, const float* w, float* out, int m, int n, int k, bool swiglu, hipStream_t s);
// interleave: 0 plain rows at row_offset, 1 / 2 gate / up of a fused SwiGLU matrix, 3 attention heads of hd rows
// with each 16-dim block followed by the block of its RoPE partners, 4 heads with each dim followed by its partner.
// rows_layout: bf16 destination row-major instead of MFMA tiles.
int launch_pack(const void* w, void* packed, int n, int k, int dtype, int row_offset, int interleave, int hd, int rows_layout,
                hipStream_t s);
