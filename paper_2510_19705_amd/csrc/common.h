// Shared declarations of libhsd's translation units (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>

#include "../../include/hsd.h"

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
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

// ---- launchers shared between translation units ----------------------------------------------
struct GemmPlan {
    int ksplit;     // cross-workgroup split of K; partial sums land in [ksplit][m][n] fp32
    int nt;         // 16-column tiles per workgroup
    int waves;      // waves per workgroup (they split the workgroup's K range)
};
GemmPlan gemm_plan(int m, int n, int k, int dtype, bool swiglu);
// y partials [ksplit][m][n] fp32 = x [m,k] (dtype) * packed W^T
int launch_gemm(const void* x, const void* wp, float* part, int m, int n, int k, int dtype, const GemmPlan& p,
                hipStream_t s);
// h [m, f] (dtype) = silu(gate) * up, W packed with gate/up rows interleaved in 16-row tiles (n = 2f)
int launch_gemm_swiglu(const void* x, const void* wp, void* h, int m, int f, int k, int dtype, const GemmPlan& p,
                       hipStream_t s);
int launch_pack(const void* w, void* packed, int n, int k, int dtype, int row_offset, int n_total,
                int interleave, hipStream_t s);
