// Small-M weight-streaming GEMMs: y[m, n] = sum_k x[m, k] W[n, k], 1 <= m <= 64.
//
// The verifier pass of Alg. 2 scores a handful of tokens against every weight of the model once
// (Sec. 3.1: loading the weights is the dominant cost, so as many tokens as possible should use each
// load), so these kernels are bound by the HBM stream of W.  bf16: W is pre-laid in 1 KiB tiles in
// the lane order of the 16x16x32 MFMA B operand, one wave-wide 16-byte load per MFMA, each wave
// walking a contiguous run of tiles; the few activation rows are the A operand, read from L2.  A
// workgroup owns NT column tiles; its waves split the K range and reduce through LDS; an optional
// cross-workgroup split of K writes partial sums that the consuming kernel adds in a fixed order
// (deterministic, no float atomics).  fp32 (small correctness configuration): one wave per output
// column with plain FMAs.
#include "common.h"

// ------------------------------------------------------------------------------------------------
// packing
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ int dest_row(int r, int row_offset, int interleave) {
    // interleave 0: rows land at row_offset + r; 1 / 2: gate / up rows of a fused SwiGLU matrix,
    // alternating in tiles of 16 rows (gate tile 2j, up tile 2j+1).
    if (interleave == 0) return row_offset + r;
    return 32 * (r >> 4) + (r & 15) + (interleave == 2 ? 16 : 0);
}

__global__ void pack_bf16_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ packed, int n, int k,
                                 int row_offset, int interleave) {
    const int k8 = k >> 3;
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)n * k8) return;
    int r = (int)(idx / k8), c = (int)(idx % k8) * 8;
    bf16x8 v = *reinterpret_cast<const bf16x8*>(w + (size_t)r * k + c);
    *reinterpret_cast<bf16x8*>(packed + packed_index(dest_row(r, row_offset, interleave), c, k)) = v;
}

__global__ void pack_f32_kernel(const float* __restrict__ w, float* __restrict__ packed, int n, int k,
                                int row_offset, int interleave) {
    const int k4 = k >> 2;
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)n * k4) return;
    int r = (int)(idx / k4), c = (int)(idx % k4) * 4;
    float4 v = *reinterpret_cast<const float4*>(w + (size_t)r * k + c);
    *reinterpret_cast<float4*>(packed + (size_t)dest_row(r, row_offset, interleave) * k + c) = v;
}

int launch_pack(const void* w, void* packed, int n, int k, int dtype, int row_offset, int n_total, int interleave,
                hipStream_t s) {
    (void)n_total;
    if (k % 32 != 0) HSD_FAIL(HSD_EINVAL, "pack: k=%d is not a multiple of 32", k);
    if (row_offset % 16 != 0) HSD_FAIL(HSD_EINVAL, "pack: row offset %d is not a multiple of 16", row_offset);
    if (interleave != 0 && n % 16 != 0) HSD_FAIL(HSD_EINVAL, "pack: interleaved matrices need n %% 16 == 0 (n=%d)", n);
    if (dtype == HSD_BF16) {
        size_t total = (size_t)n * (k / 8);
        pack_bf16_kernel<<<dim3((unsigned)((total + 255) / 256)), 256, 0, s>>>((const bf16_t*)w, (bf16_t*)packed, n, k,
                                                                              row_offset, interleave);
    } else {
        size_t total = (size_t)n * (k / 4);
        pack_f32_kernel<<<dim3((unsigned)((total + 255) / 256)), 256, 0, s>>>((const float*)w, (float*)packed, n, k,
                                                                             row_offset, interleave);
    }
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

// ------------------------------------------------------------------------------------------------
// bf16 MFMA kernel
// ------------------------------------------------------------------------------------------------
enum { EPI_PARTIAL = 0, EPI_SWIGLU = 1 };

template <int NT, int MT, int EPI>
__global__ void gemm_bf16_kernel(const bf16_t* __restrict__ x, const bf16x8* __restrict__ wp, void* __restrict__ out,
                                 int M, int N, int K, int kt_per_wg) {
    extern __shared__ float red[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int KT = K >> 5;
    const int ntiles = (N + 15) >> 4;
    const int ntile0 = blockIdx.x * NT;
    const int kt0 = blockIdx.y * kt_per_wg;
    const int kt1 = min(KT, kt0 + kt_per_wg);
    const int per = (kt1 - kt0 + nwaves - 1) / nwaves;
    const int kb = kt0 + wave * per;
    const int ke = min(kt1, kb + per);
    const int row = lane & 15, g = lane >> 4;

    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    const bf16_t* xp[MT];
    bool xv[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        int m = mt * 16 + row;
        xv[mt] = m < M;
        xp[mt] = x + (size_t)(xv[mt] ? m : 0) * K + g * 8;
    }
    const bf16x8* bp[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        int t = min(ntile0 + nt, ntiles - 1);      // clamp: tiles past the edge are computed, never stored
        bp[nt] = wp + (size_t)t * KT * 64 + lane;
    }
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};

    for (int kt = kb; kt < ke; ++kt) {
        bf16x8 b[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) b[nt] = __builtin_nontemporal_load(bp[nt] + (size_t)kt * 64);
        bf16x8 a[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
            a[mt] = xv[mt] ? *reinterpret_cast<const bf16x8*>(xp[mt] + (size_t)kt * 32) : zero;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[mt], b[nt], acc[mt][nt], 0, 0, 0);
    }

    // cross-wave reduction through LDS: red[wave][tile][r][lane]
    constexpr int TOTAL = MT * NT * 256;
    float* mine = red + wave * TOTAL;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r) mine[(mt * NT + nt) * 256 + r * 64 + lane] = acc[mt][nt][r];
    __syncthreads();

    if constexpr (EPI == EPI_PARTIAL) {
        float* part = reinterpret_cast<float*>(out) + (size_t)blockIdx.y * M * N;
        for (int idx = threadIdx.x; idx < TOTAL; idx += blockDim.x) {
            float s = 0.f;
            for (int w = 0; w < nwaves; ++w) s += red[w * TOTAL + idx];
            int tile = idx >> 8, rem = idx & 255, r = rem >> 6, l = rem & 63;
            int mt = tile / NT, nt = tile % NT;
            int m = mt * 16 + 4 * (l >> 4) + r;
            int n = (ntile0 + nt) * 16 + (l & 15);
            if (m < M && n < N) part[(size_t)m * N + n] = s;
        }
    } else if constexpr (NT >= 2) {
        // tiles alternate gate / up; N is the fused width 2F
        bf16_t* h = reinterpret_cast<bf16_t*>(out);
        const int F = N >> 1;
        constexpr int HALF = MT * (NT / 2) * 256;
        for (int idx = threadIdx.x; idx < HALF; idx += blockDim.x) {
            int pair = idx >> 8, rem = idx & 255, r = rem >> 6, l = rem & 63;
            int mt = pair / (NT / 2), j = pair % (NT / 2);
            float gt = 0.f, up = 0.f;
            for (int w = 0; w < nwaves; ++w) {
                gt += red[w * TOTAL + (mt * NT + 2 * j) * 256 + rem];
                up += red[w * TOTAL + (mt * NT + 2 * j + 1) * 256 + rem];
            }
            int m = mt * 16 + 4 * (l >> 4) + r;
            int f = ((ntile0 >> 1) + j) * 16 + (l & 15);
            if (m < M && f < F) h[(size_t)m * F + f] = (bf16_t)(gt / (1.f + __expf(-gt)) * up);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// fp32 kernel: one wave per output column (per gate/up pair for SwiGLU)
// ------------------------------------------------------------------------------------------------
template <int EPI>
__global__ void gemm_f32_kernel(const float* __restrict__ x, const float* __restrict__ w, void* __restrict__ out, int M,
                                int N, int K) {
    const int lane = threadIdx.x & 63;
    const int col = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int F = N >> 1;
    if (EPI == EPI_PARTIAL ? col >= N : col >= F) return;
    const int n0 = EPI == EPI_PARTIAL ? col : 32 * (col >> 4) + (col & 15);
    const float* w0 = w + (size_t)n0 * K;
    const float* w1 = w0 + (size_t)16 * K;
    for (int m0 = 0; m0 < M; m0 += 8) {
        float a0[8], a1[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) a0[i] = a1[i] = 0.f;
        for (int k = lane * 4; k < K; k += 256) {
            float4 wv = *reinterpret_cast<const float4*>(w0 + k);
            float4 uv = EPI == EPI_SWIGLU ? *reinterpret_cast<const float4*>(w1 + k) : float4{0, 0, 0, 0};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (m0 + i < M) {
                    float4 xv = *reinterpret_cast<const float4*>(x + (size_t)(m0 + i) * K + k);
                    a0[i] += wv.x * xv.x + wv.y * xv.y + wv.z * xv.z + wv.w * xv.w;
                    if (EPI == EPI_SWIGLU) a1[i] += uv.x * xv.x + uv.y * xv.y + uv.z * xv.z + uv.w * xv.w;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float s0 = wave_sum(a0[i]);
            float s1 = EPI == EPI_SWIGLU ? wave_sum(a1[i]) : 0.f;
            if (lane == 0 && m0 + i < M) {
                if (EPI == EPI_PARTIAL)
                    reinterpret_cast<float*>(out)[(size_t)(m0 + i) * N + col] = s0;
                else
                    reinterpret_cast<float*>(out)[(size_t)(m0 + i) * F + col] = s0 / (1.f + expf(-s0)) * s1;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
GemmPlan gemm_plan(int m, int n, int k, int dtype, bool swiglu) {
    GemmPlan p{1, 1, 4};
    if (dtype != HSD_BF16) return p;
    const int mt = ceil_div(m, 16) <= 1 ? 1 : (m <= 32 ? 2 : 4);
    const int ntiles = ceil_div(n, 16), KT = k / 32;
    p.nt = ntiles >= 2048 ? 4 : (ntiles >= 512 ? 2 : 1);
    if (swiglu) p.nt = mt > 2 ? 2 : 4;
    if (mt > 2 && p.nt > 2) p.nt = 2;
    p.waves = mt > 2 ? 4 : 8;
    while (p.waves > 1 && KT / p.waves < 2) p.waves >>= 1;
    const int groups = ceil_div(ntiles, p.nt);
    p.ksplit = 1;
    if (!swiglu) {
        int want = ceil_div(512, groups);
        int room = KT / (p.waves * 2);
        p.ksplit = want < 1 ? 1 : want;
        if (p.ksplit > room) p.ksplit = room < 1 ? 1 : room;
        if (p.ksplit > 8) p.ksplit = 8;
    }
    return p;
}

template <int NT, int MT, int EPI>
static void launch_bf16(const void* x, const void* wp, void* out, int m, int n, int k, const GemmPlan& p, hipStream_t s) {
    const int ntiles = ceil_div(n, 16), KT = k / 32;
    dim3 grid(ceil_div(ntiles, NT), p.ksplit);
    const int kt_per_wg = ceil_div(KT, p.ksplit);
    size_t lds = (size_t)p.waves * MT * NT * 256 * sizeof(float);
    gemm_bf16_kernel<NT, MT, EPI><<<grid, p.waves * 64, lds, s>>>((const bf16_t*)x, (const bf16x8*)wp, out, m, n, k,
                                                                  kt_per_wg);
}

template <int EPI>
static int dispatch_bf16(const void* x, const void* wp, void* out, int m, int n, int k, const GemmPlan& p, hipStream_t s) {
    const int mt = m <= 16 ? 1 : (m <= 32 ? 2 : 4);
#define HSD_CASE(NT_, MT_)                                              \
    if (p.nt == NT_ && mt == MT_) {                                     \
        launch_bf16<NT_, MT_, EPI>(x, wp, out, m, n, k, p, s);          \
        HSD_LAUNCH_CHECK();                                             \
        return HSD_OK;                                                  \
    }
    HSD_CASE(2, 1) HSD_CASE(4, 1) HSD_CASE(2, 2) HSD_CASE(4, 2) HSD_CASE(2, 4)
    if constexpr (EPI == EPI_PARTIAL) {
        HSD_CASE(1, 1) HSD_CASE(1, 2) HSD_CASE(1, 4)
    }
#undef HSD_CASE
    HSD_FAIL(HSD_EINVAL, "gemm: no kernel for nt=%d m=%d", p.nt, m);
}

static int check_gemm(int m, int n, int k) {
    if (m < 1 || m > HSD_MAX_PASS_ROWS) HSD_FAIL(HSD_EINVAL, "gemm: m=%d outside 1..%d", m, HSD_MAX_PASS_ROWS);
    if (n < 1 || k < 32 || k % 32 != 0) HSD_FAIL(HSD_EINVAL, "gemm: n=%d k=%d (k must be a positive multiple of 32)", n, k);
    return HSD_OK;
}

int launch_gemm(const void* x, const void* wp, float* part, int m, int n, int k, int dtype, const GemmPlan& p,
                hipStream_t s) {
    if (int rc = check_gemm(m, n, k)) return rc;
    if (dtype == HSD_BF16) return dispatch_bf16<EPI_PARTIAL>(x, wp, part, m, n, k, p, s);
    gemm_f32_kernel<EPI_PARTIAL><<<ceil_div(n, 4), 256, 0, s>>>((const float*)x, (const float*)wp, part, m, n, k);
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

int launch_gemm_swiglu(const void* x, const void* wp, void* h, int m, int f, int k, int dtype, const GemmPlan& p,
                       hipStream_t s) {
    if (int rc = check_gemm(m, 2 * f, k)) return rc;
    if (f % 16 != 0) HSD_FAIL(HSD_EINVAL, "swiglu gemm: ffn width %d is not a multiple of 16", f);
    if (dtype == HSD_BF16) return dispatch_bf16<EPI_SWIGLU>(x, wp, h, m, 2 * f, k, p, s);
    gemm_f32_kernel<EPI_SWIGLU><<<ceil_div(f, 4), 256, 0, s>>>((const float*)x, (const float*)wp, h, m, 2 * f, k);
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

// ------------------------------------------------------------------------------------------------
// C ABI
// ------------------------------------------------------------------------------------------------
__global__ void reduce_partials_kernel(const float* __restrict__ part, float* __restrict__ y, int count, int ksplit) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    float s = 0.f;
    for (int j = 0; j < ksplit; ++j) s += part[(size_t)j * count + i];
    y[i] = s;
}

int launch_reduce_partials(const float* part, float* y, int count, int ksplit, hipStream_t s) {
    reduce_partials_kernel<<<ceil_div(count, 256), 256, 0, s>>>(part, y, count, ksplit);
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

extern "C" size_t hsd_packed_bytes(int n, int k, int dtype) {
    return align_up((size_t)ceil_div(n, 16) * 16 * k * dtype_size(dtype), 256);
}

extern "C" size_t hsd_gemm_workspace_bytes(int m, int n, int k) {
    (void)k;
    return align_up((size_t)8 * m * n * sizeof(float), 256);
}

extern "C" int hsd_pack_weight(const void* w_dev, void* packed_dev, int n, int k, int dtype, void* stream) {
    if (!w_dev || !packed_dev || n < 1 || (dtype != HSD_F32 && dtype != HSD_BF16))
        HSD_FAIL(HSD_EINVAL, "hsd_pack_weight: bad arguments");
    hipStream_t s = (hipStream_t)stream;
    HSD_HIP(hipMemsetAsync(packed_dev, 0, hsd_packed_bytes(n, k, dtype), s));
    return launch_pack(w_dev, packed_dev, n, k, dtype, 0, n, 0, s);
}

extern "C" int hsd_gemm(const void* x_dev, const void* packed_dev, float* y_dev, int m, int n, int k, int dtype,
                        void* workspace_dev, void* stream) {
    if (!x_dev || !packed_dev || !y_dev || !workspace_dev || (dtype != HSD_F32 && dtype != HSD_BF16))
        HSD_FAIL(HSD_EINVAL, "hsd_gemm: bad arguments");
    if (int rc = check_gemm(m, n, k)) return rc;
    hipStream_t s = (hipStream_t)stream;
    GemmPlan p = gemm_plan(m, n, k, dtype, false);
    if (int rc = launch_gemm(x_dev, packed_dev, (float*)workspace_dev, m, n, k, dtype, p, s)) return rc;
    return launch_reduce_partials((const float*)workspace_dev, y_dev, m * n, p.ksplit, s);
}
