// Small-M weight-streaming GEMMs: y[m, n] = sum_k a[m, k] W[n, k], 1 <= m <= 64.
//
// The verifier pass of Alg. 2 scores a handful of tokens against every weight of the model once
// (Sec. 3.1: loading the weights is the dominant cost, so as many tokens as possible should use each
// load), so these kernels are bound by the HBM stream of W.
//
// bf16: W is pre-laid in 1 KiB tiles in the lane order of the 16x16x32 MFMA B operand (one wave-wide
// 16-byte load per MFMA, each wave walking a contiguous run of tiles).  A workgroup owns NT column
// tiles over the whole K range, its waves split K and reduce through LDS, so every output element is
// final inside one workgroup and the neighbouring element-wise steps are fused in:
//   A operand  - bf16 activations, or the fp32 residual stream normalised on the fly (RMSNorm: the
//                row sums of squares come from the producing kernel as fixed-point integers added
//                with atomics, so their value does not depend on the order of arrival);
//   epilogue   - plain store (LM head), residual add + sums of squares for the next norm,
//                SwiGLU on interleaved gate/up tiles, or RoPE + KV-cache append + q store.
// fp32 (small correctness configuration): one wave per output column with plain FMAs, unfused.
#include "common.h"

// ------------------------------------------------------------------------------------------------
// packing
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ int dest_row(int r, int row_offset, int interleave, int hd) {
    // 0: rows land at row_offset + r.
    // 1 / 2: gate / up rows of a fused SwiGLU matrix, alternating in tiles of 16 rows.
    // 3: rows of attention heads (hd rows each), the 16-row block of dims [16 jb, 16 jb + 16) followed
    //    by the block of its rotation partners [hd/2 + 16 jb, ...), so that one pair of tiles holds
    //    both halves of 16 RoPE pairs.
    if (interleave == 0) return row_offset + r;
    if (interleave == 3) {
        const int head = r / hd, j = r % hd, half = hd >> 1;
        const int hi = j >= half, jj = j - hi * half;
        return row_offset + head * hd + (2 * (jj >> 4) + hi) * 16 + (jj & 15);
    }
    return 32 * (r >> 4) + (r & 15) + (interleave == 2 ? 16 : 0);
}

__global__ void pack_bf16_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ packed, int n, int k,
                                 int row_offset, int interleave, int hd) {
    const int k8 = k >> 3;
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)n * k8) return;
    int r = (int)(idx / k8), c = (int)(idx % k8) * 8;
    bf16x8 v = *reinterpret_cast<const bf16x8*>(w + (size_t)r * k + c);
    *reinterpret_cast<bf16x8*>(packed + packed_index(dest_row(r, row_offset, interleave, hd), c, k)) = v;
}

__global__ void pack_f32_kernel(const float* __restrict__ w, float* __restrict__ packed, int n, int k,
                                int row_offset, int interleave, int hd) {
    const int k4 = k >> 2;
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)n * k4) return;
    int r = (int)(idx / k4), c = (int)(idx % k4) * 4;
    float4 v = *reinterpret_cast<const float4*>(w + (size_t)r * k + c);
    *reinterpret_cast<float4*>(packed + (size_t)dest_row(r, row_offset, interleave, hd) * k + c) = v;
}

int launch_pack(const void* w, void* packed, int n, int k, int dtype, int row_offset, int interleave, int hd,
                hipStream_t s) {
    if (k % 32 != 0) HSD_FAIL(HSD_EINVAL, "pack: k=%d is not a multiple of 32", k);
    if (row_offset % 16 != 0) HSD_FAIL(HSD_EINVAL, "pack: row offset %d is not a multiple of 16", row_offset);
    if (interleave != 0 && n % 16 != 0) HSD_FAIL(HSD_EINVAL, "pack: interleaved matrices need n %% 16 == 0 (n=%d)", n);
    if (interleave == 3 && (hd % 32 != 0 || n % hd != 0)) HSD_FAIL(HSD_EINVAL, "pack: head layout needs hd %% 32 == 0 and whole heads");
    if (dtype == HSD_BF16) {
        size_t total = (size_t)n * (k / 8);
        pack_bf16_kernel<<<dim3((unsigned)((total + 255) / 256)), 256, 0, s>>>((const bf16_t*)w, (bf16_t*)packed, n, k,
                                                                              row_offset, interleave, hd);
    } else {
        size_t total = (size_t)n * (k / 4);
        pack_f32_kernel<<<dim3((unsigned)((total + 255) / 256)), 256, 0, s>>>((const float*)w, (float*)packed, n, k,
                                                                             row_offset, interleave, hd);
    }
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

// ------------------------------------------------------------------------------------------------
// bf16 MFMA kernel
// ------------------------------------------------------------------------------------------------
template <int ASRC>
__device__ __forceinline__ bf16x8 load_a(const void* rowp, const float* nw, int kt, float inv, bool valid) {
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    if (!valid) return zero;
    if constexpr (ASRC == A_BF16) {
        return *reinterpret_cast<const bf16x8*>(reinterpret_cast<const bf16_t*>(rowp) + (size_t)kt * 32);
    } else {
        const float* xp = reinterpret_cast<const float*>(rowp) + (size_t)kt * 32;
        const float4 v0 = *reinterpret_cast<const float4*>(xp), v1 = *reinterpret_cast<const float4*>(xp + 4);
        const float4 w0 = *reinterpret_cast<const float4*>(nw + (size_t)kt * 32), w1 = *reinterpret_cast<const float4*>(nw + (size_t)kt * 32 + 4);
        bf16x8 a;
        a[0] = (bf16_t)(v0.x * inv * w0.x); a[1] = (bf16_t)(v0.y * inv * w0.y);
        a[2] = (bf16_t)(v0.z * inv * w0.z); a[3] = (bf16_t)(v0.w * inv * w0.w);
        a[4] = (bf16_t)(v1.x * inv * w1.x); a[5] = (bf16_t)(v1.y * inv * w1.y);
        a[6] = (bf16_t)(v1.z * inv * w1.z); a[7] = (bf16_t)(v1.w * inv * w1.w);
        return a;
    }
}

template <int NT, int MT, int ASRC, int EPI>
__global__ __launch_bounds__(512) void gemm_bf16_kernel(const GemmArgs g) {
    extern __shared__ float red[];
    constexpr int U = (8 / (NT * MT)) > 0 ? (8 / (NT * MT)) : 1;     // k-steps whose loads are issued together
    constexpr int TOTAL = MT * NT * 256;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
    const int M = g.M, N = g.N, K = g.K;
    const int KT = K >> 5;
    const int ntiles = (N + 15) >> 4;
    const int ntile0 = blockIdx.x * NT;
    const int per = (KT + nwaves - 1) / nwaves;
    const int kb = wave * per;
    const int ke = min(KT, kb + per);
    const int row = lane & 15, grp = lane >> 4;

    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    const bf16x8* bp[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int t = min(ntile0 + nt, ntiles - 1);     // clamp: tiles past the edge are computed, never stored
        bp[nt] = g.wp + (size_t)t * KT * 64 + lane;
    }

    // A rows of this lane; for the normalising source also 1/rms of those rows
    const void* ap[MT];
    bool av[MT];
    float inv[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + row;
        av[mt] = m < M;
        const size_t off = (size_t)(av[mt] ? m : 0) * K + grp * 8;
        ap[mt] = ASRC == A_BF16 ? (const void*)(reinterpret_cast<const bf16_t*>(g.a) + off)
                                : (const void*)(reinterpret_cast<const float*>(g.a) + off);
        inv[mt] = 1.f;
        if constexpr (ASRC == A_NORM) {
            const float ss = (float)((double)g.ss_in[av[mt] ? m : 0] * (1.0 / 16777216.0));
            inv[mt] = 1.0f / sqrtf(ss / (float)K + g.eps);
        }
    }
    const float* nw = ASRC == A_NORM ? g.norm_w + grp * 8 : nullptr;
    if constexpr (ASRC == A_NORM) {
        if (g.ss_zero && blockIdx.x == 0 && tid < HSD_MAX_PASS_ROWS) g.ss_zero[tid] = 0ull;   // ready for the next producer
    }

    int kt = kb;
    for (; kt + U <= ke; kt += U) {
        bf16x8 b[U][NT], a[U][MT];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) b[u][nt] = __builtin_nontemporal_load(bp[nt] + (size_t)(kt + u) * 64);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) a[u][mt] = load_a<ASRC>(ap[mt], nw, kt + u, inv[mt], av[mt]);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u][mt], b[u][nt], acc[mt][nt], 0, 0, 0);
    }
    for (; kt < ke; ++kt) {
        bf16x8 b[NT], a[MT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) b[nt] = __builtin_nontemporal_load(bp[nt] + (size_t)kt * 64);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) a[mt] = load_a<ASRC>(ap[mt], nw, kt, inv[mt], av[mt]);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[mt], b[nt], acc[mt][nt], 0, 0, 0);
    }

    // cross-wave reduction through LDS: red[wave][tile][r][lane]; element (tile, r, lane) is
    // row 16 mt + 4 (lane / 16) + r, column 16 (ntile0 + nt) + lane % 16
    float* mine = red + wave * TOTAL;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r) mine[(mt * NT + nt) * 256 + r * 64 + lane] = acc[mt][nt][r];
    __syncthreads();

    if constexpr (EPI == EPI_STORE || EPI == EPI_RESID) {
        float* sq = red + nwaves * TOTAL;                  // [MT*16][NT*16] squares of the new residual values
        for (int idx = tid; idx < TOTAL; idx += blockDim.x) {
            float s = 0.f;
            for (int w = 0; w < nwaves; ++w) s += red[w * TOTAL + idx];
            const int tile = idx >> 8, rem = idx & 255, r = rem >> 6, l = rem & 63;
            const int mt = tile / NT, nt = tile % NT;
            const int ml = mt * 16 + 4 * (l >> 4) + r;
            const int n = (ntile0 + nt) * 16 + (l & 15);
            float v = 0.f;
            if (ml < M && n < N) {
                float* dst = g.out_f32 + (size_t)ml * N + n;
                v = EPI == EPI_RESID ? *dst + s : s;
                *dst = v;
            }
            if constexpr (EPI == EPI_RESID) sq[ml * (NT * 16) + nt * 16 + (l & 15)] = v * v;
        }
        if constexpr (EPI == EPI_RESID) {
            __syncthreads();
            if (tid < M) {
                float s = 0.f;
                for (int c = 0; c < NT * 16; ++c) s += sq[tid * (NT * 16) + c];
                atomicAdd(g.ss_out + tid, (unsigned long long)((double)s * 16777216.0 + 0.5));
            }
        }
    } else if constexpr (EPI == EPI_SWIGLU) {
        // tiles alternate gate / up; N is the fused width 2F
        const int F = N >> 1;
        constexpr int HALF = MT * (NT / 2) * 256;
        for (int idx = tid; idx < HALF; idx += blockDim.x) {
            const int pair = idx >> 8, rem = idx & 255, r = rem >> 6, l = rem & 63;
            const int mt = pair / (NT / 2), j = pair % (NT / 2);
            float gt = 0.f, up = 0.f;
            for (int w = 0; w < nwaves; ++w) {
                gt += red[w * TOTAL + (mt * NT + 2 * j) * 256 + rem];
                up += red[w * TOTAL + (mt * NT + 2 * j + 1) * 256 + rem];
            }
            const int ml = mt * 16 + 4 * (l >> 4) + r;
            const int f = ((ntile0 >> 1) + j) * 16 + (l & 15);
            if (ml < M && f < F) g.out_bf16[(size_t)ml * F + f] = (bf16_t)(gt / (1.f + __expf(-gt)) * up);
        }
    } else {
        // EPI_ROPE: tile pairs hold dims [16 jb, 16 jb + 16) and their partners hd/2 further of one head
        const int hd = g.hd, half = hd >> 1, pairs_per_head = hd >> 5;
        constexpr int HALF = MT * (NT / 2) * 256;
        for (int idx = tid; idx < HALF; idx += blockDim.x) {
            const int pair = idx >> 8, rem = idx & 255, r = rem >> 6, l = rem & 63;
            const int mt = pair / (NT / 2), jp = pair % (NT / 2);
            float a = 0.f, b = 0.f;
            for (int w = 0; w < nwaves; ++w) {
                a += red[w * TOTAL + (mt * NT + 2 * jp) * 256 + rem];
                b += red[w * TOTAL + (mt * NT + 2 * jp + 1) * 256 + rem];
            }
            const int ml = mt * 16 + 4 * (l >> 4) + r;
            const int gp = (ntile0 >> 1) + jp;                      // global pair index
            const int head = gp / pairs_per_head, j = (gp % pairs_per_head) * 16 + (l & 15);
            if (ml >= M || head >= g.n_q + 2 * g.n_kv) continue;
            const int pos = g.pos0 + ml;
            const bool is_q = head < g.n_q, is_v = head >= g.n_q + g.n_kv;
            float ra = a, rb = b;
            if (!is_v) {
                const double ang = (double)pos * exp2(-2.0 * (double)j / (double)hd * log2((double)g.rope_base));
                double sn, cs;
                sincos(ang, &sn, &cs);
                ra = (float)((double)a * cs - (double)b * sn);
                rb = (float)((double)b * cs + (double)a * sn);
            }
            if (is_q) {
                bf16_t* dst = g.out_bf16 + ((size_t)ml * g.n_q + head) * hd;
                dst[j] = (bf16_t)ra;
                dst[j + half] = (bf16_t)rb;
            } else {
                const int kvh = is_v ? head - g.n_q - g.n_kv : head - g.n_q;
                const int page = g.pages[pos / HSD_KV_PAGE], ip = pos % HSD_KV_PAGE;
                bf16_t* blk = g.kv_layer + (size_t)page * kv_page_elems(g.n_kv, hd) + (size_t)kvh * 2 * kv_block_elems(hd) +
                              (is_v ? kv_block_elems(hd) : 0);
                if (is_v) {
                    blk[kv_v_index(ip, j, hd)] = (bf16_t)ra;
                    blk[kv_v_index(ip, j + half, hd)] = (bf16_t)rb;
                } else {
                    blk[kv_k_index(ip, j, hd)] = (bf16_t)ra;
                    blk[kv_k_index(ip, j + half, hd)] = (bf16_t)rb;
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// fp32 kernel: one wave per output column (per gate/up pair for SwiGLU)
// ------------------------------------------------------------------------------------------------
template <int SWIGLU>
__global__ void gemm_f32_kernel(const float* __restrict__ x, const float* __restrict__ w, float* __restrict__ out, int M,
                                int N, int K) {
    const int lane = threadIdx.x & 63;
    const int col = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const int F = N >> 1;
    if (SWIGLU ? col >= F : col >= N) return;
    const int n0 = SWIGLU ? 32 * (col >> 4) + (col & 15) : col;
    const float* w0 = w + (size_t)n0 * K;
    const float* w1 = w0 + (size_t)16 * K;
    for (int m0 = 0; m0 < M; m0 += 8) {
        float a0[8], a1[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) a0[i] = a1[i] = 0.f;
        for (int k = lane * 4; k < K; k += 256) {
            float4 wv = *reinterpret_cast<const float4*>(w0 + k);
            float4 uv = SWIGLU ? *reinterpret_cast<const float4*>(w1 + k) : float4{0, 0, 0, 0};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (m0 + i < M) {
                    float4 xv = *reinterpret_cast<const float4*>(x + (size_t)(m0 + i) * K + k);
                    a0[i] += wv.x * xv.x + wv.y * xv.y + wv.z * xv.z + wv.w * xv.w;
                    if (SWIGLU) a1[i] += uv.x * xv.x + uv.y * xv.y + uv.z * xv.z + uv.w * xv.w;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float s0 = wave_sum(a0[i]);
            float s1 = SWIGLU ? wave_sum(a1[i]) : 0.f;
            if (lane == 0 && m0 + i < M) {
                if (SWIGLU)
                    out[(size_t)(m0 + i) * F + col] = s0 / (1.f + expf(-s0)) * s1;
                else
                    out[(size_t)(m0 + i) * N + col] = s0;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
static int g_tune_nt[4] = {0, 0, 0, 0};      // optional overrides per epilogue kind (0 = heuristic)
static int g_tune_waves = 0;

void gemm_tune(int epilogue, int nt, int waves) {
    if (epilogue >= 0 && epilogue < 4) g_tune_nt[epilogue] = nt;
    g_tune_waves = waves;
}

GemmPlan gemm_plan(int m, int n, int k, int epi) {
    GemmPlan p{1, 8};
    const int mt = m <= 16 ? 1 : (m <= 32 ? 2 : 4);
    const int ntiles = ceil_div(n, 16), KT = k / 32;
    switch (epi) {
        case EPI_ROPE: p.nt = 2; break;
        case EPI_SWIGLU: p.nt = ntiles >= 1024 && mt <= 2 ? 4 : 2; break;
        case EPI_RESID: p.nt = ntiles >= 1024 ? 2 : 1; break;
        default: p.nt = ntiles >= 4096 && mt <= 2 ? 4 : (ntiles >= 512 ? 2 : 1); break;
    }
    if (epi != EPI_ROPE && epi >= 0 && epi < 4 && g_tune_nt[epi]) p.nt = g_tune_nt[epi];
    if (mt == 4 && p.nt > 2) p.nt = 2;
    p.waves = g_tune_waves ? g_tune_waves : 8;
    while (p.waves > 1 && KT < 2 * p.waves) p.waves >>= 1;
    return p;
}

static size_t gemm_lds_bytes(const GemmPlan& p, int m, int epi) {
    const int mt = m <= 16 ? 1 : (m <= 32 ? 2 : 4);
    size_t b = (size_t)p.waves * mt * p.nt * 256 * sizeof(float);
    if (epi == EPI_RESID) b += (size_t)mt * 16 * p.nt * 16 * sizeof(float);
    return b;
}

template <int NT, int MT, int ASRC, int EPI>
static void launch_inst(const GemmArgs& g, const GemmPlan& p, hipStream_t s) {
    const int ntiles = ceil_div(g.N, 16);
    gemm_bf16_kernel<NT, MT, ASRC, EPI><<<ceil_div(ntiles, NT), p.waves * 64, gemm_lds_bytes(p, g.M, EPI), s>>>(g);
}

static int check_gemm(int m, int n, int k) {
    if (m < 1 || m > HSD_MAX_PASS_ROWS) HSD_FAIL(HSD_EINVAL, "gemm: m=%d outside 1..%d", m, HSD_MAX_PASS_ROWS);
    if (n < 1 || k < 32 || k % 32 != 0) HSD_FAIL(HSD_EINVAL, "gemm: n=%d k=%d (k must be a positive multiple of 32)", n, k);
    return HSD_OK;
}

int launch_gemm_bf16(const GemmArgs& g, int asrc, int epi, const GemmPlan& p, hipStream_t s) {
    if (int rc = check_gemm(g.M, g.N, g.K)) return rc;
    const int mt = g.M <= 16 ? 1 : (g.M <= 32 ? 2 : 4);
#define HSD_CASE(NT_, MT_, A_, E_)                                         \
    if (p.nt == NT_ && mt == MT_ && asrc == A_ && epi == E_) {             \
        launch_inst<NT_, MT_, A_, E_>(g, p, s);                            \
        HSD_LAUNCH_CHECK();                                                \
        return HSD_OK;                                                     \
    }
#define HSD_MTS(NT_, A_, E_) HSD_CASE(NT_, 1, A_, E_) HSD_CASE(NT_, 2, A_, E_) HSD_CASE(NT_, 4, A_, E_)
    HSD_MTS(1, A_BF16, EPI_STORE) HSD_MTS(2, A_BF16, EPI_STORE) HSD_CASE(4, 1, A_BF16, EPI_STORE) HSD_CASE(4, 2, A_BF16, EPI_STORE)
    HSD_MTS(1, A_NORM, EPI_STORE) HSD_MTS(2, A_NORM, EPI_STORE) HSD_CASE(4, 1, A_NORM, EPI_STORE) HSD_CASE(4, 2, A_NORM, EPI_STORE)
    HSD_MTS(1, A_BF16, EPI_RESID) HSD_MTS(2, A_BF16, EPI_RESID)
    HSD_MTS(2, A_NORM, EPI_SWIGLU) HSD_CASE(4, 1, A_NORM, EPI_SWIGLU) HSD_CASE(4, 2, A_NORM, EPI_SWIGLU)
    HSD_MTS(2, A_NORM, EPI_ROPE)
#undef HSD_MTS
#undef HSD_CASE
    HSD_FAIL(HSD_EINVAL, "gemm: no kernel for nt=%d m=%d source=%d epilogue=%d", p.nt, g.M, asrc, epi);
}

int launch_gemm_f32(const float* x, const float* w, float* out, int m, int n, int k, bool swiglu, hipStream_t s) {
    if (int rc = check_gemm(m, n, k)) return rc;
    if (swiglu)
        gemm_f32_kernel<1><<<ceil_div(n / 2, 4), 256, 0, s>>>(x, w, out, m, n, k);
    else
        gemm_f32_kernel<0><<<ceil_div(n, 4), 256, 0, s>>>(x, w, out, m, n, k);
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

// ------------------------------------------------------------------------------------------------
// C ABI
// ------------------------------------------------------------------------------------------------
extern "C" size_t hsd_packed_bytes(int n, int k, int dtype) {
    return align_up((size_t)ceil_div(n, 16) * 16 * k * dtype_size(dtype), 256);
}

extern "C" int hsd_pack_weight(const void* w_dev, void* packed_dev, int n, int k, int dtype, void* stream) {
    if (!w_dev || !packed_dev || n < 1 || (dtype != HSD_F32 && dtype != HSD_BF16))
        HSD_FAIL(HSD_EINVAL, "hsd_pack_weight: bad arguments");
    hipStream_t s = (hipStream_t)stream;
    HSD_HIP(hipMemsetAsync(packed_dev, 0, hsd_packed_bytes(n, k, dtype), s));
    return launch_pack(w_dev, packed_dev, n, k, dtype, 0, 0, 0, s);
}

extern "C" int hsd_gemm(const void* x_dev, const void* packed_dev, float* y_dev, int m, int n, int k, int dtype,
                        void* stream) {
    if (!x_dev || !packed_dev || !y_dev || (dtype != HSD_F32 && dtype != HSD_BF16))
        HSD_FAIL(HSD_EINVAL, "hsd_gemm: bad arguments");
    if (int rc = check_gemm(m, n, k)) return rc;
    hipStream_t s = (hipStream_t)stream;
    if (dtype == HSD_F32) return launch_gemm_f32((const float*)x_dev, (const float*)packed_dev, y_dev, m, n, k, false, s);
    GemmArgs g = {};
    g.a = x_dev;
    g.wp = (const bf16x8*)packed_dev;
    g.M = m; g.N = n; g.K = k;
    g.out_f32 = y_dev;
    return launch_gemm_bf16(g, A_BF16, EPI_STORE, gemm_plan(m, n, k, EPI_STORE), s);
}
