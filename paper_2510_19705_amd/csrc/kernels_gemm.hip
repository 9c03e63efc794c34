// Small-M weight-streaming GEMMs: y[m, n] = sum_k a[m, k] W[n, k], 1 <= m <= 64.
//
// The verifier pass of Alg. 2 scores a handful of tokens against every weight of the model once
// (Sec. 3.1: loading the weights is the dominant cost, so as many tokens as possible should use each
// load), so these kernels are bound by the HBM stream of W.
//
// bf16: W is pre-laid in 1 KiB tiles in the lane order of the 16x16x32 MFMA B operand (one wave-wide
// 16-byte load per MFMA, each wave walking a contiguous run of tiles).  HBM peak needs every CU
// pulling, so the grid is (column groups of NT tiles) x (ksplit slices of K), about a thousand
// workgroups whatever the matrix shape.  Inside a workgroup the waves split the slice and reduce
// through LDS; across the ksplit workgroups of a column group the partial tiles go through memory and
// the LAST one to arrive (a ticket counter) adds them in slice order, so the result does not depend
// on arrival order, and runs the epilogue.  The element-wise neighbours of each projection are fused:
//   RMSNorm   - the producer of the residual stream also stores bf16(x * w_norm) and adds each row's
//               sum of squares, as a fixed-point integer, into an accumulator with atomics (integer
//               addition: order-free); since a GEMM is linear in a per-row scale, the consumer feeds
//               the un-normalised rows to the MFMAs and multiplies by 1/rms in its epilogue;
//   epilogue  - plain store (LM head), residual add (+ the two products above), SwiGLU on interleaved
//               gate/up tiles, or RoPE + KV-cache append + q store.
// fp32 (small correctness configuration): one wave per output column with plain FMAs, unfused.
#include <algorithm>

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
    if (interleave == 4) {      // heads of hd rows, each dim directly followed by its RoPE partner: 2 j, 2 j + 1
        const int head = r / hd, j = r % hd, half = hd >> 1;
        const int hi = j >= half, jj = j - hi * half;
        return row_offset + head * hd + 2 * jj + hi;
    }
    if (interleave == 3) {
        const int head = r / hd, j = r % hd, half = hd >> 1;
        const int hi = j >= half, jj = j - hi * half;
        return row_offset + head * hd + (2 * (jj >> 4) + hi) * 16 + (jj & 15);
    }
    return 32 * (r >> 4) + (r & 15) + (interleave == 2 ? 16 : 0);
}

__global__ void pack_bf16_kernel(const bf16_t* __restrict__ w, bf16_t* __restrict__ packed, int n, int k,
                                 int row_offset, int interleave, int hd, int rows_layout) {
    const int k8 = k >> 3;
    size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)n * k8) return;
    int r = (int)(idx / k8), c = (int)(idx % k8) * 8;
    bf16x8 v = *reinterpret_cast<const bf16x8*>(w + (size_t)r * k + c);
    const int dr = dest_row(r, row_offset, interleave, hd);
    bf16_t* dst = rows_layout ? packed + (size_t)dr * k + c : packed + packed_index(dr, c, k);
    *reinterpret_cast<bf16x8*>(dst) = v;
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
                int rows_layout, hipStream_t s) {
    if (k % 32 != 0) HSD_FAIL(HSD_EINVAL, "pack: k=%d is not a multiple of 32", k);
    if (row_offset % 16 != 0) HSD_FAIL(HSD_EINVAL, "pack: row offset %d is not a multiple of 16", row_offset);
    if (interleave != 0 && n % 16 != 0) HSD_FAIL(HSD_EINVAL, "pack: interleaved matrices need n %% 16 == 0 (n=%d)", n);
    if ((interleave == 3 || interleave == 4) && (hd % 32 != 0 || n % hd != 0)) HSD_FAIL(HSD_EINVAL, "pack: head layout needs hd %% 32 == 0 and whole heads");
    if (dtype == HSD_BF16) {
        size_t total = (size_t)n * (k / 8);
        pack_bf16_kernel<<<dim3((unsigned)((total + 255) / 256)), 256, 0, s>>>((const bf16_t*)w, (bf16_t*)packed, n, k,
                                                                              row_offset, interleave, hd, rows_layout);
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
// 1 / sqrt(mean(x^2) + eps) of row m from its fixed-point sum of squares (times 2^24), which the
// producers spread over SS_SLOTS accumulators to keep the atomics from queueing on one address
__device__ __forceinline__ float row_inv_rms(const unsigned long long* ss, int m, int d, float eps) {
    unsigned long long t = 0;
#pragma unroll
    for (int sl = 0; sl < SS_SLOTS; ++sl) t += ss[sl * HSD_MAX_PASS_ROWS + m];
    const float v = (float)((double)t * (1.0 / 16777216.0));
    return 1.0f / sqrtf(v / (float)d + eps);
}

__device__ __forceinline__ void ss_clear(unsigned long long* ss, int tid, int nthreads) {
    for (int i = tid; i < SS_SLOTS * HSD_MAX_PASS_ROWS; i += nthreads) ss[i] = 0ull;
}

__device__ __forceinline__ void ss_add(unsigned long long* ss, int m, float sum_sq) {
    atomicAdd(ss + (blockIdx.x % SS_SLOTS) * HSD_MAX_PASS_ROWS + m, (unsigned long long)((double)sum_sq * 16777216.0 + 0.5));
}

// RoPE on one (dim j, dim j + hd/2) pair of token row ml of `head` (q heads, then k heads, then v heads, which are
// not rotated), then the q store or the KV-cache append through the page table.  Angle in fp64.  In two parts:
// rope_prepare needs only the element's coordinates (the rotation and the page-table entry), so the kernels run it
// before their weight stream, whose latency hides the fp64 sincos and the page lookup; rope_finish needs the sums.
struct RopePre {
    double cs, sn;
    int page;
};

__device__ __forceinline__ RopePre rope_prepare(const GemmArgs& g, int head, int j, int ml) {
    RopePre r{1.0, 0.0, 0};
    const int32_t* ptab;
    const int pos = gemm_row_position(g, ml, &ptab);
    if (head < g.n_q + g.n_kv) {
        const double ang = (double)pos * exp2(-2.0 * (double)j / (double)g.hd * log2((double)g.rope_base));
        sincos(ang, &r.sn, &r.cs);
    }
    if (head >= g.n_q) r.page = ptab[pos / HSD_KV_PAGE];
    return r;
}

__device__ __forceinline__ void rope_finish(const GemmArgs& g, int head, int j, int ml, float a, float b, const RopePre& pre) {
    const int hd = g.hd, half = hd >> 1;
    const int32_t* ptab;
    const int pos = gemm_row_position(g, ml, &ptab);
    const bool is_q = head < g.n_q, is_v = head >= g.n_q + g.n_kv;
    float ra = a, rb = b;
    if (!is_v) {
        ra = (float)((double)a * pre.cs - (double)b * pre.sn);
        rb = (float)((double)b * pre.cs + (double)a * pre.sn);
    }
    if (is_q) {
        bf16_t* dst = g.out_bf16 + ((size_t)ml * g.n_q + head) * hd;
        dst[j] = (bf16_t)ra;
        dst[j + half] = (bf16_t)rb;
        return;
    }
    const int kvh = is_v ? head - g.n_q - g.n_kv : head - g.n_q;
    const int ip = pos % HSD_KV_PAGE;
    bf16_t* blk = g.kv_layer + (size_t)pre.page * kv_page_elems(g.n_kv, hd) + (size_t)kvh * 2 * kv_block_elems(hd) +
                  (is_v ? kv_block_elems(hd) : 0);
    if (is_v) {
        blk[kv_v_index(ip, j, hd)] = (bf16_t)ra;
        blk[kv_v_index(ip, j + half, hd)] = (bf16_t)rb;
    } else {
        blk[kv_k_index(ip, j, hd)] = (bf16_t)ra;
        blk[kv_k_index(ip, j + half, hd)] = (bf16_t)rb;
    }
}

// DEEP: twice as many k-steps' loads issued together.  Used for 4096 <= K < 8192 per workgroup (16-31 steps per wave):
// +16 % on the 7B-shaped gate/up; with 8 steps per wave the extra registers only cost occupancy, and from 32 steps on
// the shallower batches measured 2-3 % faster (70B-shaped gate/up).
template <int NT, int MT, int EPI, bool DEEP>
__global__ __launch_bounds__(512) void gemm_bf16_kernel(const GemmArgs g) {
    extern __shared__ float red[];
    __shared__ bool sh_last;
    constexpr int UB = (DEEP ? 16 : 8) / (NT * MT);
    constexpr int U = UB > 8 ? 8 : (UB > 0 ? UB : 1);                // k-steps whose loads are issued together
    constexpr int TOTAL = MT * NT * 256;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), nwaves = blockDim.x >> 6;
    const int M = g.M, N = g.N, K = g.K;
    const int KT = K >> 5;
    const int ntiles = (N + 15) >> 4;
    // halves: two workgroups share a column group, each loads and owns 8 of the 16 columns of every tile (in the
    // packed tile those are every other 128-byte line; for RoPE pairs the same columns of both tiles, i.e. whole
    // pairs); the other half of the MFMA's columns multiplies zeros
    const bool halves = g.halves != 0;
    const int ntile0 = (halves ? (int)(blockIdx.x >> 1) : (int)blockIdx.x) * NT;
    const bool my_col = !halves || (int)((threadIdx.x & 15) >> 3) == (int)(blockIdx.x & 1);   // this lane's column (lane % 16) is the workgroup's
    const int ksplit = gridDim.y;
    const int per_wg = (KT + ksplit - 1) / ksplit;
    const int kt0 = blockIdx.y * per_wg, kt1 = min(KT, kt0 + per_wg);
    // The waves form groups of kstep (1, 2, 4 or 8) waves: every group owns a contiguous run of the workgroup's k-steps,
    // and the waves of a group take the steps of that run round-robin (kstep = 1: every wave its own contiguous
    // slice; kstep = 8: the eight waves' requests of one round are one contiguous 8 KB run per tile).
    const int kstep = g.interleave > 1 ? g.interleave : 1;
    const int ngroups = nwaves / kstep;
    const int per = (kt1 - kt0 + ngroups - 1) / ngroups;
    const int gbeg = kt0 + (wave / kstep) * per, gend = min(kt1, gbeg + per);
    const int kb = gbeg + wave % kstep;
    const int cnt = gend > kb ? (gend - kb + kstep - 1) / kstep : 0;      // this wave's steps: kb, kb + kstep, ...
    const int row = lane & 15, grp = lane >> 4;

    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto koff = [&](int kt) -> size_t { return (size_t)kt * 32 + grp * 8; };   // of this lane group's 8 elements in an A row
    const bf16x8* bp[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int t = min(ntile0 + nt, ntiles - 1);     // clamp: tiles past the edge are computed, never stored
        bp[nt] = g.wp + (size_t)t * KT * 64 + lane;
    }
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    auto load_b = [&](int nt, int kt) -> bf16x8 { return my_col ? __builtin_nontemporal_load(bp[nt] + (size_t)kt * 64) : zero; };
    const bf16_t* ap[MT];
    bool av[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = mt * 16 + row;
        av[mt] = m < M;
        ap[mt] = g.a + (size_t)(av[mt] ? m : 0) * K;
    }
    if (g.ss_zero && blockIdx.x == 0 && blockIdx.y == 0) ss_clear(g.ss_zero, tid, blockDim.x);   // for the next producer

    // ---- operands of this thread's epilogue elements: requested, and the rotary angles evaluated, before the
    // weight stream, whose latency covers them (workgroups are 512 threads; element i of thread tid is
    // tid + 512 i in the epilogue's order) ----
    constexpr int OUTS = (EPI == EPI_STORE || EPI == EPI_RESID) ? TOTAL : MT * (NT / 2) * 256;
    constexpr int EPT = (OUTS + 511) / 512;
    float pre_inv[EPT], pre_x[EPT], pre_nw[EPT];
    RopePre pre_rope[EPT];
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
        const int idx = tid + 512 * i;
        pre_inv[i] = 1.f;
        pre_x[i] = 0.f;
        pre_nw[i] = 0.f;
        pre_rope[i] = RopePre{1.0, 0.0, 0};
        if (idx >= OUTS) continue;
        const int tile = idx >> 8, rem = idx & 255, r = rem >> 6, l = rem & 63;
        if constexpr (EPI == EPI_STORE || EPI == EPI_RESID) {
            const int mt = tile / NT, nt = tile % NT;
            const int ml = mt * 16 + 4 * (l >> 4) + r;
            const int n = (ntile0 + nt) * 16 + (l & 15);
            const bool own = !halves || (int)((l & 15) >> 3) == (int)(blockIdx.x & 1);
            if (ml < M && n < N && own) {
                if constexpr (EPI == EPI_RESID) {
                    pre_x[i] = g.out_f32[(size_t)ml * N + n];
                    if (g.out_bf16) pre_nw[i] = g.norm_w[n];
                } else if (g.ss_in) {
                    pre_inv[i] = row_inv_rms(g.ss_in, ml, K, g.eps);
                }
            }
        } else {
            const int mt = tile / (NT / 2), jp = tile % (NT / 2);
            const int ml = mt * 16 + 4 * (l >> 4) + r;
            const bool own = !halves || (int)((l & 15) >> 3) == (int)(blockIdx.x & 1);
            if (ml < M && own) {
                pre_inv[i] = row_inv_rms(g.ss_in, ml, K, g.eps);
                if constexpr (EPI == EPI_ROPE) {
                    const int pairs_per_head = g.hd >> 5;
                    const int gp = (ntile0 >> 1) + jp;
                    const int head = gp / pairs_per_head, j = (gp % pairs_per_head) * 16 + (l & 15);
                    if (head < g.n_q + 2 * g.n_kv) pre_rope[i] = rope_prepare(g, head, j, ml);
                }
            }
        }
    }

    // Batches of U k-steps: all loads of a batch are issued before its MFMAs.  A last, partial batch requests its
    // missing steps at the wave's last tile again (cache hits) and feeds them zero activations, so that no step is
    // ever a load-wait-multiply round trip of its own.
    // With the interleaved order every workgroup also starts its walk at its own offset (a hash of its column group):
    // column groups lie a power of two apart in memory for the usual K, so workgroups that advance in step would
    // otherwise ask the same few memory channels at the same moment, which is what held these launches at 6.2 TB/s.
    const int rot = g.rotate && cnt > 0 ? (int)((blockIdx.x * 2654435761u >> 8) % (unsigned)cnt) : 0;
    auto step_of = [&](int i) -> int {                 // the wave's i-th step, i < cnt
        int ii = i + rot;
        if (ii >= cnt) ii -= cnt;
        return kb + kstep * ii;
    };
    for (int i0 = 0; i0 < cnt; i0 += U) {
        bf16x8 b[U][NT], a[U][MT];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int kk = step_of(min(i0 + u, cnt - 1));
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) b[u][nt] = load_b(nt, kk);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int kk = step_of(min(i0 + u, cnt - 1));
            const bool live = i0 + u < cnt;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const bf16x8 v = *reinterpret_cast<const bf16x8*>(ap[mt] + koff(kk));     // row 0 for lanes past M: always mapped
                a[u][mt] = av[mt] && live ? v : zero;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u][mt], b[u][nt], acc[mt][nt], 0, 0, 0);
    }

    // cross-wave reduction through LDS: red[wave][tile][r][lane]; element (tile, r, lane) is
    // row 16 mt + 4 (lane / 16) + r, column 16 (ntile0 + nt) + lane % 16.  Result in red[0 .. TOTAL).
    float* mine = red + wave * TOTAL;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 4; ++r) mine[(mt * NT + nt) * 256 + r * 64 + lane] = acc[mt][nt][r];
    __syncthreads();
    if (ksplit == 1) {
        for (int idx = tid; idx < TOTAL; idx += blockDim.x) {
            float s = 0.f;
            for (int w = 0; w < nwaves; ++w) s += red[w * TOTAL + idx];
            red[idx] = s;
        }
    } else {
        // Partial tile of this K slice to memory; the last slice to arrive adds them in slice order.
        // The exchange uses device-scope relaxed atomic stores and loads (performed at the level all
        // XCDs share, no cache-wide write-back or invalidate as a device-scope fence would cost on
        // every one of ~1000 workgroups).  Ordering: every wave waits until the memory system has
        // acknowledged its own write-through stores (vmcnt counts stores on this architecture, and a
        // workgroup-scope fence alone emits no such wait), then the barrier collects all waves, and only
        // then thread 0 takes the ticket; the last arriver's device-scope loads are issued after its own
        // ticket returned, i.e. after every other slice's stores were acknowledged.
        float* slot = g.part + ((size_t)blockIdx.x * ksplit) * TOTAL;
        for (int idx = tid; idx < TOTAL; idx += blockDim.x) {
            float s = 0.f;
            for (int w = 0; w < nwaves; ++w) s += red[w * TOTAL + idx];
            __hip_atomic_store(slot + (size_t)blockIdx.y * TOTAL + idx, s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");           // this wave's stores have been acknowledged
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();
        if (tid == 0)
            sh_last = __hip_atomic_fetch_add(g.tickets + blockIdx.x, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == ksplit - 1;
        __syncthreads();
        if (!sh_last) return;
        for (int idx = tid; idx < TOTAL; idx += blockDim.x) {
            float s = 0.f;
            for (int k = 0; k < ksplit; ++k)
                s += __hip_atomic_load(slot + (size_t)k * TOTAL + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            red[idx] = s;
        }
        if (tid == 0) __hip_atomic_store(g.tickets + blockIdx.x, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next launch
    }
    __syncthreads();

    // ---- epilogue on the final sums red[tile][r][lane] ----
    if constexpr (EPI == EPI_STORE || EPI == EPI_RESID) {
        float* sq = red + nwaves * TOTAL;                  // [MT*16][NT*16] squares of the new residual values
#pragma unroll
        for (int i = 0; i < EPT; ++i) {
            const int idx = tid + 512 * i;
            if (idx >= TOTAL) continue;
            const float s = red[idx];
            const int tile = idx >> 8, rem = idx & 255, r = rem >> 6, l = rem & 63;
            const int mt = tile / NT, nt = tile % NT;
            const int ml = mt * 16 + 4 * (l >> 4) + r;
            const int n = (ntile0 + nt) * 16 + (l & 15);
            const bool own = !halves || (int)((l & 15) >> 3) == (int)(blockIdx.x & 1);
            float v = 0.f;
            if (ml < M && n < N && own) {
                float* dst = g.out_f32 + (size_t)ml * N + n;
                if constexpr (EPI == EPI_RESID) {
                    v = pre_x[i] + s;
                    if (g.out_bf16) g.out_bf16[(size_t)ml * N + n] = (bf16_t)(v * pre_nw[i]);
                    if (g.tap) g.tap[(size_t)ml * N + n] = v;
                } else {
                    v = s * pre_inv[i];
                }
                *dst = v;
            }
            if constexpr (EPI == EPI_RESID) sq[ml * (NT * 16) + nt * 16 + (l & 15)] = v * v;
        }
        if constexpr (EPI == EPI_RESID) {
            __syncthreads();
            if (tid < M) {
                float s = 0.f;
                for (int c = 0; c < NT * 16; ++c) s += sq[tid * (NT * 16) + c];
                ss_add(g.ss_out, tid, s);
            }
        }
    } else if constexpr (EPI == EPI_SWIGLU) {
        // tiles alternate gate / up; N is the fused width 2F
        const int F = N >> 1;
#pragma unroll
        for (int i = 0; i < EPT; ++i) {
            const int idx = tid + 512 * i;
            if (idx >= OUTS) continue;
            const int pair = idx >> 8, rem = idx & 255, r = rem >> 6, l = rem & 63;
            const int mt = pair / (NT / 2), j = pair % (NT / 2);
            const int ml = mt * 16 + 4 * (l >> 4) + r;
            const int f = ((ntile0 >> 1) + j) * 16 + (l & 15);
            const bool own = !halves || (int)((l & 15) >> 3) == (int)(blockIdx.x & 1);
            if (ml < M && f < F && own) {
                const float gt = red[(mt * NT + 2 * j) * 256 + rem] * pre_inv[i];
                const float up = red[(mt * NT + 2 * j + 1) * 256 + rem] * pre_inv[i];
                g.out_bf16[(size_t)ml * F + f] = (bf16_t)(gt / (1.f + __expf(-gt)) * up);
            }
        }
    } else {
        // EPI_ROPE: tile pairs hold dims [16 jb, 16 jb + 16) and their partners hd/2 further of one head
        const int pairs_per_head = g.hd >> 5;
#pragma unroll
        for (int i = 0; i < EPT; ++i) {
            const int idx = tid + 512 * i;
            if (idx >= OUTS) continue;
            const int pair = idx >> 8, rem = idx & 255, r = rem >> 6, l = rem & 63;
            const int mt = pair / (NT / 2), jp = pair % (NT / 2);
            const int ml = mt * 16 + 4 * (l >> 4) + r;
            const int gp = (ntile0 >> 1) + jp;                      // global pair index
            const int head = gp / pairs_per_head, j = (gp % pairs_per_head) * 16 + (l & 15);
            const bool own = !halves || (int)((l & 15) >> 3) == (int)(blockIdx.x & 1);
            if (ml >= M || head >= g.n_q + 2 * g.n_kv || !own) continue;
            const float a = red[(mt * NT + 2 * jp) * 256 + rem] * pre_inv[i];
            const float b = red[(mt * NT + 2 * jp + 1) * 256 + rem] * pre_inv[i];
            rope_finish(g, head, j, ml, a, b, pre_rope[i]);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// bf16 row kernel for the narrow projections (q/k/v, attention output, FFN down) with m <= 16 rows.
// With N / 16 column tiles in the low hundreds the MFMA tiling cannot give every CU its share of the
// stream without exchanging partial sums between workgroups, which costs more than it saves.  Here W
// is row-major, a workgroup owns only R output features over the whole K range (its waves split K and
// reduce through LDS), so there are N / R workgroups and every output is final where it is computed.
// The dot products use the packed bf16 dot instruction; the activations are read from L1/L2.
// ------------------------------------------------------------------------------------------------
template <int R, int MB, int EPI>
__global__ __launch_bounds__(512) void gemv_bf16_kernel(const GemmArgs g) {
    constexpr int LPR = 64 / R;                        // lanes per weight row
    __shared__ float red[8][R][MB];
    __shared__ float sq[R][MB];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), nwaves = blockDim.x >> 6;
    const int M = g.M, N = g.N, K = g.K;
    const int KC = K >> 3;                             // 16-byte chunks per row
    const int n0 = blockIdx.x * R;
    const int r = lane / LPR, cl = lane % LPR;
    const int n = min(n0 + r, N - 1);                  // clamp: rows past the edge are computed, never stored
    const int per = (KC + nwaves - 1) / nwaves;
    const int c0 = wave * per, c1 = min(KC, c0 + per);
    if (g.ss_zero && blockIdx.x == 0) ss_clear(g.ss_zero, tid, blockDim.x);

    // epilogue operands first: their latency (and the rotary sincos) hides behind the weight stream
    const int er = tid / MB, em = tid % MB;            // epilogue element of this thread: row er, token em
    const bool active = tid < R * MB && em < M && n0 + er < N;
    float pre_inv = 1.f, pre_x = 0.f, pre_nw = 0.f;
    RopePre pre_rope{1.0, 0.0, 0};
    if constexpr (EPI == EPI_STORE) {
        if (active && g.ss_in) pre_inv = row_inv_rms(g.ss_in, em, K, g.eps);
    } else if constexpr (EPI == EPI_RESID) {
        if (active) {
            pre_x = g.out_f32[(size_t)em * N + n0 + er];
            if (g.out_bf16) pre_nw = g.norm_w[n0 + er];
        }
    } else {
        const int half = g.hd >> 1;
        const int head = blockIdx.x / half, j = blockIdx.x % half;
        if (tid < M && head < g.n_q + 2 * g.n_kv) {
            pre_inv = row_inv_rms(g.ss_in, tid, K, g.eps);
            pre_rope = rope_prepare(g, head, j, tid);
        }
    }

    float acc[MB];
#pragma unroll
    for (int m = 0; m < MB; ++m) acc[m] = 0.f;
    const bf16x8* wrow = reinterpret_cast<const bf16x8*>(g.wp) + (size_t)n * KC;
    const bf16x8* arow = reinterpret_cast<const bf16x8*>(g.a);
#pragma unroll 4
    for (int c = c0 + cl; c < c1; c += LPR) {
        const bf16x8 w = __builtin_nontemporal_load(wrow + c);
#pragma unroll
        for (int m = 0; m < MB; ++m) {
            if (m < M) {
                const bf16x8 a = arow[(size_t)m * KC + c];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bf16x2 wp2 = {w[2 * e], w[2 * e + 1]}, ap2 = {a[2 * e], a[2 * e + 1]};
                    acc[m] = __builtin_amdgcn_fdot2_f32_bf16(wp2, ap2, acc[m], false);
                }
            }
        }
    }
#pragma unroll
    for (int m = 0; m < MB; ++m) {
#pragma unroll
        for (int o = LPR / 2; o > 0; o >>= 1) acc[m] += __shfl_xor(acc[m], o, 64);
        if (cl == 0) red[wave][r][m] = acc[m];
    }
    __syncthreads();
    float s = 0.f;
    if (tid < R * MB)
        for (int w = 0; w < nwaves; ++w) s += red[w][er][em];

    if constexpr (EPI == EPI_STORE) {
        if (active) g.out_f32[(size_t)em * N + n0 + er] = s * pre_inv;
    } else if constexpr (EPI == EPI_RESID) {
        float v = 0.f;
        if (active) {
            const size_t at = (size_t)em * N + n0 + er;
            v = pre_x + s;
            g.out_f32[at] = v;
            if (g.out_bf16) g.out_bf16[at] = (bf16_t)(v * pre_nw);
            if (g.tap) g.tap[at] = v;
        }
        if (tid < R * MB) sq[er][em] = v * v;
        __syncthreads();
        if (tid < M) {
            float t = 0.f;
#pragma unroll
            for (int i = 0; i < R; ++i) t += sq[i][tid];
            ss_add(g.ss_out, tid, t);
        }
    } else {
        // EPI_ROPE (R == 2): the two rows are dim j of a head and its rotation partner j + hd/2
        if (tid < R * MB) sq[er][em] = s;
        __syncthreads();
        const int half = g.hd >> 1;
        const int head = blockIdx.x / half, j = blockIdx.x % half;
        if (tid < M && head < g.n_q + 2 * g.n_kv) rope_finish(g, head, j, tid, sq[0][tid] * pre_inv, sq[1][tid] * pre_inv, pre_rope);
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
// The library's own launch choices.  Most tokens of a pass that a projection serves from its row-major copy (1B
// shape, microseconds, row kernel against tile kernel: q/k/v 6.9 / 6.1 at one row, 7.9 / 6.3 at two: the tile kernel
// with two workgroups per column group always wins; attention output 4.4 / 4.9 and 5.2 / 5.0; FFN down 7.8 / 9.4 and
// 9.5 / 9.5).
const hsd_kernel_tuning& default_kernel_tuning() {
    static const hsd_kernel_tuning t = {{0, 0, 0, 0}, {0, 0, 0, 0}, 0, {0, 0, 0, 0}, 0, 1, 2, 128, 1 << 30, 0, 256, 1, 0, 0};
    return t;
}

const hsd_driver_tuning& default_driver_tuning() {
    static const hsd_driver_tuning t = {32768, 1, 1};
    return t;
}

extern "C" void hsd_kernel_tuning_default(hsd_kernel_tuning* t) {
    if (t) *t = default_kernel_tuning();
}

extern "C" void hsd_driver_tuning_default(hsd_driver_tuning* t) {
    if (t) *t = default_driver_tuning();
}

// Above 64 rows the tiled kernel wins at every shape measured (7B-shaped layer, 128 rows: 42-100 us against 48-130 us
// for two weight streams; 256 rows: 1.8-4 x); the per-64-rows path stays as the alternative the setting selects.
static bool use_wide_kernel(int m, const hsd_kernel_tuning& t) {
    if (m <= HSD_MAX_PASS_ROWS) return false;
    return t.wide_min_rows > 0 ? m >= t.wide_min_rows : true;
}

GemmPlan gemm_plan(int m, int n, int k, int epi, const hsd_kernel_tuning& t) {
    GemmPlan p{1, 1, 8, 0, t.gemm_deep, 0};
    const int mt = m <= 16 ? 1 : (m <= 32 ? 2 : 4);
    const int ntiles = ceil_div(n, 16), KT = k / 32;
    switch (epi) {
        // wide q/k/v matrices (640 tiles and more: the 7B and 70B shapes) in passes of few rows: two rotary pairs per
        // workgroup and no K split, 160-192 workgroups that each stream 0.5-1 MB in the interleaved order, instead of
        // 384-960 short ones (70B-shaped 31.6 -> 28.8 us at one row, 32.6 -> 30.6 at four; 7B-shaped 23.8 -> 21.1 at 16);
        // with K = 8192 it loses from 12 rows on, with 384 tiles (8B shape) or fewer at every row count
        case EPI_ROPE: p.nt = mt <= 2 && ntiles >= 640 && (m <= 8 || k <= 4096) ? 4 : 2; break;
        // from 16 rows on, four tiles per workgroup where that still leaves 448 workgroups: the activations cross the L2
        // half as often (70B-shaped gate/up at 32 rows 193 -> 176 us, 8B-shaped 59.8 -> 48.9; the 7B shape, 344
        // workgroups, loses)
        case EPI_SWIGLU: p.nt = mt <= 2 && (ntiles >= 4096 || (m >= 16 && ntiles >= 1792)) ? 4 : 2; break;
        // long K (the FFN down projections, the widest attention output): two column tiles per workgroup halve how often
        // the activations (K values per row, re-read by every workgroup) cross the L2, which at 8 rows and K = 28672 is
        // as many bytes as the weights (70B-shaped down 78.9 -> 70.1 us at 8 rows, 72.2 -> 70.6 at 4)
        case EPI_RESID: p.nt = ntiles >= 2048 || (k >= 8192 && ntiles >= 256) ? 2 : 1; break;
        default: p.nt = ntiles >= 8192 && mt <= 2 ? 4 : (ntiles >= 1024 ? 2 : 1); break;
    }
    if (t.gemm_nt[epi] && (epi != EPI_ROPE || t.gemm_nt[epi] == 2 || (t.gemm_nt[epi] == 4 && mt <= 2))) p.nt = t.gemm_nt[epi];
    if (mt == 4 && p.nt > 2) p.nt = 2;
    // about a thousand workgroups: every CU must be pulling for the HBM stream to reach its peak
    // Splitting K across workgroups costs a round trip through memory for the partial tiles, which only pays for
    // plain stores of narrow matrices; the fused epilogues keep K inside the workgroup.
    // Two measured exceptions: a RoPE matrix of 128 MB or more in at most 384 groups (1.25-1.5 workgroups per CU:
    // the uneven second round costs a third of the bandwidth; 3 slices, 4 above 8 rows, even it out), and a residual matrix with at
    // most 128 groups and K >= 8192 (half the CUs idle; 2 slices).
    const int groups = ceil_div(ntiles, p.nt);
    p.ksplit = epi == EPI_STORE ? (1024 + groups / 2) / groups : 1;
    if (epi == EPI_ROPE && p.nt == 2 && groups <= 384 && (size_t)n * k * 2 >= ((size_t)128 << 20)) p.ksplit = m <= 8 ? 3 : 4;
    if (epi == EPI_RESID && groups <= 128 && k >= 8192) p.ksplit = 2;
    // Narrow matrices (at most 128 column groups: half the CUs would idle) with few rows: two workgroups per group,
    // each owning 8 of the 16 columns of its tiles, instead of slices of K: twice the workgroups without an exchange
    // (1B shape, 4-8 rows: down 10.8 -> 10.2 us, q/k/v 7.4 -> 6.9; 16 layers: -3.5 % per pass).  Each half reads all the
    // activations, which from 16 rows on costs the residual projections more than the extra workgroups give
    // (32 rows: down 16.6 -> 21 us), and 256-group matrices (7B shape) lose at every row count.
    if (epi == EPI_RESID && p.nt == 1 && groups <= t.halves_max_groups && m <= 8) {
        p.halves = 1;
        p.ksplit = 1;
    }
    if (epi == EPI_ROPE && p.ksplit == 1 && groups <= t.halves_max_groups && m <= 32) p.halves = 1;
    if (t.gemm_ksplit[epi]) { p.ksplit = t.gemm_ksplit[epi]; p.halves = 0; }
    if (p.ksplit > 8) p.ksplit = 8;
    if (p.ksplit > KT) p.ksplit = KT;
    if (p.ksplit < 1) p.ksplit = 1;
    // How the eight waves of a workgroup share its k-steps.  With a contiguous slice per wave a workgroup streams eight
    // far-apart runs per tile; with the steps dealt round-robin to groups of four waves, the requests of a round are
    // two contiguous 4 KB runs per tile, which the memory system serves faster once a workgroup's share of K is long
    // (>= 4096: 16 KB or more per wave and tile) and the pass is a few rows (one row tile).  Measured at 1-8 rows:
    // 70B-shaped gate/up 151 -> 136 us (6.9 TB/s), 128256 x 8192 head 337 -> 302, 128256 x 4096 head 163 -> 152,
    // 8B-shaped gate/up 43.5 -> 38.5 and q/k/v 12.4 -> 11.3, 7B-shaped gate/up 35.2 -> 30.2 and q/k/v 23.0 -> 20.0,
    // 70B-shaped attention output 24.6 -> 23.5; with the deeper load batches it gains less, so those go.  The kernel
    // then also starts every workgroup's walk at its own offset (another 0.5-1 %).  Groups of two or eight waves gain
    // less or lose; shorter K (1B shape) is indifferent; passes of more than 16 rows lose up to 8 % and keep the
    // contiguous slices, as does the longest residual projection (K = 28672) from five rows on.
    const int k_wg = k / p.ksplit;
    if (t.gemm_interleave[epi]) {
        p.interleave = t.gemm_interleave[epi] > 0 ? t.gemm_interleave[epi] : 1;
    } else if (k_wg >= 4096 && (m <= 16 || (epi == EPI_SWIGLU && p.nt == 4 && m <= 32)) && !p.halves) {
        if (epi != EPI_RESID) {
            p.interleave = 4;
            if (!p.deep) p.deep = -1;
        } else if (m <= 4 || (m <= 8 && k <= 16384) || (k >= 8192 && k <= 16384)) {
            // residual projections: every K up to four rows (70B-shaped down 70.7 -> 70.1 us), K up to 16384 up to eight
            // (7B-shaped down 20.4 -> 19.3), 8192..16384 up to sixteen; beyond, the contiguous slices are ahead
            p.interleave = 4;
        }
    }
    if (p.ksplit > 8) p.ksplit = 8;
    if (p.ksplit > KT) p.ksplit = KT;
    if (p.ksplit < 1) p.ksplit = 1;
    p.waves = 8;                 // always 512 threads: the epilogue addresses its elements by that stride
    return p;
}

size_t gemm_part_bytes(int m, int n, int k, int epi) {
    const GemmPlan p = gemm_plan(m, n, k, epi);
    const int mt = m <= 16 ? 1 : (m <= 32 ? 2 : 4);
    return p.ksplit == 1 ? 0 : (size_t)ceil_div(ceil_div(n, 16), p.nt) * p.ksplit * mt * p.nt * 256 * sizeof(float);
}

static size_t gemm_lds_bytes(const GemmPlan& p, int m, int epi) {
    const int mt = m <= 16 ? 1 : (m <= 32 ? 2 : 4);
    size_t b = (size_t)p.waves * mt * p.nt * 256 * sizeof(float);
    if (epi == EPI_RESID) b += (size_t)mt * 16 * p.nt * 16 * sizeof(float);
    return b;
}

template <int NT, int MT, int EPI>
static void launch_inst(const GemmArgs& g, const GemmPlan& p, hipStream_t s) {
    const int ntiles = ceil_div(g.N, 16);
    GemmArgs a = g;
    a.halves = p.halves && p.ksplit == 1;
    a.interleave = p.interleave;
    a.rotate = p.interleave > 1;
    dim3 grid(ceil_div(ntiles, NT) * (a.halves ? 2 : 1), p.ksplit);
    const bool deep = p.deep ? p.deep > 0 : (a.K / p.ksplit >= 4096 && a.K / p.ksplit < 8192);
    const size_t lds = gemm_lds_bytes(p, a.M, EPI);
    // four row tiles x two column tiles of a residual projection need 72 KB: above 64 KB a kernel must be told once
    if (lds > 64 * 1024) {
        static bool told[2] = {false, false};
        if (!told[deep]) {
            const void* fn = deep ? (const void*)gemm_bf16_kernel<NT, MT, EPI, true> : (const void*)gemm_bf16_kernel<NT, MT, EPI, false>;
            if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess) told[deep] = true;
            else (void)hipGetLastError();      // the launch below reports what is wrong, if anything
        }
    }
    if (deep)
        gemm_bf16_kernel<NT, MT, EPI, true><<<grid, p.waves * 64, lds, s>>>(a);
    else
        gemm_bf16_kernel<NT, MT, EPI, false><<<grid, p.waves * 64, lds, s>>>(a);
}

// Name of the kernel instance launch_gemm_bf16 runs for a plan, as a profiler prints it.
void gemm_kernel_name(int m, int k, int epi, const GemmPlan& p, char* out, size_t cap) {
    const int mt = m <= 16 ? 1 : (m <= 32 ? 2 : 4);
    const bool deep = p.deep ? p.deep > 0 : (k / p.ksplit >= 4096 && k / p.ksplit < 8192);
    snprintf(out, cap, "gemm_bf16_kernel<%d, %d, %d, %s>", p.nt, mt, epi, deep ? "true" : "false");
}

static int check_gemm(int m, int n, int k, int max_rows = HSD_MAX_PASS_ROWS) {
    if (m < 1 || m > max_rows) HSD_FAIL(HSD_EINVAL, "gemm: m=%d outside 1..%d", m, max_rows);
    if (n < 1 || k < 32 || k % 32 != 0) HSD_FAIL(HSD_EINVAL, "gemm: n=%d k=%d (k must be a positive multiple of 32)", n, k);
    return HSD_OK;
}

int launch_gemm_bf16(const GemmArgs& g, int epi, const GemmPlan& plan, hipStream_t s) {
    if (int rc = check_gemm(g.M, g.N, g.K)) return rc;
    GemmPlan p = plan;
    const int mt = g.M <= 16 ? 1 : (g.M <= 32 ? 2 : 4);
    if (p.ksplit > 1) {
        if (!g.part || !g.tickets) HSD_FAIL(HSD_EINVAL, "gemm: split-K launch without partial / ticket buffers");
        // the partial tiles must fit the caller's buffer (plans can change after it was sized: tuning overrides)
        const size_t need = (size_t)ceil_div(ceil_div(g.N, 16), p.nt) * p.ksplit * mt * p.nt * 256 * sizeof(float);
        if (need > g.part_bytes) p.ksplit = 1;
    }
#define HSD_CASE(NT_, MT_, E_)                                  \
    if (p.nt == NT_ && mt == MT_ && epi == E_) {                \
        launch_inst<NT_, MT_, E_>(g, p, s);                     \
        HSD_LAUNCH_CHECK();                                     \
        return HSD_OK;                                          \
    }
#define HSD_MTS(NT_, E_) HSD_CASE(NT_, 1, E_) HSD_CASE(NT_, 2, E_) HSD_CASE(NT_, 4, E_)
    HSD_MTS(1, EPI_STORE) HSD_MTS(2, EPI_STORE) HSD_CASE(4, 1, EPI_STORE) HSD_CASE(4, 2, EPI_STORE)
    HSD_MTS(1, EPI_RESID) HSD_MTS(2, EPI_RESID)
    HSD_MTS(2, EPI_SWIGLU) HSD_CASE(4, 1, EPI_SWIGLU) HSD_CASE(4, 2, EPI_SWIGLU)
    HSD_MTS(2, EPI_ROPE) HSD_CASE(4, 1, EPI_ROPE) HSD_CASE(4, 2, EPI_ROPE)
#undef HSD_MTS
#undef HSD_CASE
    HSD_FAIL(HSD_EINVAL, "gemm: no kernel for nt=%d m=%d epilogue=%d", p.nt, g.M, epi);
}

template <int R, int EPI>
static int launch_gemv_mb(const GemmArgs& g, hipStream_t s) {
    const int grid = ceil_div(g.N, R);
    int waves = 8;
    while (waves > 1 && (g.K >> 3) < waves * (64 / R)) waves >>= 1;     // at least one chunk per lane
    const int mb = g.M <= 1 ? 1 : (g.M <= 2 ? 2 : (g.M <= 4 ? 4 : (g.M <= 8 ? 8 : 16)));
    switch (mb) {
        case 1: gemv_bf16_kernel<R, 1, EPI><<<grid, waves * 64, 0, s>>>(g); break;
        case 2: gemv_bf16_kernel<R, 2, EPI><<<grid, waves * 64, 0, s>>>(g); break;
        case 4: gemv_bf16_kernel<R, 4, EPI><<<grid, waves * 64, 0, s>>>(g); break;
        case 8: gemv_bf16_kernel<R, 8, EPI><<<grid, waves * 64, 0, s>>>(g); break;
        default: gemv_bf16_kernel<R, 16, EPI><<<grid, waves * 64, 0, s>>>(g); break;
    }
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

// Row-major W: 16 tokens per launch (the pass only sends one or two tokens here; more would make the
// per-token activation reads outweigh the weight stream, and the tiled kernel serves them).
int launch_gemv_bf16(const GemmArgs& g0, int epi, hipStream_t s) {
    if (int rc = check_gemm(g0.M, g0.N, g0.K, HSD_MAX_GEMM_ROWS)) return rc;
    if (epi == EPI_ROPE && g0.N != (g0.n_q + 2 * g0.n_kv) * g0.hd) HSD_FAIL(HSD_EINVAL, "gemv: q/k/v width mismatch");
    for (int m0 = 0; m0 < g0.M; m0 += 16) {
        GemmArgs g = g0;
        g.M = g0.M - m0 < 16 ? g0.M - m0 : 16;
        g.a = g0.a + (size_t)m0 * g0.K;
        if (g.ss_in) g.ss_in = g0.ss_in + m0;
        if (g.ss_out) g.ss_out = g0.ss_out + m0;
        if (m0 > 0) g.ss_zero = nullptr;
        if (epi == EPI_ROPE) {
            if (g0.pos0_arr && g0.M > 16) HSD_FAIL(HSD_EINVAL, "gemv: a batch of sequences takes at most 16 rows here");
            g.out_bf16 = g0.out_bf16 + (size_t)m0 * g0.n_q * g0.hd;
            g.pos0 = g0.pos0 + m0;
        } else {
            g.out_f32 = g0.out_f32 + (size_t)m0 * g0.N;
            if (g0.out_bf16) g.out_bf16 = g0.out_bf16 + (size_t)m0 * g0.N;
            if (g0.tap) g.tap = g0.tap + (size_t)m0 * g0.N;
        }
        int rc;
        if (epi == EPI_ROPE) rc = launch_gemv_mb<2, EPI_ROPE>(g, s);
        else if (epi == EPI_RESID) rc = g.N <= 4096 ? launch_gemv_mb<2, EPI_RESID>(g, s) : launch_gemv_mb<4, EPI_RESID>(g, s);
        else rc = g.N <= 4096 ? launch_gemv_mb<2, EPI_STORE>(g, s) : launch_gemv_mb<4, EPI_STORE>(g, s);
        if (rc) return rc;
    }
    return HSD_OK;
}

int launch_gemm_f32(const float* x, const float* w, float* out, int m, int n, int k, bool swiglu, hipStream_t s) {
    if (int rc = check_gemm(m, n, k, HSD_MAX_GEMM_ROWS)) return rc;
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

extern "C" int hsd_pack_weight(const void* w_dev, void* packed_dev, int n, int k, int dtype, int layout, void* stream) {
    if (!w_dev || !packed_dev || n < 1 || (dtype != HSD_F32 && dtype != HSD_BF16) || (layout != HSD_LAYOUT_TILES && layout != HSD_LAYOUT_ROWS))
        HSD_FAIL(HSD_EINVAL, "hsd_pack_weight: bad arguments");
    hipStream_t s = (hipStream_t)stream;
    HSD_HIP(hipMemsetAsync(packed_dev, 0, hsd_packed_bytes(n, k, dtype), s));
    return launch_pack(w_dev, packed_dev, n, k, dtype, 0, 0, 0, layout == HSD_LAYOUT_ROWS, s);
}

// split-K partial tiles of the widest plan any 64-row block of an m-row product may use
static size_t gemm_store_part_bytes(int m, int n, int k) {
    size_t b = gemm_part_bytes(std::min(m, (int)HSD_MAX_PASS_ROWS), n, k, EPI_STORE);       // the full blocks
    if (m > HSD_MAX_PASS_ROWS && m % HSD_MAX_PASS_ROWS) b = std::max(b, gemm_part_bytes(m % HSD_MAX_PASS_ROWS, n, k, EPI_STORE));
    return align_up(b, 256);
}

extern "C" size_t hsd_gemm_workspace_bytes(int m, int n, int k) {
    if (m < 1 || m > HSD_MAX_GEMM_ROWS || n < 1 || k < 32) return 0;
    return gemm_store_part_bytes(m, n, k) + align_up((size_t)ceil_div(n, 16) * sizeof(int), 256);
}

static int gemm_entry(const void* x_dev, const void* packed_dev, float* y_dev, int m, int n, int k, int dtype, int layout,
                      void* workspace_dev, void* stream, const hsd_kernel_tuning& t, const char* who) {
    if (!x_dev || !packed_dev || !y_dev || !workspace_dev || (dtype != HSD_F32 && dtype != HSD_BF16) ||
        (layout != HSD_LAYOUT_TILES && layout != HSD_LAYOUT_ROWS))
        HSD_FAIL(HSD_EINVAL, "%s: bad arguments", who);
    if (int rc = check_gemm(m, n, k, HSD_MAX_GEMM_ROWS)) return rc;
    hipStream_t s = (hipStream_t)stream;
    if (dtype == HSD_F32) return launch_gemm_f32((const float*)x_dev, (const float*)packed_dev, y_dev, m, n, k, false, s);
    if (layout == HSD_LAYOUT_ROWS) {
        GemmArgs g = {};
        g.a = (const bf16_t*)x_dev;
        g.wp = (const bf16x8*)packed_dev;
        g.M = m; g.N = n; g.K = k;
        g.out_f32 = y_dev;
        return launch_gemv_bf16(g, EPI_STORE, s);
    }
    if (use_wide_kernel(m, t))
        return launch_gemm_wide_bf16((const bf16_t*)x_dev, (const bf16x8*)packed_dev, y_dev, m, n, k, t.wide_cols, s);
    const size_t part_bytes = gemm_store_part_bytes(m, n, k);
    GemmArgs g = {};
    g.wp = (const bf16x8*)packed_dev;
    g.N = n; g.K = k;
    g.part = (float*)workspace_dev;
    g.part_bytes = part_bytes;
    g.tickets = (int*)((char*)workspace_dev + part_bytes);
    HSD_HIP(hipMemsetAsync(g.tickets, 0, (size_t)ceil_div(n, 16) * sizeof(int), s));
    // one weight stream per block of 64 rows; the blocks share the workspace, in stream order (the last arriver of a
    // column group leaves its ticket at zero for the next launch)
    for (int m0 = 0; m0 < m; m0 += HSD_MAX_PASS_ROWS) {
        g.M = std::min((int)HSD_MAX_PASS_ROWS, m - m0);
        g.a = (const bf16_t*)x_dev + (size_t)m0 * k;
        g.out_f32 = y_dev + (size_t)m0 * n;
        if (int rc = launch_gemm_bf16(g, EPI_STORE, gemm_plan(g.M, n, k, EPI_STORE, t), s)) return rc;
    }
    return HSD_OK;
}

extern "C" int hsd_gemm(const void* x_dev, const void* packed_dev, float* y_dev, int m, int n, int k, int dtype, int layout,
                        void* workspace_dev, void* stream) {
    return gemm_entry(x_dev, packed_dev, y_dev, m, n, k, dtype, layout, workspace_dev, stream, default_kernel_tuning(), "hsd_gemm");
}

extern "C" int hsd_gemm_tuned(const void* x_dev, const void* packed_dev, float* y_dev, int m, int n, int k, int dtype, int layout,
                              void* workspace_dev, void* stream, const hsd_kernel_tuning* t) {
    return gemm_entry(x_dev, packed_dev, y_dev, m, n, k, dtype, layout, workspace_dev, stream, t ? *t : default_kernel_tuning(),
                      "hsd_gemm_tuned");
}
