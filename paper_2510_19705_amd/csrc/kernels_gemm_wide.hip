// Many-row GEMM y[m, n] = sum_k a[m, k] W[n, k] for 64 < m: the batched verification cells of the layer
// microbenchmark (a batch of sequences times k drafted tokens each gives hundreds of rows per weight load,
// Sec. 3.1: every load of the weights should serve as many tokens as possible).  From a few hundred rows on the
// matrix cores, not the weight stream, bound the time, so this kernel is tiled for them:
//
//   workgroup = 4 waves, 128 rows x 256 columns of y; wave w owns four 16-column tiles and all 128 rows
//   (32 accumulator tiles of the 16x16x32 MFMA, 128 registers).  Per MFMA cycle a 128 x 64 wave tile needs half
//   of what the LDS and a quarter of what the vector cache can deliver; smaller tiles would saturate one of them.
//   W operand: the packed 1 KiB tiles are already in B-operand lane order, so each wave loads its own tiles straight
//   from memory into a ring of eight register sets, seven 32-wide k steps ahead of their use (nothing of W is shared
//   between the waves of a workgroup).
//   A operand: every wave needs all 128 rows, so slabs of 128 rows x 128 k go through LDS, stored in A-operand lane
//   order (a wave's 16-byte reads are one contiguous KiB: no bank conflicts), double-buffered, one barrier per slab;
//   their global loads are spread over the slab before the one that copies them into LDS.
//   The accumulators leave one wave per SIMD, so nothing but the wave's own instruction order hides a latency: every
//   k step issues the LDS reads of the next step's A operand and its share of the global loads in between its 32
//   MFMAs (scheduling groups pin that order), and no load sits under a branch (the compiler would lose count of the
//   loads in flight and wait for all of them at every use): addresses are clamped instead, and what a clamped load
//   brought in is replaced by zeros on its way into LDS.
//
// Workgroups that share a column block (the row blocks of one 256-column strip) get consecutive slots on one XCD
// (block id mod 8 picks the XCD), so W comes from HBM once and from that XCD's L2 for the other row blocks.
#include "common.h"

namespace {

constexpr int WIDE_ROWS = 128;                          // rows per workgroup
constexpr int WIDE_MT = WIDE_ROWS / 16;                 // 16-row tiles per workgroup (every wave computes all)
constexpr int WIDE_WAVES = 4;
constexpr int WIDE_SKT = 4;                             // 32-wide k steps per LDS slab
constexpr int WIDE_NB = 8;                              // ring of W register sets, one per k step in flight
constexpr int WIDE_APT = WIDE_SKT * WIDE_MT * 64 / (WIDE_WAVES * 64);   // 16-byte A chunks per thread and slab: 8
static_assert(WIDE_NB == 2 * WIDE_SKT && WIDE_APT == 2 * WIDE_SKT, "the main loop is unrolled over two slabs");

// WIDE_NT: 16-column tiles per wave (4: 256 columns per workgroup; 2: 128 columns: twice the LDS reads per MFMA, ~80 %
// of the LDS rate, but half the registers, so two workgroups share a CU and each covers the other's first loads,
// last stores and barriers)
template <int WIDE_NT>
__device__ __forceinline__ void gemm_wide_body(const bf16_t* __restrict__ a, const bf16x8* __restrict__ wp, float* __restrict__ out,
                                               int M, int N, int K, int mblocks, int nblocks) {
    constexpr int WIDE_COLS = WIDE_WAVES * WIDE_NT * 16;
    __shared__ bf16x8 lds_a[2][WIDE_SKT][WIDE_MT][64];          // 64 KiB
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int mblk = slot % mblocks, nblk = (slot / mblocks) * 8 + xcd;
    if (nblk >= nblocks) return;                                 // the padding of the last group of eight strips
    const int KT = K >> 5;
    const int slabs = (KT + WIDE_SKT - 1) / WIDE_SKT;
    const int ntiles = (N + 15) >> 4;
    const int row0 = mblk * WIDE_ROWS;

    // A chunk i of this thread and slab: k step i / 2, row tile wave + 4 (i % 2), lane's place in the operand;
    // LDS slot (k step, row tile, lane) in storage order
    const bf16_t* ap[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int r = min(row0 + (wave + 4 * h) * 16 + (lane & 15), M - 1);   // clamp: rows past the edge are computed, never stored
        ap[h] = a + (size_t)r * K + (lane >> 4) * 8;
    }
    const bf16x8* bp[WIDE_NT];
#pragma unroll
    for (int nt = 0; nt < WIDE_NT; ++nt) {
        const int t = min(nblk * (WIDE_COLS / 16) + wave * WIDE_NT + nt, ntiles - 1);
        bp[nt] = wp + (size_t)t * KT * 64 + lane;
    }
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    auto load_a = [&](int slab, int j, bf16x8 (&r)[WIDE_APT]) {                // the two chunks of k step j
        const int kt = min(slab * WIDE_SKT + j, KT - 1);
#pragma unroll
        for (int h = 0; h < 2; ++h) r[2 * j + h] = *reinterpret_cast<const bf16x8*>(ap[h] + (size_t)kt * 32);
    };
    auto store_a = [&](int slab, int i0, int i1, const bf16x8 (&r)[WIDE_APT]) {   // chunks [i0, i1); k steps past the end: zero rows of A
#pragma unroll
        for (int i = i0; i < i1; ++i)
            lds_a[slab & 1][i >> 1][wave + 4 * (i & 1)][lane] = slab * WIDE_SKT + (i >> 1) < KT ? r[i] : zero;
    };
    auto load_b = [&](int kt, bf16x8 (&b)[WIDE_NT]) {
        const int k = min(kt, KT - 1);                                         // past the end: any valid tile, its A rows are zero
#pragma unroll
        for (int nt = 0; nt < WIDE_NT; ++nt) b[nt] = bp[nt][(size_t)k * 64];
    };

    f32x4 acc[WIDE_MT][WIDE_NT];
#pragma unroll
    for (int mt = 0; mt < WIDE_MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < WIDE_NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    bf16x8 aq[2][WIDE_APT], bq[WIDE_NB][WIDE_NT], af[2][WIDE_MT];
#pragma unroll
    for (int j = 0; j < WIDE_SKT; ++j) load_a(0, j, aq[0]);
    store_a(0, 0, WIDE_APT, aq[0]);
#pragma unroll
    for (int j = 0; j < WIDE_SKT; ++j) load_a(1, j, aq[1]);                    // stored during slab 0
#pragma unroll
    for (int u = 0; u < WIDE_NB - 1; ++u) load_b(u, bq[u]);
    __syncthreads();
#pragma unroll
    for (int mt = 0; mt < WIDE_MT; ++mt) af[0][mt] = lds_a[0][0][mt][lane];

    // Two slabs per trip, so that every ring index is a constant; the slab count is rounded up to even (a padding
    // slab multiplies zeros).  Slab s computes from LDS buffer s & 1 and, in its second and third steps, fills the
    // other buffer with slab s + 1 (loaded from memory during slab s - 1).  The one barrier of a slab stands before
    // its last step: by then the other buffer is complete, so that step can already fetch the first operands of
    // slab s + 1, and the buffer it overwrites two steps later has been read for the last time.
    const int padded = (slabs + 1) & ~1;
    for (int s0 = 0; s0 < padded; s0 += 2) {
#pragma unroll
        for (int sp = 0; sp < 2; ++sp) {
            const int s = s0 + sp;                                             // LDS buffer sp
#pragma unroll
            for (int j = 0; j < WIDE_SKT; ++j) {
                const int u = sp * WIDE_SKT + j;                               // W set of this step
                __builtin_amdgcn_sched_barrier(0);
                if (j == WIDE_SKT - 1) {
                    __syncthreads();
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int mt = 0; mt < WIDE_MT; ++mt)
                    af[(j + 1) & 1][mt] = j + 1 < WIDE_SKT ? lds_a[sp][j + 1][mt][lane] : lds_a[sp ^ 1][0][mt][lane];
                load_b(s * WIDE_SKT + j + WIDE_NB - 1, bq[(u + WIDE_NB - 1) % WIDE_NB]);   // into the set the step before used
                load_a(s + 2, j, aq[sp]);                                      // stored during slab s + 1
                if (j == 1) store_a(s + 1, 0, WIDE_APT / 2, aq[sp ^ 1]);
                if (j == 2) store_a(s + 1, WIDE_APT / 2, WIDE_APT, aq[sp ^ 1]);
#pragma unroll
                for (int mt = 0; mt < WIDE_MT; ++mt)
#pragma unroll
                    for (int nt = 0; nt < WIDE_NT; ++nt)
                        acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[j & 1][mt], bq[u][nt], acc[mt][nt], 0, 0, 0);
                // order within the step: after every WIDE_NT MFMAs (one row tile) one LDS read, then the step's global
                // loads one by one and, in the steps that fill the other buffer, four times one LDS write
#pragma unroll
                for (int g = 0; g < 8; ++g) {
                    __builtin_amdgcn_sched_group_barrier(0x008, WIDE_NT, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    if (g < WIDE_NT + 2) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
                    if ((j == 1 || j == 2) && g >= 4) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
                }
            }
        }
    }

    // accumulator element r of lane (j, grp): row 16 mt + 4 grp + r, column 16 tile + j
    const int j = lane & 15, grp = lane >> 4;
#pragma unroll
    for (int nt = 0; nt < WIDE_NT; ++nt) {
        const int tile = nblk * (WIDE_COLS / 16) + wave * WIDE_NT + nt;
        const int n = tile * 16 + j;
        if (tile >= ntiles || n >= N) continue;
#pragma unroll
        for (int mt = 0; mt < WIDE_MT; ++mt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int m = row0 + mt * 16 + 4 * grp + r;
                if (m < M) out[(size_t)m * N + n] = acc[mt][nt][r];
            }
    }
}

__global__ __launch_bounds__(WIDE_WAVES * 64) void gemm_wide_bf16_kernel_256(const bf16_t* __restrict__ a, const bf16x8* __restrict__ wp,
                                                                             float* __restrict__ out, int M, int N, int K, int mblocks,
                                                                             int nblocks) {
    gemm_wide_body<4>(a, wp, out, M, N, K, mblocks, nblocks);
}

// register budget of two waves per SIMD (256): fits without spills
__global__ __launch_bounds__(WIDE_WAVES * 64) __attribute__((amdgpu_waves_per_eu(2))) void gemm_wide_bf16_kernel_128(
    const bf16_t* __restrict__ a, const bf16x8* __restrict__ wp, float* __restrict__ out, int M, int N, int K, int mblocks, int nblocks) {
    gemm_wide_body<2>(a, wp, out, M, N, K, mblocks, nblocks);
}

}  // namespace

// Column strips of 256, unless they leave at least half of the 256 CUs idle: then strips of 128 (twice the workgroups,
// still one round).  wide_cols = 128 or 256 fixes the width (a tuning setting), 0 takes the rule.
static int wide_nt(int m, int n, int wide_cols) {
    if (wide_cols == 128) return 2;
    if (wide_cols == 256) return 4;
    return ceil_div(m, WIDE_ROWS) * ceil_div(n, 256) <= 128 ? 2 : 4;
}

// bf16, packed tiles.  Shapes are the caller's to check (m >= 1, k a positive multiple of 32).
int launch_gemm_wide_bf16(const bf16_t* a, const bf16x8* wp, float* out, int m, int n, int k, int wide_cols, hipStream_t s) {
    const int nt = wide_nt(m, n, wide_cols);
    const int mblocks = ceil_div(m, WIDE_ROWS), nblocks = ceil_div(n, WIDE_WAVES * nt * 16);
    const long long grid = 8ll * mblocks * ceil_div(nblocks, 8);
    if (grid > 0x7fffffffll) HSD_FAIL(HSD_EINVAL, "gemm: %d x %d is too large for one launch", m, n);
    if (nt == 2)
        gemm_wide_bf16_kernel_128<<<dim3((unsigned)grid), WIDE_WAVES * 64, 0, s>>>(a, wp, out, m, n, k, mblocks, nblocks);
    else
        gemm_wide_bf16_kernel_256<<<dim3((unsigned)grid), WIDE_WAVES * 64, 0, s>>>(a, wp, out, m, n, k, mblocks, nblocks);
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}
