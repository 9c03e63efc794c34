// The rejection rule of Alg. 2 (App. B.1) / Sec. 2 on the device: accept tests for the t drafted tokens, then the
// corrected token from the normalised residual max(0, p - q) or the bonus token from p_{t+1}.  Random numbers are
// Philox4x32-10 blocks addressed by (seed; slot, call, level), so nothing depends on launch geometry; sums are over
// integer fixed-point weights, so any reduction order gives the same token.  Three kernels:
//  * accept_resample_kernel (any vocabulary): every workgroup evaluates the t accept tests (lane i tests draft i,
//    first rejection by ballot), sums the weights of its slice of the chosen row; the last workgroup to finish
//    (device-scope ticket) scans the slice totals, locates the slice that holds the threshold and scans inside it;
//  * accept_resample_small_kernel (vocabulary <= 32768): the same in one workgroup that holds the row in registers;
//  * softmax_verify_kernel (vocabulary <= 32768): softmax of the logit rows, the accept tests and the draw fused, one
//    workgroup per row, plus what the driver needs next (results in pinned host memory, the emitted token embedded).
#include <algorithm>

#include "common.h"
#include "softmax_row.h"
#include "model.h"

namespace {

constexpr int SLICE = 2048;          // elements per workgroup
constexpr int THREADS = 256;
constexpr int PER_THREAD = SLICE / THREADS;

// `coin` in the kernels below: negative = Alg. 2's test; in [0, 1] = the ablation of the appendix on the assumptions
// of HSD, where every draft is accepted with that fixed probability (u < coin, same Philox word).
struct Philox4 { uint32_t w[4]; };

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return Philox4{{c0, c1, c2, c3}};
}

// floor(r * 2^62) for an fp32 r in [0, 1], exactly, with integer operations only (a double multiply and a
// double -> uint64 conversion cost several times more): r = mant * 2^(exp - 150), so the weight is mant shifted by
// exp - 88 (at most 39 to the left for r = 1).  Values below 2^-62, subnormals included, give 0.
__device__ __forceinline__ uint64_t fixed_weight(float r) {
    const uint32_t bits = __float_as_uint(r);
    const int exp = (int)(bits >> 23) & 0xFF;
    const uint64_t mant = (uint64_t)((bits & 0x7FFFFFu) | 0x800000u);
    const int shift = exp - 88;
    if (exp == 0 || shift <= -24) return 0;
    return shift >= 0 ? mant << shift : mant >> -shift;
}

// scratch layout: [0] ticket counter (uint32), then slice totals: resid[nslices], plain[nslices] (uint64)
__global__ __launch_bounds__(THREADS) void accept_resample_kernel(const float* __restrict__ p, const float* __restrict__ q,
                                                                  int32_t* __restrict__ x, int t, int V, uint32_t k0,
                                                                  uint32_t k1, uint32_t level, uint32_t call,
                                                                  int32_t* __restrict__ result, uint32_t* ticket,
                                                                  uint64_t* totals, float coin) {
    __shared__ int sh_n;
    __shared__ uint64_t sh_a[THREADS / 64], sh_b[THREADS / 64];
    __shared__ bool sh_last;
    __shared__ uint64_t sh_scan[THREADS];
    __shared__ int sh_slice;
    __shared__ uint64_t sh_before;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nslices = gridDim.x;

    // ---- accept tests: lane i < t of wave 0 tests draft i+1 (t <= 64) ----
    if (wave == 0) {
        bool reject = false;
        if (lane < t) {
            const int xi = min(max(x[lane], 0), V - 1);      // ids are validated on the host; never read out of bounds
            const Philox4 rnd = philox4x32_10((uint32_t)lane, call, level, 0u, k0, k1);
            const float u = (float)(rnd.w[0] >> 8) * 5.9604644775390625e-8f;          // 2^-24 grid in [0,1)
            const float px = p[(size_t)lane * V + xi], qx = q[(size_t)lane * V + xi];
            reject = coin >= 0.f ? !(u < coin) : !(__fmul_rn(u, qx) < px);
        }
        const unsigned long long mask = __ballot(reject);
        if (lane == 0) sh_n = mask ? (int)__ffsll((long long)mask) - 1 : t;
    }
    __syncthreads();
    const int n = sh_n;
    const float* prow = p + (size_t)n * V;
    const float* qrow = n < t ? q + (size_t)n * V : nullptr;

    // ---- slice totals of the residual weights and of the plain weights ----
    uint64_t a = 0, b = 0;
    const int base = blockIdx.x * SLICE + tid * PER_THREAD;
#pragma unroll
    for (int e = 0; e < PER_THREAD; ++e) {
        const int i = base + e;
        if (i < V) {
            const float pv = prow[i];
            b += fixed_weight(pv);
            if (qrow) a += fixed_weight(fmaxf(0.f, __fsub_rn(pv, qrow[i])));
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        a += __shfl_xor(a, o, 64);
        b += __shfl_xor(b, o, 64);
    }
    if (lane == 0) { sh_a[wave] = a; sh_b[wave] = b; }
    __syncthreads();
    if (tid == 0) {
        uint64_t ta = 0, tb = 0;
        for (int w = 0; w < THREADS / 64; ++w) { ta += sh_a[w]; tb += sh_b[w]; }
        totals[blockIdx.x] = ta;
        totals[nslices + blockIdx.x] = tb;
        __threadfence();                                   // publish the totals before taking a ticket
        const uint32_t done = atomicAdd(ticket, 1u);
        sh_last = done == (uint32_t)nslices - 1;
    }
    __syncthreads();
    if (!sh_last) return;
    __threadfence();                                       // see the other workgroups' totals

    // ---- last workgroup: total, threshold, slice search ----
    volatile const uint64_t* vt = totals;
    uint64_t sa = 0, sb = 0;
    for (int s = tid; s < nslices; s += THREADS) { sa += vt[s]; sb += vt[nslices + s]; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        sa += __shfl_xor(sa, o, 64);
        sb += __shfl_xor(sb, o, 64);
    }
    if (lane == 0) { sh_a[wave] = sa; sh_b[wave] = sb; }
    __syncthreads();
    sa = sb = 0;
    for (int w = 0; w < THREADS / 64; ++w) { sa += sh_a[w]; sb += sh_b[w]; }
    const bool use_resid = qrow != nullptr && sa != 0;     // residual identically zero: fall back to p
    const uint64_t S = use_resid ? sa : sb;
    const int off = use_resid ? 0 : nslices;
    const Philox4 rnd = philox4x32_10((uint32_t)t, call, level, 0u, k0, k1);
    const uint64_t thr = __umul64hi(S, (uint64_t)rnd.w[1] << 32);          // floor(S * U / 2^32) < S
    if (tid == 0) {
        uint64_t before = 0;
        int s = 0;
        for (; s < nslices - 1; ++s) {
            const uint64_t v = vt[off + s];
            if (before + v > thr) break;
            before += v;
        }
        sh_slice = s;
        sh_before = before;
    }
    __syncthreads();
    const int slice = sh_slice;
    const uint64_t before = sh_before;

    // ---- scan inside the slice: smallest index whose inclusive prefix exceeds thr ----
    uint64_t wv[PER_THREAD];
    uint64_t mine = 0;
    const int sbase = slice * SLICE + tid * PER_THREAD;
#pragma unroll
    for (int e = 0; e < PER_THREAD; ++e) {
        const int i = sbase + e;
        uint64_t w = 0;
        if (i < V) {
            const float pv = prow[i];
            w = use_resid ? fixed_weight(fmaxf(0.f, __fsub_rn(pv, qrow[i]))) : fixed_weight(pv);
        }
        wv[e] = w;
        mine += w;
    }
    sh_scan[tid] = mine;
    __syncthreads();
    if (tid == 0) {
        uint64_t run = before;
        for (int i = 0; i < THREADS; ++i) { const uint64_t v = sh_scan[i]; sh_scan[i] = run; run += v; }   // exclusive
    }
    __syncthreads();
    uint64_t run = sh_scan[tid];
    int found = 0x7fffffff;
#pragma unroll
    for (int e = 0; e < PER_THREAD; ++e) {
        run += wv[e];
        if (found == 0x7fffffff && run > thr) found = sbase + e;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) found = min(found, __shfl_xor(found, o, 64));
    __shared__ int sh_found[THREADS / 64];
    if (lane == 0) sh_found[wave] = found;
    __syncthreads();
    if (tid == 0) {
        int m = sh_found[0];
        for (int w = 1; w < THREADS / 64; ++w) m = min(m, sh_found[w]);
        if (m >= V) m = V - 1;                                  // unreachable for a non-zero row
        result[0] = n;
        result[1] = m;
        x[n] = m;
        *ticket = 0;                                            // leave the scratch ready for the next launch
    }
}

// ---- one-workgroup search -------------------------------------------------------------------------
// Rows of up to 32768 tokens are held by one workgroup of 1024 threads in 8 chunks of 4096 tokens; in chunk k
// thread i owns tokens 4096 k + 4 i .. + 3 (a wave reads 1 KiB contiguous).  Token order is therefore
// (chunk, wave, lane, element).
constexpr int SMALL_THREADS = SOFTMAX_THREADS, SMALL_CHUNKS = 8, SMALL_MAX_V = SMALL_THREADS * 4 * SMALL_CHUNKS;
constexpr int SMALL_WAVES = SMALL_THREADS / 64;

struct SearchShared {
    uint64_t tot[SMALL_CHUNKS * SMALL_WAVES];     // [chunk][wave] sums, i.e. in token order
    int token;
};

// Sums of 8 values over the 64 lanes with 10 exchanges instead of 48: each step halves the values a lane
// carries.  Afterwards every lane holds the wave's sum of value number lane >> 3.
__device__ __forceinline__ uint64_t wave_sum8(const uint64_t (&v)[8], int lane) {
    uint64_t a[4], b[2];
    const bool h5 = lane & 32, h4 = lane & 16, h3 = lane & 8;
#pragma unroll
    for (int j = 0; j < 4; ++j) a[j] = (h5 ? v[j + 4] : v[j]) + __shfl_xor(h5 ? v[j] : v[j + 4], 32, 64);
#pragma unroll
    for (int j = 0; j < 2; ++j) b[j] = (h4 ? a[j + 2] : a[j]) + __shfl_xor(h4 ? a[j] : a[j + 2], 16, 64);
    uint64_t c = (h3 ? b[1] : b[0]) + __shfl_xor(h3 ? b[0] : b[1], 8, 64);
    c += __shfl_xor(c, 4, 64);
    c += __shfl_xor(c, 2, 64);
    c += __shfl_xor(c, 1, 64);
    return c;
}

__device__ __forceinline__ uint64_t wave_inclusive_scan(uint64_t v, int lane) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint64_t up = __shfl_up(v, o, 64);
        if (lane >= o) v += up;
    }
    return v;
}

// Inverse-CDF draw over the integer weights of this thread's tokens, which weights4(k, w) yields for chunk k
// (recomputed where needed rather than kept: 32 64-bit weights would not fit the register budget): with S their total over the
// workgroup and thr = floor(S * U32 / 2^32), the smallest token whose inclusive prefix exceeds thr goes to
// sh.token (one thread writes it; the caller puts a barrier before reading).  Returns S to every thread; for
// S == 0 nothing is written.  One barrier inside; sh.tot must not be in use by slower waves on entry.
template <typename F>
__device__ __forceinline__ uint64_t search_token(F&& weights4, uint32_t U32, SearchShared& sh) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint64_t cs[SMALL_CHUNKS];
#pragma unroll
    for (int k = 0; k < SMALL_CHUNKS; ++k) {
        uint64_t w4[4];
        weights4(k, w4);
        cs[k] = (w4[0] + w4[1]) + (w4[2] + w4[3]);
    }
    const uint64_t wsum = wave_sum8(cs, lane);
    if ((lane & 7) == 0) sh.tot[(lane >> 3) * SMALL_WAVES + wave] = wsum;
    __syncthreads();
    // every wave scans the 128 (chunk, wave) totals, two per lane
    const uint64_t e0 = sh.tot[2 * lane], e1 = sh.tot[2 * lane + 1];
    const uint64_t inc = wave_inclusive_scan(e0 + e1, lane);
    const uint64_t S = __shfl(inc, 63, 64);
    if (S == 0) return 0;
    const uint64_t thr = __umul64hi(S, (uint64_t)U32 << 32);                  // floor(S * U / 2^32) < S
    const uint64_t exc = inc - (e0 + e1);
    const bool here = exc <= thr && thr < inc;                               // exactly one lane
    const bool second = thr >= exc + e0;
    const unsigned long long mask = __ballot(here);
    const int src = (int)__ffsll((long long)mask) - 1;
    const int entry = __shfl(2 * lane + (second ? 1 : 0), src, 64);
    const uint64_t before = __shfl(second ? exc + e0 : exc, src, 64);
    if (wave != (entry & (SMALL_WAVES - 1))) return S;
    const int kk = entry / SMALL_WAVES;
    uint64_t mine = 0;
#pragma unroll
    for (int k = 0; k < SMALL_CHUNKS; ++k)
        if (k == kk) mine = cs[k];
    const uint64_t linc = wave_inclusive_scan(mine, lane);
    const uint64_t lexc = before + linc - mine;
    if (mine != 0 && lexc <= thr && thr < lexc + mine) {                     // exactly one lane
        uint64_t w4[4] = {0, 0, 0, 0};
#pragma unroll
        for (int k = 0; k < SMALL_CHUNKS; ++k)
            if (k == kk) weights4(k, w4);
        const uint64_t r0 = lexc + w4[0], r1 = r0 + w4[1], r2 = r1 + w4[2];
        const int e = r0 > thr ? 0 : r1 > thr ? 1 : r2 > thr ? 2 : 3;
        sh.token = (kk * SMALL_THREADS + tid) * 4 + e;
    }
    return S;
}

// Loads this thread's 32 values of a row (0 beyond V).
__device__ __forceinline__ void load_row_chunks(const float* __restrict__ row, int V, bool vec, float4 (&c)[SMALL_CHUNKS]) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int k = 0; k < SMALL_CHUNKS; ++k) {
        const int i = (k * SMALL_THREADS + tid) * 4;
        float4 v = {0.f, 0.f, 0.f, 0.f};
        if (vec) {
            if (i < V) v = *reinterpret_cast<const float4*>(row + i);
        } else {
            if (i < V) v.x = row[i];
            if (i + 1 < V) v.y = row[i + 1];
            if (i + 2 < V) v.z = row[i + 2];
            if (i + 3 < V) v.w = row[i + 3];
        }
        c[k] = v;
    }
}

// Token drawn from the normalised max(0, p - q) (q != null and the residual not identically zero) or from p,
// per Alg. 2; p and q are this thread's chunks.  The token lands in sh.token (barrier included).
__device__ __forceinline__ void draw_corrected(const float4 (&pc)[SMALL_CHUNKS], const float4 (&qc)[SMALL_CHUNKS], bool have_q,
                                               uint32_t U32, int V, SearchShared& sh) {
    uint64_t S = 0;
    if (have_q) {
        S = search_token([&](int k, uint64_t (&w)[4]) {
            w[0] = fixed_weight(fmaxf(0.f, __fsub_rn(pc[k].x, qc[k].x)));
            w[1] = fixed_weight(fmaxf(0.f, __fsub_rn(pc[k].y, qc[k].y)));
            w[2] = fixed_weight(fmaxf(0.f, __fsub_rn(pc[k].z, qc[k].z)));
            w[3] = fixed_weight(fmaxf(0.f, __fsub_rn(pc[k].w, qc[k].w)));
        }, U32, sh);
        if (S == 0) __syncthreads();                       // all waves are past the totals before they are rewritten
    }
    if (S == 0) {                                          // bonus row, or residual identically zero: draw from p
        S = search_token([&](int k, uint64_t (&w)[4]) {
            w[0] = fixed_weight(pc[k].x);
            w[1] = fixed_weight(pc[k].y);
            w[2] = fixed_weight(pc[k].z);
            w[3] = fixed_weight(pc[k].w);
        }, U32, sh);
    }
    if (S == 0 && threadIdx.x == 0) sh.token = V - 1;      // unreachable for a distribution row
    __syncthreads();
}

// Alg. 2 in ONE workgroup for vocabularies up to 32768: no exchange between workgroups, no fences.
__global__ __launch_bounds__(SMALL_THREADS) void accept_resample_small_kernel(const float* __restrict__ p, const float* __restrict__ q,
                                                                              int32_t* __restrict__ x, int t, int V, uint32_t k0,
                                                                              uint32_t k1, uint32_t level, uint32_t call,
                                                                              int32_t* __restrict__ result, float coin) {
    __shared__ int sh_n;
    __shared__ SearchShared sh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (wave == 0) {
        bool reject = false;
        if (lane < t) {
            const int xi = min(max(x[lane], 0), V - 1);
            const Philox4 rnd = philox4x32_10((uint32_t)lane, call, level, 0u, k0, k1);
            const float u = (float)(rnd.w[0] >> 8) * 5.9604644775390625e-8f;
            const float px = p[(size_t)lane * V + xi], qx = q[(size_t)lane * V + xi];
            reject = coin >= 0.f ? !(u < coin) : !(__fmul_rn(u, qx) < px);
        }
        const unsigned long long mask = __ballot(reject);
        if (lane == 0) sh_n = mask ? (int)__ffsll((long long)mask) - 1 : t;
    }
    __syncthreads();
    const int n = sh_n;
    const float* prow = p + (size_t)n * V;
    const float* qrow = n < t ? q + (size_t)n * V : nullptr;
    const bool vec = (V & 3) == 0 && ((uintptr_t)prow & 15) == 0 && (!qrow || ((uintptr_t)qrow & 15) == 0);
    float4 pc[SMALL_CHUNKS], qc[SMALL_CHUNKS];
    load_row_chunks(prow, V, vec, pc);
    if (qrow) load_row_chunks(qrow, V, vec, qc);
    const Philox4 rnd = philox4x32_10((uint32_t)t, call, level, 0u, k0, k1);
    draw_corrected(pc, qc, qrow != nullptr, rnd.w[1], V, sh);
    if (tid == 0) {
        const int m = sh.token;
        result[0] = n;
        result[1] = m;
        x[n] = m;
    }
}

// Softmax of the verifier's t+1 logit rows, the t accept tests and the corrected / bonus token in ONE launch:
// workgroup i turns logit row i into p_i in registers (same bits as the softmax kernel), stores it, tests
// draft i (i < t) and draws the token Alg. 2 would emit IF the first rejection were at i (i = t: the bonus
// token), all with the call's one sampling draw, as only one row's token is used.  Rejecting rows and row t
// then race an atomic max of ~(i << 32 | token): the largest is the smallest i, i.e. n and its token.  The
// last workgroup to take a ticket publishes them (result, x[n], and a pinned host mailbox if given) and
// resets key and ticket.  The ticket increment depends on the returned value of the max, so the max is
// performed before the ticket is taken.
__device__ __forceinline__ void softmax_verify_row(const int row, const float* __restrict__ z, const float* __restrict__ q,
                                                   int32_t* __restrict__ x, int t, int V, float temperature, uint32_t k0, uint32_t k1,
                                                   uint32_t level, uint32_t call, float* __restrict__ p_out, int32_t* __restrict__ result,
                                                   uint32_t* ticket, unsigned long long* key, int32_t* __restrict__ mailbox,
                                                   const EmbedNext& next, float coin, int mailbox_seq) {
    __shared__ float shv[16];
    __shared__ int shi[16];
    __shared__ SearchShared sh;
    __shared__ int sh_reject;
    __shared__ int sh_last, sh_emit;
    const int tid = threadIdx.x;
    const float* zr = z + (size_t)row * V;
    const float* qr = row < t ? q + (size_t)row * V : nullptr;
    float* pr = p_out ? p_out + (size_t)row * V : nullptr;
    const bool vec = (V & 3) == 0 && ((uintptr_t)zr & 15) == 0 && (!qr || ((uintptr_t)qr & 15) == 0) && (!pr || ((uintptr_t)pr & 15) == 0);
    const int xi = row < t ? min(max(x[row], 0), V - 1) : -1;
    float4 pc[SMALL_CHUNKS], qc[SMALL_CHUNKS];
    if (qr) load_row_chunks(qr, V, vec, qc);
    softmax_row_cached<SMALL_CHUNKS>(zr, V, temperature, vec, pc, shv, shi);
    if (pr) store_row_cached<SMALL_CHUNKS>(pr, V, vec, pc);
    if (row < t) {
        // the thread that owns the drafted token tests it: accept iff fl32(u * q(x)) < p(x)
        if (((xi >> 2) & (SMALL_THREADS - 1)) == tid) {
            const int kk = xi >> 12, e = xi & 3;
            float px = 0.f, qx = 0.f;
#pragma unroll
            for (int k = 0; k < SMALL_CHUNKS; ++k)
                if (k == kk) {
                    px = e == 0 ? pc[k].x : e == 1 ? pc[k].y : e == 2 ? pc[k].z : pc[k].w;
                    qx = e == 0 ? qc[k].x : e == 1 ? qc[k].y : e == 2 ? qc[k].z : qc[k].w;
                }
            const Philox4 rnd = philox4x32_10((uint32_t)row, call, level, 0u, k0, k1);
            const float u = (float)(rnd.w[0] >> 8) * 5.9604644775390625e-8f;
            sh_reject = coin >= 0.f ? !(u < coin) : !(__fmul_rn(u, qx) < px);
        }
    } else if (tid == 0) {
        sh_reject = 1;                                     // the bonus row always takes part
    }
    const Philox4 rnd = philox4x32_10((uint32_t)t, call, level, 0u, k0, k1);
    draw_corrected(pc, qc, qr != nullptr, rnd.w[1], V, sh);           // ends with a barrier: sh_reject and sh.token are visible
    if (tid < 64) {
        int last = 0;
        unsigned long long best = 0;
        if (t == 0) {                                          // one row (a draft step): nothing to agree on
            last = 1;
            best = (unsigned long long)(uint32_t)sh.token;
        } else if (tid == 0) {
            unsigned long long old = 0;
            if (sh_reject) {
                const unsigned long long mine = ~(((unsigned long long)row << 32) | (unsigned long long)(uint32_t)sh.token);
                old = __hip_atomic_fetch_max(key, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            const uint32_t step = 1u + (uint32_t)(old == 1ull);           // old is 0 or has bit 63 set: always 1, but data-dependent
            const uint32_t done = __hip_atomic_fetch_add(ticket, step, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (done == (uint32_t)t) {
                last = 1;
                best = ~__hip_atomic_exchange(key, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        if (t != 0) {
            last = __shfl(last, 0, 64);
            best = __shfl(best, 0, 64);
        }
        if (last) {
            const int n = (int)(best >> 32), m = (int)(uint32_t)best;
            if (tid == 0) {
                result[0] = n;
                result[1] = m;
                x[n] = m;
                if (mailbox) { mailbox[0] = n; mailbox[1] = m; }
                sh_emit = m;
            }
            if (mailbox) {                                     // the accepted drafts and the new token, for the host
                if (tid < n) mailbox[2 + tid] = x[tid];
                if (tid == 0) mailbox[2 + n] = m;
                if (mailbox_seq) {
                    // a host that polls instead of waiting for the stream: the payload above is made visible system-wide
                    // by every lane that wrote it, then the sequence number follows
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "");
                    if (tid == 0)
                        __hip_atomic_store(mailbox + MAILBOX_SEQ_SLOT, mailbox_seq, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                }
            }
        }
        if (tid == 0) sh_last = last;
    }
    if (!next.E) return;
    __syncthreads();
    if (!sh_last) return;
    // The emitted token, embedded for a one-token pass that may follow: the arithmetic (256 strided partial sums, four
    // wave sums, their sum in wave order) is the embedding kernel's, so the pass sees the same bits either way.
    int tk = sh_emit;
    tk = tk < 0 ? 0 : (tk >= next.vocab ? next.vocab - 1 : tk);
    float acc = 0.f;
    if (tid < 256) {
        for (int i = tid; i < next.d; i += 256) {
            const float v = next.dtype == HSD_BF16 ? (float)((const bf16_t*)next.E)[(size_t)tk * next.d + i]
                                                   : ((const float*)next.E)[(size_t)tk * next.d + i];
            next.x[i] = v;
            if (next.xn) ((bf16_t*)next.xn)[i] = (bf16_t)(v * next.norm_w[i]);
            acc += v * v;
        }
        acc = wave_sum(acc);
        if ((tid & 63) == 0) shv[tid >> 6] = acc;
    }
    __syncthreads();
    if (next.ss && tid < SS_SLOTS) {
        float s4 = 0.f;
        for (int w = 0; w < 4; ++w) s4 += shv[w];
        next.ss[tid * HSD_MAX_PASS_ROWS] = tid == 0 ? (unsigned long long)((double)s4 * 16777216.0 + 0.5) : 0ull;
        next.ss_other[tid * HSD_MAX_PASS_ROWS] = 0ull;
    }
}

__global__ __launch_bounds__(SMALL_THREADS) void softmax_verify_kernel(const float* __restrict__ z, const float* __restrict__ q,
                                                                       int32_t* __restrict__ x, int t, int V, float temperature,
                                                                       uint32_t k0, uint32_t k1, uint32_t level, uint32_t call,
                                                                       float* __restrict__ p_out, int32_t* __restrict__ result,
                                                                       uint32_t* ticket, unsigned long long* key,
                                                                       int32_t* __restrict__ mailbox, const EmbedNext next, float coin,
                                                                       int mailbox_seq) {
    softmax_verify_row((int)blockIdx.x, z, q, x, t, V, temperature, k0, k1, level, call, p_out, result, ticket, key, mailbox, next, coin,
                       mailbox_seq);
}

// The same for several independent calls (the sequences of a batch) in one launch: grid (most rows of a call, calls);
// call c has its own rows, tokens, seed, call index, result, mailbox and its own ticket / key pair at scratch + 16 c.
__global__ __launch_bounds__(SMALL_THREADS) void softmax_verify_batch_kernel(const VerifyCalls calls, int V, float temperature,
                                                                             uint32_t level, char* scratch) {
    const VerifyCall& c = calls.c[blockIdx.y];
    if ((int)blockIdx.x > c.t) return;
    softmax_verify_row((int)blockIdx.x, c.z, c.q, c.x, c.t, V, temperature, (uint32_t)c.seed, (uint32_t)(c.seed >> 32), level, c.call,
                       c.p_out, c.result, (uint32_t*)(scratch + 16 * blockIdx.y), (unsigned long long*)(scratch + 16 * blockIdx.y + 8),
                       c.mailbox, EmbedNext{}, -1.f, 0);
}

// z[r, v] += std * n(level, pos0 + r, v): the synthetic closeness of a drafter to a deeper level (workload
// construction, not part of the method).  n = Box-Muller on the words of the Philox block with counter
// (v / 4, position, level | 2^31, 0x4E4F4953), two normals per word pair, evaluated in fp64.
__global__ __launch_bounds__(256) void add_noise_kernel(float* __restrict__ z, int V, uint32_t k0, uint32_t k1, uint32_t level,
                                                        int pos0, float std) {
    const int blk = blockIdx.x * blockDim.x + threadIdx.x, row = blockIdx.y;
    if (blk * 4 >= V) return;
    const Philox4 w = philox4x32_10((uint32_t)blk, (uint32_t)(pos0 + row), level | 0x80000000u, 0x4E4F4953u, k0, k1);
    float* zr = z + (size_t)row * V + (size_t)blk * 4;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const double u1 = ((double)w.w[2 * h] + 0.5) * 2.3283064365386963e-10;          // 2^-32
        const double u2 = ((double)w.w[2 * h + 1] + 0.5) * 2.3283064365386963e-10;
        const double r = sqrt(-2.0 * log(u1));
        double sn, cs;
        sincos(6.283185307179586 * u2, &sn, &cs);
        const int v = blk * 4 + 2 * h;
        if (v < V) zr[2 * h] = (float)((double)zr[2 * h] + (double)std * (r * cs));
        if (v + 1 < V) zr[2 * h + 1] = (float)((double)zr[2 * h + 1] + (double)std * (r * sn));
    }
}

}  // namespace

int launch_add_noise(float* z, int rows, int vocab, uint64_t seed, uint32_t level, int pos0, float std, hipStream_t s) {
    if (rows < 1) return HSD_OK;
    add_noise_kernel<<<dim3(ceil_div(ceil_div(vocab, 4), 256), rows), 256, 0, s>>>(z, vocab, (uint32_t)seed, (uint32_t)(seed >> 32), level,
                                                                                  pos0, std);
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

extern "C" size_t hsd_sampler_scratch_bytes(int vocab) {
    const int nslices = ceil_div(vocab < 1 ? 1 : vocab, SLICE);
    return align_up(16 + (size_t)2 * nslices * sizeof(uint64_t), 256);
}

int launch_accept_resample(const float* p, const float* q, int32_t* x, int t, int vocab, uint64_t seed, uint32_t level,
                           uint32_t call, int32_t* result, void* scratch, float coin, hipStream_t s) {
    if (vocab <= SMALL_MAX_V) {
        accept_resample_small_kernel<<<1, SMALL_THREADS, 0, s>>>(p, q, x, t, vocab, (uint32_t)seed, (uint32_t)(seed >> 32), level,
                                                              call, result, coin);
        HSD_LAUNCH_CHECK();
        return HSD_OK;
    }
    const int nslices = ceil_div(vocab, SLICE);
    accept_resample_kernel<<<nslices, THREADS, 0, s>>>(p, q, x, t, vocab, (uint32_t)seed, (uint32_t)(seed >> 32), level, call,
                                                       result, (uint32_t*)scratch, (uint64_t*)((char*)scratch + 16), coin);
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

// Fused softmax + Alg. 2 (vocabularies up to 32768 only); scratch as for launch_accept_resample (ticket in word 0,
// the key in bytes 8..15, both zero between launches).
bool softmax_verify_supported(int vocab, int max_v) { return vocab <= SMALL_MAX_V && vocab <= max_v; }

int launch_softmax_verify(const float* z, const float* q, int32_t* x, int t, int vocab, float temperature, uint64_t seed,
                          uint32_t level, uint32_t call, float* p_out, int32_t* result, void* scratch, int32_t* mailbox,
                          const EmbedNext& next, float coin, int mailbox_seq, hipStream_t s) {
    if (!softmax_verify_supported(vocab)) HSD_FAIL(HSD_ECAPACITY, "fused softmax + verify: vocabulary %d above %d", vocab, SMALL_MAX_V);
    softmax_verify_kernel<<<t + 1, SMALL_THREADS, 0, s>>>(z, q, x, t, vocab, temperature, (uint32_t)seed, (uint32_t)(seed >> 32), level,
                                                          call, p_out, result, (uint32_t*)scratch,
                                                          (unsigned long long*)((char*)scratch + 8), mailbox, next, coin, mailbox_seq);
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

int launch_softmax_verify_batch(const VerifyCall* calls, int n_calls, int vocab, float temperature, uint32_t level, void* scratch,
                                hipStream_t s) {
    if (!softmax_verify_supported(vocab)) HSD_FAIL(HSD_ECAPACITY, "fused softmax + verify: vocabulary %d above %d", vocab, SMALL_MAX_V);
    for (int c0 = 0; c0 < n_calls; c0 += VERIFY_CALLS_MAX) {
        VerifyCalls group;
        const int n = std::min(VERIFY_CALLS_MAX, n_calls - c0);
        int rows = 1;
        for (int c = 0; c < n; ++c) {
            group.c[c] = calls[c0 + c];
            if (group.c[c].t < 0 || group.c[c].t > 64) HSD_FAIL(HSD_EINVAL, "fused softmax + verify: t=%d outside 0..64", group.c[c].t);
            rows = std::max(rows, group.c[c].t + 1);
        }
        softmax_verify_batch_kernel<<<dim3(rows, n), SMALL_THREADS, 0, s>>>(group, vocab, temperature, level, (char*)scratch + 16 * (size_t)c0);
        HSD_LAUNCH_CHECK();
    }
    return HSD_OK;
}

extern "C" int hsd_accept_resample(const float* p_dev, const float* q_dev, int32_t* x_dev, int t, int vocab, uint64_t seed,
                                   uint32_t level, uint32_t call, int32_t* result_dev, void* scratch_dev, void* stream) {
    if (!p_dev || !x_dev || !result_dev || !scratch_dev) HSD_FAIL(HSD_EINVAL, "hsd_accept_resample: null pointer");
    if (t < 0 || t > 64) HSD_FAIL(HSD_EINVAL, "hsd_accept_resample: t=%d outside 0..64", t);
    if (t > 0 && !q_dev) HSD_FAIL(HSD_EINVAL, "hsd_accept_resample: draft rows missing for t=%d", t);
    if (vocab < 1) HSD_FAIL(HSD_EINVAL, "hsd_accept_resample: vocab=%d", vocab);
    return launch_accept_resample(p_dev, q_dev, x_dev, t, vocab, seed, level, call, result_dev, scratch_dev, -1.f,
                                  (hipStream_t)stream);
}

extern "C" int hsd_softmax_verify(const float* logits_dev, const float* q_dev, int32_t* x_dev, int t, int vocab, float temperature,
                                  uint64_t seed, uint32_t level, uint32_t call, float* probs_dev, int32_t* result_dev,
                                  void* scratch_dev, int32_t* host_mailbox, void* stream) {
    if (!logits_dev || !x_dev || !result_dev || !scratch_dev) HSD_FAIL(HSD_EINVAL, "hsd_softmax_verify: null pointer");
    if (t < 0 || t > 64) HSD_FAIL(HSD_EINVAL, "hsd_softmax_verify: t=%d outside 0..64", t);
    if (t > 0 && !q_dev) HSD_FAIL(HSD_EINVAL, "hsd_softmax_verify: draft rows missing for t=%d", t);
    if (vocab < 1 || !(temperature >= 0.f)) HSD_FAIL(HSD_EINVAL, "hsd_softmax_verify: vocab=%d temperature=%g", vocab, temperature);
    return launch_softmax_verify(logits_dev, q_dev, x_dev, t, vocab, temperature, seed, level, call, probs_dev, result_dev,
                                 scratch_dev, host_mailbox, EmbedNext{}, -1.f, 0, (hipStream_t)stream);
}

// ------------------------------------------------------------------------------------------------
// hsd_accept_resample for callers that cannot allocate device memory: the ticket and the slice totals live in a
// file-scope device array instead of a caller's scratch buffer.
// ------------------------------------------------------------------------------------------------
constexpr int STATIC_MAX_V = HSD_STATIC_SAMPLER_MAX_VOCAB;
constexpr int STATIC_SCRATCH_BYTES = 16 + 2 * (STATIC_MAX_V / 2048) * (int)sizeof(uint64_t);   // ticket + two totals per 2048-token slice
// One copy per GPU the library runs on, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress: the kernels get the device address it resolves to, never the name.
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {

static_assert(STATIC_MAX_V % SLICE == 0 && SLICE == 2048, "the static sampler's vocabulary limit must be whole slices");
constexpr int STATIC_MAX_DEVICES = 64;
void* g_static_scratch[STATIC_MAX_DEVICES];       // device address of `scratch` on each GPU, null until resolved

// The first 16 bytes (ticket, padding) must read zero when accept_resample_kernel starts.  A kernel, not a memset:
// callers may be recording a graph.
__global__ void clear_ticket_kernel(uint32_t* words) {
    if (threadIdx.x < 4) words[threadIdx.x] = 0u;
}

int static_scratch_of_current_device(void** out) {
    int dev = -1;
    HSD_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= STATIC_MAX_DEVICES) HSD_FAIL(HSD_ECAPACITY, "hsd_accept_resample_static: device %d beyond the %d supported", dev, STATIC_MAX_DEVICES);
    void* ptr = __atomic_load_n(&g_static_scratch[dev], __ATOMIC_ACQUIRE);
    if (!ptr) {
        // resolved with this device current; two threads racing here get the same address
        HSD_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) HSD_FAIL(HSD_EHIP, "hsd_accept_resample_static: the scratch symbol resolved to null on device %d", dev);
        __atomic_store_n(&g_static_scratch[dev], ptr, __ATOMIC_RELEASE);
    }
    *out = ptr;
    return HSD_OK;
}

}  // namespace

extern "C" int hsd_accept_resample_static(const float* p_dev, const float* q_dev, int32_t* x_dev, int t, int vocab, uint64_t seed,
                                          uint32_t level, uint32_t call, int32_t* result_dev, void* stream) {
    if (!p_dev || !x_dev || !result_dev) HSD_FAIL(HSD_EINVAL, "hsd_accept_resample_static: null pointer");
    if (t < 0 || t > 64) HSD_FAIL(HSD_EINVAL, "hsd_accept_resample_static: t=%d outside 0..64", t);
    if (t > 0 && !q_dev) HSD_FAIL(HSD_EINVAL, "hsd_accept_resample_static: draft rows missing for t=%d", t);
    if (vocab < 1) HSD_FAIL(HSD_EINVAL, "hsd_accept_resample_static: vocab=%d", vocab);
    if (vocab > STATIC_MAX_V)
        HSD_FAIL(HSD_ECAPACITY, "hsd_accept_resample_static: vocabulary %d above the %d the built-in scratch holds (use hsd_accept_resample)",
                 vocab, STATIC_MAX_V);
    void* ptr = nullptr;
    if (int rc = static_scratch_of_current_device(&ptr)) return rc;
    hipStream_t s = (hipStream_t)stream;
    if (vocab > SMALL_MAX_V) {          // the one-workgroup kernel below that size exchanges nothing through memory
        clear_ticket_kernel<<<1, 64, 0, s>>>((uint32_t*)ptr);
        HSD_LAUNCH_CHECK();
    }
    return launch_accept_resample(p_dev, q_dev, x_dev, t, vocab, seed, level, call, result_dev, ptr, -1.f, s);
}
