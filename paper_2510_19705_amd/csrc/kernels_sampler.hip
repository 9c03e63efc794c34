// Fused rejection rule of Alg. 2 (App. B.1) / Sec. 2: accept tests for the t drafted tokens, then
// the corrected token from the normalised residual max(0, p - q) or the bonus token from p_{t+1},
// in ONE launch.  Every workgroup first evaluates the t accept tests (lane i tests draft i, the
// first rejection is found with a ballot), so all agree on n; each then sums the fixed-point weights
// of its slice of the chosen row (integer sums: any order gives the same bits); the last workgroup
// to finish (device-scope ticket) scans the slice totals, locates the slice that holds the
// threshold and scans inside it.  Random numbers are Philox4x32-10 blocks addressed by
// (seed; slot, call, level), so nothing depends on launch geometry.
#include "common.h"

namespace {

constexpr int SLICE = 2048;          // elements per workgroup
constexpr int THREADS = 256;
constexpr int PER_THREAD = SLICE / THREADS;

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
                                                                  uint64_t* totals) {
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
            reject = !(__fmul_rn(u, qx) < px);
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

// Same rule in ONE workgroup for vocabularies up to 32768: no exchange between workgroups, no fences.
// The row is cut in 8 chunks of 4096 tokens; in chunk k thread i owns tokens 4096 k + 4 i .. + 3 (so a
// wave reads 1 KiB contiguous).  Per chunk an exclusive scan of the threads' integer sums, chunk totals
// chained in order: together the prefix sums in token order, which locate the one (chunk, thread) whose
// four tokens hold the threshold.
constexpr int SMALL_THREADS = 1024, SMALL_CHUNKS = 8, SMALL_MAX_V = SMALL_THREADS * 4 * SMALL_CHUNKS;

__global__ __launch_bounds__(SMALL_THREADS) void accept_resample_small_kernel(const float* __restrict__ p, const float* __restrict__ q,
                                                                              int32_t* __restrict__ x, int t, int V, uint32_t k0,
                                                                              uint32_t k1, uint32_t level, uint32_t call,
                                                                              int32_t* __restrict__ result) {
    constexpr int NWAVE = SMALL_THREADS / 64;
    __shared__ int sh_n;
    __shared__ uint64_t sh_a[NWAVE], sh_b[NWAVE];
    __shared__ uint64_t sh_tot[NWAVE][SMALL_CHUNKS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (wave == 0) {
        bool reject = false;
        if (lane < t) {
            const int xi = min(max(x[lane], 0), V - 1);
            const Philox4 rnd = philox4x32_10((uint32_t)lane, call, level, 0u, k0, k1);
            const float u = (float)(rnd.w[0] >> 8) * 5.9604644775390625e-8f;
            const float px = p[(size_t)lane * V + xi], qx = q[(size_t)lane * V + xi];
            reject = !(__fmul_rn(u, qx) < px);
        }
        const unsigned long long mask = __ballot(reject);
        if (lane == 0) sh_n = mask ? (int)__ffsll((long long)mask) - 1 : t;
    }
    __syncthreads();
    const int n = sh_n;
    const float* prow = p + (size_t)n * V;
    const float* qrow = n < t ? q + (size_t)n * V : nullptr;
    const bool vec = (V & 3) == 0 && ((uintptr_t)prow & 15) == 0 && (!qrow || ((uintptr_t)qrow & 15) == 0);
    float pv[SMALL_CHUNKS][4], rv[SMALL_CHUNKS][4];
    uint64_t a = 0, b = 0;
#pragma unroll
    for (int k = 0; k < SMALL_CHUNKS; ++k) {
        const int i = (k * SMALL_THREADS + tid) * 4;
        float4 pp = {0.f, 0.f, 0.f, 0.f}, qq = {0.f, 0.f, 0.f, 0.f};
        if (vec) {
            if (i < V) {
                pp = *reinterpret_cast<const float4*>(prow + i);
                if (qrow) qq = *reinterpret_cast<const float4*>(qrow + i);
            }
        } else {
            if (i < V) { pp.x = prow[i]; if (qrow) qq.x = qrow[i]; }
            if (i + 1 < V) { pp.y = prow[i + 1]; if (qrow) qq.y = qrow[i + 1]; }
            if (i + 2 < V) { pp.z = prow[i + 2]; if (qrow) qq.z = qrow[i + 2]; }
            if (i + 3 < V) { pp.w = prow[i + 3]; if (qrow) qq.w = qrow[i + 3]; }
        }
        pv[k][0] = pp.x; pv[k][1] = pp.y; pv[k][2] = pp.z; pv[k][3] = pp.w;
        rv[k][0] = qrow ? fmaxf(0.f, __fsub_rn(pp.x, qq.x)) : 0.f;
        rv[k][1] = qrow ? fmaxf(0.f, __fsub_rn(pp.y, qq.y)) : 0.f;
        rv[k][2] = qrow ? fmaxf(0.f, __fsub_rn(pp.z, qq.z)) : 0.f;
        rv[k][3] = qrow ? fmaxf(0.f, __fsub_rn(pp.w, qq.w)) : 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            b += fixed_weight(pv[k][e]);
            a += fixed_weight(rv[k][e]);
        }
    }
    uint64_t ta = a, tb = b;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        ta += __shfl_xor(ta, o, 64);
        tb += __shfl_xor(tb, o, 64);
    }
    if (lane == 0) { sh_a[wave] = ta; sh_b[wave] = tb; }
    __syncthreads();
    ta = tb = 0;
    for (int w = 0; w < NWAVE; ++w) { ta += sh_a[w]; tb += sh_b[w]; }
    const bool use_resid = qrow != nullptr && ta != 0;     // residual identically zero: fall back to p
    const uint64_t S = use_resid ? ta : tb;
    const Philox4 rnd = philox4x32_10((uint32_t)t, call, level, 0u, k0, k1);
    const uint64_t thr = __umul64hi(S, (uint64_t)rnd.w[1] << 32);
    // per chunk: this thread's sum and its inclusive scan inside the wave
    uint64_t mine[SMALL_CHUNKS], inc[SMALL_CHUNKS];
#pragma unroll
    for (int k = 0; k < SMALL_CHUNKS; ++k) {
        uint64_t m4 = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) m4 += fixed_weight(use_resid ? rv[k][e] : pv[k][e]);
        mine[k] = m4;
        uint64_t v = m4;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint64_t up = __shfl_up(v, o, 64);
            if (lane >= o) v += up;
        }
        inc[k] = v;
        if (lane == 63) sh_tot[wave][k] = v;
    }
    __syncthreads();
    uint64_t chunk_base = 0;                               // tokens before chunk k
#pragma unroll
    for (int k = 0; k < SMALL_CHUNKS; ++k) {
        uint64_t before = chunk_base + inc[k] - mine[k];
        uint64_t chunk_total = 0;
        for (int w = 0; w < NWAVE; ++w) {
            const uint64_t v = sh_tot[w][k];
            if (w < wave) before += v;
            chunk_total += v;
        }
        if (mine[k] != 0 && before <= thr && thr < before + mine[k]) {      // exactly one (chunk, thread)
            uint64_t run = before;
            int m = (k * SMALL_THREADS + tid) * 4;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                run += fixed_weight(use_resid ? rv[k][e] : pv[k][e]);
                if (run > thr) { m += e; break; }
            }
            result[0] = n;
            result[1] = m;
            x[n] = m;
        }
        chunk_base += chunk_total;
    }
    if (S == 0 && tid == 0) {                              // unreachable for a distribution row
        result[0] = n;
        result[1] = V - 1;
        x[n] = V - 1;
    }
}

}  // namespace

extern "C" size_t hsd_sampler_scratch_bytes(int vocab) {
    const int nslices = ceil_div(vocab < 1 ? 1 : vocab, SLICE);
    return align_up(16 + (size_t)2 * nslices * sizeof(uint64_t), 256);
}

int launch_accept_resample(const float* p, const float* q, int32_t* x, int t, int vocab, uint64_t seed, uint32_t level,
                           uint32_t call, int32_t* result, void* scratch, hipStream_t s) {
    if (vocab <= SMALL_MAX_V) {
        accept_resample_small_kernel<<<1, SMALL_THREADS, 0, s>>>(p, q, x, t, vocab, (uint32_t)seed, (uint32_t)(seed >> 32), level,
                                                              call, result);
        HSD_LAUNCH_CHECK();
        return HSD_OK;
    }
    const int nslices = ceil_div(vocab, SLICE);
    accept_resample_kernel<<<nslices, THREADS, 0, s>>>(p, q, x, t, vocab, (uint32_t)seed, (uint32_t)(seed >> 32), level, call,
                                                       result, (uint32_t*)scratch, (uint64_t*)((char*)scratch + 16));
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

extern "C" int hsd_accept_resample(const float* p_dev, const float* q_dev, int32_t* x_dev, int t, int vocab, uint64_t seed,
                                   uint32_t level, uint32_t call, int32_t* result_dev, void* scratch_dev, void* stream) {
    if (!p_dev || !x_dev || !result_dev || !scratch_dev) HSD_FAIL(HSD_EINVAL, "hsd_accept_resample: null pointer");
    if (t < 0 || t > 64) HSD_FAIL(HSD_EINVAL, "hsd_accept_resample: t=%d outside 0..64", t);
    if (t > 0 && !q_dev) HSD_FAIL(HSD_EINVAL, "hsd_accept_resample: draft rows missing for t=%d", t);
    if (vocab < 1) HSD_FAIL(HSD_EINVAL, "hsd_accept_resample: vocab=%d", vocab);
    return launch_accept_resample(p_dev, q_dev, x_dev, t, vocab, seed, level, call, result_dev, scratch_dev,
                                  (hipStream_t)stream);
}
