// Element-wise and row-wise kernels of the decoder pass: embedding gather, residual-accumulate +
// RMSNorm, rotary embedding + KV append, vocabulary softmax.  None of them is bandwidth-relevant
// next to the weight and KV streams; they exist to keep every step of the pass on the device.
#include "common.h"
#include "softmax_row.h"

__device__ __forceinline__ float block_sum_256(float v, float* sh) {
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    float s = 0.f;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) s += sh[w];
    __syncthreads();
    return s;
}

// x[m, :] = E[tok[m], :] as fp32 (the residual stream is fp32 for both storage types).  With ss != null
// also what the first normalising GEMM of the pass reads: xn = bf16(x * norm_w), the row's sum of squares
// in fixed point (times 2^24), and the second accumulator cleared for the first producer of the pass.
template <typename T>
__global__ void embed_kernel(const int32_t* __restrict__ tok, const T* __restrict__ E, float* __restrict__ x, int d,
                             int vocab, unsigned long long* __restrict__ ss, unsigned long long* __restrict__ ss_other,
                             const float* __restrict__ norm_w, bf16_t* __restrict__ xn) {
    __shared__ float sh[16];
    int t = tok[blockIdx.x];
    t = t < 0 ? 0 : (t >= vocab ? vocab - 1 : t);          // ids are validated on the host; never read out of bounds
    const T* src = E + (size_t)t * d;
    float* dst = x + (size_t)blockIdx.x * d;
    float acc = 0.f;
    for (int i = threadIdx.x; i < d; i += blockDim.x) {
        const float v = to_f32(src[i]);
        dst[i] = v;
        if (xn) xn[(size_t)blockIdx.x * d + i] = (bf16_t)(v * norm_w[i]);
        acc += v * v;
    }
    if (ss) {
        acc = block_sum_256(acc, sh);
        if (threadIdx.x < SS_SLOTS) {      // the row's total in slot 0, every other slot of both accumulators cleared
            const int at = threadIdx.x * HSD_MAX_PASS_ROWS + blockIdx.x;
            ss[at] = threadIdx.x == 0 ? (unsigned long long)((double)acc * 16777216.0 + 0.5) : 0ull;
            ss_other[at] = 0ull;
        }
    }
}

// The pass resumes above an exit another pass has already reached (hidden-state reuse between exits of one
// network): x[m, :] = rows[m, :], the residual stream kept at that exit, and, with ss != null, what the next layer's
// normalising GEMM reads, exactly as the embedding kernel leaves it for the first layer.
__global__ void resume_rows_kernel(const float* __restrict__ rows, float* __restrict__ x, int d, unsigned long long* __restrict__ ss,
                                   unsigned long long* __restrict__ ss_other, const float* __restrict__ norm_w, bf16_t* __restrict__ xn) {
    __shared__ float sh[16];
    const float* src = rows + (size_t)blockIdx.x * d;
    float* dst = x + (size_t)blockIdx.x * d;
    float acc = 0.f;
    for (int i = threadIdx.x; i < d; i += blockDim.x) {
        const float v = src[i];
        dst[i] = v;
        if (xn) xn[(size_t)blockIdx.x * d + i] = (bf16_t)(v * norm_w[i]);
        acc += v * v;
    }
    if (ss) {
        acc = block_sum_256(acc, sh);
        if (threadIdx.x < SS_SLOTS) {
            const int at = threadIdx.x * HSD_MAX_PASS_ROWS + blockIdx.x;
            ss[at] = threadIdx.x == 0 ? (unsigned long long)((double)acc * 16777216.0 + 0.5) : 0ull;
            ss_other[at] = 0ull;
        }
    }
}

// Row r (grid.x) of x: x += sum_s part[s][r] (fixed order; part may be null), then
// xn[r] = x * w / sqrt(mean(x^2) + eps).  `part` rows and xn rows are indexed from 0, x rows from row0.
template <typename T>
__global__ void resid_rmsnorm_kernel(float* __restrict__ x, const float* __restrict__ part, int ksplit, int part_rows,
                                     int part_row0, const float* __restrict__ w, T* __restrict__ xn, int d, float eps,
                                     int row0) {
    __shared__ float sh[16];
    const int r = blockIdx.x;
    float* xr = x + (size_t)(row0 + r) * d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += blockDim.x) {
        float v = xr[i];
        if (part) {
            for (int s = 0; s < ksplit; ++s) v += part[((size_t)s * part_rows + part_row0 + r) * d + i];
            xr[i] = v;
        }
        ss += v * v;
    }
    ss = block_sum_256(ss, sh);
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
    T* o = xn + (size_t)r * d;
    for (int i = threadIdx.x; i < d; i += blockDim.x) o[i] = from_f32<T>(xr[i] * w[i] * inv);
}

// out[r, :] = bf16(x[r, :] * w): the rows an exit's head GEMM reads when the pass goes on to deeper layers (the
// producing GEMM has stored x * w of the NEXT layer's norm; the rows' sums of squares are the same for both).
__global__ void scale_rows_bf16_kernel(const float* __restrict__ x, const float* __restrict__ w, bf16_t* __restrict__ out, int d) {
    const float* xr = x + (size_t)blockIdx.x * d;
    bf16_t* o = out + (size_t)blockIdx.x * d;
    for (int i = threadIdx.x; i < d; i += blockDim.x) o[i] = (bf16_t)(xr[i] * w[i]);
}

// qkv = sum of the QKV GEMM partials [ksplit][m][(n_q + 2 n_kv) hd]; rotates q and k (pairs j, j+hd/2 by
// angle pos * base^(-2j/hd), computed in fp64), writes q [m][n_q][hd] and appends k, v at pos0 + m
// through the page table.  grid (m, n_q + 2 n_kv), 64 threads.
template <typename T>
__global__ void rope_kv_kernel(const float* __restrict__ part, int ksplit, int M, T* __restrict__ q, T* __restrict__ kv_layer,
                               const int32_t* __restrict__ pages, int pos0, int n_q, int n_kv, int hd, float rope_base,
                               const int32_t* __restrict__ pos0_arr, int m_seq, int max_pages) {
    const int m = blockIdx.x, head = blockIdx.y;
    const int width = (n_q + 2 * n_kv) * hd;
    const int half = hd >> 1;
    // a batch of sequences: row m is token m % m_seq of sequence m / m_seq, with that sequence's page table
    const int pos = pos0_arr ? pos0_arr[m / m_seq] + m % m_seq : pos0 + m;
    if (pos0_arr) pages += (size_t)(m / m_seq) * max_pages;
    const size_t stride = (size_t)M * width;
    const float* src = part + (size_t)m * width + (size_t)head * hd;
    const bool is_v = head >= n_q + n_kv;
    const bool is_q = head < n_q;
    const int kvh = is_q ? 0 : (is_v ? head - n_q - n_kv : head - n_q);
    const int page = pages[pos / HSD_KV_PAGE], inpage = pos % HSD_KV_PAGE;
    T* blk = kv_layer + (size_t)page * kv_page_elems(n_kv, hd) + (size_t)kvh * 2 * kv_block_elems(hd) +
             (is_v ? kv_block_elems(hd) : 0);
    for (int j = threadIdx.x; j < half; j += blockDim.x) {
        float a = 0.f, b = 0.f;
        for (int s = 0; s < ksplit; ++s) {
            a += src[s * stride + j];
            b += src[s * stride + j + half];
        }
        float ra = a, rb = b;
        if (!is_v) {
            double inv = exp2(-2.0 * (double)j / (double)hd * log2((double)rope_base));
            double sn, cs;
            sincos((double)pos * inv, &sn, &cs);
            ra = (float)((double)a * cs - (double)b * sn);
            rb = (float)((double)b * cs + (double)a * sn);
        }
        if (is_q) {
            T* dst = q + ((size_t)m * n_q + head) * hd;
            dst[j] = from_f32<T>(ra);
            dst[j + half] = from_f32<T>(rb);
        } else if constexpr (sizeof(T) == 4) {
            blk[(size_t)inpage * hd + j] = from_f32<T>(ra);
            blk[(size_t)inpage * hd + j + half] = from_f32<T>(rb);
        } else if (is_v) {
            blk[kv_v_index(inpage, j, hd)] = from_f32<T>(ra);
            blk[kv_v_index(inpage, j + half, hd)] = from_f32<T>(rb);
        } else {
            blk[kv_k_index(inpage, j, hd)] = from_f32<T>(ra);
            blk[kv_k_index(inpage, j + half, hd)] = from_f32<T>(rb);
        }
    }
}

// p = softmax(z / temperature) per row (grid.x rows, 1024 threads); temperature 0: one-hot at the
// lowest-index maximum.  The row fits the workgroup's registers (vocab <= 1024 * 4 * CH), so it is read once.
template <int CH>
__global__ __launch_bounds__(SOFTMAX_THREADS) void softmax_kernel(const float* __restrict__ z, float* __restrict__ p, int V,
                                                                  float temperature) {
    __shared__ float shv[16];
    __shared__ int shi[16];
    const float* zr = z + (size_t)blockIdx.x * V;
    float* pr = p + (size_t)blockIdx.x * V;
    const bool vec = (V & 3) == 0 && ((uintptr_t)zr & 15) == 0 && ((uintptr_t)pr & 15) == 0;
    float4 c[CH];
    softmax_row_cached<CH>(zr, V, temperature, vec, c, shv, shi);
    store_row_cached<CH>(pr, V, vec, c);
}

// Larger vocabularies: a row is cut in slices of SLICE_V tokens, one workgroup each (a single workgroup streams a
// row at one CU's ~40 GB/s, which for 128256 tokens costs tens of microseconds).  First launch: every slice's
// maximum (lowest index on ties) and sum of exp((z - slice max) / temperature); second launch: the row's maximum and
// the sum of the slice sums rescaled to it, in slice order, then p = exp((z - max) / temperature) / sum for the slice.
constexpr int SLICE_V = SOFTMAX_THREADS * 8;

__global__ __launch_bounds__(SOFTMAX_THREADS) void softmax_slice_stats_kernel(const float* __restrict__ z, int V, float temperature,
                                                                              float* __restrict__ stats, int nslices) {
    __shared__ float shv[16];
    __shared__ int shi[16];
    const int row = blockIdx.x, sl = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* zr = z + (size_t)row * V;
    const int lo = sl * SLICE_V, hi = min(V, lo + SLICE_V);
    float v[8];
    float mx = -INFINITY;
    int arg = 0x7fffffff;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int i = lo + k * SOFTMAX_THREADS + tid;
        v[k] = i < hi ? zr[i] : -INFINITY;
        if (v[k] > mx) { mx = v[k]; arg = i; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float om = __shfl_xor(mx, o, 64);
        const int oa = __shfl_xor(arg, o, 64);
        if (om > mx || (om == mx && oa < arg)) { mx = om; arg = oa; }
    }
    if (lane == 0) { shv[wave] = mx; shi[wave] = arg; }
    __syncthreads();
    mx = shv[0];
    arg = shi[0];
    for (int w = 1; w < 16; ++w)
        if (shv[w] > mx || (shv[w] == mx && shi[w] < arg)) { mx = shv[w]; arg = shi[w]; }
    __syncthreads();
    float sum = 0.f;
    if (temperature != 0.f) {
        const float it = 1.0f / temperature;
#pragma unroll
        for (int k = 0; k < 8; ++k) sum = __fadd_rn(sum, expf(__fmul_rn(__fsub_rn(v[k], mx), it)));     // exp(-inf) = 0 for the padding
        sum = wave_sum(sum);
        if (lane == 0) shv[wave] = sum;
        __syncthreads();
        sum = 0.f;
        for (int w = 0; w < 16; ++w) sum += shv[w];
    }
    if (tid == 0) {
        float* st = stats + ((size_t)row * nslices + sl) * 4;
        st[0] = mx;
        st[1] = sum;
        st[2] = __int_as_float(arg);
    }
}

__global__ __launch_bounds__(SOFTMAX_THREADS) void softmax_slice_write_kernel(const float* __restrict__ z, float* __restrict__ p, int V,
                                                                              float temperature, const float* __restrict__ stats,
                                                                              int nslices) {
    const int row = blockIdx.x, sl = blockIdx.y, tid = threadIdx.x;
    const float* st = stats + (size_t)row * nslices * 4;
    float mx = st[0];
    int arg = __float_as_int(st[2]);
    for (int s = 1; s < nslices; ++s) {                    // slices ascend in index, so ties keep the earlier one
        const float m = st[s * 4];
        if (m > mx) { mx = m; arg = __float_as_int(st[s * 4 + 2]); }
    }
    const float* zr = z + (size_t)row * V;
    float* pr = p + (size_t)row * V;
    const int lo = sl * SLICE_V, hi = min(V, lo + SLICE_V);
    if (temperature == 0.f) {
        for (int i = lo + tid; i < hi; i += SOFTMAX_THREADS) pr[i] = i == arg ? 1.f : 0.f;
        return;
    }
    const float it = 1.0f / temperature;
    float sum = 0.f;
    for (int s = 0; s < nslices; ++s) sum = __fadd_rn(sum, __fmul_rn(st[s * 4 + 1], expf(__fmul_rn(__fsub_rn(st[s * 4], mx), it))));
    const float inv = 1.0f / sum;
    for (int i = lo + tid; i < hi; i += SOFTMAX_THREADS) pr[i] = __fmul_rn(expf(__fmul_rn(__fsub_rn(zr[i], mx), it)), inv);
}

// ---- launchers --------------------------------------------------------------------------------
int launch_embed(const int32_t* tok, const void* E, float* x, int m, int d, int vocab, int dtype, unsigned long long* ss,
                 unsigned long long* ss_other, const float* norm_w, void* xn, hipStream_t s) {
    if (dtype == HSD_BF16)
        embed_kernel<bf16_t><<<m, 256, 0, s>>>(tok, (const bf16_t*)E, x, d, vocab, ss, ss_other, norm_w, (bf16_t*)xn);
    else
        embed_kernel<float><<<m, 256, 0, s>>>(tok, (const float*)E, x, d, vocab, nullptr, nullptr, nullptr, nullptr);
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

int launch_resume_rows(const float* rows, float* x, int m, int d, unsigned long long* ss, unsigned long long* ss_other,
                       const float* norm_w, void* xn, hipStream_t s) {
    resume_rows_kernel<<<m, 256, 0, s>>>(rows, x, d, ss, ss_other, norm_w, (bf16_t*)xn);
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

int launch_resid_rmsnorm(float* x, const float* part, int ksplit, int part_rows, int part_row0, const float* w, void* xn,
                         int rows, int row0, int d, float eps, int dtype, hipStream_t s) {
    if (dtype == HSD_BF16)
        resid_rmsnorm_kernel<bf16_t><<<rows, 256, 0, s>>>(x, part, ksplit, part_rows, part_row0, w, (bf16_t*)xn, d, eps, row0);
    else
        resid_rmsnorm_kernel<float><<<rows, 256, 0, s>>>(x, part, ksplit, part_rows, part_row0, w, (float*)xn, d, eps, row0);
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

int launch_scale_rows_bf16(const float* x, const float* w, void* out, int rows, int d, hipStream_t s) {
    scale_rows_bf16_kernel<<<rows, 256, 0, s>>>(x, w, (bf16_t*)out, d);
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

int launch_rope_kv(const float* part, int ksplit, int m, void* q, void* kv_layer, const int32_t* pages, int pos0, int n_q,
                   int n_kv, int hd, float rope_base, int dtype, hipStream_t s, const int32_t* pos0_arr, int m_seq, int max_pages) {
    dim3 grid(m, n_q + 2 * n_kv);
    if (dtype == HSD_BF16)
        rope_kv_kernel<bf16_t><<<grid, 64, 0, s>>>(part, ksplit, m, (bf16_t*)q, (bf16_t*)kv_layer, pages, pos0, n_q, n_kv, hd,
                                                   rope_base, pos0_arr, m_seq, max_pages);
    else
        rope_kv_kernel<float><<<grid, 64, 0, s>>>(part, ksplit, m, (float*)q, (float*)kv_layer, pages, pos0, n_q, n_kv, hd,
                                                  rope_base, pos0_arr, m_seq, max_pages);
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

// Bytes of device scratch launch_softmax needs beyond the rows (slice statistics of the large-vocabulary path).
size_t softmax_scratch_bytes(int rows, int vocab) {
    if (vocab <= SOFTMAX_THREADS * 4 * 8) return 0;
    return align_up((size_t)rows * ceil_div(vocab, SLICE_V) * 4 * sizeof(float), 256);
}

int launch_softmax(const float* z, float* p, int rows, int vocab, float temperature, float* scratch, hipStream_t s) {
    if (vocab <= SOFTMAX_THREADS * 4 * 2) {
        softmax_kernel<2><<<rows, SOFTMAX_THREADS, 0, s>>>(z, p, vocab, temperature);
    } else if (vocab <= SOFTMAX_THREADS * 4 * 8) {
        softmax_kernel<8><<<rows, SOFTMAX_THREADS, 0, s>>>(z, p, vocab, temperature);
    } else {
        if (!scratch) HSD_FAIL(HSD_EINVAL, "softmax: vocabulary %d needs the slice scratch", vocab);
        const int nslices = ceil_div(vocab, SLICE_V);
        softmax_slice_stats_kernel<<<dim3(rows, nslices), SOFTMAX_THREADS, 0, s>>>(z, vocab, temperature, scratch, nslices);
        HSD_LAUNCH_CHECK();
        softmax_slice_write_kernel<<<dim3(rows, nslices), SOFTMAX_THREADS, 0, s>>>(z, p, vocab, temperature, scratch, nslices);
    }
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

extern "C" size_t hsd_softmax_scratch_bytes(int rows, int vocab) {
    return rows < 1 || vocab < 1 ? 0 : softmax_scratch_bytes(rows, vocab);
}

extern "C" int hsd_softmax(const float* logits_dev, float* probs_dev, int rows, int vocab, float temperature, void* scratch_dev,
                           void* stream) {
    if (!logits_dev || !probs_dev || rows < 0 || vocab < 1 || !(temperature >= 0.f))
        HSD_FAIL(HSD_EINVAL, "hsd_softmax: bad arguments (rows=%d vocab=%d temperature=%g)", rows, vocab, temperature);
    if (rows == 0) return HSD_OK;
    if (softmax_scratch_bytes(rows, vocab) > 0 && (!scratch_dev || ((uintptr_t)scratch_dev & 15)))
        HSD_FAIL(HSD_EINVAL, "hsd_softmax: vocabulary %d needs 16-byte aligned scratch of hsd_softmax_scratch_bytes()", vocab);
    return launch_softmax(logits_dev, probs_dev, rows, vocab, temperature, (float*)scratch_dev, (hipStream_t)stream);
}
