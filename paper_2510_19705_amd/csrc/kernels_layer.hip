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
                               const int32_t* __restrict__ pages, int pos0, int n_q, int n_kv, int hd, float rope_base) {
    const int m = blockIdx.x, head = blockIdx.y;
    const int width = (n_q + 2 * n_kv) * hd;
    const int half = hd >> 1;
    const int pos = pos0 + m;
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
// lowest-index maximum.  CH > 0: the row fits the workgroup's registers (vocab <= 1024 * 4 * CH), so it is
// read once; CH == 0: it is re-read from L2 for the sum and the final pass.
template <int CH>
__global__ __launch_bounds__(SOFTMAX_THREADS) void softmax_kernel(const float* __restrict__ z, float* __restrict__ p, int V,
                                                                  float temperature) {
    __shared__ float shv[16];
    __shared__ int shi[16];
    const float* zr = z + (size_t)blockIdx.x * V;
    float* pr = p + (size_t)blockIdx.x * V;
    if constexpr (CH > 0) {
        const bool vec = (V & 3) == 0 && ((uintptr_t)zr & 15) == 0 && ((uintptr_t)pr & 15) == 0;
        float4 c[CH];
        softmax_row_cached<CH>(zr, V, temperature, vec, c, shv, shi);
        store_row_cached<CH>(pr, V, vec, c);
    } else {
        const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
        float mx = -INFINITY;
        int arg = 0x7fffffff;
        for (int i = tid; i < V; i += blockDim.x) {
            const float v = zr[i];
            if (v > mx) { mx = v; arg = i; }
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
        for (int w = 1; w < nw; ++w)
            if (shv[w] > mx || (shv[w] == mx && shi[w] < arg)) { mx = shv[w]; arg = shi[w]; }
        __syncthreads();
        if (temperature == 0.f) {
            for (int i = tid; i < V; i += blockDim.x) pr[i] = i == arg ? 1.f : 0.f;
            return;
        }
        const float it = 1.0f / temperature;
        float sum = 0.f;
        for (int i = tid; i < V; i += blockDim.x) sum += expf(__fmul_rn(__fsub_rn(zr[i], mx), it));
        sum = wave_sum(sum);
        if (lane == 0) shv[wave] = sum;
        __syncthreads();
        sum = 0.f;
        for (int w = 0; w < nw; ++w) sum += shv[w];
        const float inv = 1.0f / sum;
        for (int i = tid; i < V; i += blockDim.x) pr[i] = __fmul_rn(expf(__fmul_rn(__fsub_rn(zr[i], mx), it)), inv);
    }
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
                   int n_kv, int hd, float rope_base, int dtype, hipStream_t s) {
    dim3 grid(m, n_q + 2 * n_kv);
    if (dtype == HSD_BF16)
        rope_kv_kernel<bf16_t><<<grid, 64, 0, s>>>(part, ksplit, m, (bf16_t*)q, (bf16_t*)kv_layer, pages, pos0, n_q, n_kv, hd,
                                                   rope_base);
    else
        rope_kv_kernel<float><<<grid, 64, 0, s>>>(part, ksplit, m, (float*)q, (float*)kv_layer, pages, pos0, n_q, n_kv, hd,
                                                  rope_base);
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

int launch_softmax(const float* z, float* p, int rows, int vocab, float temperature, hipStream_t s) {
    if (vocab <= SOFTMAX_THREADS * 4 * 2)
        softmax_kernel<2><<<rows, SOFTMAX_THREADS, 0, s>>>(z, p, vocab, temperature);
    else if (vocab <= SOFTMAX_THREADS * 4 * 8)
        softmax_kernel<8><<<rows, SOFTMAX_THREADS, 0, s>>>(z, p, vocab, temperature);
    else
        softmax_kernel<0><<<rows, SOFTMAX_THREADS, 0, s>>>(z, p, vocab, temperature);
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

extern "C" int hsd_softmax(const float* logits_dev, float* probs_dev, int rows, int vocab, float temperature, void* stream) {
    if (!logits_dev || !probs_dev || rows < 0 || vocab < 1 || !(temperature >= 0.f))
        HSD_FAIL(HSD_EINVAL, "hsd_softmax: bad arguments (rows=%d vocab=%d temperature=%g)", rows, vocab, temperature);
    if (rows == 0) return HSD_OK;
    return launch_softmax(logits_dev, probs_dev, rows, vocab, temperature, (hipStream_t)stream);
}
