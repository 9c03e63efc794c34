// One vocabulary row's softmax held in the registers of a 1024-thread workgroup, shared by the stand-alone
// softmax kernel and the fused softmax + Verify kernel so that both produce the same bits: thread tid owns
// elements (k * 1024 + tid) * 4 .. + 3 of chunk k, every product and difference is a single rounded fp32
// operation (no contraction across them), and sums are taken in one fixed order.
#pragma once
#include "common.h"

constexpr int SOFTMAX_THREADS = 1024;

// Loads the row (padding reads as -inf), leaves p = softmax(z / temperature) in c (padding 0) and returns the
// lowest index of the row maximum.  temperature 0: one-hot at that index.  Contains two workgroup barriers;
// shv/shi are 16-entry shared arrays the caller may reuse afterwards (after a barrier of its own).
template <int CH>
__device__ __forceinline__ int softmax_row_cached(const float* __restrict__ zr, int V, float temperature, bool vec,
                                                  float4 (&c)[CH], float* shv, int* shi) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int NW = SOFTMAX_THREADS / 64;
    float mx = -INFINITY;
    int arg = 0x7fffffff;
#pragma unroll
    for (int k = 0; k < CH; ++k) {
        const int i = (k * SOFTMAX_THREADS + tid) * 4;
        float4 v = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        if (vec) {
            if (i < V) v = *reinterpret_cast<const float4*>(zr + i);
        } else {
            if (i < V) v.x = zr[i];
            if (i + 1 < V) v.y = zr[i + 1];
            if (i + 2 < V) v.z = zr[i + 2];
            if (i + 3 < V) v.w = zr[i + 3];
        }
        c[k] = v;
        if (v.x > mx) { mx = v.x; arg = i; }
        if (v.y > mx) { mx = v.y; arg = i + 1; }
        if (v.z > mx) { mx = v.z; arg = i + 2; }
        if (v.w > mx) { mx = v.w; arg = i + 3; }
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
    for (int w = 1; w < NW; ++w)
        if (shv[w] > mx || (shv[w] == mx && shi[w] < arg)) { mx = shv[w]; arg = shi[w]; }
    __syncthreads();
    if (temperature == 0.f) {
#pragma unroll
        for (int k = 0; k < CH; ++k) {
            const int i = (k * SOFTMAX_THREADS + tid) * 4;
            c[k].x = i == arg ? 1.f : 0.f;
            c[k].y = i + 1 == arg ? 1.f : 0.f;
            c[k].z = i + 2 == arg ? 1.f : 0.f;
            c[k].w = i + 3 == arg ? 1.f : 0.f;
        }
        return arg;
    }
    const float it = 1.0f / temperature;
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < CH; ++k) {                       // exp(-inf) = 0 for the padding
        c[k].x = expf(__fmul_rn(__fsub_rn(c[k].x, mx), it));
        c[k].y = expf(__fmul_rn(__fsub_rn(c[k].y, mx), it));
        c[k].z = expf(__fmul_rn(__fsub_rn(c[k].z, mx), it));
        c[k].w = expf(__fmul_rn(__fsub_rn(c[k].w, mx), it));
        sum = __fadd_rn(sum, __fadd_rn(__fadd_rn(c[k].x, c[k].y), __fadd_rn(c[k].z, c[k].w)));
    }
    sum = wave_sum(sum);
    if (lane == 0) shv[wave] = sum;
    __syncthreads();
    sum = 0.f;
    for (int w = 0; w < NW; ++w) sum += shv[w];
    const float inv = 1.0f / sum;
#pragma unroll
    for (int k = 0; k < CH; ++k) {
        c[k].x = __fmul_rn(c[k].x, inv);
        c[k].y = __fmul_rn(c[k].y, inv);
        c[k].z = __fmul_rn(c[k].z, inv);
        c[k].w = __fmul_rn(c[k].w, inv);
    }
    return arg;
}

// Stores the chunks held in c to the row pr (vec: 16-byte stores allowed).
template <int CH>
__device__ __forceinline__ void store_row_cached(float* __restrict__ pr, int V, bool vec, const float4 (&c)[CH]) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int k = 0; k < CH; ++k) {
        const int i = (k * SOFTMAX_THREADS + tid) * 4;
        if (vec) {
            if (i < V) *reinterpret_cast<float4*>(pr + i) = c[k];
        } else {
            if (i < V) pr[i] = c[k].x;
            if (i + 1 < V) pr[i + 1] = c[k].y;
            if (i + 2 < V) pr[i + 2] = c[k].z;
            if (i + 3 < V) pr[i + 3] = c[k].w;
        }
    }
}
