// k-query attention over the paged KV cache: each of the m new tokens of a verifier pass (Alg. 2:
// the verifier scores every prefix context + x_1..x_i in one pass) attends to all cached positions
// and, causally, to the new tokens before it.
//
// The KV stream is split along the sequence: every wave owns a run of 32-position steps of one KV
// head and produces an online-softmax partial (running max, running sum, unnormalised output) for
// all query rows of that head (m tokens x n_q/n_kv grouped heads); a merge kernel combines the
// partials.  bf16 path: S^T = K Q^T and O^T = V^T P^T on 16x16x32 MFMAs.  K and V are stored in the
// cache already in A-operand tile order (common.h), V with the position order that makes the
// accumulator layout of S^T directly usable as the B operand P^T, so probabilities never leave
// registers; row max / sum are reduced across the four 16-lane groups with wave shuffles.
// fp32 path (small correctness configuration): lanes = positions for the scores, lanes = head
// dims for the output, through LDS.
#include "common.h"

// ------------------------------------------------------------------------------------------------
// bf16 MFMA kernel.  grid (nsplit, n_kv, batch * qgroups), NW waves per workgroup.  The waves of a
// workgroup take the 32-position steps of the workgroup's range round-robin and combine their
// online-softmax states through LDS.  With nsplit == 1 the normalised output is written directly;
// otherwise one partial per workgroup goes to the merge kernel.
// ------------------------------------------------------------------------------------------------
// One step = SP blocks of 32 positions (SP = 2, a whole page, for hd 64; SP = 1 for hd 128, where the tiles of a
// page would not fit the registers twice).
template <int HD, int SP>
struct KvTiles {
    bf16x8 k[2 * SP][HD / 32];     // 16-position tiles x 32-dim chunks
    bf16x8 v[SP][HD / 16];         // 32-position blocks x 16-dim tiles
};

template <int HD, int SP>
__device__ __forceinline__ void load_kv(KvTiles<HD, SP>& t, const bf16_t* __restrict__ kv_layer, int page, int step, int n_kv,
                                        int g, int lane) {
    constexpr int KC = HD / 32, DT = HD / 16;
    const int p0 = step * 32 * SP;
    const int inpage = p0 % HSD_KV_PAGE;
    const size_t blk = kv_block_elems(HD);
    const bf16_t* kblk = kv_layer + ((size_t)page * n_kv + g) * 2 * blk;
    const bf16_t* vblk = kblk + blk;
#pragma unroll
    for (int h = 0; h < 2 * SP; ++h)
#pragma unroll
        for (int c = 0; c < KC; ++c)
            t.k[h][c] = *reinterpret_cast<const bf16x8*>(kblk + (size_t)(((inpage >> 4) + h) * KC + c) * 512 + lane * 8);
#pragma unroll
    for (int sb = 0; sb < SP; ++sb)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
            t.v[sb][dt] = *reinterpret_cast<const bf16x8*>(vblk + (size_t)(((inpage >> 5) + sb) * DT + dt) * 512 + lane * 8);
}

template <int HD, int QT>
__global__ __launch_bounds__(512) void attn_mfma_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ kv_layer,
                                                        const int32_t* __restrict__ pages, int max_pages,
                                                        const int32_t* __restrict__ pos0_arr, int pos0_all, int M, int n_q,
                                                        int n_kv, float scale_log2, int steps_per_split, int qgroups,
                                                        float* __restrict__ part_o, float* __restrict__ part_ml, int rpad,
                                                        bf16_t* __restrict__ att) {
    extern __shared__ float lds[];                 // [NW][QT*16][HD + 2]: o, then running max and sum
    constexpr int SP = HD == 64 ? 2 : 1;
    constexpr int KC = HD / 32;   // K chunks of 32 dims per 16-position tile
    constexpr int DT = HD / 16;   // 16-dim tiles of the output
    constexpr int RS = HD + 2;
    constexpr int NV = 8 * SP;    // scores per lane and query tile in one step
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, NW = blockDim.x >> 6;
    const int j = lane & 15, grp = lane >> 4;
    const int split = blockIdx.x, nsplit = gridDim.x, g = blockIdx.y;
    const int b = blockIdx.z / qgroups, qg = blockIdx.z % qgroups;
    const int group = n_q / n_kv;
    const int R = M * group;
    const int pos0 = pos0_arr ? pos0_arr[b] : pos0_all;
    const int S = pos0 + M;
    const int total_steps = (S + 32 * SP - 1) / (32 * SP);
    const int step0 = split * steps_per_split;
    const int step1 = min(total_steps, step0 + steps_per_split);

    // K/V of this wave's first two steps are requested before anything else.  The page-table entry a load needs
    // is fetched one round earlier (pg[i]: the page of the step buffer i loads next), so that no K/V request waits
    // behind a page lookup.
    const int32_t* ptab = pages + (size_t)b * max_pages;
    auto page_of = [&](int st) -> int { return st < step1 ? ptab[st * (32 * SP) / HSD_KV_PAGE] : 0; };
    KvTiles<HD, SP> buf[2];
    int pg[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) pg[i] = page_of(step0 + wave + i * NW);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int st = step0 + wave + i * NW;
        if (st < step1) load_kv<HD, SP>(buf[i], kv_layer, pg[i], st, n_kv, g, lane);
        pg[i] = page_of(st + 2 * NW);
    }

    bf16x8 qreg[QT][KC];
    int limit[QT];
    float m_run[QT], l_run[QT];    // l_run: this lane's share of the row sum (its own positions), reduced at the end
    f32x4 o[QT][DT];
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const int r = (qg * QT + qt) * 16 + j;
        const bool valid = r < R;
        const int i = valid ? r / group : 0, hq = valid ? r % group : 0;
        const bf16_t* qrow = q + (((size_t)b * M + i) * n_q + g * group + hq) * HD + grp * 8;
#pragma unroll
        for (int c = 0; c < KC; ++c) qreg[qt][c] = valid ? *reinterpret_cast<const bf16x8*>(qrow + c * 32) : zero;
        limit[qt] = valid ? pos0 + i + 1 : S;
        m_run[qt] = -INFINITY;
        l_run[qt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[qt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    for (int base = step0 + wave; base < step1; base += 2 * NW) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int step = base + i * NW;
            if (step < step1) {
                const KvTiles<HD, SP>& cur = buf[i];
                const int p0 = step * 32 * SP;
                // scores of all query tiles first, then their maxima, then the exponentials: independent chains
                // next to each other so that MFMA and cross-lane latencies overlap
                float v[QT][NV], mx[QT];
#pragma unroll
                for (int qt = 0; qt < QT; ++qt) {
                    mx[qt] = -INFINITY;
#pragma unroll
                    for (int h = 0; h < 2 * SP; ++h) {
                        f32x4 sc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int c = 0; c < KC; ++c) sc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur.k[h][c], qreg[qt][c], sc, 0, 0, 0);
                        // lane (j, grp): sc[r] is position p0 + 16 h + 4 grp + r of query row j
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int pa = p0 + 16 * h + 4 * grp + r;
                            const float val = pa < limit[qt] ? sc[r] * scale_log2 : -INFINITY;
                            v[qt][4 * h + r] = val;
                            mx[qt] = fmaxf(mx[qt], val);
                        }
                    }
                }
#pragma unroll
                for (int qt = 0; qt < QT; ++qt) mx[qt] = fmaxf(mx[qt], __shfl_xor(mx[qt], 16, 64));
#pragma unroll
                for (int qt = 0; qt < QT; ++qt) mx[qt] = fmaxf(mx[qt], __shfl_xor(mx[qt], 32, 64));
#pragma unroll
                for (int qt = 0; qt < QT; ++qt) {
                    const float m_new = fmaxf(m_run[qt], mx[qt]);
                    const float m_use = m_new == -INFINITY ? 0.f : m_new;      // row fully masked so far: all p = 0
                    const float alpha = exp2f(m_run[qt] - m_use);
                    m_run[qt] = m_new;
                    float sum = 0.f;
                    bf16x8 pb[SP];
#pragma unroll
                    for (int sb = 0; sb < SP; ++sb)
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            // B-operand element e of block sb: position 32 sb + 16 (e / 4) + 4 grp + e % 4
                            const float pe = exp2f(v[qt][8 * sb + e] - m_use);
                            sum += pe;
                            pb[sb][e] = (bf16_t)pe;
                        }
                    l_run[qt] = l_run[qt] * alpha + sum;
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) {
                        o[qt][dt] *= alpha;
#pragma unroll
                        for (int sb = 0; sb < SP; ++sb)
                            o[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur.v[sb][dt], pb[sb], o[qt][dt], 0, 0, 0);
                    }
                }
                const int nxt = step + 2 * NW;
                if (nxt < step1) {
                    load_kv<HD, SP>(buf[i], kv_layer, pg[i], nxt, n_kv, g, lane);
                    pg[i] = page_of(nxt + 2 * NW);
                }
            }
        }
    }
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {          // row sums: the four lane groups hold disjoint positions
        l_run[qt] += __shfl_xor(l_run[qt], 16, 64);
        l_run[qt] += __shfl_xor(l_run[qt], 32, 64);
    }

    // this wave's state to LDS: o^T accumulators hold d = 16 dt + 4 grp + r for query row j
    float* mine = lds + (size_t)wave * (QT * 16) * RS;
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        float* rowp = mine + (qt * 16 + j) * RS;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 4; ++r) rowp[dt * 16 + grp * 4 + r] = o[qt][dt][r];
        if (grp == 0) {
            rowp[HD] = m_run[qt];
            rowp[HD + 1] = l_run[qt];
        }
    }
    __syncthreads();
    const size_t pbase = (((size_t)b * n_kv + g) * nsplit + split) * rpad;
    for (int idx = tid; idx < QT * 16 * HD; idx += blockDim.x) {
        const int rl = idx / HD, d = idx % HD;
        const int r = qg * QT * 16 + rl;
        float m = -INFINITY;
        for (int w = 0; w < NW; ++w) m = fmaxf(m, lds[((size_t)w * QT * 16 + rl) * RS + HD]);
        float L = 0.f, acc = 0.f;
        if (m != -INFINITY) {
            for (int w = 0; w < NW; ++w) {
                const float* rowp = lds + ((size_t)w * QT * 16 + rl) * RS;
                const float wgt = exp2f(rowp[HD] - m);          // exp2(-inf) = 0 for idle waves
                L += wgt * rowp[HD + 1];
                acc += wgt * rowp[d];
            }
        }
        if (nsplit == 1) {
            if (r < R) {
                const int i = r / group, hq = r % group;
                att[(((size_t)b * M + i) * n_q + g * group + hq) * HD + d] = (bf16_t)(acc / L);
            }
        } else if (r < rpad) {
            part_o[(pbase + r) * HD + d] = acc;
            if (d == 0) {
                part_ml[(pbase + r) * 2] = m;
                part_ml[(pbase + r) * 2 + 1] = L;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// generic partial kernel (fp32 cache in natural layout; also reads the tiled bf16 layout).
// grid (nsplit, n_q, batch * M), 64 threads.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(64) void attn_simple_kernel(const T* __restrict__ q, const T* __restrict__ kv_layer,
                                                         const int32_t* __restrict__ pages, int max_pages,
                                                         const int32_t* __restrict__ pos0_arr, int pos0_all, int M, int n_q,
                                                         int n_kv, int hd, float scale_log2, int steps_per_split,
                                                         float* __restrict__ part_o, float* __restrict__ part_ml, int rpad) {
    __shared__ float qs[256];
    __shared__ float ps[64];
    const int lane = threadIdx.x;
    const int split = blockIdx.x, nsplit = gridDim.x, head = blockIdx.y;
    const int b = blockIdx.z / M, i = blockIdx.z % M;
    const int group = n_q / n_kv, g = head / group, hq = head % group;
    const int pos0 = pos0_arr ? pos0_arr[b] : pos0_all;
    const int limit = pos0 + i + 1;
    const int total_steps = (pos0 + M + 31) >> 5;
    const int step0 = split * steps_per_split;
    const int step1 = min(total_steps, step0 + steps_per_split);
    const T* qrow = q + (((size_t)b * M + i) * n_q + head) * hd;
    for (int d = lane; d < hd; d += 64) qs[d] = to_f32(qrow[d]);
    __syncthreads();
    const size_t blk = kv_block_elems(hd);
    float m_run = -INFINITY, l_run = 0.f;
    float o[4] = {0.f, 0.f, 0.f, 0.f};                 // dims lane, lane+64, ... (hd <= 256)
    for (int p0 = step0 << 5; p0 < min(step1 << 5, limit); p0 += 64) {
        // both 32-steps of a 64-chunk lie in one page only if aligned; handle per lane
        const int pos = p0 + lane;
        float s = -INFINITY;
        if (pos < limit && pos < (step1 << 5)) {
            const int page = pages[(size_t)b * max_pages + pos / HSD_KV_PAGE], ip = pos % HSD_KV_PAGE;
            const T* kblk = kv_layer + ((size_t)page * n_kv + g) * 2 * blk;
            float acc = 0.f;
            for (int d = 0; d < hd; ++d) {
                float kv = sizeof(T) == 4 ? to_f32(kblk[(size_t)ip * hd + d]) : to_f32(kblk[kv_k_index(ip, d, hd)]);
                acc += qs[d] * kv;
            }
            s = acc * scale_log2;
        }
        const float m_new = fmaxf(m_run, wave_max(s));
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = exp2f(m_run - m_use);
        const float p = exp2f(s - m_use);
        l_run = l_run * alpha + wave_sum(p);
        m_run = m_new;
        ps[lane] = p;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] *= alpha;
        const int cnt = min(64, min(step1 << 5, limit) - p0);
        for (int pp = 0; pp < cnt; ++pp) {
            const int ppos = p0 + pp;
            const int page = pages[(size_t)b * max_pages + ppos / HSD_KV_PAGE], ip = ppos % HSD_KV_PAGE;
            const T* vblk = kv_layer + ((size_t)page * n_kv + g) * 2 * blk + blk;
            const float w = ps[pp];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int d = lane + 64 * k;
                if (d < hd)
                    o[k] += w * (sizeof(T) == 4 ? to_f32(vblk[(size_t)ip * hd + d]) : to_f32(vblk[kv_v_index(ip, d, hd)]));
            }
        }
        __syncthreads();
    }
    const int r = i * group + hq;
    const size_t pbase = (((size_t)b * n_kv + g) * nsplit + split) * rpad + r;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int d = lane + 64 * k;
        if (d < hd) part_o[pbase * hd + d] = o[k];
    }
    if (lane == 0) {
        part_ml[pbase * 2] = m_run;
        part_ml[pbase * 2 + 1] = l_run;
    }
}

// ------------------------------------------------------------------------------------------------
// merge: one wave per (query row, KV head, batch).  grid (R, n_kv, batch), 64 threads.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(64) void attn_merge_kernel(const float* __restrict__ part_o, const float* __restrict__ part_ml,
                                                        int nsplit, int rpad, int M, int n_q, int n_kv, int hd,
                                                        T* __restrict__ att) {
    const int r = blockIdx.x, g = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
    const int group = n_q / n_kv, i = r / group, hq = r % group;
    const size_t base = ((size_t)b * n_kv + g) * nsplit;
    float m = -INFINITY;
    for (int s = 0; s < nsplit; ++s) m = fmaxf(m, part_ml[((base + s) * rpad + r) * 2]);
    float L = 0.f;
    float o[4] = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < nsplit; ++s) {
        const size_t pr = (base + s) * rpad + r;
        const float ms = part_ml[pr * 2];
        if (ms == -INFINITY) continue;
        const float w = exp2f(ms - m);
        L += w * part_ml[pr * 2 + 1];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int d = lane + 64 * k;
            if (d < hd) o[k] += w * part_o[pr * hd + d];
        }
    }
    T* dst = att + (((size_t)b * M + i) * n_q + g * group + hq) * hd;
    const float inv = 1.0f / L;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int d = lane + 64 * k;
        if (d < hd) dst[d] = from_f32<T>(o[k] * inv);
    }
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
struct AttnPlan {
    int nsplit, steps_per_split, rpad, qt, qgroups, nw;
};

// Up to this many query rows per KV head, one 16-row tile per workgroup (more workgroups, each re-reading the
// head's K/V from L2, instead of more tiles per workgroup): measured faster at every pass size up to 64 tokens and
// contexts up to 4096 (two tiles per workgroup double the registers and halve what is in flight).  Beyond it two
// tiles per workgroup; a tuning knob (hsd_tune key 101).
int g_attn_qt1_rows = 1 << 30;
int g_attn_steps_per_wave = 0;      // tuning override (hsd_tune key 102); 0: the default below

AttnPlan attn_plan(int batch, int m, int n_q, int n_kv, int hd, int max_len, bool mfma) {
    AttnPlan p;
    const int R = m * (n_q / n_kv);
    p.qt = R <= 16 || R <= g_attn_qt1_rows ? 1 : 2;
    p.qgroups = ceil_div(R, 16 * p.qt);
    p.rpad = p.qgroups * p.qt * 16;
    int total_steps = ceil_div(max_len, 32);
    if (mfma) {
        total_steps = ceil_div(max_len, hd == 64 ? 64 : 32);     // the MFMA kernel steps over a whole page for hd 64
        const int per_wave = p.qt * 16 * (hd + 2) * 4;               // LDS bytes of one wave's state
        p.nw = 65536 / per_wave;
        if (p.nw > 8) p.nw = 8;
        if (p.nw < 1) p.nw = 1;
        // one workgroup per (head, query group) while its waves get at most ~6 steps each; beyond that split the
        // sequence over workgroups and merge, but only up to about 160 workgroups in all: measured on sequences of
        // 4096 to 32768 positions, 100-250 fat workgroups stream K/V faster than a thousand thin ones (the partial
        // states and their merge cost more than the extra parallelism gives)
        const int spw = g_attn_steps_per_wave > 0 ? g_attn_steps_per_wave : (hd == 64 ? 3 : 6);
        int want = ceil_div(total_steps, p.nw * spw);
        const int heads = batch * n_kv * p.qgroups;
        const int cap = g_attn_steps_per_wave > 0 ? 64 : (160 / heads > 0 ? 160 / heads : 1);
        if (want > cap) want = cap;
        if (want > 64) want = 64;
        if (want < 1) want = 1;
        p.steps_per_split = ceil_div(total_steps, want);
        p.nsplit = ceil_div(total_steps, p.steps_per_split);
        return p;
    }
    p.nw = 1;
    int want = 2048 / (batch * n_kv * p.qgroups);
    if (want < 1) want = 1;
    if (want > 64) want = 64;
    int sps = ceil_div(total_steps, want);
    if (sps < 4) sps = 4;
    p.steps_per_split = sps;
    p.nsplit = ceil_div(total_steps, sps);
    return p;
}

size_t attn_workspace_bytes(int batch, int m, int n_q, int n_kv, int hd, int max_len) {
    // worst case over the lengths a plan may be made for: nsplit <= 64
    const int R = m * (n_q / n_kv);
    const int rpad = ceil_div(R, 16) * 16 + 48;
    return align_up((size_t)batch * n_kv * 64 * rpad * (hd + 2) * sizeof(float), 256);
}

int launch_attention(const void* q, const void* kv_layer, const int32_t* pages, int max_pages, const int32_t* pos0_dev,
                     int pos0_all, int batch, int m, int max_len, int n_q, int n_kv, int hd, int dtype, void* att, float* workspace,
                     int force_simple, hipStream_t s) {
    if (n_q % n_kv != 0) HSD_FAIL(HSD_EINVAL, "attention: n_q=%d not a multiple of n_kv=%d", n_q, n_kv);
    if (hd % 32 != 0 || hd > 256) HSD_FAIL(HSD_EINVAL, "attention: head dim %d must be a multiple of 32, at most 256", hd);
    const bool mfma = dtype == HSD_BF16 && !force_simple && (hd == 64 || hd == 128);
    AttnPlan p = attn_plan(batch, m, n_q, n_kv, hd, max_len, mfma);
    const int R = m * (n_q / n_kv);
    float* part_o = workspace;
    float* part_ml = workspace + (size_t)batch * n_kv * p.nsplit * p.rpad * hd;
    const float scale_log2 = 1.4426950408889634f / sqrtf((float)hd);
    if (mfma) {
        dim3 grid(p.nsplit, n_kv, batch * p.qgroups);
#define HSD_ATT(HD_, QT_)                                                                                              \
    if (hd == HD_ && p.qt == QT_)                                                                                      \
        attn_mfma_kernel<HD_, QT_><<<grid, p.nw * 64, (size_t)p.nw * QT_ * 16 * (HD_ + 2) * 4, s>>>(                    \
            (const bf16_t*)q, (const bf16_t*)kv_layer, pages, max_pages, pos0_dev, pos0_all, m, n_q, n_kv, scale_log2, \
            p.steps_per_split, p.qgroups, part_o, part_ml, p.rpad, (bf16_t*)att);
        HSD_ATT(64, 1) HSD_ATT(64, 2) HSD_ATT(128, 1) HSD_ATT(128, 2)
#undef HSD_ATT
    } else {
        dim3 grid(p.nsplit, n_q, batch * m);
        if (dtype == HSD_BF16)
            attn_simple_kernel<bf16_t><<<grid, 64, 0, s>>>((const bf16_t*)q, (const bf16_t*)kv_layer, pages, max_pages,
                                                           pos0_dev, pos0_all, m, n_q, n_kv, hd, scale_log2,
                                                           p.steps_per_split, part_o, part_ml, p.rpad);
        else
            attn_simple_kernel<float><<<grid, 64, 0, s>>>((const float*)q, (const float*)kv_layer, pages, max_pages,
                                                          pos0_dev, pos0_all, m, n_q, n_kv, hd, scale_log2,
                                                          p.steps_per_split, part_o, part_ml, p.rpad);
    }
    HSD_LAUNCH_CHECK();
    if (mfma && p.nsplit == 1) return HSD_OK;            // the kernel wrote the normalised output itself
    dim3 mg(R, n_kv, batch);
    if (dtype == HSD_BF16)
        attn_merge_kernel<bf16_t><<<mg, 64, 0, s>>>(part_o, part_ml, p.nsplit, p.rpad, m, n_q, n_kv, hd, (bf16_t*)att);
    else
        attn_merge_kernel<float><<<mg, 64, 0, s>>>(part_o, part_ml, p.nsplit, p.rpad, m, n_q, n_kv, hd, (float*)att);
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

// ------------------------------------------------------------------------------------------------
// stand-alone entry points: cache fill from logical K/V, attention over a batch of sequences
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void kv_write_kernel(T* __restrict__ kv_layer, const int32_t* __restrict__ pages, int max_pages,
                                const int32_t* __restrict__ pos0_arr, int n, int n_kv, int hd, const T* __restrict__ k,
                                const T* __restrict__ v) {
    const int b = blockIdx.z, i = blockIdx.x, kvh = blockIdx.y;
    const int pos = pos0_arr[b] + i;
    const int page = pages[(size_t)b * max_pages + pos / HSD_KV_PAGE], ip = pos % HSD_KV_PAGE;
    T* kblk = kv_layer + ((size_t)page * n_kv + kvh) * 2 * kv_block_elems(hd);
    T* vblk = kblk + kv_block_elems(hd);
    const size_t src = (((size_t)b * n + i) * n_kv + kvh) * hd;
    for (int d = threadIdx.x; d < hd; d += blockDim.x) {
        if constexpr (sizeof(T) == 4) {
            kblk[(size_t)ip * hd + d] = k[src + d];
            vblk[(size_t)ip * hd + d] = v[src + d];
        } else {
            kblk[kv_k_index(ip, d, hd)] = k[src + d];
            vblk[kv_v_index(ip, d, hd)] = v[src + d];
        }
    }
}

extern "C" size_t hsd_kv_layer_bytes(int n_pages, int n_kv, int hd, int dtype) {
    if (n_pages < 1 || n_kv < 1 || hd < 32 || hd % 32 != 0) return 0;
    return (size_t)n_pages * kv_page_elems(n_kv, hd) * dtype_size(dtype);
}

extern "C" size_t hsd_attention_workspace_bytes(int batch, int m, int n_q, int n_kv, int hd, int max_len) {
    if (batch < 1 || m < 1 || n_q < 1 || n_kv < 1 || n_q % n_kv != 0 || max_len < 1) return 0;
    return attn_workspace_bytes(batch, m, n_q, n_kv, hd, max_len);
}

static int check_attn_args(int batch, int m, int n_q, int n_kv, int hd, int dtype) {
    if (batch < 1 || m < 1 || m > HSD_MAX_PASS_ROWS) HSD_FAIL(HSD_EINVAL, "attention: batch=%d m=%d (m within 1..%d)", batch, m, HSD_MAX_PASS_ROWS);
    if (n_kv < 1 || n_q < 1 || n_q % n_kv != 0) HSD_FAIL(HSD_EINVAL, "attention: n_q=%d n_kv=%d", n_q, n_kv);
    if (hd % 32 != 0 || hd < 32 || hd > 256) HSD_FAIL(HSD_EINVAL, "attention: head dim %d", hd);
    if (dtype != HSD_F32 && dtype != HSD_BF16) HSD_FAIL(HSD_EINVAL, "attention: dtype %d", dtype);
    return HSD_OK;
}

extern "C" int hsd_kv_write(void* kv_layer_dev, const int32_t* pages_dev, int max_pages, const int32_t* pos0_dev, int batch, int n,
                            int n_kv, int hd, int dtype, const void* k_dev, const void* v_dev, void* stream) {
    if (!kv_layer_dev || !pages_dev || !pos0_dev || !k_dev || !v_dev) HSD_FAIL(HSD_EINVAL, "hsd_kv_write: null pointer");
    if (int rc = check_attn_args(batch, 1, n_kv, n_kv, hd, dtype)) return rc;
    if (n < 1 || max_pages < 1) HSD_FAIL(HSD_EINVAL, "hsd_kv_write: n=%d max_pages=%d", n, max_pages);
    dim3 grid(n, n_kv, batch);
    if (dtype == HSD_BF16)
        kv_write_kernel<bf16_t><<<grid, 64, 0, (hipStream_t)stream>>>((bf16_t*)kv_layer_dev, pages_dev, max_pages, pos0_dev, n, n_kv, hd,
                                                                      (const bf16_t*)k_dev, (const bf16_t*)v_dev);
    else
        kv_write_kernel<float><<<grid, 64, 0, (hipStream_t)stream>>>((float*)kv_layer_dev, pages_dev, max_pages, pos0_dev, n, n_kv, hd,
                                                                     (const float*)k_dev, (const float*)v_dev);
    HSD_LAUNCH_CHECK();
    return HSD_OK;
}

extern "C" int hsd_attention(const void* q_dev, const void* kv_layer_dev, const int32_t* pages_dev, int max_pages,
                             const int32_t* pos0_dev, int batch, int m, int max_len, int n_q, int n_kv, int hd, int dtype,
                             void* att_dev, void* workspace_dev, void* stream) {
    if (!q_dev || !kv_layer_dev || !pages_dev || !pos0_dev || !att_dev || !workspace_dev) HSD_FAIL(HSD_EINVAL, "hsd_attention: null pointer");
    if (int rc = check_attn_args(batch, m, n_q, n_kv, hd, dtype)) return rc;
    if (max_len < m || max_len > max_pages * HSD_KV_PAGE) HSD_FAIL(HSD_EINVAL, "hsd_attention: max_len=%d outside %d..%d", max_len, m, max_pages * HSD_KV_PAGE);
    return launch_attention(q_dev, kv_layer_dev, pages_dev, max_pages, pos0_dev, 0, batch, m, max_len, n_q, n_kv, hd, dtype, att_dev,
                            (float*)workspace_dev, 0, (hipStream_t)stream);
}
