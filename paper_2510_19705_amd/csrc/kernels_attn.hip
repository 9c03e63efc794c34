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
#include <algorithm>

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

constexpr size_t ATTN_TICKET_BYTES = 64 * 1024;  // arrival counters at the start of every attention workspace
int attn_max_splits(int batch, int m, int n_q, int n_kv);
constexpr int ATTN_FUSED_MAX_SPLITS = 16;     // most splits the attention kernel merges itself (last arriver)

template <int HD, int QT>
__global__ __launch_bounds__(512) void attn_mfma_kernel(const bf16_t* __restrict__ q, const bf16_t* __restrict__ kv_layer,
                                                        const int32_t* __restrict__ pages, int max_pages,
                                                        const int32_t* __restrict__ pos0_arr, int pos0_all, int M, int n_q,
                                                        int n_kv, float scale_log2, int steps_per_split, int nsplit, int qgroups,
                                                        int n_units, float* __restrict__ part_o, float* __restrict__ part_ml,
                                                        int rpad, bf16_t* __restrict__ att, int* __restrict__ tickets) {
    extern __shared__ float lds[];                 // [NW][QT*16][HD + 2]: o, then running max and sum
    constexpr int SP = HD == 64 ? 2 : 1;
    constexpr int KC = HD / 32;   // K chunks of 32 dims per 16-position tile
    constexpr int DT = HD / 16;   // 16-dim tiles of the output
    constexpr int RS = HD + 2;
    constexpr int NV = 8 * SP;    // scores per lane and query tile in one step
    // the wave index is the same in all lanes: telling the compiler so keeps the page-table lookups and the step
    // arithmetic on the scalar unit
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), NW = blockDim.x >> 6;
    const int j = lane & 15, grp = lane >> 4;
    // One-dimensional grid, decoded so that the query groups of one (sequence, KV head, split) unit sit 8 apart in
    // launch order: workgroups go to the 8 XCDs round-robin, so those groups land on the same XCD one after the
    // other and all but the first read the unit's K/V from that XCD's L2.
    const int xcd = blockIdx.x & 7, rr = blockIdx.x >> 3;
    const int qg = rr % qgroups, unit = (rr / qgroups) * 8 + xcd;
    if (unit >= n_units) return;
    const int split = unit % nsplit, g = (unit / nsplit) % n_kv, b = unit / (nsplit * n_kv);
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
        } else if (r < R) {
            if (tickets) {          // the last split to arrive merges: device-scope stores, performed where all XCDs see them
                __hip_atomic_store(part_o + (pbase + r) * HD + d, acc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (d == 0) {
                    __hip_atomic_store(part_ml + (pbase + r) * 2, m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(part_ml + (pbase + r) * 2 + 1, L, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            } else {
                part_o[(pbase + r) * HD + d] = acc;
                if (d == 0) {
                    part_ml[(pbase + r) * 2] = m;
                    part_ml[(pbase + r) * 2 + 1] = L;
                }
            }
        }
    }
    if (nsplit == 1 || !tickets) return;

    // ---- merge of the splits inside this launch (few splits, one query tile: the partial states of a
    // (sequence, KV head, query group) are a few KB).  Every wave waits until its device-scope stores have been
    // acknowledged, the barrier collects the waves, thread 0 takes a ticket; the last of the nsplit workgroups
    // reads all partial states back with device-scope loads (issued after its own ticket returned, i.e. after
    // every other split's stores were acknowledged) and writes the normalised rows.  Splits are added in split
    // order, so the result does not depend on who arrives last.
    __shared__ bool sh_last;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
    int* ticket = tickets + ((size_t)b * n_kv + g) * qgroups + qg;
    if (tid == 0) sh_last = __hip_atomic_fetch_add(ticket, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == nsplit - 1;
    __syncthreads();
    if (!sh_last) return;
    if (tid == 0) __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);     // for the next launch
    const size_t hbase = ((size_t)b * n_kv + g) * nsplit;
    float* wl = lds;                                    // [QT*16][nsplit] normalised weights; the waves' states are no longer needed
    for (int idx = tid; idx < QT * 16 * nsplit; idx += blockDim.x) {
        const int rl = idx / nsplit, sp = idx % nsplit;
        const int r = qg * QT * 16 + rl;
        float ms = -INFINITY, ls = 0.f;
        if (r < R) {
            ms = __hip_atomic_load(part_ml + ((hbase + sp) * rpad + r) * 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ls = __hip_atomic_load(part_ml + ((hbase + sp) * rpad + r) * 2 + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        wl[idx] = ms;
        wl[QT * 16 * nsplit + idx] = ls;
    }
    __syncthreads();
    for (int idx = tid; idx < QT * 16 * HD; idx += blockDim.x) {
        const int rl = idx / HD, d = idx % HD;
        const int r = qg * QT * 16 + rl;
        if (r >= R) continue;
        float v[ATTN_FUSED_MAX_SPLITS];                 // all splits' values requested together: one memory latency
#pragma unroll
        for (int sp = 0; sp < ATTN_FUSED_MAX_SPLITS; ++sp)
            v[sp] = sp < nsplit ? __hip_atomic_load(part_o + ((hbase + sp) * rpad + r) * HD + d, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.f;
        float mx = -INFINITY;
        for (int sp = 0; sp < nsplit; ++sp) mx = fmaxf(mx, wl[rl * nsplit + sp]);
        float L = 0.f, acc = 0.f;
#pragma unroll
        for (int sp = 0; sp < ATTN_FUSED_MAX_SPLITS; ++sp) {
            if (sp < nsplit) {
                const float ms = wl[rl * nsplit + sp];
                const float w = ms == -INFINITY ? 0.f : exp2f(ms - mx);
                L += w * wl[QT * 16 * nsplit + rl * nsplit + sp];
                acc += w == 0.f ? 0.f : w * v[sp];
            }
        }
        const int i = r / group, hq = r % group;
        att[(((size_t)b * M + i) * n_q + g * group + hq) * HD + d] = (bf16_t)(acc / L);
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
// merge of the sequence splits: one workgroup of four waves per (query row, KV head, batch).  grid (R, n_kv, batch).
// Wave 0 turns the splits' (max, sum) pairs into one weight per split (at most 64 splits: one per lane); then every
// wave adds up its quarter of the splits' outputs (independent loads, four dims per lane) and the four partial sums
// are added in wave order.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void attn_merge_kernel(const float* __restrict__ part_o, const float* __restrict__ part_ml,
                                                         int nsplit, int rpad, int M, int n_q, int n_kv, int hd,
                                                         T* __restrict__ att) {
    __shared__ float4 sh_acc[4][64];
    const int r = blockIdx.x, g = blockIdx.y, b = blockIdx.z, tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int group = n_q / n_kv, i = r / group, hq = r % group;
    const size_t base = ((size_t)b * n_kv + g) * nsplit;
    const int nvec = hd >> 2;                          // float4 chunks of a row, at most 64
    // every wave requests the (max, sum) pairs of all splits (lane s: split s) together with its own quarter of the
    // splits' outputs, so that one memory latency covers both; the weights are then computed redundantly per wave
    float ms = -INFINITY, ls = 0.f;
    if (lane < nsplit) {
        const float2 ml = *reinterpret_cast<const float2*>(part_ml + ((base + lane) * rpad + r) * 2);
        ms = ml.x;
        ls = ml.y;
    }
    constexpr int PER = 16;                            // splits per wave: 64 / 4
    float4 v[PER];
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int s = wave + 4 * k;
        v[k] = float4{0.f, 0.f, 0.f, 0.f};
        if (s < nsplit && lane < nvec) v[k] = *reinterpret_cast<const float4*>(part_o + ((base + s) * rpad + r) * hd + 4 * lane);
    }
    const float m = wave_max(ms);
    const float wgt = ms == -INFINITY ? 0.f : exp2f(ms - m);
    const float L = wave_sum(wgt * ls);
    const float wn = wgt / L;                          // lane s: normalised weight of split s
    float4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < PER; ++k) {
        const int s = wave + 4 * k;
        const float w = __shfl(wn, s & 63, 64);
        if (s < nsplit && w != 0.f) {
            acc.x += w * v[k].x; acc.y += w * v[k].y; acc.z += w * v[k].z; acc.w += w * v[k].w;
        }
    }
    sh_acc[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && lane < nvec) {
        float4 o = sh_acc[0][lane];
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const float4 v = sh_acc[w][lane];
            o.x += v.x; o.y += v.y; o.z += v.z; o.w += v.w;
        }
        T* dst = att + (((size_t)b * M + i) * n_q + g * group + hq) * hd + 4 * lane;
        dst[0] = from_f32<T>(o.x);
        dst[1] = from_f32<T>(o.y);
        dst[2] = from_f32<T>(o.z);
        dst[3] = from_f32<T>(o.w);
    }
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
struct AttnPlan {
    int nsplit, steps_per_split, rpad, qt, qgroups, nw;
    bool fused_merge;     // the kernel's last split to arrive merges (no second launch)
};

// Query tiles: up to attn_qt1_rows query rows per KV head every workgroup takes one 16-row tile (more workgroups, each
// re-reading the head's K/V from L2, instead of more tiles per workgroup): measured faster at every pass size up to
// 64 tokens and contexts up to 4096 (two tiles per workgroup double the registers and halve what is in flight), so
// the default never takes two.
AttnPlan attn_plan(int batch, int m, int n_q, int n_kv, int hd, int max_len, bool mfma, const hsd_kernel_tuning& t) {
    AttnPlan p;
    const int R = m * (n_q / n_kv);
    p.qt = R <= 16 || R <= t.attn_qt1_rows ? 1 : 2;
    p.qgroups = ceil_div(R, 16 * p.qt);
    p.rpad = p.qgroups * p.qt * 16;
    int total_steps = ceil_div(max_len, 32);
    if (mfma) {
        total_steps = ceil_div(max_len, hd == 64 ? 64 : 32);     // the MFMA kernel steps over a whole page for hd 64
        const int per_wave = p.qt * 16 * (hd + 2) * 4;               // LDS bytes of one wave's state
        p.nw = (144 * 1024) / per_wave;
        if (p.nw > 8) p.nw = 8;
        if (p.nw < 1) p.nw = 1;
        // One workgroup per (sequence, KV head, query group) while the sequence is short: up to 24 steps (16 KB of
        // K/V each) a second launch for the merge costs more than the idle CUs.  Beyond that the sequence is split so
        // that the launch has about one workgroup per CU (a CU pulls only ~40 GB/s, so the stream needs all 256 of
        // them, evenly loaded), each keeping at least 4 steps.
        const int heads = batch * n_kv * p.qgroups;
        int want = 1;
        if (t.attn_steps_per_wave > 0) {
            want = ceil_div(total_steps, p.nw * t.attn_steps_per_wave);
        } else if (total_steps > 24) {
            want = ((t.attn_target_wgs > 0 ? t.attn_target_wgs : 256) + heads / 2) / heads;
            if (want > total_steps / 4) want = total_steps / 4;
        }
        want = std::min(want, attn_max_splits(batch, m, n_q, n_kv));
        if (want < 1) want = 1;
        p.steps_per_split = ceil_div(total_steps, want);
        p.nsplit = ceil_div(total_steps, p.steps_per_split);
        // few splits of very few rows (7B shape, context 4096, 8 splits; microseconds, merged by the last arriver /
        // by a second launch: 1 row 18.3 / 19.3, 4 rows 18.5 / 19.5, 8 rows 20.1 / 19.6, 16 rows 23.4 / 20.1): the
        // last arriver's serial tail (acknowledged stores, ticket, two rounds of loads) grows with the rows
        p.fused_merge = t.attn_fused_merge && p.nsplit > 1 && p.nsplit <= ATTN_FUSED_MAX_SPLITS && p.nsplit * R <= 32 &&
                        (size_t)heads * sizeof(int) <= ATTN_TICKET_BYTES;
        return p;
    }
    p.fused_merge = false;
    p.nw = 1;
    int want = 2048 / (batch * n_kv * p.qgroups);
    if (want < 1) want = 1;
    want = std::min(want, attn_max_splits(batch, m, n_q, n_kv));
    int sps = ceil_div(total_steps, want);
    if (sps < 4) sps = 4;
    p.steps_per_split = sps;
    p.nsplit = ceil_div(total_steps, sps);
    return p;
}

// workspace: [arrival counters of the in-kernel merge, one per (sequence, KV head, query group), zero between
// launches: a region of fixed size, so that the counters sit at the same place whatever the launch][partial
// outputs][partial (max, sum) pairs]
size_t attn_ticket_bytes() { return ATTN_TICKET_BYTES; }

// Most splits of a sequence a launch may use: the plans aim for a few hundred workgroups, so launches with many
// (sequence, KV head, query group) units split less; the bound sizes the partial buffers.
int attn_max_splits(int batch, int m, int n_q, int n_kv) {
    const int R = m * (n_q / n_kv);
    const long long heads = (long long)batch * n_kv * ceil_div(R, 16);
    const long long s = (1024 + heads - 1) / heads;
    return (int)(s > 64 ? 64 : (s < 1 ? 1 : s));
}

size_t attn_workspace_bytes(int batch, int m, int n_q, int n_kv, int hd, int max_len) {
    (void)max_len;
    const int R = m * (n_q / n_kv);
    const int rpad = ceil_div(R, 16) * 16 + 16;        // + 16: two query tiles per workgroup round the rows up to 32
    return attn_ticket_bytes() +
           align_up((size_t)batch * n_kv * attn_max_splits(batch, m, n_q, n_kv) * rpad * (hd + 2) * sizeof(float), 256);
}

int launch_attention(const void* q, const void* kv_layer, const int32_t* pages, int max_pages, const int32_t* pos0_dev,
                     int pos0_all, int batch, int m, int max_len, int n_q, int n_kv, int hd, int dtype, void* att, float* workspace,
                     int force_simple, hipStream_t s, const hsd_kernel_tuning& t) {
    if (n_q % n_kv != 0) HSD_FAIL(HSD_EINVAL, "attention: n_q=%d not a multiple of n_kv=%d", n_q, n_kv);
    if (hd % 32 != 0 || hd > 256) HSD_FAIL(HSD_EINVAL, "attention: head dim %d must be a multiple of 32, at most 256", hd);
    const bool mfma = dtype == HSD_BF16 && !force_simple && (hd == 64 || hd == 128);
    AttnPlan p = attn_plan(batch, m, n_q, n_kv, hd, max_len, mfma, t);
    const int R = m * (n_q / n_kv);
    int* tickets = (int*)workspace;
    float* part_o = (float*)((char*)workspace + attn_ticket_bytes());
    float* part_ml = part_o + (size_t)batch * n_kv * p.nsplit * p.rpad * hd;
    const float scale_log2 = 1.4426950408889634f / sqrtf((float)hd);
    if (mfma) {
        const int n_units = batch * n_kv * p.nsplit;
        dim3 grid(ceil_div(n_units, 8) * 8 * p.qgroups);
#define HSD_ATT(HD_, QT_)                                                                                              \
    if (hd == HD_ && p.qt == QT_) {                                                                                    \
        const size_t lds_bytes = (size_t)p.nw * QT_ * 16 * (HD_ + 2) * 4;                                              \
        static size_t lds_allowed = 64 * 1024;   /* above the default limit the kernel needs an attribute, once */    \
        if (lds_bytes > lds_allowed) {                                                                                 \
            HSD_HIP(hipFuncSetAttribute((const void*)attn_mfma_kernel<HD_, QT_>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes)); \
            lds_allowed = lds_bytes;                                                                                   \
        }                                                                                                              \
        attn_mfma_kernel<HD_, QT_><<<grid, p.nw * 64, lds_bytes, s>>>(                                                 \
            (const bf16_t*)q, (const bf16_t*)kv_layer, pages, max_pages, pos0_dev, pos0_all, m, n_q, n_kv, scale_log2, \
            p.steps_per_split, p.nsplit, p.qgroups, n_units, part_o, part_ml, p.rpad, (bf16_t*)att,                    \
            p.fused_merge ? tickets : nullptr);                                                                        \
    }
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
    if (mfma && (p.nsplit == 1 || p.fused_merge)) return HSD_OK;            // the kernel wrote the normalised output itself
    dim3 mg(R, n_kv, batch);
    if (dtype == HSD_BF16)
        attn_merge_kernel<bf16_t><<<mg, 256, 0, s>>>(part_o, part_ml, p.nsplit, p.rpad, m, n_q, n_kv, hd, (bf16_t*)att);
    else
        attn_merge_kernel<float><<<mg, 256, 0, s>>>(part_o, part_ml, p.nsplit, p.rpad, m, n_q, n_kv, hd, (float*)att);
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

static int attention_entry(const void* q_dev, const void* kv_layer_dev, const int32_t* pages_dev, int max_pages,
                           const int32_t* pos0_dev, int batch, int m, int max_len, int n_q, int n_kv, int hd, int dtype,
                           void* att_dev, void* workspace_dev, void* stream, const hsd_kernel_tuning& t, const char* who) {
    if (!q_dev || !kv_layer_dev || !pages_dev || !pos0_dev || !att_dev || !workspace_dev) HSD_FAIL(HSD_EINVAL, "%s: null pointer", who);
    if (int rc = check_attn_args(batch, m, n_q, n_kv, hd, dtype)) return rc;
    if (max_len < m || max_len > max_pages * HSD_KV_PAGE) HSD_FAIL(HSD_EINVAL, "%s: max_len=%d outside %d..%d", who, max_len, m, max_pages * HSD_KV_PAGE);
    return launch_attention(q_dev, kv_layer_dev, pages_dev, max_pages, pos0_dev, 0, batch, m, max_len, n_q, n_kv, hd, dtype, att_dev,
                            (float*)workspace_dev, 0, (hipStream_t)stream, t);
}

extern "C" int hsd_attention(const void* q_dev, const void* kv_layer_dev, const int32_t* pages_dev, int max_pages,
                             const int32_t* pos0_dev, int batch, int m, int max_len, int n_q, int n_kv, int hd, int dtype,
                             void* att_dev, void* workspace_dev, void* stream) {
    return attention_entry(q_dev, kv_layer_dev, pages_dev, max_pages, pos0_dev, batch, m, max_len, n_q, n_kv, hd, dtype, att_dev,
                           workspace_dev, stream, default_kernel_tuning(), "hsd_attention");
}

extern "C" int hsd_attention_tuned(const void* q_dev, const void* kv_layer_dev, const int32_t* pages_dev, int max_pages,
                                   const int32_t* pos0_dev, int batch, int m, int max_len, int n_q, int n_kv, int hd, int dtype,
                                   void* att_dev, void* workspace_dev, void* stream, const hsd_kernel_tuning* t) {
    return attention_entry(q_dev, kv_layer_dev, pages_dev, max_pages, pos0_dev, batch, m, max_len, n_q, n_kv, hd, dtype, att_dev,
                           workspace_dev, stream, t ? *t : default_kernel_tuning(), "hsd_attention_tuned");
}
