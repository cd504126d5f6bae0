// seer_verify_attention: entry point, device-side split-K plan, the general
// (any supported shape) partition kernel, and the split-K combine.
//
// What is computed (paper, Section 2.2: the target model verifies all draft
// tokens of a request in one pass, which beats serial decoding because the
// context is read from memory once instead of once per token): every one of the
// T = gamma + 1 verify slots of a request attends to the request's cached
// prefix and to the draft slots on its own root path (chain or multi-path tree,
// Section 3.4.2).  One read of a KV page must therefore serve all T slots and
// all G query heads that share the KV head.
#include "seer_attention.h"
#include "../../include/seer_verify_diag.h"

#include <stdio.h>

#include "seer_device.h"

namespace seer {

// ---------------------------------------------------------------------------
// Plan: one workgroup turns ctx_len[B] into the tile line, the stretch of every
// partition workgroup, and the table of (request, stretch) pieces; a second one,
// beside it, compares neighbouring block-table rows (plan_shared_pages).
// ---------------------------------------------------------------------------
constexpr int kPlanThreads = 256;

struct PlanArgs {
    const int32_t* ctx_len;
    const int32_t* block_table;
    int B, T, max_ctx, wgs_per_head, max_splits, max_items, fixed_split, max_pages, page_size;
    PlanHeader* header;
    int32_t* split_off;
    int32_t* tile_off;
    int32_t* wg_first;
    int32_t* wg_start;
    int32_t* req_first;
    int32_t* shared_tiles;
    uint32_t* fb_time;
    uint32_t* fb_tiles;
    float* fb_speed;
    WorkItem* items;
};

// Block-wide primitives for the 256 threads of the plan kernel (4 waves): wave shuffles, then one
// value per wave through LDS.  s_tmp: at least 2 * (kPlanThreads / kWave) words, reused call after call.
template <typename T>
__device__ __forceinline__ T plan_excl_scan(T v, T* s_tmp, T& total) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    T incl = v;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const T up = __shfl_up(incl, o, kWave);
        if (lane >= o) incl += up;
    }
    __syncthreads();                     // s_tmp may still be read by the previous call
    if (lane == kWave - 1) s_tmp[wave] = incl;
    __syncthreads();
    T base = 0, sum = 0;
#pragma unroll
    for (int w = 0; w < kPlanThreads / kWave; ++w) {
        const T x = s_tmp[w];
        if (w < wave) base += x;
        sum += x;
    }
    total = sum;
    return base + incl - v;
}
__device__ __forceinline__ float plan_sum(float v, float* s_tmp) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, kWave);
    __syncthreads();
    if (lane == 0) s_tmp[wave] = v;
    __syncthreads();
    float sum = 0.f;
#pragma unroll
    for (int w = 0; w < kPlanThreads / kWave; ++w) sum += s_tmp[w];
    return sum;
}
__device__ __forceinline__ int plan_max(int v, int* s_tmp) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = max(v, __shfl_xor(v, o, kWave));
    __syncthreads();
    if (lane == 0) s_tmp[wave] = v;
    __syncthreads();
    int m = s_tmp[0];
#pragma unroll
    for (int w = 1; w < kPlanThreads / kWave; ++w) m = max(m, s_tmp[w]);
    return m;
}

// The plan's second workgroup.  Leading pages that a request has in common with the request before or after it
// (the prompt that the rollouts of a group share sits in the same physical pages): the partition kernel loads such
// tiles with the cache policy that keeps them, so that the repeats are served by the memory-side cache.  This is a
// hint only, results do not depend on it, so the length of the common run is found by probing instead of comparing
// every entry: sixteen entries at doubling distances, then sixteen evenly spaced ones between the last equal probe
// and the first unequal one (two dependent rounds of loads; exact for runs of up to 32 pages, else short by less
// than a sixteenth of the run if the tables are equal up to a point and differ behind it).  It runs beside the
// first workgroup, which needs about as long for the tile line and the stretches.
__device__ __forceinline__ void plan_shared_pages(const PlanArgs& p) {
    for (int b = threadIdx.x; b < p.B; b += kPlanThreads) {
        const int n = p.ctx_len[b];
        int best = 0;
        if (n >= p.T && n <= p.max_ctx) {
            const int32_t* mine = p.block_table + static_cast<size_t>(b) * p.max_pages;
            const int pages = (n + p.page_size - 1) / p.page_size;
            int m[2] = {0, 0};                 // entries that can be compared with the neighbour
            const int32_t* other[2] = {mine, mine};
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int nb = s ? b + 1 : b - 1;
                if (nb < 0 || nb >= p.B) continue;
                const int nn = p.ctx_len[nb];
                if (nn < p.T || nn > p.max_ctx) continue;
                m[s] = min(pages, (nn + p.page_size - 1) / p.page_size);
                other[s] = p.block_table + static_cast<size_t>(nb) * p.max_pages;
            }
            uint32_t eq[2] = {0u, 0u};        // bit k: probe k found equal entries
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    const int i = (1 << k) - 1;
                    const int ic = min(i, max(m[s] - 1, 0));
                    eq[s] |= static_cast<uint32_t>((i < m[s]) & (mine[ic] == other[s][ic])) << k;
                }
            int lo[2], step[2], hi[2];
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int k = __builtin_ctz(~eq[s]);          // first probe that differs or lies outside (<= 16)
                lo[s] = k ? (1 << (k - 1)) : 0;               // number of leading entries taken as equal
                hi[s] = k ? min((1 << k) - 1, m[s]) : 0;      // entry hi differs or does not exist
                step[s] = max(1, (hi[s] - lo[s] + 15) / 16);
                eq[s] = 0u;
            }
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int i = lo[s] + (j + 1) * step[s] - 1;
                    const int ic = min(i, max(m[s] - 1, 0));
                    eq[s] |= static_cast<uint32_t>((i < hi[s]) & (mine[ic] == other[s][ic])) << j;
                }
#pragma unroll
            for (int s = 0; s < 2; ++s) best = max(best, min(lo[s] + __builtin_ctz(~eq[s]) * step[s], hi[s]));
        }
        p.shared_tiles[b] = static_cast<int>(static_cast<long long>(best) * p.page_size / kPlanTile);
    }
}

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(PlanArgs p) {
    if (blockIdx.x == 1) {
        plan_shared_pages(p);
        return;
    }
    __shared__ int s_tmp[2 * kPlanThreads / kWave];
    __shared__ int s_start[kMaxWgsPerHead + 1];
    const int tid = threadIdx.x;
    const int W = p.wgs_per_head;
    for (int w = tid; w < W; w += kPlanThreads) p.wg_first[w] = -1;

    // thread `tid` owns a contiguous run of requests
    const int per = (p.B + kPlanThreads - 1) / kPlanThreads;
    const int b0 = min(p.B, tid * per), b1 = min(p.B, b0 + per);
    auto tiles_of = [&](int b) -> int {
        const int n = p.ctx_len[b];
        if (n < p.T || n > p.max_ctx) return 0;   // flagged, gets a zero output
        return (n + kPlanTile - 1) / kPlanTile;
    };

    // 1. tile line: exclusive prefix of tiles per request, and the longest request
    int cnt = 0, mx = 0, bad = 0;
    for (int b = b0; b < b1; ++b) {
        const int n = p.ctx_len[b];
        if (n < p.T || n > p.max_ctx) bad = 1;
        const int t = tiles_of(b);
        cnt += t;
        mx = max(mx, t);
    }
    int total = 0;
    const int my_tile_off = plan_excl_scan(cnt, s_tmp, total);
    const int longest = plan_max(mx, s_tmp);
    bad = plan_max(bad, s_tmp);
    {
        int off = my_tile_off;
        for (int b = b0; b < b1; ++b) {
            p.tile_off[b] = off;
            off += tiles_of(b);
        }
        if (tid == 0) p.tile_off[p.B] = total;
    }

    // 2. the stretches (balanced mode; L = 0 means one workgroup per request)
    int L = 0;
    if (p.max_splits > 1) {
        L = max((total + W - 1) / W, 1);
        // a request of t tiles touches at most ceil(t / Lmin) + 1 stretches, which must fit max_splits
        const int Lmin = max(kMinTilesPerWg, (longest + p.max_splits - 2) / (p.max_splits - 1));
        // relative speed of each stretch index from the history in the workspace; thread t owns the
        // stretch indices [t * per_w, t * per_w + per_w)
        constexpr int kPerW = kMaxWgsPerHead / kPlanThreads;
        const int per_w = (W + kPlanThreads - 1) / kPlanThreads;
        const int w0 = min(W, tid * per_w);
        const bool have = !p.fixed_split && p.header->fb_magic == kFeedbackMagic && p.header->fb_w == W;
        float speed[kPerW];
        float sum = 0.f, known = 0.f;
#pragma unroll
        for (int i = 0; i < kPerW; ++i) {
            const int w = w0 + i;
            speed[i] = 0.f;
            if (i < per_w && w < W) {
                float est = have ? p.fb_speed[w] : 0.f;
                const uint32_t ticks = have ? p.fb_time[w] : 0u, tiles = have ? p.fb_tiles[w] : 0u;
                if (ticks > 0u && tiles > 0u) {
                    const float meas = static_cast<float>(tiles) / static_cast<float>(ticks);
                    est = est > 0.f ? 0.5f * est + 0.5f * meas : meas;
                }
                if (!(est > 0.f) || !(est < 1e30f)) est = 0.f;     // unknown (also whatever a stale workspace held)
                if (!p.fixed_split) {
                    p.fb_speed[w] = est;
                    p.fb_time[w] = 0u;
                    p.fb_tiles[w] = 0u;
                }
                speed[i] = est;
                if (est > 0.f) {
                    sum += est;
                    known += 1.f;
                }
            }
        }
        sum = plan_sum(sum, reinterpret_cast<float*>(s_tmp));
        known = plan_sum(known, reinterpret_cast<float*>(s_tmp));
        const float mean = known > 0.f ? sum / known : 1.f;
        // Stretch w begins at the tile nearest to total * (r_0 + .. + r_{w-1}) / R.  When the line is too
        // short for that to keep every stretch at Lmin tiles or more, cut it into equal stretches of
        // max(Lmin, ceil(total / W)) tiles instead (the last ones are then short or empty).
        const bool weighted = static_cast<long long>(total) >= 2ll * Lmin * W;
        float rsum = 0.f;
#pragma unroll
        for (int i = 0; i < kPerW; ++i) {
            if (i < per_w && w0 + i < W) {
                const float r = (weighted && speed[i] > 0.f) ? speed[i] / mean : 1.f;
                speed[i] = fminf(fmaxf(r, 0.75f), 4.f / 3.f);
                rsum += speed[i];
            }
        }
        float R = 0.f;
        float before = plan_excl_scan(rsum, reinterpret_cast<float*>(s_tmp), R);
        const int L_equal = max(Lmin, L);
#pragma unroll
        for (int i = 0; i < kPerW; ++i) {
            if (i < per_w && w0 + i < W) {
                const int w = w0 + i;
                const long long cut = weighted ? static_cast<long long>(static_cast<double>(total) * before / R + 0.5)
                                               : static_cast<long long>(w) * L_equal;
                s_start[w] = static_cast<int>(cut < total ? cut : total);
                before += speed[i];
            }
        }
        if (tid == 0) s_start[W] = total;
        __syncthreads();
        for (int w = tid; w <= W; w += kPlanThreads) p.wg_start[w] = s_start[w];
    }
    // stretch that holds tile x (x < total): the last one that starts at or before it
    auto stretch_of = [&](int x) -> int {
        int lo = 0, hi = W - 1;
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (s_start[mid] <= x) lo = mid; else hi = mid - 1;
        }
        return lo;
    };

    // 3. pieces per request -> first partial slot of each request
    cnt = 0;
    {
        int lo = my_tile_off;
        for (int b = b0; b < b1; ++b) {
            const int hi = lo + tiles_of(b);
            if (hi > lo) cnt += L ? stretch_of(hi - 1) - stretch_of(lo) + 1 : 1;
            lo = hi;
        }
    }
    int n_pieces = 0;
    int slot = plan_excl_scan(cnt, s_tmp, n_pieces);
    if (tid == 0) {
        p.header->status = bad ? 1u : 0u;
        p.header->n_items = min(n_pieces, p.max_items);
        p.header->tiles_per_wg = L;
        p.header->total_tiles = total;
        if (!p.fixed_split) {
            p.header->fb_magic = kFeedbackMagic;
            p.header->fb_w = W;
        }
        p.split_off[p.B] = n_pieces;
    }

    // 4. piece table and the request each stretch starts in
    int lo = my_tile_off;
    for (int b = b0; b < b1; ++b) {
        const int hi = lo + tiles_of(b);
        p.split_off[b] = slot;
        const int n = p.ctx_len[b];
        const int w_first = hi > lo ? (L ? stretch_of(lo) : b) : 0;
        const int np = hi > lo ? (L ? stretch_of(hi - 1) - w_first + 1 : 1) : 0;
        p.req_first[b] = w_first;
        for (int s = 0; s < np; ++s) {
            const int w = w_first + s;
            const int w_begin = L ? s_start[w] : lo, w_end = L ? s_start[w + 1] : hi;
            const int t_begin = max(lo, w_begin);
            const int t_end = min(hi, w_end);
            if (slot + s < p.max_items) {
                WorkItem it;
                it.b = b;
                it.begin = (t_begin - lo) * kPlanTile;
                it.end = min(n, (t_end - lo) * kPlanTile);
                it.split = s;
                p.items[slot + s] = it;
            }
            if (t_begin == w_begin && w < W) p.wg_first[w] = b;   // stretch w starts here
        }
        slot += np;
        lo = hi;
    }
}

hipError_t launch_plan(const AttnArgs& a, const WorkspaceLayout& w, hipStream_t stream) {
    const long long max_ctx_ll = static_cast<long long>(a.max_pages) * a.P;
    PlanArgs p;
    p.ctx_len = a.ctx_len;
    p.block_table = a.block_table;
    p.max_pages = a.max_pages;
    p.page_size = a.P;
    p.shared_tiles = const_cast<int32_t*>(a.shared_tiles);
    p.B = a.B;
    p.T = a.T;
    p.max_ctx = max_ctx_ll > 0x7fffffffLL - kPlanTile ? 0x7fffffff - kPlanTile : static_cast<int>(max_ctx_ll);
    p.wgs_per_head = w.wgs_per_head;
    p.max_splits = w.max_splits;
    p.max_items = w.max_items;
    p.header = a.header;
    p.split_off = const_cast<int32_t*>(a.split_off);
    p.tile_off = const_cast<int32_t*>(a.tile_off);
    p.wg_first = const_cast<int32_t*>(a.wg_first);
    p.wg_start = const_cast<int32_t*>(a.wg_start);
    p.req_first = const_cast<int32_t*>(a.req_first);
    p.fb_time = a.fb_time;
    p.fb_tiles = a.fb_tiles;
    p.fb_speed = a.fb_speed;
    p.fixed_split = a.fixed_split;
    p.items = const_cast<WorkItem*>(a.items);
    hipLaunchKernelGGL(plan_kernel, dim3(2), dim3(kPlanThreads), 0, stream, p);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// General partition kernel: one workgroup per (item, query head, slot).
// Plain vector arithmetic, one KV token per wave iteration: lanes split the
// head dimension, the dot product is reduced with shuffles, the running
// (max, sum, acc) is kept per wave and the four waves are merged through LDS.
// Slow, but it covers every supported head size and page size, and serves as
// the on-device cross-check of the tiled kernels.
// ---------------------------------------------------------------------------
constexpr int kGenThreads = 256;
constexpr int kGenWaves = kGenThreads / kWave;

template <int DQK, int DV>
__global__ __launch_bounds__(kGenThreads) void attn_general_kernel(AttnArgs a) {
    constexpr int NQ = (DQK + 127) / 128;  // bf16 pairs per lane
    constexpr int NV = (DV + 127) / 128;
    const int item_idx = blockIdx.x;
    if (item_idx >= a.header->n_items) return;
    const WorkItem item = a.items[item_idx];
    const int hq = blockIdx.y, t = blockIdx.z;
    const int kvh = hq / a.G;
    const int b = item.b;
    const int n = a.ctx_len[b];
    const int n0 = n - a.T;
    const uint64_t word = a.tree_mask ? a.tree_mask[static_cast<size_t>(b) * a.T + t]
                                      : (t >= 63 ? ~0ull : ((1ull << (t + 1)) - 1));
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const uint16_t* __restrict__ kp = static_cast<const uint16_t*>(a.k_pages);
    const uint16_t* __restrict__ vp = static_cast<const uint16_t*>(a.v_pages);
    const uint16_t* __restrict__ qrow =
        static_cast<const uint16_t*>(a.q) + ((static_cast<size_t>(b) * a.T + t) * a.Hq + hq) * DQK;

    float qlo[NQ], qhi[NQ];
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
        const int d = 2 * lane + 128 * i;
        const uint32_t pr = (d < DQK) ? *reinterpret_cast<const uint32_t*>(qrow + d) : 0u;
        qlo[i] = bf16lo_to_f32(pr);
        qhi[i] = bf16hi_to_f32(pr);
    }
    float m = kNegInf, l = 0.f;
    float alo[NV], ahi[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) alo[i] = ahi[i] = 0.f;

    const int32_t* __restrict__ table = a.block_table + static_cast<size_t>(b) * a.max_pages;
    bool bad_page = false;
    for (int j = item.begin + wave; j < item.end; j += kGenWaves) {
        const bool visible = (j < n0) || ((word >> (j - n0)) & 1ull);
        if (!visible) continue;  // uniform across the wave
        int page = table[j / a.P];
        if (page < 0 || page >= a.num_pages) {
            bad_page = true;
            page = min(max(page, 0), a.num_pages - 1);
        }
        const size_t tok = (static_cast<size_t>(page) * a.Hkv + kvh) * a.P + (j % a.P);
        const uint16_t* __restrict__ krow = kp + tok * DQK;
        float part = 0.f;
        uint32_t kpair[NQ];
#pragma unroll
        for (int i = 0; i < NQ; ++i) {
            const int d = 2 * lane + 128 * i;
            kpair[i] = (d < DQK) ? *reinterpret_cast<const uint32_t*>(krow + d) : 0u;
            part = fmaf(qlo[i], bf16lo_to_f32(kpair[i]), part);
            part = fmaf(qhi[i], bf16hi_to_f32(kpair[i]), part);
        }
        const float s = wave_sum(part) * a.scale_log2;
        const float m_new = fmaxf(m, s);
        const float alpha = fast_exp2(m - m_new);
        const float p = fast_exp2(s - m_new);
        l = l * alpha + p;
        m = m_new;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int d = 2 * lane + 128 * i;
            uint32_t vpair;
            if (vp) vpair = (d < DV) ? *reinterpret_cast<const uint32_t*>(vp + tok * DV + d) : 0u;
            else vpair = (i < NQ) ? kpair[i < NQ ? i : 0] : 0u;  // shared latent: V = K[..., :DV]
            alo[i] = fmaf(p, bf16lo_to_f32(vpair), alo[i] * alpha);
            ahi[i] = fmaf(p, bf16hi_to_f32(vpair), ahi[i] * alpha);
        }
    }
    if (bad_page && lane == 0) atomicOr(&a.header->status, 2u);

    __shared__ float s_m[kGenWaves], s_l[kGenWaves];
    __shared__ float s_acc[kGenWaves][DV];
    if (lane == 0) {
        s_m[wave] = m;
        s_l[wave] = l;
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int d = 2 * lane + 128 * i;
        if (d < DV) {
            s_acc[wave][d] = alo[i];
            s_acc[wave][d + 1] = ahi[i];
        }
    }
    __syncthreads();
    float M = s_m[0];
#pragma unroll
    for (int w = 1; w < kGenWaves; ++w) M = fmaxf(M, s_m[w]);
    float f[kGenWaves];
    float L = 0.f;
#pragma unroll
    for (int w = 0; w < kGenWaves; ++w) {
        f[w] = (s_m[w] == kNegInf) ? 0.f : fast_exp2(s_m[w] - M);
        L += s_l[w] * f[w];
    }
    const size_t prow = (static_cast<size_t>(item_idx) * a.T + t) * a.Hq + hq;
    if (threadIdx.x == 0) {
        a.part_ml[2 * prow] = M;
        a.part_ml[2 * prow + 1] = L;
    }
    for (int d = threadIdx.x; d < DV; d += kGenThreads) {
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < kGenWaves; ++w) v += s_acc[w][d] * f[w];
        a.part_acc[prow * DV + d] = v;
    }
}

bool general_supports(int Dqk, int Dv) {
    return (Dqk == 64 && Dv == 64) || (Dqk == 128 && Dv == 128) || (Dqk == 256 && Dv == 256) ||
           (Dqk == 192 && Dv == 128) || (Dqk == 576 && Dv == 512);
}

hipError_t launch_general(const AttnArgs& a, hipStream_t stream) {
    const dim3 grid(a.max_items, a.Hq, a.T), block(kGenThreads);
#define SEER_GEN_CASE(DQK_, DV_)                                                                   \
    if (a.Dqk == DQK_ && a.Dv == DV_) {                                                            \
        hipLaunchKernelGGL((attn_general_kernel<DQK_, DV_>), grid, block, 0, stream, a);           \
        return hipGetLastError();                                                                  \
    }
    SEER_GEN_CASE(64, 64)
    SEER_GEN_CASE(128, 128)
    SEER_GEN_CASE(256, 256)
    SEER_GEN_CASE(192, 128)
    SEER_GEN_CASE(576, 512)
#undef SEER_GEN_CASE
    return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------
// Combine: out = sum_s acc_s * 2^(m_s - M) / sum_s l_s * 2^(m_s - M), M = max_s m_s.
// A thread owns 4 consecutive output values of one row (16-byte loads of the fp32
// partials, one 8-byte bf16 store); a 256-thread workgroup covers 1024 / Dv rows,
// so the launch has a few thousand workgroups instead of one per row.
// ---------------------------------------------------------------------------
constexpr int kCombineThreads = 256;

__global__ __launch_bounds__(kCombineThreads) void combine_kernel(AttnArgs a, long long n_rows) {
    const int per_row = a.Dv >> 2;                       // threads per output row (Dv is a multiple of 64)
    const long long gid = static_cast<long long>(blockIdx.x) * kCombineThreads + threadIdx.x;
    const long long row = gid / per_row;                 // (b*T + t)*Hq + h
    if (row >= n_rows) return;
    const int d = static_cast<int>(gid - row * per_row) << 2;
    const int per_b = a.T * a.Hq;
    const int b = static_cast<int>(row / per_b);
    const int r = static_cast<int>(row - static_cast<long long>(b) * per_b);
    const int first = a.split_off[b];
    int ns = a.split_off[b + 1] - first;
    if (first + ns > a.max_items) ns = max(0, a.max_items - first);

    // Both passes request the partial results of several pieces before using any of them (no branch
    // between the loads): a thread otherwise waits one round trip per piece.
    const float2* ml = reinterpret_cast<const float2*>(a.part_ml) + static_cast<size_t>(first) * per_b + r;
    const float* acc = a.part_acc + (static_cast<size_t>(first) * per_b + r) * a.Dv + d;
    const size_t acc_stride = static_cast<size_t>(per_b) * a.Dv;
    float M = kNegInf;
    int s = 0;
    if (ns >= 1 && ns <= 4) {
        // The common case, a request cut into a handful of pieces: everything is requested at once (the pieces past
        // ns re-read the last one and count as having seen nothing), one round trip instead of one per piece and
        // pass.  Same operations in the same order as the general path below.
        float2 msl[4];
        f32x4 p[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int su = min(u, ns - 1);
            msl[u] = ml[static_cast<size_t>(su) * per_b];
            p[u] = *reinterpret_cast<const f32x4*>(acc + su * acc_stride);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (u >= ns) msl[u].x = kNegInf;
            M = fmaxf(M, msl[u].x);
        }
        float L = 0.f;
        f32x4 v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const bool live = msl[u].x != kNegInf;
            const float w = live ? fast_exp2(msl[u].x - M) : 0.f;
            L += live ? msl[u].y * w : 0.f;
#pragma unroll
            for (int c = 0; c < 4; ++c) v[c] += live ? p[u][c] * w : 0.f;
        }
        const float inv = (L > 0.f) ? 1.f / L : 0.f;
        u32x2 o;
        o[0] = pack_bf16x2(v[0] * inv, v[1] * inv);
        o[1] = pack_bf16x2(v[2] * inv, v[3] * inv);
        *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(a.out) + row * a.Dv + d) = o;
        return;
    }
    for (; s + 4 <= ns; s += 4) {
        float m4[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) m4[u] = ml[static_cast<size_t>(s + u) * per_b].x;
#pragma unroll
        for (int u = 0; u < 4; ++u) M = fmaxf(M, m4[u]);
    }
    for (; s < ns; ++s) M = fmaxf(M, ml[static_cast<size_t>(s) * per_b].x);
    float L = 0.f;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    auto add = [&](float2 msl, f32x4 p) {
        // a piece that saw nothing for this row (m = -inf) may hold anything in its accumulator
        const bool live = msl.x != kNegInf;
        const float w = live ? fast_exp2(msl.x - M) : 0.f;
        L += live ? msl.y * w : 0.f;
#pragma unroll
        for (int c = 0; c < 4; ++c) v[c] += live ? p[c] * w : 0.f;
    };
    s = 0;
    for (; s + 4 <= ns; s += 4) {
        float2 msl[4];
        f32x4 p[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            msl[u] = ml[static_cast<size_t>(s + u) * per_b];
            p[u] = *reinterpret_cast<const f32x4*>(acc + (s + u) * acc_stride);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) add(msl[u], p[u]);
    }
    for (; s < ns; ++s) add(ml[static_cast<size_t>(s) * per_b], *reinterpret_cast<const f32x4*>(acc + s * acc_stride));
    const float inv = (L > 0.f) ? 1.f / L : 0.f;         // a row that saw nothing: zeros
    u32x2 o;
    o[0] = pack_bf16x2(v[0] * inv, v[1] * inv);
    o[1] = pack_bf16x2(v[2] * inv, v[3] * inv);
    *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(a.out) + row * a.Dv + d) = o;
}

hipError_t launch_combine(const AttnArgs& a, hipStream_t stream) {
    const long long rows = static_cast<long long>(a.B) * a.T * a.Hq;
    const long long threads = rows * (a.Dv >> 2);
    const unsigned blocks = static_cast<unsigned>((threads + kCombineThreads - 1) / kCombineThreads);
    hipLaunchKernelGGL(combine_kernel, dim3(blocks), dim3(kCombineThreads), 0, stream, a, rows);
    return hipGetLastError();
}

}  // namespace seer

// ---------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------
namespace {

int validate_params(const seer_attn_params* p) {
    if (!p) return SEER_EINVAL;
    if (p->B < 0 || p->num_pages < 1 || p->max_pages_per_seq < 1 || p->page_size < 1) return SEER_EINVAL;
    if (p->T < 1 || p->T > SEER_MAX_T || p->Hq < 1 || p->Hkv < 1 || p->Hq % p->Hkv != 0) return SEER_ESHAPE;
    if (p->max_splits < 0 || p->max_splits > 256) return SEER_ESHAPE;
    if (p->flags & ~(SEER_ATTN_GENERAL_KERNEL | SEER_ATTN_FIXED_SPLIT | SEER_ATTN_STREAM_ONLY | SEER_ATTN_REUSE_PLAN))
        return SEER_EINVAL;
    if (p->Hq > 65535 || p->T * (int64_t)p->Hq * p->B > 0x7fffffffLL) return SEER_ESHAPE;
    if (!(p->scale > 0.f) || p->scale > 3.0e38f) return SEER_EINVAL;   // positive and finite
    if (!seer::general_supports(p->Dqk, p->Dv)) return SEER_EUNSUPPORTED;
    if (p->kv_shared_latent && p->Dv > p->Dqk) return SEER_ESHAPE;
    return SEER_OK;
}

}  // namespace

extern "C" size_t seer_verify_attention_workspace(const seer_attn_params* p) {
    if (validate_params(p) != SEER_OK || p->B == 0) return 0;
    return seer::workspace_layout(*p).total;
}

extern "C" size_t seer_verify_attention_status_offset(void) { return offsetof(seer::PlanHeader, status); }

extern "C" size_t seer_verify_attention_shared_tiles_offset(const seer_attn_params* p) {
    if (validate_params(p) != SEER_OK || p->B == 0) return 0;
    return seer::workspace_layout(*p).off_shared;
}

extern "C" const char* seer_verify_attention_kernel(const seer_attn_params* p) {
    if (validate_params(p) != SEER_OK) return nullptr;
    // the same tests, on the same fields, as the dispatch in run_verify_attention
    seer::AttnArgs a{};
    a.Dqk = p->Dqk, a.Dv = p->Dv, a.P = p->page_size, a.Hkv = p->Hkv;
    a.v_pages = p->kv_shared_latent ? nullptr : static_cast<const void*>(p);   // only null / non-null is looked at
    const bool tiled_ok = !(p->flags & SEER_ATTN_GENERAL_KERNEL);
    if (tiled_ok && seer::gqa128_supports(a)) {
        struct Names {
            char text[9][40];
            Names() {
                for (int nw = 1; nw <= 8; ++nw)
                    snprintf(text[nw], sizeof(text[nw]), "attn_gqa128_kernel<%d,%d>", nw, seer::gqa_pipe_depth(nw));
            }
        };
        static const Names names;
        const int rows = (p->Hq / p->Hkv) * p->T;
        if (seer::gqa_block_uses_helpers(seer::gqa_rows_per_block(rows))) return "attn_gqa128_kernel<4,2,helpers=4>";
        return names.text[seer::gqa_rows_per_block(rows) / 32];
    }
    if (tiled_ok && seer::mla_supports(a)) return "attn_mla_kernel";
    if (p->Dqk == 64) return "attn_general_kernel<64,64>";
    if (p->Dqk == 128) return "attn_general_kernel<128,128>";
    if (p->Dqk == 256) return "attn_general_kernel<256,256>";
    if (p->Dqk == 192) return "attn_general_kernel<192,128>";
    return "attn_general_kernel<576,512>";
}

namespace {

int run_verify_attention(void* out, const void* q, const void* k_pages, const void* v_pages,
                         const int32_t* block_table, const int32_t* ctx_len, const uint64_t* tree_mask,
                         const seer_attn_params* p, void* workspace, size_t workspace_bytes, void* hip_stream,
                         hipEvent_t ev_begin, hipEvent_t ev_end) {
    const int rc = validate_params(p);
    if (rc != SEER_OK) return rc;
    if (p->B == 0) return SEER_OK;
    if (!out || !q || !k_pages || !block_table || !ctx_len) return SEER_EINVAL;
    if (p->kv_shared_latent ? (v_pages != nullptr) : (v_pages == nullptr)) return SEER_EINVAL;
    const seer::WorkspaceLayout w = seer::workspace_layout(*p);
    if (!workspace || workspace_bytes < w.total) return SEER_EWORKSPACE;
    auto misaligned = [](const void* ptr, uintptr_t a) { return reinterpret_cast<uintptr_t>(ptr) % a != 0; };
    if (misaligned(out, 16) || misaligned(q, 16) || misaligned(k_pages, 16) || misaligned(v_pages, 16) ||
        misaligned(workspace, 256) || misaligned(block_table, 4) || misaligned(ctx_len, 4) ||
        misaligned(tree_mask, 8))
        return SEER_EALIGN;

    char* ws = static_cast<char*>(workspace);
    seer::AttnArgs a{};
    a.out = out;
    a.q = q;
    a.k_pages = k_pages;
    a.v_pages = v_pages;
    a.block_table = block_table;
    a.ctx_len = ctx_len;
    a.tree_mask = tree_mask;
    a.header = reinterpret_cast<seer::PlanHeader*>(ws + w.off_header);
    a.split_off = reinterpret_cast<const int32_t*>(ws + w.off_split);
    a.tile_off = reinterpret_cast<const int32_t*>(ws + w.off_tiles);
    a.wg_first = reinterpret_cast<const int32_t*>(ws + w.off_first);
    a.wg_start = reinterpret_cast<const int32_t*>(ws + w.off_start);
    a.req_first = reinterpret_cast<const int32_t*>(ws + w.off_reqfirst);
    a.shared_tiles = reinterpret_cast<const int32_t*>(ws + w.off_shared);
    a.fb_time = reinterpret_cast<uint32_t*>(ws + w.off_fb);
    a.fb_tiles = a.fb_time + (w.wgs_per_head + 1);
    a.fb_speed = reinterpret_cast<float*>(a.fb_tiles + (w.wgs_per_head + 1));
    a.fixed_split = (p->flags & SEER_ATTN_FIXED_SPLIT) ? 1 : 0;
    a.stream_only = (p->flags & SEER_ATTN_STREAM_ONLY) ? 1 : 0;
    a.stream_partials = (w.total - w.off_acc) < seer::kStreamPartialsBelow ? 1 : 0;
    a.row_blocks = seer::gqa_row_blocks((p->Hq / p->Hkv) * p->T);
    a.rows_per_block = seer::gqa_rows_per_block((p->Hq / p->Hkv) * p->T);
    a.items = reinterpret_cast<const seer::WorkItem*>(ws + w.off_items);
    a.part_ml = reinterpret_cast<float*>(ws + w.off_ml);
    a.part_acc = reinterpret_cast<float*>(ws + w.off_acc);
    a.B = p->B;
    a.T = p->T;
    a.Hq = p->Hq;
    a.Hkv = p->Hkv;
    a.G = p->Hq / p->Hkv;
    a.Dqk = p->Dqk;
    a.Dv = p->Dv;
    a.P = p->page_size;
    a.num_pages = p->num_pages;
    a.max_pages = p->max_pages_per_seq;
    a.max_items = w.max_items;
    a.wgs_per_head = w.wgs_per_head;
    a.scale_log2 = p->scale * seer::kLog2e;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // the plan depends on the shape and on ctx_len only: the layers of one step can share it
    hipError_t err = (p->flags & SEER_ATTN_REUSE_PLAN) ? hipSuccess : seer::launch_plan(a, w, stream);
    if (err != hipSuccess) return static_cast<int>(err);
    if (ev_begin && (err = hipEventRecord(ev_begin, stream)) != hipSuccess) return static_cast<int>(err);
    const bool tiled_ok = !(p->flags & SEER_ATTN_GENERAL_KERNEL);
    if (tiled_ok && seer::gqa128_supports(a)) err = seer::launch_gqa128(a, stream);
    else if (tiled_ok && seer::mla_supports(a)) err = seer::launch_mla(a, stream);
    else err = seer::launch_general(a, stream);
    if (err != hipSuccess) return static_cast<int>(err);
    if (ev_end && (err = hipEventRecord(ev_end, stream)) != hipSuccess) return static_cast<int>(err);
    err = seer::launch_combine(a, stream);
    return err == hipSuccess ? SEER_OK : static_cast<int>(err);
}

}  // namespace

extern "C" int seer_verify_attention(void* out, const void* q, const void* k_pages, const void* v_pages,
                                     const int32_t* block_table, const int32_t* ctx_len,
                                     const uint64_t* tree_mask, const seer_attn_params* p, void* workspace,
                                     size_t workspace_bytes, void* hip_stream) {
    return run_verify_attention(out, q, k_pages, v_pages, block_table, ctx_len, tree_mask, p, workspace,
                                workspace_bytes, hip_stream, nullptr, nullptr);
}

extern "C" int seer_verify_attention_timed(void* out, const void* q, const void* k_pages, const void* v_pages,
                                           const int32_t* block_table, const int32_t* ctx_len,
                                           const uint64_t* tree_mask, const seer_attn_params* p,
                                           void* workspace, size_t workspace_bytes, void* hip_stream,
                                           void* event_begin, void* event_end) {
    if (!event_begin || !event_end) return SEER_EINVAL;
    return run_verify_attention(out, q, k_pages, v_pages, block_table, ctx_len, tree_mask, p, workspace,
                                workspace_bytes, hip_stream, static_cast<hipEvent_t>(event_begin),
                                static_cast<hipEvent_t>(event_end));
}

extern "C" const char* seer_strerror(int code) {
    switch (code) {
        case SEER_OK: return "ok";
        case SEER_EINVAL: return "null pointer or non-positive size";
        case SEER_ESHAPE: return "shape outside the supported range";
        case SEER_EUNSUPPORTED: return "no kernel for these head dimensions";
        case SEER_EWORKSPACE: return "workspace missing or too small";
        case SEER_EALIGN: return "pointer not aligned as required";
        case SEER_ELIMIT: return "problem larger than this fixed-size entry point holds";
        default: break;
    }
    if (code > 0) return hipGetErrorString(static_cast<hipError_t>(code));
    return "unknown seer error";
}
