// Tiled verify-attention partition kernel for grouped-query heads with
// D = 128 and 16-token pages (the shape of the paper's dense 8B- to 72B-class
// rollout models), on the gfx950 matrix cores.
//
// Why matrix cores although decoding is "memory bound": verification reads a
// KV page once for ALL T = gamma + 1 slots and all G heads of the group
// (Section 2.2: verifying n tokens in parallel beats n serial steps because
// memory is touched once).  That makes every 512 bytes of K+V feed G*T query
// rows (36 to 132 in the workloads here), i.e. 36-132 flop per byte: at HBM
// speed this is several hundred TFLOP/s, beyond the vector ALUs, so scores and
// P.V are MFMA contractions; everything else in this kernel exists to keep
// HBM streaming.
//
// Work decomposition
//   grid = (W, Hkv); workgroup (w, kv head) streams stretch w of the head's tile line
//   (see the plan in seer_attention.h) and, for each request the stretch touches,
//   handles all R = G*T query rows of that head.  Wave i owns rows [32i, 32i+32);
//   NW = ceil(R/32) waves per workgroup.
//
// Data flow per 32-token tile (two pages)
//   HBM -> VGPR (16-byte lanes, whole 4 KB page-head blocks, coalesced)
//       -> LDS  K as [token][d] (row pitch 272 B: conflict-free 16-byte reads)
//               V as [token/4][d][token%4] (4x8 bf16 blocks transposed in registers
//                 on the way in, so the P.V operand is two 8-byte LDS reads)
//   S^T = K . Q^T    v_mfma_f32_32x32x16_bf16, M = tokens, N = rows, 8 steps over d
//   softmax          each lane owns ONE query row (N index = lane % 32) and 16 of the
//                    tile's 32 tokens, so max/sum are in-lane plus one cross-half
//                    exchange; the C registers of S^T are, as they stand, the
//                    B operand of the next product (no shuffle, no LDS round trip)
//   O^T += V^T . P^T M = d (4 tiles of 32), N = rows, 2 steps over the tokens
//   Q^T (the B operand of the first product) stays in 32 VGPRs for the whole
//   partition; K/V of tile i+1 are in flight from HBM while tile i is computed.
#include <type_traits>

#include "seer_attention.h"
#include "seer_device.h"

namespace seer {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kD = 128;          // head dim
constexpr int kPage = 16;        // tokens per page
constexpr int kTile = 32;        // tokens per tile
constexpr int kKPitch = 272;     // bytes per K row in LDS (256 + 16)
constexpr int kKBytes = kTile * kKPitch;         // 8704
constexpr int kVQuadPitch = kD * 8 + 8 * 16;     // 1152: [d][4 tokens], 16 bytes of padding every 16 d
constexpr int kVBytes = (kTile / 4) * kVQuadPitch;   // 9216
// byte offset of (d, token%4 = 0) inside a token quad of V: the padding makes both the 64-byte
// row-block writes of staging and the 8-byte operand reads hit 32 distinct banks
__device__ __forceinline__ int v_quad_offset(int d) { return d * 8 + (d >> 4) * 16; }
constexpr int kBufBytes = kKBytes + kVBytes;
static_assert(kTile == kPlanTile, "the plan counts work in tiles of this kernel");

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
    typedef __attribute__((ext_vector_type(2))) float f32x2;
    f32x2 v = {lo, hi};
    bf16x2 r = __builtin_convertvector(v, bf16x2);   // round-to-nearest-even (v_cvt_pk_bf16_f32)
    return __builtin_bit_cast(uint32_t, r);
}

template <int NW>
__global__ __launch_bounds__(NW * kWave) __attribute__((amdgpu_waves_per_eu(NW == 1 ? 1 : 2, 2)))
void attn_gqa128_kernel(AttnArgs a) {
    constexpr int NT = NW * kWave;
    constexpr int K_CHUNKS = kTile * kD * 2 / 16;      // 512 16-byte pieces of K per tile
    constexpr int K_PER = (K_CHUNKS + NT - 1) / NT;
    constexpr int V_UNITS = (kTile / 4) * (kD / 8);    // 128 (token quad, 8-wide d chunk) units
    constexpr int V_PER = (V_UNITS + NT - 1) / NT;

    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * kBufBytes];

    const int kvh = blockIdx.y;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int ln = lane & 31;      // N / M index inside a 32-wide tile
    const int lg = lane >> 5;      // which half of the contraction index this lane feeds

    // ---- this workgroup's stretch of the per-head tile line ---------------------------
    const int wg = blockIdx.x;
    const int L = a.header->tiles_per_wg;          // 0: one workgroup per request
    int b = a.wg_first[wg];
    if (b < 0) return;                             // idle stretch (uniform for the workgroup)
    int g = L ? wg * L : a.tile_off[b];
    const int g_end = L ? min((wg + 1) * L, a.header->total_tiles) : a.tile_off[b + 1];
    bool bad_page = false;

  for (; g < g_end; ++b) {
    const int t_lo = a.tile_off[b], t_hi = a.tile_off[b + 1];
    if (t_hi == t_lo) continue;                    // request without tiles (flagged ctx_len)
    const int item_idx = a.split_off[b] + (L ? wg - t_lo / L : 0);
    WorkItem item;
    item.b = b;
    item.begin = (g - t_lo) * kTile;
    const int n = a.ctx_len[b];
    item.end = min(n, (min(g_end, t_hi) - t_lo) * kTile);
    g = t_hi;
    const int n0 = n - a.T;
    __syncthreads();                               // the previous piece is done with the LDS buffers

    // ---- this lane's query row -------------------------------------------------
    const int R = a.G * a.T;
    const int r = wave * 32 + ln;
    const bool row_ok = r < R;
    const int t = row_ok ? r / a.G : 0;
    const int hq = kvh * a.G + (row_ok ? r - t * a.G : 0);
    uint64_t word = 0;
    if (row_ok) word = a.tree_mask ? a.tree_mask[static_cast<size_t>(b) * a.T + t]
                                   : (t >= 63 ? ~0ull : ((1ull << (t + 1)) - 1));
    bf16x8 qreg[8];
    {
        const u32x4* qp = reinterpret_cast<const u32x4*>(
            static_cast<const uint16_t*>(a.q) + ((static_cast<size_t>(b) * a.T + t) * a.Hq + hq) * kD + lg * 8);
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (row_ok) v = qp[kk * 2];      // d = kk*16 + lg*8 .. +7
            qreg[kk] = as_bf16x8(v);
        }
    }

    f32x16 acc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[dt][i] = 0.f;
    float m_run = kNegInf, l_run = 0.f;

    // ---- tile streaming ----------------------------------------------------------
    const int32_t* __restrict__ table = a.block_table + static_cast<size_t>(b) * a.max_pages;
    const unsigned char* __restrict__ kbase = static_cast<const unsigned char*>(a.k_pages);
    const unsigned char* __restrict__ vbase = static_cast<const unsigned char*>(a.v_pages);
    const size_t page_bytes = static_cast<size_t>(a.Hkv) * kPage * kD * 2;   // one page, all kv heads
    const size_t head_off = static_cast<size_t>(kvh) * kPage * kD * 2;
    const int n_tiles = (item.end - item.begin + kTile - 1) / kTile;

    // Page ids are fetched 64 at a time (lane l holds logical page cache_base + l) and handed
    // out with v_readlane: one vector load per 32 tiles instead of a dependent table read --
    // and a full drain of the loads in flight -- in front of every tile.
    int cache_base = -0x40000000;
    int pg_cache = 0;
    const int last_page = (n - 1) / kPage;
    auto page_offset = [&](int logical_page) -> size_t {
        if (logical_page < cache_base || logical_page >= cache_base + kWave) {   // uniform
            cache_base = logical_page;
            const int idx = cache_base + lane;
            int pg = table[min(idx, a.max_pages - 1)];
            if (pg < 0 || pg >= a.num_pages) {
                if (idx <= last_page) bad_page = true;
                pg = min(max(pg, 0), a.num_pages - 1);
            }
            pg_cache = pg;
        }
        const int pg = __builtin_amdgcn_readlane(pg_cache, __builtin_amdgcn_readfirstlane(logical_page - cache_base));
        return static_cast<size_t>(pg) * page_bytes + head_off;
    };

    // two tiles are in flight from HBM per workgroup (register sets 0 and 1)
    u32x4 kst[2][K_PER];        // K pieces in flight
    u32x4 vst[2][V_PER][4];     // V: 4 tokens x 16 bytes per unit

    auto issue_loads = [&](int tile, auto set_tag) {
        constexpr int set = decltype(set_tag)::value;
        const int tb = item.begin + tile * kTile;
        const size_t p0 = page_offset(tb / kPage);
        const size_t p1 = page_offset(tb / kPage + 1);
#pragma unroll
        for (int j = 0; j < K_PER; ++j) {
            const int u = tid + j * NT;
            if (K_CHUNKS % NT == 0 || u < K_CHUNKS) {
                const size_t off = (u < 256 ? p0 : p1) + static_cast<size_t>(u & 255) * 16;
                kst[set][j] = *reinterpret_cast<const u32x4*>(kbase + off);
            }
        }
#pragma unroll
        for (int j = 0; j < V_PER; ++j) {
            const int u = tid + j * NT;
            if (V_UNITS % NT == 0 || u < V_UNITS) {
                const int quad = u >> 4, c = u & 15;
                const size_t off = (quad < 4 ? p0 : p1) + static_cast<size_t>((quad & 3) * 4) * 256 + c * 16;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    vst[set][j][e] = *reinterpret_cast<const u32x4*>(vbase + off + e * 256);
                }
            }
        }
    };

    auto stage_to_lds = [&](int tile, auto set_tag) {
        constexpr int set = decltype(set_tag)::value;
        const int tb = item.begin + tile * kTile;
        const bool ragged = tb + kTile > n;     // only the last tile of a request
        unsigned char* kl = lds + set * kBufBytes;
        unsigned char* vl = kl + kKBytes;
#pragma unroll
        for (int j = 0; j < K_PER; ++j) {
            const int u = tid + j * NT;
            if (K_CHUNKS % NT == 0 || u < K_CHUNKS)
                *reinterpret_cast<u32x4*>(kl + (u >> 4) * kKPitch + (u & 15) * 16) = kst[set][j];
        }
#pragma unroll
        for (int j = 0; j < V_PER; ++j) {
            const int u = tid + j * NT;
            if (V_UNITS % NT == 0 || u < V_UNITS) {
                const int quad = u >> 4, c = u & 15;
                unsigned char* dst = vl + quad * kVQuadPitch + v_quad_offset(c * 8);
                if (ragged) {
                    // values of slots past the end of the context are never used: zero them so
                    // that whatever the page holds there (NaN included) cannot reach 0 * x.
                    // (Done here, where the data is consumed, not where the loads are issued.)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (tb + quad * 4 + e >= n) vst[set][j][e] = u32x4{0u, 0u, 0u, 0u};
                }
                // 4 tokens x 8 d  ->  8 d x 4 tokens
#pragma unroll
                for (int e = 0; e < 4; ++e) {   // dword e of each token row holds d = 2e, 2e+1
                    const uint32_t t0 = vst[set][j][0][e], t1 = vst[set][j][1][e], t2 = vst[set][j][2][e],
                                   t3 = vst[set][j][3][e];
                    u32x4 o;
                    o[0] = (t0 & 0xffffu) | (t1 << 16);          // d = 2e   : tokens 0,1
                    o[1] = (t2 & 0xffffu) | (t3 << 16);          //            tokens 2,3
                    o[2] = (t0 >> 16) | (t1 & 0xffff0000u);      // d = 2e+1 : tokens 0,1
                    o[3] = (t2 >> 16) | (t3 & 0xffff0000u);      //            tokens 2,3
                    *reinterpret_cast<u32x4*>(dst + e * 16) = o;
                }
            }
        }
    };

    auto tile_step = [&](int tile, auto set_tag) {
        constexpr int buf = decltype(set_tag)::value;
        stage_to_lds(tile, set_tag);
        __syncthreads();
        if (tile + 2 < n_tiles) issue_loads(tile + 2, set_tag);

        const unsigned char* kl = lds + buf * kBufBytes;
        const unsigned char* vl = kl + kKBytes;
        const int tb = item.begin + tile * kTile;

        // S^T[token][row] = sum_d K[token][d] * Q[row][d]
        f32x16 s;
#pragma unroll
        for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            const u32x4 kv = *reinterpret_cast<const u32x4*>(kl + ln * kKPitch + kk * 32 + lg * 16);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kv), qreg[kk], s, 0, 0, 0);
        }

        // register i of s holds token  (i/4)*8 + lg*4 + i%4  of the tile, for this lane's row
        const bool need_mask = (tb + kTile > n0);
        float mx = kNegInf;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            float v = s[i] * a.scale_log2;
            if (need_mask) {
                const int j = tb + (i >> 2) * 8 + lg * 4 + (i & 3);
                const bool vis = (j < n0) || (j < n && ((word >> (j - n0)) & 1ull));
                v = vis ? v : kNegInf;
            }
            s[i] = v;
            mx = fmaxf(mx, v);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
        const float m_new = fmaxf(m_run, mx);
        const float m_use = (m_new == kNegInf) ? 0.f : m_new;   // nothing visible yet: keep exp2 finite
        const float alpha = fast_exp2(m_run - m_use);
        m_run = m_new;
        float psum = 0.f;
        uint32_t pk[8];
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
            const float p0 = fast_exp2(s[i] - m_use);
            const float p1 = fast_exp2(s[i + 1] - m_use);
            psum += p0 + p1;
            pk[i >> 1] = cvt_pk_bf16(p0, p1);
        }
        l_run = l_run * alpha + psum;
        if (__any(alpha != 1.f)) {
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[dt][i] *= alpha;
        }

        // O^T[d][row] += sum_token V[token][d] * P[row][token]
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const bf16x8 pb = as_bf16x8(u32x4{pk[ks * 4], pk[ks * 4 + 1], pk[ks * 4 + 2], pk[ks * 4 + 3]});
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) {
                const int d = dt * 32 + ln;
                const u32x2 lo = *reinterpret_cast<const u32x2*>(vl + (ks * 4 + lg) * kVQuadPitch + v_quad_offset(d));
                const u32x2 hi = *reinterpret_cast<const u32x2*>(vl + (ks * 4 + 2 + lg) * kVQuadPitch + v_quad_offset(d));
                const bf16x8 va = as_bf16x8(u32x4{lo[0], lo[1], hi[0], hi[1]});
                acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb, acc[dt], 0, 0, 0);
            }
        }
    };   // tile_step

    using Set0 = std::integral_constant<int, 0>;
    using Set1 = std::integral_constant<int, 1>;
    if (n_tiles > 0) issue_loads(0, Set0{});
    if (n_tiles > 1) issue_loads(1, Set1{});
    for (int tile = 0; tile < n_tiles; tile += 2) {
        tile_step(tile, Set0{});
        if (tile + 1 < n_tiles) tile_step(tile + 1, Set1{});
    }

    // ---- partial result: (running max, sum, unnormalised O) per row -------------------
    const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
    if (row_ok) {
        const size_t prow = (static_cast<size_t>(item_idx) * a.T + t) * a.Hq + hq;
        if (lg == 0) {
            a.part_ml[2 * prow] = m_run;
            a.part_ml[2 * prow + 1] = l_tot;
        }
        float* __restrict__ po = a.part_acc + prow * kD;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const f32x4 v = {acc[dt][i4 * 4], acc[dt][i4 * 4 + 1], acc[dt][i4 * 4 + 2], acc[dt][i4 * 4 + 3]};
                *reinterpret_cast<f32x4*>(po + dt * 32 + i4 * 8 + lg * 4) = v;
            }
    }
  }  // pieces of the stretch
    if (bad_page && lane == 0) atomicOr(&a.header->status, 2u);
}

bool gqa128_supports(const AttnArgs& a) {
    return a.Dqk == kD && a.Dv == kD && a.P == kPage && a.v_pages != nullptr && a.G * a.T <= 8 * 32 &&
           a.Hkv <= 65535;
}

hipError_t launch_gqa128(const AttnArgs& a, hipStream_t stream) {
    const int R = a.G * a.T;
    const int nw = (R + 31) / 32;
    const dim3 grid(a.wgs_per_head, a.Hkv);
    switch (nw) {
#define SEER_GQA_CASE(NW_)                                                                               \
    case NW_:                                                                                            \
        hipLaunchKernelGGL((attn_gqa128_kernel<NW_>), grid, dim3(NW_ * kWave), 0, stream, a);            \
        break;
        SEER_GQA_CASE(1)
        SEER_GQA_CASE(2)
        SEER_GQA_CASE(3)
        SEER_GQA_CASE(4)
        SEER_GQA_CASE(5)
        SEER_GQA_CASE(6)
        SEER_GQA_CASE(7)
        SEER_GQA_CASE(8)
#undef SEER_GQA_CASE
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace seer
