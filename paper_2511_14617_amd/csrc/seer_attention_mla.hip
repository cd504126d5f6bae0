// Tiled verify-attention partition kernel for the shared-latent (MLA, absorbed
// form) shape: all query heads of a request attend to ONE compressed KV latent
// of 576 dims per token (512 latent + 64 rope); the value of a token is the
// first 512 dims of that same vector.  Pages hold 64 tokens.
//
// This is the shape of the paper's largest rollout model (a 1 TB MoE served with
// data + expert parallelism, so each GPU sees all 128 attention heads of its own
// requests): with T = gamma + 1 verify slots a request has 128*T query rows over
// one latent stream, about 1200 flop per KV byte -- the kernel is bound by the
// matrix cores (and, on this hardware, by LDS bandwidth feeding them), not HBM.
//
// Work decomposition
//   A workgroup = 4 waves = 128 query rows (wave i owns rows 32i..32i+31) of one request
//   piece; the R = G*T rows of a request are cut into RB = ceil(R/128) row blocks, and the
//   RB workgroups that walk the same stretch of the tile line are placed on the same XCD
//   (workgroup ids are dealt round-robin to the 8 XCDs), so that one of them pulls a latent
//   tile from HBM and the others find it in that XCD's L2.
// Data flow per 32-token tile (36 KB: 32 rows of 1152 B)
//   HBM/L2 -> LDS directly (global_load_lds_dwordx4), ring of 3 stages; 16-byte chunks of a
//   row XOR-swizzled by a 3-bit function of row bits 1..3 (bit 1 of the row moves the chunk by 64
//   bytes), which spreads both read patterns below over all 64 LDS banks.
//   S^T = K . Q^T : 36 steps of v_mfma_f32_32x32x16_bf16 (M = tokens, N = rows); K operand =
//                   ds_read_b128, Q^T (32 rows x 576) lives in 144 VGPRs
//   softmax       : one query row per lane, as in the D = 128 kernel
//   O^T += V^T.P^T: 16 d-tiles x 2 steps; V^T operand from the same LDS tile through the
//                   transposing read ds_read_b64_tr_b16; O^T (32 rows x 512) = 256 accumulators
#include "seer_attention.h"
#include "seer_device.h"
#include "seer_tile.h"

namespace seer {

namespace mla {
constexpr int kDqk = 576, kDv = 512;
constexpr int kPage = 64;
constexpr int kTile = 32;
constexpr int kRowBytes = kDqk * 2;               // 1152
constexpr int kChunksPerRow = kRowBytes / 16;      // 72
constexpr int kStageBytes = kTile * kRowBytes;     // 36864
constexpr int kBlocks = kStageBytes / 1024;        // 36 one-KB wave loads per tile
constexpr int kWaves = 4;
constexpr int kRowsPerWg = 32 * kWaves;            // 128
constexpr int kStages = 3;
constexpr int kLoadsPerWave = kBlocks / kWaves;    // 9
constexpr int kKSteps = kDqk / 16;                 // 36
constexpr int kDTiles = kDv / 32;                  // 16
constexpr int kQRegSteps = 24;                     // contraction steps whose Q^T operand stays in registers
constexpr int kQLdsSteps = kKSteps - kQRegSteps;   // the remaining 12 are re-read from LDS every tile
static_assert(kTile == kPlanTile, "the plan counts work in tiles of this kernel");
static_assert(kBlocks % kWaves == 0, "every wave issues the same number of loads");

// Row r starts 1152 r bytes into the stage, i.e. at bank group (in 16-byte units) 8 (r & 1) of the 16
// that make up the 64 banks, so row parity supplies one bit of spread and the swizzle the other three.
__device__ __forceinline__ int swz(int row) { return (((row >> 1) & 1) << 2) | (((row >> 2) & 1) << 1) | ((row >> 3) & 1); }
}  // namespace mla

// 8 transposing reads (an even and an odd d-tile x {step 0 lo, step 0 hi, step 1 lo, step 1 hi}) and the
// wait for them, as one asm block (see the D = 128 kernel for why these do not go through the builtin).
// a_even / a_odd: lane address for even / odd d-tiles; OFF: byte offset of the d-tile pair.
// The token rows +8 and +24 differ from +0 and +16 in row bit 3, which the swizzle uses: they go
// through addresses of their own (a_even8 / a_odd8).
#define SEER_MLA_TR8(vr, a_even, a_even8, a_odd, a_odd8, OFF)                                              \
    asm volatile(                                                                                          \
        "ds_read_b64_tr_b16 %0, %8 offset:%12\n"                                                           \
        "ds_read_b64_tr_b16 %1, %9 offset:%13\n"                                                           \
        "ds_read_b64_tr_b16 %2, %8 offset:%14\n"                                                           \
        "ds_read_b64_tr_b16 %3, %9 offset:%15\n"                                                           \
        "ds_read_b64_tr_b16 %4, %10 offset:%12\n"                                                          \
        "ds_read_b64_tr_b16 %5, %11 offset:%13\n"                                                          \
        "ds_read_b64_tr_b16 %6, %10 offset:%14\n"                                                          \
        "ds_read_b64_tr_b16 %7, %11 offset:%15\n"                                                          \
        "s_waitcnt lgkmcnt(0)"                                                                             \
        : "=&v"(vr[0][0]), "=&v"(vr[0][1]), "=&v"(vr[0][2]), "=&v"(vr[0][3]), "=&v"(vr[1][0]), "=&v"(vr[1][1]), \
          "=&v"(vr[1][2]), "=&v"(vr[1][3])                                                                 \
        : "v"(a_even), "v"(a_even8), "v"(a_odd), "v"(a_odd8), "n"((OFF)), "n"((OFF) + 8 * mla::kRowBytes),  \
          "n"((OFF) + 16 * mla::kRowBytes), "n"((OFF) + 24 * mla::kRowBytes))

// acc += A . B with the accumulator pinned to the AGPR half of the register file.  Written as asm
// because the compiler, left to choose, keeps part of the 256 accumulators in VGPRs and then
// spills the Q^T operands; with the accumulators forced into AGPRs everything else fits in VGPRs.
// The compiler does not see an MFMA here, so the code that later reads the accumulators with
// ordinary instructions (rescale, epilogue) first idles past the MFMA pipeline depth itself
// (mfma_drain).  Dependent MFMAs on one accumulator are interlocked by the hardware.
__device__ __forceinline__ void mfma_acc(f32x16& acc, u32x4 a, u32x4 b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// The score accumulator, pinned to VGPRs (all AGPRs hold O^T).
__device__ __forceinline__ void mfma_vgpr(f32x16& acc, u32x4 a, bf16x8 b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma_drain() { asm volatile("s_nop 15\n\ts_nop 15" ::: "memory"); }

__global__ __launch_bounds__(mla::kWaves* kWave) __attribute__((amdgpu_waves_per_eu(1, 1)))
void attn_mla_kernel(AttnArgs a, int row_blocks) {
    using namespace mla;
    constexpr int NT = kWaves * kWave;
    __shared__ __attribute__((aligned(1024))) unsigned char lds[kStages * kStageBytes];
    // Q^T operands of the last kQLdsSteps contraction steps, [wave][step][lane]: 256 accumulators and all
    // 144 Q registers do not fit one wave's register file, so a third of Q^T is parked here (each lane
    // writes and re-reads only its own 16 bytes).  A separate array, so that the compiler can tell these
    // accesses apart from the tile stages that the direct-to-LDS loads write.
    __shared__ __attribute__((aligned(16))) u32x4 q_tail[kWaves][kQLdsSteps][kWave];

    const int kvh = blockIdx.y;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int ln = lane & 31;
    const int lg = lane >> 5;
    const int l16 = lane >> 4;
    const int p16 = lane & 15;

    // ---- which stretch and which row block: siblings (same stretch) share an XCD -----------
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int wg = (slot / row_blocks) * 8 + xcd;
    const int rb = slot % row_blocks;
    if (wg >= a.wgs_per_head) return;
    const int L = uniform_load(&a.header->tiles_per_wg);
    int b = uniform_load(a.wg_first + wg);
    if (b < 0) return;
    int g = L ? wg * L : uniform_load(a.tile_off + b);
    const int g_end = L ? min((wg + 1) * L, uniform_load(&a.header->total_tiles)) : uniform_load(a.tile_off + b + 1);
    bool bad_page = false;

    const unsigned char* __restrict__ kbase = static_cast<const unsigned char*>(a.k_pages);
    const size_t page_bytes = static_cast<size_t>(a.Hkv) * kPage * kRowBytes;
    const size_t head_off = static_cast<size_t>(kvh) * kPage * kRowBytes;

    // K operand: row ln, chunk 2*kk + lg; the swizzle only touches the low 3 bits of the chunk index
    int k_rd[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) k_rd[j] = ln * kRowBytes + (((2 * j + lg) ^ swz(ln)) << 4);
    // V operand through the transposing read (lane s = 4k + c4 of a 16-lane group points at token
    // row k, d columns 4c4..4c4+3 of the group's 16).  Token rows are 4lg + k (+8, +16, +24).
    const int v_k = p16 >> 2, v_c4 = p16 & 3, v_dhalf = l16 & 1;
    const int v_swz = swz(lg * 4 + v_k);          // for +0 and +16; +8 and +24 flip the swizzle's bit 0
    const int v_row0 = (lg * 4 + v_k) * kRowBytes;
    // d-tile dt: chunk = 4dt + 2dhalf + (c4 >> 1); even and odd dt differ in bit 2, which the swizzle touches
    const int v_even = v_row0 + (((v_dhalf * 2 + (v_c4 >> 1)) ^ v_swz) << 4) + (v_c4 & 1) * 8;
    const int v_odd = v_row0 + (((4 + v_dhalf * 2 + (v_c4 >> 1)) ^ v_swz) << 4) + (v_c4 & 1) * 8;
    const int v_even8 = v_row0 + (((v_dhalf * 2 + (v_c4 >> 1)) ^ v_swz ^ 1) << 4) + (v_c4 & 1) * 8;
    const int v_odd8 = v_row0 + (((4 + v_dhalf * 2 + (v_c4 >> 1)) ^ v_swz ^ 1) << 4) + (v_c4 & 1) * 8;

  for (; g < g_end; ++b) {
    const int t_lo = uniform_load(a.tile_off + b), t_hi = uniform_load(a.tile_off + b + 1);
    if (t_hi == t_lo) continue;
    const int item_idx = uniform_load(a.split_off + b) + (L ? wg - t_lo / L : 0);
    const int n = uniform_load(a.ctx_len + b);
    const int tok_begin = (g - t_lo) * kTile;
    const int tok_end = min(n, (min(g_end, t_hi) - t_lo) * kTile);
    g = t_hi;
    const int n0 = n - a.T;
    const int n_tiles = (tok_end - tok_begin + kTile - 1) / kTile;
    bare_barrier();

    // ---- this lane's query row -------------------------------------------------------------
    const int R = a.G * a.T;
    const int r = rb * kRowsPerWg + wave * 32 + ln;
    const bool row_ok = r < R;
    const int t = row_ok ? r / a.G : 0;
    const int hq = kvh * a.G + (row_ok ? r - t * a.G : 0);
    uint64_t word = 0;
    if (row_ok) {
        word = a.tree_mask ? a.tree_mask[static_cast<size_t>(b) * a.T + t]
                           : (t >= 63 ? ~0ull : ((1ull << (t + 1)) - 1));
        if (a.T < 64) word &= (1ull << a.T) - 1;
    }
    bf16x8 qreg[kQRegSteps];
    {
        const u32x4* qp = reinterpret_cast<const u32x4*>(
            static_cast<const uint16_t*>(a.q) + ((static_cast<size_t>(b) * a.T + t) * a.Hq + hq) * kDqk + lg * 8);
#pragma unroll
        for (int kk = 0; kk < kQLdsSteps; ++kk) {
            u32x4 v = u32x4{0u, 0u, 0u, 0u};
            if (row_ok) v = qp[(kQRegSteps + kk) * 2];
            q_tail[wave][kk][lane] = v;
        }
        u32x4 qv[kQRegSteps];
#pragma unroll
        for (int kk = 0; kk < kQRegSteps; ++kk) {
            qv[kk] = u32x4{0u, 0u, 0u, 0u};
            if (row_ok) qv[kk] = qp[kk * 2];
        }
#pragma unroll
        for (int kk = 0; kk < kQRegSteps; ++kk) {   // pin the arrival of these loads before the tile loop
            asm volatile("" : "+v"(qv[kk]));
            qreg[kk] = as_bf16x8(qv[kk]);
        }
        uint32_t w_lo = static_cast<uint32_t>(word), w_hi = static_cast<uint32_t>(word >> 32);
        asm volatile("" : "+v"(w_lo), "+v"(w_hi));
        word = (static_cast<uint64_t>(w_hi) << 32) | w_lo;
    }

    f32x16 acc[kDTiles];
#pragma unroll
    for (int dt = 0; dt < kDTiles; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[dt][i] = 0.f;
    float m_run = kNegInf, l_run = 0.f;

    // ---- page ids, 64 at a time, handed out by v_readlane ------------------------------------
    const int32_t* __restrict__ table = a.block_table + static_cast<size_t>(b) * a.max_pages;
    int cache_base = -0x40000000;
    int pg_cache = 0;
    const int last_page = (n - 1) / kPage;
    auto page_offset = [&](int logical_page) __attribute__((always_inline)) -> size_t {
        if (logical_page < cache_base || logical_page >= cache_base + kWave) {
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
    auto issue_tile = [&](int tile) __attribute__((always_inline)) {
        const int tb = tok_begin + tile * kTile;
        const unsigned char* src = kbase + page_offset(tb / kPage) + static_cast<size_t>(tb % kPage) * kRowBytes;
        unsigned char* stage = lds + (tile % kStages) * kStageBytes;
#pragma unroll
        for (int i = 0; i < kLoadsPerWave; ++i) {
            // LDS slot c = block*64 + lane holds chunk (c % 72) ^ swz(row) of row c / 72 (recomputed per
            // load: nine more live registers per lane would not fit beside Q^T and the accumulators)
            const unsigned c = static_cast<unsigned>((wave + i * kWaves) * 64 + lane);
            const unsigned row = c / kChunksPerRow, pos = c - row * kChunksPerRow;
            const int goff = static_cast<int>(row * kRowBytes + ((pos ^ static_cast<unsigned>(swz(static_cast<int>(row)))) << 4));
            __builtin_amdgcn_global_load_lds((const SEER_AS1 void*)(src + goff),
                                             (SEER_AS3 void*)(stage + (wave + i * kWaves) * 1024), 16, 0, 0);
        }
    };

#pragma unroll
    for (int s = 0; s < kStages - 1; ++s)
        if (s < n_tiles) issue_tile(s);

    for (int tile = 0; tile < n_tiles; ++tile) {
        if (tile + 1 < n_tiles) wait_vmcnt<kLoadsPerWave>(); else wait_vmcnt<0>();
        bare_barrier();
        if (tile + kStages - 1 < n_tiles) issue_tile(tile + kStages - 1);

        const int stage_off = (tile % kStages) * kStageBytes;
        const unsigned char* kl = lds + stage_off;
        const int tb = tok_begin + tile * kTile;

        if (tb + kTile > n) {
            // ragged last tile: clear the rows past the end (0 * NaN must not reach the output)
            const int first_bad = n - tb;
            for (int c = tid; c < kTile * kChunksPerRow; c += NT)
                if (c / kChunksPerRow >= first_bad)
                    *reinterpret_cast<u32x4*>(const_cast<unsigned char*>(kl) + c * 16) = u32x4{0u, 0u, 0u, 0u};
            __builtin_amdgcn_s_waitcnt(0xc07f);
            bare_barrier();
        }

        // S^T[token][row] = sum_d K[token][d] * Q[row][d]
        f32x16 s;
#pragma unroll
        for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
        for (int kk = 0; kk < kKSteps; ++kk) {
            const u32x4 kv = *reinterpret_cast<const u32x4*>(kl + k_rd[kk & 3] + (kk >> 2) * 128);
            const bf16x8 qb = kk < kQRegSteps ? qreg[kk < kQRegSteps ? kk : 0]
                                              : as_bf16x8(q_tail[wave][kk < kQRegSteps ? 0 : kk - kQRegSteps][lane]);
            mfma_vgpr(s, kv, qb);
        }
        mfma_drain();   // the vector ALU reads s next, and the compiler does not know an MFMA wrote it

        float mx = kNegInf;
        if (tb + kTile > n0) {
            const int rel = tb - n0;
            uint32_t vis = rel >= 0 ? static_cast<uint32_t>(word >> rel)
                                    : (static_cast<uint32_t>(word << (-rel)) | ((1u << (-rel)) - 1u));
            vis >>= lg * 4;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const bool on = (vis >> ((i >> 2) * 8 + (i & 3))) & 1u;
                const float v = on ? s[i] * a.scale_log2 : kNegInf;
                s[i] = v;
                mx = fmaxf(mx, v);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                s[i] *= a.scale_log2;
                mx = fmaxf(mx, s[i]);
            }
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
        // Lazy reference: m_run is the exponent reference of (l, acc), not necessarily the true
        // maximum; it moves only when the tile maximum exceeds it by more than 2^8, so p stays
        // below 256 (bf16 and fp32 have the range) and the 256-register rescale is rare.
        const bool move_ref = mx > m_run + 8.f;
        const float m_new = move_ref ? mx : m_run;
        const float m_use = (m_new == kNegInf) ? 0.f : m_new;
        const float alpha = move_ref ? fast_exp2(m_run - m_use) : 1.f;
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
            mfma_drain();
            // one d-tile at a time through VGPRs (the empty asm statements keep the compiler from
            // pulling all 256 accumulators out of the AGPRs at once, which would spill)
#pragma unroll
            for (int dt = 0; dt < kDTiles; ++dt) {
                f32x16 tmp = acc[dt];
                asm volatile("" : "+v"(tmp));
#pragma unroll
                for (int i = 0; i < 16; ++i) tmp[i] *= alpha;
                acc[dt] = tmp;
                asm volatile("" : "+a"(acc[dt]));
            }
        }

        // O^T[d][row] += sum_token V[token][d] * P[row][token], V = first 512 dims of the latent
        const u32x4 pb0 = {pk[0], pk[1], pk[2], pk[3]};
        const u32x4 pb1 = {pk[4], pk[5], pk[6], pk[7]};
        const int a_even = stage_off + v_even, a_odd = stage_off + v_odd;
        const int a_even8 = stage_off + v_even8, a_odd8 = stage_off + v_odd8;
#define SEER_MLA_PV(G2)                                                                                   \
        {                                                                                                 \
            u32x2 vr[2][4];   /* [even | odd d-tile of the pair][step*2 + (tokens +0..3 | +8..11)] */      \
            SEER_MLA_TR8(vr, a_even, a_even8, a_odd, a_odd8, (G2) * 128);                                 \
            const u32x4 e0 = {vr[0][0][0], vr[0][0][1], vr[0][1][0], vr[0][1][1]};                        \
            const u32x4 o0 = {vr[1][0][0], vr[1][0][1], vr[1][1][0], vr[1][1][1]};                        \
            const u32x4 e1 = {vr[0][2][0], vr[0][2][1], vr[0][3][0], vr[0][3][1]};                        \
            const u32x4 o1 = {vr[1][2][0], vr[1][2][1], vr[1][3][0], vr[1][3][1]};                        \
            mfma_acc(acc[(G2) * 2], e0, pb0);                                                             \
            mfma_acc(acc[(G2) * 2 + 1], o0, pb0);                                                         \
            mfma_acc(acc[(G2) * 2], e1, pb1);                                                             \
            mfma_acc(acc[(G2) * 2 + 1], o1, pb1);                                                         \
        }
        SEER_MLA_PV(0)
        SEER_MLA_PV(1)
        SEER_MLA_PV(2)
        SEER_MLA_PV(3)
        SEER_MLA_PV(4)
        SEER_MLA_PV(5)
        SEER_MLA_PV(6)
        SEER_MLA_PV(7)
#undef SEER_MLA_PV
    }

    // ---- partial result ------------------------------------------------------------------------
    mfma_drain();
    const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
    if (row_ok) {
        const size_t prow = (static_cast<size_t>(item_idx) * a.T + t) * a.Hq + hq;
        if (lg == 0) {
            a.part_ml[2 * prow] = m_run;
            a.part_ml[2 * prow + 1] = l_tot;
        }
        float* __restrict__ po = a.part_acc + prow * kDv;
#pragma unroll
        for (int dt = 0; dt < kDTiles; ++dt)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const f32x4 v = {acc[dt][i4 * 4], acc[dt][i4 * 4 + 1], acc[dt][i4 * 4 + 2], acc[dt][i4 * 4 + 3]};
                *reinterpret_cast<f32x4*>(po + dt * 32 + i4 * 8 + lg * 4) = v;
            }
    }
  }
    if (bad_page && lane == 0) atomicOr(&a.header->status, 2u);
}

bool mla_supports(const AttnArgs& a) {
    return a.Dqk == mla::kDqk && a.Dv == mla::kDv && a.P == mla::kPage && a.v_pages == nullptr && a.Hkv <= 65535;
}

hipError_t launch_mla(const AttnArgs& a, hipStream_t stream) {
    const int row_blocks = (a.G * a.T + mla::kRowsPerWg - 1) / mla::kRowsPerWg;
    const unsigned groups = (a.wgs_per_head + 7) / 8;
    const dim3 grid(8u * groups * row_blocks, a.Hkv);
    hipLaunchKernelGGL(attn_mla_kernel, grid, dim3(mla::kWaves * kWave), 0, stream, a, row_blocks);
    return hipGetLastError();
}

}  // namespace seer
