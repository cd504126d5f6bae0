// Tiled verify-attention partition kernel for the shared-latent (MLA, absorbed
// form) shape: all query heads of a request attend to ONE compressed KV latent
// of 576 dims per token (512 latent + 64 rope); the value of a token is the
// first 512 dims of that same vector.  Pages hold 32 tokens or a larger power of two (64 in the workload).
//
// This is the shape of the paper's largest rollout model (a 1 TB MoE served with
// data + expert parallelism, so each GPU sees all 128 attention heads of its own
// requests): with T = gamma + 1 verify slots a request has 128*T query rows over
// one latent stream, about 1200 flop per KV byte -- the kernel is bound by the
// matrix cores and by what the one wave per SIMD issues between its MFMAs (nothing else feeds the
// SIMD's matrix core while that wave requests a tile load or awaits an operand), not by HBM and not by
// LDS bandwidth (counters: the LDS data path is busy a third of the time, the matrix cores 57 % of it).
//
// Work decomposition
//   A workgroup = 4 waves = 128 query rows (wave i owns rows 32i..32i+31) of one request
//   piece; the R = G*T rows of a request are cut into RB = ceil(R/128) row blocks, and the
//   RB workgroups that walk the same stretch of the tile line are placed on the same XCD
//   (workgroup ids are dealt round-robin to the 8 XCDs), so that one of them pulls a latent
//   tile from HBM and the others find it in that XCD's L2.
// Data flow per 32-token tile (36 KB: 32 rows of 1152 B)
//   HBM/L2 -> LDS directly (buffer_load_dwordx4 ... lds, requested inside the score phase), ring of 3 stages; 16-byte chunks of a
//   row XOR-swizzled by a 3-bit function of row bits 1..3 (bit 1 of the row moves the chunk by 64
//   bytes), which spreads both read patterns below over all 64 LDS banks.
//   S^T = K . Q^T : 36 steps of v_mfma_f32_32x32x16_bf16 (M = tokens, N = rows); K operand =
//                   ds_read_b128; Q^T (32 rows x 576 = 144 registers' worth per lane) is held in VGPRs for 24 of
//                   the 36 steps, the other 12 are parked in LDS and re-read every tile (the 256 output
//                   accumulators take the other half of the register file)
//   softmax       : one query row per lane, as in the D = 128 kernel
//   O^T += V^T.P^T: 16 d-tiles x 2 steps; V^T operand from the same LDS tile through the
//                   transposing read ds_read_b64_tr_b16; O^T (32 rows x 512) = 256 accumulators
#include <type_traits>
#include <utility>

#include "seer_attention.h"
#include "seer_device.h"
#include "seer_tile.h"

namespace seer {

namespace mla {
constexpr int kDqk = 576, kDv = 512;
constexpr int kMinPage = 32;                       // pages of 32 tokens or a larger power of two: a tile lies inside one page
constexpr int kTile = 32;
constexpr int kRowBytes = kDqk * 2;               // 1152
constexpr int kChunksPerRow = kRowBytes / 16;      // 72
constexpr int kStageBytes = kTile * kRowBytes;     // 36864
constexpr int kBlocks = kStageBytes / 1024;        // 36 one-KB wave loads per tile
constexpr int kWaves = 4;
constexpr int kRowsPerWg = 32 * kWaves;            // 128
constexpr int kStages = 3;                        // tile u (K operand), tile u-1 (V operand), one in flight
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

// LDS byte address of an object in LDS, for the address operands of the asm blocks below.
template <typename T>
__device__ __forceinline__ int lds_addr(T* p) {
    return static_cast<int>(reinterpret_cast<uintptr_t>((SEER_AS3 void*)(p)));
}

// Operand reads whose issue and completion are separated by hand (LDS returns in order, so
// "s_waitcnt lgkmcnt(N)" with N = the reads issued after a group means that group has arrived).
// The issuing block names the destination registers as outputs although they are only written
// when the read returns; the matching wait block takes them as read-write operands, so every use
// of the data is ordered after the wait.  They do not go through the builtins: the compiler puts a
// vmcnt(0) in front of those, because it cannot tell the reads apart from the direct-to-LDS loads
// still in flight.
//
// one read, one wait
#define SEER_MLA_READ128(dst, addr, OFF) \
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(dst) : "v"(addr), "n"(OFF))
#define SEER_MLA_READ_TR2(dst, addr_lo, addr_hi, OFF_LO, OFF_HI)                                           \
    asm volatile("ds_read_b64_tr_b16 %0, %2 offset:%4\n"                                                   \
                 "ds_read_b64_tr_b16 %1, %3 offset:%5"                                                     \
                 : "=&v"(dst[0]), "=&v"(dst[1])                                                            \
                 : "v"(addr_lo), "v"(addr_hi), "n"(OFF_LO), "n"(OFF_HI))
template <int N>
__device__ __forceinline__ void wait_lgkm() {
    static_assert(N >= 0 && N < 16, "lgkmcnt is a 4-bit counter");
    // (through the builtin: an instruction the compiler knows between two asm MFMAs on one accumulator keeps it from
    // padding them with a wait state of its own; vmcnt and expcnt fields at their maxima = no wait on those)
    __builtin_amdgcn_s_waitcnt(0xc07f | (N << 8));
}
#define SEER_MLA_FENCE() __builtin_amdgcn_sched_barrier(0)
// Keeps the computation of x at the place where it is written (see the D = 128 kernel).
#define SEER_MLA_PIN(x) asm volatile("" : "+v"(x))

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
__device__ __forceinline__ void mfma_vgpr(f32x16& acc, u32x4 a, u32x4 b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}
// ... starting from zero
__device__ __forceinline__ void mfma_vgpr_first(f32x16& acc, u32x4 a, u32x4 b) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma_drain() { asm volatile("s_nop 15\n\ts_nop 15" ::: "memory"); }

namespace mla {

template <typename F, int... I>
__device__ __forceinline__ void for_each_index(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}

// max over the two lanes that share a query row (lane and lane ^ 32): see the D = 128 kernel
__device__ __forceinline__ float max_across_halves(float x) {
    float a = x, b = x;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    return fmaxf(a, b);
}

// A wave issues in order, and an MFMA holds the matrix core for 32 cycles: whatever else a step has
// to issue (operand reads from LDS, the softmax arithmetic) only runs in the shadow of the MFMAs
// if it sits BETWEEN them, one MFMA at a time.  Both phases below are written that way: after
// every MFMA come the one or two LDS reads that feed an MFMA a fixed distance ahead, and a slice
// of vector-ALU work.

constexpr int kKAhead = 8;    // the K operand of score step kk is read kKAhead MFMAs before it is used
constexpr int kQAhead = 4;    // ... the parked Q^T operands kQAhead MFMAs before
constexpr int kVAhead = 6;    // the V^T operand of a P.V MFMA (two transposing reads) kVAhead MFMAs before
constexpr int kLoadFirst = 1, kLoadEvery = 4;   // load i of the next tile goes behind score MFMA kLoadFirst + i kLoadEvery
static_assert(kLoadFirst + (kLoadsPerWave - 1) * kLoadEvery < kKSteps, "all loads of a tile fit in one score phase");

// LDS reads outstanding behind the operand(s) of score step kk at the point where that step waits,
// from the order in which phase_a issues them
// (with V_AHEAD, the last kVAhead score steps are each followed by the two transposing reads of one of the first
// kVAhead P.V MFMAs of the phase that comes next)
constexpr int kVFirst = kKSteps - kVAhead;
constexpr int qk_wait_count(int kk, bool v_ahead) {
    int seq = 0, pos_k[kKSteps] = {}, pos_q[kKSteps] = {}, before[kKSteps] = {};
    for (int i = 0; i < kKAhead; ++i) pos_k[i] = seq++;
    for (int m = 0; m < kKSteps; ++m) {
        before[m] = seq;
        if (m + kKAhead < kKSteps) pos_k[m + kKAhead] = seq++;
        if (m + kQAhead >= kQRegSteps && m + kQAhead < kKSteps) pos_q[m + kQAhead] = seq++;
        if (v_ahead && m >= kVFirst) seq += 2;
    }
    int need = pos_k[kk];
    if (kk >= kQRegSteps && pos_q[kk] > need) need = pos_q[kk];
    return before[kk] - 1 - need;
}
static_assert(kQRegSteps >= kQAhead && qk_wait_count(0, false) == kKAhead - 1 && qk_wait_count(kKSteps - 1, false) == 0, "");
static_assert(qk_wait_count(kKSteps - 1, true) < 16, "lgkmcnt is a 4-bit counter");

// The V^T operand of P.V MFMA m (see phase_b) : two transposing reads into ring slot m % kVAhead.
template <int m>
__device__ __forceinline__ void v_read(u32x2 (&vr)[kVAhead][2], int a_even, int a_even8, int a_odd, int a_odd8) {
    constexpr int G2 = m >> 2, w = m & 3;
    constexpr int off_lo = G2 * 128 + (w >= 2 ? 16 : 0) * kRowBytes, off_hi = off_lo + 8 * kRowBytes;
    if constexpr (w & 1) SEER_MLA_READ_TR2(vr[m % kVAhead], a_odd, a_odd8, off_lo, off_hi);
    else SEER_MLA_READ_TR2(vr[m % kVAhead], a_even, a_even8, off_lo, off_hi);
}

// Phase A of a pipeline step: the scores of tile u (36 MFMAs into s_new) with, in their shadow, the
// probabilities of tile u-1 (s_old -> pk, l_run; the exponent reference m_use and the factor alpha of that
// tile were set during the phase B before).  ka: LDS addresses of this lane's K
// operand chunks for contraction steps 0..3 of the tile (steps 4g + j are 128 g bytes further);
// qt: LDS address of this lane's parked Q^T operands.  s_old must already carry -inf in masked slots.
// With DO_SM, the V^T operands of the first kVAhead P.V MFMAs of tile u-1 (addresses va) are requested behind the
// last score MFMAs, so that phase B starts without waiting for LDS.
// load(i): request load i of the next tile; extra(kk): other arithmetic for the shadow of score MFMA kk (no LDS traffic;
// it may write va before step kVFirst).
template <bool DO_QK, bool DO_SM, typename LOAD, typename EXTRA>
__device__ __forceinline__ void phase_a(const int (&ka)[4], int qt, const u32x4 (&qreg)[kQRegSteps], f32x16& s_new,
                                        f32x16& s_old, uint32_t (&pk)[8], float m_use, float& l_run, float alpha,
                                        float scale_log2, int (&va)[4], u32x2 (&vr)[kVAhead][2], LOAD&& load,
                                        EXTRA&& extra) {
    u32x4 kr[kKAhead], qr[kQAhead];
    if constexpr (DO_QK) {
        for_each_index([&](auto ic) __attribute__((always_inline)) {
            constexpr int I = decltype(ic)::value;
            (void)&kr, (void)&ka;   // (asm operands alone do not capture)
            SEER_MLA_READ128(kr[I], ka[I & 3], (I >> 2) * 128);
        }, std::make_integer_sequence<int, kKAhead>{});
    }
    float psum = 0.f, p_even = 0.f;
    if constexpr (!DO_QK && DO_SM) {
        for_each_index([&](auto ic) __attribute__((always_inline)) {
            (void)&vr, (void)&va;
            v_read<decltype(ic)::value>(vr, va[0], va[1], va[2], va[3]);
        }, std::make_integer_sequence<int, kVAhead>{});
    }
    // probability of slot i; two of them make one packed register
    auto element = [&](auto ic) __attribute__((always_inline)) {
        constexpr int i = decltype(ic)::value;
        if constexpr (DO_SM) {
            const float p = fast_exp2(fmaf(s_old[i], scale_log2, -m_use));
            if constexpr (i % 2 == 0) {
                p_even = p;
                SEER_MLA_PIN(p_even);
                // the sum takes the probabilities as the P.V product will see them, a pair per instruction,
                // one pair behind (not right after the packing that produces its operand)
                if constexpr (i >= 2) {
                    psum = add_bf16_pair(pk[(i >> 1) - 1], psum);
                    SEER_MLA_PIN(psum);
                }
            } else {
                pk[i >> 1] = cvt_pk_bf16(p_even, p);
                SEER_MLA_PIN(pk[i >> 1]);
            }
        }
    };
    SEER_MLA_FENCE();
    if constexpr (DO_QK) {
        for_each_index([&](auto ic) __attribute__((always_inline)) {
            constexpr int kk = decltype(ic)::value;
            (void)&kr, (void)&qr, (void)&ka, (void)&qt;   // (asm operands alone do not capture)
            wait_lgkm<qk_wait_count(kk, DO_SM)>();
            const u32x4 qv = kk < kQRegSteps ? qreg[kk < kQRegSteps ? kk : 0] : qr[kk % kQAhead];
            if constexpr (kk == 0) mfma_vgpr_first(s_new, kr[0], qv); else mfma_vgpr(s_new, kr[kk % kKAhead], qv);
            if constexpr (kk + kKAhead < kKSteps)
                SEER_MLA_READ128(kr[kk % kKAhead], ka[(kk + kKAhead) & 3], ((kk + kKAhead) >> 2) * 128);
            if constexpr (kk + kQAhead >= kQRegSteps && kk + kQAhead < kKSteps)
                SEER_MLA_READ128(qr[kk % kQAhead], qt, (kk + kQAhead - kQRegSteps) * 1024);
            if constexpr (DO_SM && kk >= kVFirst) {
                (void)&vr, (void)&va;
                v_read<kk - kVFirst>(vr, va[0], va[1], va[2], va[3]);
            }
            // one probability in the shadow of every second MFMA
            if constexpr (kk >= 2 && kk % 2 == 0 && (kk - 2) / 2 < 16) element(std::integral_constant<int, (kk - 2) / 2>{});
            // ... and one of this wave's loads of the next tile behind every kLoadEvery-th
            if constexpr (kk >= kLoadFirst && (kk - kLoadFirst) % kLoadEvery == 0 && (kk - kLoadFirst) / kLoadEvery < kLoadsPerWave)
                load(std::integral_constant<int, (kk - kLoadFirst) / kLoadEvery>{});
            extra(ic);
            SEER_MLA_FENCE();
        }, std::make_integer_sequence<int, kKSteps>{});
    } else {
        for_each_index(element, std::make_integer_sequence<int, 16>{});
    }
    if constexpr (DO_SM) {
        psum = add_bf16_pair(pk[7], psum);
        l_run = l_run * alpha + psum;
        SEER_MLA_PIN(l_run);
    }
}

// Phase B: O^T[d][row] += sum_token V[token][d] * P[row][token] for one tile (32 MFMAs), V = first 512
// dims of the latent through the transposing read.  MFMA m = 4 G2 + w works on the pair of d-tiles G2:
// w = 0, 1: even, odd d-tile, tokens 0..15;  w = 2, 3: even, odd d-tile, tokens 16..31.
// va = {a_even, a_even8, a_odd, a_odd8}: lane address for even / odd d-tiles; the token rows +8 and +24 differ
// from +0 and +16 in row bit 3, which the swizzle uses: they go through addresses of their own.
// The operands of MFMAs 0..kVAhead-1 are already on their way into vr (requested by phase A); shadow(m) is vector
// arithmetic to issue behind MFMA m (it must not touch LDS).
template <typename SHADOW>
__device__ __forceinline__ void phase_b(const int (&va)[4], u32x2 (&vr)[kVAhead][2], const uint32_t (&pk)[8],
                                        f32x16 (&acc)[kDTiles], SHADOW&& shadow) {
    const u32x4 pb0 = {pk[0], pk[1], pk[2], pk[3]};
    const u32x4 pb1 = {pk[4], pk[5], pk[6], pk[7]};
    for_each_index([&](auto ic) __attribute__((always_inline)) {
        constexpr int m = decltype(ic)::value;
        constexpr int left = kDTiles * 2 - 1 - m;                       // MFMAs after this one
        (void)&vr, (void)&va;                                           // (asm operands alone do not capture)
        wait_lgkm<2 * (left < kVAhead - 1 ? left : kVAhead - 1)>();
        const u32x4 v = {vr[m % kVAhead][0][0], vr[m % kVAhead][0][1], vr[m % kVAhead][1][0], vr[m % kVAhead][1][1]};
        mfma_acc(acc[(m >> 2) * 2 + (m & 1)], v, (m & 2) ? pb1 : pb0);
        if constexpr (m + kVAhead < kDTiles * 2) v_read<m + kVAhead>(vr, va[0], va[1], va[2], va[3]);
        shadow(ic);
        SEER_MLA_FENCE();
    }, std::make_integer_sequence<int, kDTiles * 2>{});
}

}  // namespace mla

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
    int g = uniform_load(L ? a.wg_start + wg : a.tile_off + b);
    const int g_end = uniform_load(L ? a.wg_start + wg + 1 : a.tile_off + b + 1);
    bool bad_page = false;

    const unsigned char* __restrict__ kbase = static_cast<const unsigned char*>(a.k_pages);
    const int page_shift = __builtin_ctz(static_cast<unsigned>(a.P));
    const size_t page_bytes = static_cast<size_t>(a.Hkv) * a.P * kRowBytes;
    const size_t head_off = static_cast<size_t>(kvh) * a.P * kRowBytes;

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
    // tile loads: byte offset in the tile (global side) of what LDS slot c of the first 18 blocks receives
    int pat[5];
#pragma unroll
    for (int j = 0; j < 5; ++j) {
        const unsigned c = static_cast<unsigned>((j < 4 ? wave + 4 * j : 16 + (wave & 1)) * 64 + lane);
        const unsigned row = c / kChunksPerRow, pos = c - row * kChunksPerRow;
        pat[j] = static_cast<int>(row * kRowBytes + ((pos ^ static_cast<unsigned>(swz(static_cast<int>(row)))) << 4));
    }

  for (; g < g_end; ++b) {
    const int t_lo = uniform_load(a.tile_off + b), t_hi = uniform_load(a.tile_off + b + 1);
    if (t_hi == t_lo) continue;
    const int item_idx = uniform_load(a.split_off + b) + (L ? wg - uniform_load(a.req_first + b) : 0);
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
    u32x4 qreg[kQRegSteps];
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
            qreg[kk] = qv[kk];
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
    float m_run = kNegInf, l_run = 0.f, alpha = 1.f;

    // ---- page ids, 64 at a time, handed out by v_readlane ------------------------------------
    const int32_t* __restrict__ table = a.block_table + static_cast<size_t>(b) * a.max_pages;
    int cache_base = -0x40000000;
    int pg_cache = 0;
    const int last_page = (n - 1) >> page_shift;
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
    // Tile loads go through a buffer descriptor of the tile (base = the tile's first row, 36 KB long): a
    // 32-bit lane offset and a scalar offset per load instead of 64-bit address arithmetic.  LDS slot
    // c = block * 64 + lane holds chunk (c % 72) ^ swz(row) of row c / 72; blocks k and k + 18 lie 16 rows
    // apart (same swizzle), so 18 lane patterns serve the 36 blocks.  Wave w takes the blocks w + 4j and
    // w + 4j + 18 (j = 0..3) and one of 16, 17, 34, 35: five pattern registers.
    auto tile_rsrc = [&](int tile) __attribute__((always_inline)) {
        const int tb = tok_begin + tile * kTile;
        const unsigned char* src = kbase + page_offset(tb >> page_shift) + static_cast<size_t>(tb & (a.P - 1)) * kRowBytes;
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(src), 0, kStageBytes, 0x00020000);
    };
    auto issue_load = [&](auto ic, __amdgpu_buffer_rsrc_t rsrc, int stage_off) __attribute__((always_inline)) {
        constexpr int i = decltype(ic)::value;
        const int half = i < 8 ? (i & 1) : (wave >> 1);
        const int block = (i < 8 ? wave + 4 * (i >> 1) : 16 + (wave & 1)) + 18 * half;
        unsigned char* stage = lds + stage_off;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (SEER_AS3 void*)(stage + block * 1024), 16, pat[i < 8 ? (i >> 1) : 4],
                                                 half * (16 * kRowBytes), 0, 0);
    };
    auto issue_tile = [&](int tile, int stage_off) __attribute__((always_inline)) {
        const __amdgpu_buffer_rsrc_t rsrc = tile_rsrc(tile);
        for_each_index([&](auto ic) __attribute__((always_inline)) { issue_load(ic, rsrc, stage_off); },
                       std::make_integer_sequence<int, kLoadsPerWave>{});
    };

    // ---- the pipeline: step u = scores of tile u | softmax of tile u-1, then P.V of tile u-1 ------
    // Tile u + 1 is requested at step u, into the stage that tile u-2 left at the end of step u-1.
    // Byte offsets of the stages that hold tiles u-1, u and u+1 at step u: they rotate, no arithmetic.
    static_assert(kStages == 3, "the three stage offsets below rotate");
    int st_prev = 2 * kStageBytes, st_cur = 0, st_next = kStageBytes;
    const int lds_base = lds_addr(lds);
    const int qt = lds_addr(&q_tail[wave][0][lane]);
    f32x16 s_a, s_b;
    uint32_t pk[8];
    // top of step u: tile u has landed for every wave, every wave is done with step u-1
    auto step_top = [&](int u) __attribute__((always_inline)) {
        if (kStages > 3 && u + 1 < n_tiles) wait_vmcnt<(kStages > 3 ? kLoadsPerWave : 0)>(); else wait_vmcnt<0>();
        bare_barrier();
        if (u == n_tiles - 1 && tok_begin + (u + 1) * kTile > n) {
            // ragged last tile: clear the rows past the end (0 * NaN must not reach the output)
            unsigned char* kl = lds + st_cur;
            const int first_bad = n - (tok_begin + u * kTile);
            for (int c = tid; c < kTile * kChunksPerRow; c += NT)
                if (c / kChunksPerRow >= first_bad) *reinterpret_cast<u32x4*>(kl + c * 16) = u32x4{0u, 0u, 0u, 0u};
            __builtin_amdgcn_s_waitcnt(0xc07f);
            bare_barrier();
        }
    };
    // -inf into the slots of tile j that this lane's row does not see
    auto apply_mask = [&](int j, f32x16& sc) __attribute__((always_inline)) {
        const int rel = tok_begin + j * kTile - n0;        // uniform; a tile with masked slots has rel > -32
        if (rel <= -kTile) return;
        uint32_t vis = rel >= 0 ? static_cast<uint32_t>(word >> rel)
                                : (static_cast<uint32_t>(word << (-rel)) | ((1u << (-rel)) - 1u));
        vis >>= lg * 4;
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (!((vis >> ((i >> 2) * 8 + (i & 3))) & 1u)) sc[i] = kNegInf;
    };
    // K operand addresses of the tile in the stage at byte offset stage_off
    auto k_addrs = [&](int stage_off, int (&ka)[4]) __attribute__((always_inline)) {
        const int st = lds_base + stage_off;
#pragma unroll
        for (int j = 0; j < 4; ++j) ka[j] = st + k_rd[j];
    };
    // V^T operand addresses
    auto v_addrs = [&](int stage_off, int (&va)[4]) __attribute__((always_inline)) {
        const int st = lds_base + stage_off;
        va[0] = st + v_even, va[1] = st + v_even8, va[2] = st + v_odd, va[3] = st + v_odd8;
    };
    // The exponent reference for the scores sc of one tile, in four slices (issued in the shadow of P.V MFMAs, or in
    // one go).  Lazy reference: m_run is the exponent reference of (l, acc), not necessarily the true maximum; it
    // moves only when the tile maximum exceeds it by more than 8 (log2 units), so p stays below 2^8 (bf16 and fp32
    // have the range) and the 256-register rescale is rare.  Sets m_use and alpha for the tile, and m_run.
    // Register i of sc holds token (i/4)*8 + lg*4 + i%4 of the tile, for this lane's row.
    float m_use = 0.f, mx_part = 0.f;
    auto reference = [&](auto ic, const f32x16& sc) __attribute__((always_inline)) {
        constexpr int part = decltype(ic)::value;
        if constexpr (part == 0) {
            mx_part = fmaxf(fmaxf(sc[0], sc[1]), sc[2]);
#pragma unroll
            for (int i = 3; i < 9; i += 2) mx_part = fmaxf(fmaxf(mx_part, sc[i]), sc[i + 1]);
            SEER_MLA_PIN(mx_part);
        } else if constexpr (part == 1) {
#pragma unroll
            for (int i = 9; i < 15; i += 2) mx_part = fmaxf(fmaxf(mx_part, sc[i]), sc[i + 1]);
            mx_part = fmaxf(mx_part, sc[15]);
            SEER_MLA_PIN(mx_part);
        } else if constexpr (part == 2) {
            mx_part = max_across_halves(mx_part) * a.scale_log2;
            SEER_MLA_PIN(mx_part);
        } else {
            const float m_new = (mx_part > m_run + 8.f) ? mx_part : m_run;
            m_use = (m_new == kNegInf) ? 0.f : m_new;
            alpha = fast_exp2(m_run - m_use);
            m_run = m_new;
            SEER_MLA_PIN(m_use);
            SEER_MLA_PIN(alpha);
            SEER_MLA_PIN(m_run);
        }
    };
    // P.V of tile j (probabilities pk, first operands already requested into vr) with, in its shadow, the exponent
    // reference of the scores of tile j + 1 (sc_next; NEXT = false: there is none).  The accumulators are rescaled
    // first if any row of the wave moved its reference for tile j.
    u32x2 vr[kVAhead][2];   // [ring slot][tokens +0..3 | +8..11 of the MFMA's 16]
    int va[4];
    auto pv = [&](int j, auto next, f32x16& sc_next, auto&& prepare) __attribute__((always_inline)) {
        constexpr bool NEXT = decltype(next)::value;
        if constexpr (NEXT) {
            // -inf into the slots of tile j + 1 that this lane's row does not see (only the tiles that reach the draft
            // slots have any); the scores were written by MFMAs the compiler knows nothing of: idle past them first
            const int rel = tok_begin + (j + 1) * kTile - n0;
            if (rel > -kTile) {
                mfma_drain();
                apply_mask(j + 1, sc_next);
            }
        }
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
            asm volatile("s_nop 7");
        }
        // the score MFMAs of sc_next were issued before the phase began; its first use here sits behind P.V MFMA
        // kRefFirst, more than an MFMA's depth later
        constexpr int kRefFirst = 4;
        phase_b(va, vr, pk, acc, [&](auto ic) __attribute__((always_inline)) {
            constexpr int m = decltype(ic)::value;
            if constexpr (NEXT && m >= kRefFirst && (m - kRefFirst) % 2 == 0 && (m - kRefFirst) / 2 < 4)
                reference(std::integral_constant<int, (m - kRefFirst) / 2>{}, sc_next);
            prepare(ic);
        });
    };
    using yes = std::true_type;
    using no = std::false_type;

    issue_tile(0, st_cur);

    int ka[4];
    // the loads of tile u + 1, requested inside step u's score phase (its stage held tile u - 2, which every
    // wave left before the barrier at the top of step u)
    __amdgpu_buffer_rsrc_t next_rsrc = tile_rsrc(0);
    bool next_ok = false;
    auto next_setup = [&](int u) __attribute__((always_inline)) {
        next_ok = u + 1 < n_tiles;
        if (next_ok) next_rsrc = tile_rsrc(u + 1);
    };
    auto next_load = [&](auto ic) __attribute__((always_inline)) {
        if (next_ok) issue_load(ic, next_rsrc, st_next);
    };
    auto nothing = [](auto) {};
    // What step u + 1 needs before its first LDS read, done in the shadow of step u's P.V MFMAs instead of behind the
    // barrier: the stage offsets move on, the K operand addresses, the descriptor of the tile after.
    int u = 0;
    auto prepare_next = [&](auto ic) __attribute__((always_inline)) {
        constexpr int m = decltype(ic)::value;
        if constexpr (m == 14) {
            const int t = st_prev;
            st_prev = st_cur, st_cur = st_next, st_next = t;
            k_addrs(st_cur, ka);
        } else if constexpr (m == 18) {
            next_setup(u + 1);
        }
    };
    // the V^T operand addresses of tile u - 1, early in step u's score phase (first used behind score MFMA kVFirst)
    auto v_addrs_early = [&](auto ic) __attribute__((always_inline)) {
        if constexpr (decltype(ic)::value == 2) v_addrs(st_prev, va);
    };
    k_addrs(st_cur, ka);
    next_setup(0);
    step_top(0);
    phase_a<true, false>(ka, qt, qreg, s_a, s_b, pk, m_use, l_run, alpha, a.scale_log2, va, vr, next_load, nothing);
    // the first tile's exponent reference, with nothing to hide behind
    mfma_drain();
    apply_mask(0, s_a);
    for_each_index([&](auto ic) __attribute__((always_inline)) { reference(ic, s_a); }, std::make_integer_sequence<int, 4>{});
    prepare_next(std::integral_constant<int, 14>{});
    prepare_next(std::integral_constant<int, 18>{});
    // steps 1 .. n_tiles - 1, two per iteration so that s_a and s_b swap roles without register moves
    for (u = 1; u + 1 < n_tiles;) {
        step_top(u);
        phase_a<true, true>(ka, qt, qreg, s_b, s_a, pk, m_use, l_run, alpha, a.scale_log2, va, vr, next_load, v_addrs_early);
        pv(u - 1, yes{}, s_b, prepare_next);
        ++u;
        step_top(u);
        phase_a<true, true>(ka, qt, qreg, s_a, s_b, pk, m_use, l_run, alpha, a.scale_log2, va, vr, next_load, v_addrs_early);
        pv(u - 1, yes{}, s_a, prepare_next);
        ++u;
    }
    if (u < n_tiles) {
        step_top(u);
        phase_a<true, true>(ka, qt, qreg, s_b, s_a, pk, m_use, l_run, alpha, a.scale_log2, va, vr, next_load, v_addrs_early);
        pv(u - 1, yes{}, s_b, prepare_next);
        asm volatile("" : "+v"(s_b));       // the copy below reads s_b after the P.V MFMAs, not right behind the score MFMAs
#pragma unroll
        for (int i = 0; i < 16; ++i) s_a[i] = s_b[i];
    }
    // the last tile's scores are in s_a, masked, and its reference is set; its stage is the one before the current
    v_addrs(st_prev, va);
    phase_a<false, true>(ka, qt, qreg, s_b, s_a, pk, m_use, l_run, alpha, a.scale_log2, va, vr, nothing, nothing);
    pv(n_tiles - 1, no{}, s_a, nothing);

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
    return a.Dqk == mla::kDqk && a.Dv == mla::kDv && a.P >= mla::kMinPage && a.P <= 1024 && (a.P & (a.P - 1)) == 0 &&
           a.v_pages == nullptr && a.Hkv <= 65535;
}

hipError_t launch_mla(const AttnArgs& a, hipStream_t stream) {
    const int row_blocks = (a.G * a.T + mla::kRowsPerWg - 1) / mla::kRowsPerWg;
    const unsigned groups = (a.wgs_per_head + 7) / 8;
    const dim3 grid(8u * groups * row_blocks, a.Hkv);
    hipLaunchKernelGGL(attn_mla_kernel, grid, dim3(mla::kWaves * kWave), 0, stream, a, row_blocks);
    return hipGetLastError();
}

}  // namespace seer
