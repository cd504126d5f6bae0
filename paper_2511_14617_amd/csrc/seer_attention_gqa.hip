// Tiled verify-attention partition kernel for grouped-query heads with
// D = 128 and pages of 16 (or a larger power of two) tokens (the shape of the paper's dense 8B- to 72B-class
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
// Data flow per 32-token tile (two pages, 8 KB of K and 8 KB of V)
//   HBM -> LDS directly (global_load_lds_dwordx4: 16 bytes per lane, 1 KB per wave
//          instruction, no staging registers), into a ring of K slots and a ring of V slots,
//          D tiles in flight per workgroup while one is computed.  Rows are 256 B, unpadded;
//          the 16-byte chunks of a row are stored XOR-swizzled (the lane picks which
//          global chunk lands in its fixed LDS slot), which makes the operand reads
//          below free of bank conflicts.  Completion is tracked by hand: s_waitcnt
//          vmcnt(loads of the younger steps) then s_barrier.
//   S^T = K . Q^T    v_mfma_f32_32x32x16_bf16, M = tokens, N = rows, 8 steps over d;
//                    K operand = one ds_read_b128 per step, Q^T stays in 32 VGPRs
//   softmax          each lane owns ONE query row (N index = lane % 32) and 16 of the
//                    tile's 32 tokens, so max/sum are in-lane plus one cross-half
//                    exchange; the C registers of S^T are, as they stand, the
//                    B operand of the next product (no shuffle, no LDS round trip)
//   O^T += V^T . P^T M = d (4 tiles of 32), N = rows, 2 steps over the tokens; the
//                    V^T operand (8 tokens at one d) comes from the token-major tile
//                    through two transposing LDS reads (ds_read_b64_tr_b16)
//
// Software pipeline
//   A wave that ran a tile's three phases one after the other (scores on the matrix core,
//   softmax on the vector ALU, P.V on the matrix core) would leave each unit idle while the other
//   works, and waves sharing a SIMD would not fill each other's gaps either, because the per-tile
//   barrier keeps them in the same phase.  So one loop step works on three consecutive tiles,
//   with no dependence between the three parts:
//       step u:   P.V of tile u-2 (MFMA)  |  softmax of tile u-1 (VALU)  |  scores of tile u (MFMA)
//   K is needed two steps before the V of the same tile, hence the two rings (D+1 slots of 8 KB
//   each): step u issues the loads of K tile u+D and V tile u+D-2; both are consumed D steps
//   after they were issued, with the loads of D-1 steps in flight behind them.
//   The exponent reference of a row only moves when the new maximum exceeds it by more than 8
//   (in log2 units: the probabilities then stay below 2^8, as exact in bf16's 8 bits as values
//   below 1), which makes the rescaling of the 64 output accumulators rare.
#include <type_traits>
#include <utility>

#include "seer_attention.h"
#include "seer_device.h"
#include "seer_tile.h"

namespace seer {

constexpr int kD = 128;                  // head dim
constexpr int kMinPage = 16;             // tokens per page: 16, or a larger power of two (a 32-token tile is then inside one page)
constexpr int kTile = 32;                // tokens per tile
constexpr int kRowBytes = kD * 2;        // 256
constexpr int kKBytes = kTile * kRowBytes;   // 8192
static_assert(kTile == kPlanTile, "the plan counts work in tiles of this kernel");

// Swizzles: a row's 16-byte chunk c is stored at chunk position c ^ f(row).  LDS has 64 banks of
// 4 bytes (256 bytes per clock): a row is exactly one pass over the banks, so without a swizzle
// every row starts at bank 0.
//   K: f = row & 15        -> 16 consecutive rows, same chunk (one ds_read_b128 quarter-wave):
//                             16 distinct 16-byte bank groups
//   V: f = (row & 3) << 2  -> 4 consecutive rows, same 64-byte quarter of the row (half a wave of
//                             the transposing read): 4 distinct 64-byte groups
// (measured with several waves reading at once: these reach the rate of a linear access pattern,
// twice that of swizzles which only spread over 128 bytes)
__device__ __forceinline__ int k_swz(int row) { return row & 15; }
__device__ __forceinline__ int v_swz(int row) { return (row & 3) << 2; }

// Which waves issue the tile loads.  A direct-to-LDS load holds the issuing wave for about 27 ns (the
// vector memory path of a CU moves 64 bytes per clock), and with five waves on four SIMDs, waves 0 and 4
// share a SIMD and are the ones every step waits for: they are left out, waves 1..3 load.
template <int NW> struct Loaders { static constexpr int kFirst = 0, kCount = NW; };
template <> struct Loaders<5> { static constexpr int kFirst = 1, kCount = 3; };

// Cache policy of the tile loads: non-temporal.  A KV tile is used once per call by one workgroup, and
// streaming it (no allocation for reuse in the L2 and the memory-side cache) is what lets a gather of 4 KB
// blocks reach 6.9 TB/s on this part; the default policy tops out at 6.1 TB/s (bare read loops, plain loads
// and loads into LDS alike).
constexpr int kTileLoadPolicy = 2;   // the "nt" bit of the instruction's cache-policy field

// Loads of one half tile (K or V): its 8 one-KB blocks dealt round-robin to the loading waves.
template <int NW, int POLICY = kTileLoadPolicy>
__device__ __forceinline__ void issue_half_tile(unsigned char* slot, int wave, size_t p0, size_t p1,
                                                const unsigned char* base, int goff, bool is_k) {
    constexpr int NL = Loaders<NW>::kCount;
    const int li = wave - Loaders<NW>::kFirst;
    if (li < 0 || li >= NL) return;
#pragma unroll
    for (int i = 0; i < (8 + NL - 1) / NL; ++i) {
        const int j = li + i * NL;
        if (j < 8) {
            const size_t pg = (j < 4) ? p0 : p1;
            const int lane_off = is_k ? goff ^ ((j & 3) << 6) : goff;   // K rows 4j + l16: f = 4(j & 3) + l16
            const unsigned char* src = base + pg + (j & 3) * (4 * kRowBytes) + lane_off;
            __builtin_amdgcn_global_load_lds((const SEER_AS1 void*)(src), (SEER_AS3 void*)(slot + j * 1024), 16, 0, POLICY);
        }
    }
}

// 8 transposing reads: for each of the 4 d-tiles, the tokens +0..3 and +8..11 of one 16-token half.
// Within a 16-lane group, lane s = 4k + c points at token row k (of the 4 the group covers) and d
// columns 4c..4c+3 of the group's 16; lane i of the group receives the 4 tokens of column i.
// The reads are issued from an asm block that ends in its own s_waitcnt lgkmcnt(0): through the
// builtin, the compiler puts a vmcnt(0) in front of them (it cannot tell them apart from the
// direct-to-LDS loads still in flight), which would drain the ring on every tile.
#define SEER_GQA_TR8(vr_, a0_, a1_, a2_, a3_, OFF0, OFF1)                                                  \
    asm volatile("ds_read_b64_tr_b16 %0, %8 offset:" #OFF0 "\n"                                            \
                 "ds_read_b64_tr_b16 %1, %8 offset:" #OFF1 "\n"                                            \
                 "ds_read_b64_tr_b16 %2, %9 offset:" #OFF0 "\n"                                            \
                 "ds_read_b64_tr_b16 %3, %9 offset:" #OFF1 "\n"                                            \
                 "ds_read_b64_tr_b16 %4, %10 offset:" #OFF0 "\n"                                           \
                 "ds_read_b64_tr_b16 %5, %10 offset:" #OFF1 "\n"                                           \
                 "ds_read_b64_tr_b16 %6, %11 offset:" #OFF0 "\n"                                           \
                 "ds_read_b64_tr_b16 %7, %11 offset:" #OFF1 "\n"                                           \
                 "s_waitcnt lgkmcnt(0)"                                                                    \
                 : "=&v"(vr_[0][0]), "=&v"(vr_[0][1]), "=&v"(vr_[1][0]), "=&v"(vr_[1][1]), "=&v"(vr_[2][0]), \
                   "=&v"(vr_[2][1]), "=&v"(vr_[3][0]), "=&v"(vr_[3][1])                                    \
                 : "v"(a0_), "v"(a1_), "v"(a2_), "v"(a3_))

// max over the two lanes that share a query row (lane and lane ^ 32), without touching LDS:
// v_permlane32_swap exchanges the upper 32 lanes of its first operand with the lower 32 lanes of
// its second, so from two copies of x one register ends up with the lower half's values in both
// halves and the other with the upper half's.  (Issued from an asm block: with the builtin this
// compiler keeps only the first of the two results.  The s_nop covers the wait states the
// instruction needs after a vector-ALU write of its operands.)
__device__ __forceinline__ float max_across_halves(float x) {
    float a = x, b = x;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    float m;
    asm("v_max_f32 %0, %1, %2" : "=v"(m) : "v"(a), "v"(b));   // (fmaxf would first quieten both operands: two more instructions)
    return m;
}

// Softmax bookkeeping of one tile for this lane's row, from the row's raw score maximum mx_raw
// (masked slots excluded): moves the exponent reference m_run only when the new maximum exceeds
// it by more than 8 (probabilities then stay below 2^8), returns the reference to subtract (in
// units of log2 e, scores scaled) and leaves in alpha the factor that brings sums taken under the
// old reference to the new one.  scale_log2 > 0.
__device__ __forceinline__ float move_reference(float mx_raw, float scale_log2, float& m_run, float& alpha) {
    const float mx = max_across_halves(mx_raw) * scale_log2;
    const float m_new = (mx > m_run + 8.f) ? mx : m_run;      // m_run = -inf: any finite mx moves it
    const float m_use = (m_new == kNegInf) ? 0.f : m_new;      // nothing visible yet: keep exp2 finite
    alpha = fast_exp2(m_run - m_use);
    m_run = m_new;
    return m_use;
}

__device__ __forceinline__ void rescale_if_moved(f32x16 (&acc)[4], float alpha) {
    if (__any(alpha != 1.f)) {
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[dt][i] *= alpha;
    }
}

// One pipeline step at the ends of a piece, where not all three parts exist (the steady state is
// fused_step below).  k_off / v_off: byte offsets in LDS of the K slot the scores read and of the
// V slot (row part of the lane's address included) the P.V product reads.  alpha is the
// rescaling factor the previous step's softmax left for the output accumulators: it is applied
// before this step's P.V, and replaced by this step's softmax.
template <bool DO_QK, bool DO_SM, bool DO_PV, bool MASKED = true>
__device__ __forceinline__ void pipe_step(const unsigned char* lds, int k_off, int v_off, const int (&k_rd)[8],
                                          const int (&v_rd)[4], const bf16x8 (&qreg)[8], f32x16& s_sm,
                                          f32x16& s_qk, const uint32_t (&pk_pv)[8], uint32_t (&pk_sm)[8],
                                          f32x16 (&acc)[4], float& m_run, float& l_run, float& alpha,
                                          float scale_log2, uint32_t vis) {
    if constexpr (DO_PV) {
        rescale_if_moved(acc, alpha);
        alpha = 1.f;
        // O^T[d][row] += sum_token V[token][d] * P[row][token], 16 tokens at a time
        const int a0 = v_off + v_rd[0], a1 = v_off + v_rd[1], a2 = v_off + v_rd[2], a3 = v_off + v_rd[3];
        u32x2 vr[4][2];
        SEER_GQA_TR8(vr, a0, a1, a2, a3, 0, 2048);
        const bf16x8 pb0 = as_bf16x8(u32x4{pk_pv[0], pk_pv[1], pk_pv[2], pk_pv[3]});
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
            const bf16x8 va = as_bf16x8(u32x4{vr[dt][0][0], vr[dt][0][1], vr[dt][1][0], vr[dt][1][1]});
            acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb0, acc[dt], 0, 0, 0);
        }
        u32x2 vq[4][2];
        SEER_GQA_TR8(vq, a0, a1, a2, a3, 4096, 6144);
        const bf16x8 pb1 = as_bf16x8(u32x4{pk_pv[4], pk_pv[5], pk_pv[6], pk_pv[7]});
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
            const bf16x8 va = as_bf16x8(u32x4{vq[dt][0][0], vq[dt][0][1], vq[dt][1][0], vq[dt][1][1]});
            acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb1, acc[dt], 0, 0, 0);
        }
    }
    if constexpr (DO_QK) {
        // S^T[token][row] = sum_d K[token][d] * Q[row][d]
#pragma unroll
        for (int i = 0; i < 16; ++i) s_qk[i] = 0.f;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            u32x4 kv[4];
            const int b0 = k_off + k_rd[4 * h], b1 = k_off + k_rd[4 * h + 1], b2 = k_off + k_rd[4 * h + 2],
                      b3 = k_off + k_rd[4 * h + 3];
            asm volatile("ds_read_b128 %0, %4\n"
                         "ds_read_b128 %1, %5\n"
                         "ds_read_b128 %2, %6\n"
                         "ds_read_b128 %3, %7\n"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(kv[0]), "=&v"(kv[1]), "=&v"(kv[2]), "=&v"(kv[3])
                         : "v"(b0), "v"(b1), "v"(b2), "v"(b3));
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                s_qk = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kv[kk]), qreg[4 * h + kk], s_qk, 0, 0, 0);
        }
    }
    if constexpr (DO_SM) {
        // register i of s_sm holds token (i/4)*8 + lg*4 + i%4 of the tile (vis is already shifted by lg*4)
        float mx = kNegInf;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            if constexpr (MASKED)
                if (!((vis >> ((i >> 2) * 8 + (i & 3))) & 1u)) s_sm[i] = kNegInf;
            mx = fmaxf(mx, s_sm[i]);
        }
        const float m_use = move_reference(mx, scale_log2, m_run, alpha);
        float psum = 0.f;
#pragma unroll
        for (int i = 0; i < 16; i += 2) {
            const float p0 = fast_exp2(fmaf(s_sm[i], scale_log2, -m_use));
            const float p1 = fast_exp2(fmaf(s_sm[i + 1], scale_log2, -m_use));
            pk_sm[i >> 1] = cvt_pk_bf16(p0, p1);
            psum = add_bf16_pair(pk_sm[i >> 1], psum);
        }
        l_run = l_run * alpha + psum;
    }
}

// Operand reads whose issue and completion are separated by hand.  The issuing block names the
// destination registers as outputs although they are only written when the read returns; the
// matching SEER_LGKM_WAIT block (s_waitcnt lgkmcnt(N), N = reads issued after the group: LDS
// returns in order) takes them as read-write operands, so every use of the data is ordered after
// the wait, and nothing between the two blocks has a reason to touch them.
#define SEER_TR8_ISSUE(vr_, a0_, a1_, a2_, a3_, OFF0, OFF1)                                                \
    asm volatile("ds_read_b64_tr_b16 %0, %8 offset:%12\n"                                                  \
                 "ds_read_b64_tr_b16 %1, %8 offset:%13\n"                                                  \
                 "ds_read_b64_tr_b16 %2, %9 offset:%12\n"                                                  \
                 "ds_read_b64_tr_b16 %3, %9 offset:%13\n"                                                  \
                 "ds_read_b64_tr_b16 %4, %10 offset:%12\n"                                                 \
                 "ds_read_b64_tr_b16 %5, %10 offset:%13\n"                                                 \
                 "ds_read_b64_tr_b16 %6, %11 offset:%12\n"                                                 \
                 "ds_read_b64_tr_b16 %7, %11 offset:%13"                                                   \
                 : "=&v"(vr_[0][0]), "=&v"(vr_[0][1]), "=&v"(vr_[1][0]), "=&v"(vr_[1][1]), "=&v"(vr_[2][0]), \
                   "=&v"(vr_[2][1]), "=&v"(vr_[3][0]), "=&v"(vr_[3][1])                                    \
                 : "v"(a0_), "v"(a1_), "v"(a2_), "v"(a3_), "n"(OFF0), "n"(OFF1))
#define SEER_TR8_WAIT(N, vr_)                                                                              \
    asm volatile("s_waitcnt lgkmcnt(" #N ")"                                                               \
                 : "+v"(vr_[0][0]), "+v"(vr_[0][1]), "+v"(vr_[1][0]), "+v"(vr_[1][1]), "+v"(vr_[2][0]),    \
                   "+v"(vr_[2][1]), "+v"(vr_[3][0]), "+v"(vr_[3][1]))
#define SEER_K4_ISSUE(kv_, b0_, b1_, b2_, b3_, OFF)                                                        \
    asm volatile("ds_read_b128 %0, %4 offset:%8\n"                                                         \
                 "ds_read_b128 %1, %5 offset:%8\n"                                                         \
                 "ds_read_b128 %2, %6 offset:%8\n"                                                         \
                 "ds_read_b128 %3, %7 offset:%8"                                                           \
                 : "=&v"(kv_[0]), "=&v"(kv_[1]), "=&v"(kv_[2]), "=&v"(kv_[3])                              \
                 : "v"(b0_), "v"(b1_), "v"(b2_), "v"(b3_), "n"(OFF))
#define SEER_K4_WAIT(N, kv_)                                                                               \
    asm volatile("s_waitcnt lgkmcnt(" #N ")" : "+v"(kv_[0]), "+v"(kv_[1]), "+v"(kv_[2]), "+v"(kv_[3]))
#define SEER_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)
// Keeps the computation of x in the block (and at the place) where it is written: a value whose
// only uses are in a later block is otherwise sunk there, out of the shadow of the MFMAs.
#define SEER_PIN(x) asm volatile("" : "+v"(x))

// The steady-state step: P.V of tile u-2 (8 MFMAs), scores of tile u (8 MFMAs) and the softmax of
// tile u-1 (about 80 vector-ALU instructions), with the instruction order fixed by hand: one
// MFMA, then the slice of softmax work that fits in the 32 cycles the matrix core is busy with
// it.  The compiler's scheduler, left alone, issues the sixteen MFMAs back to back and the
// softmax after them, which serialises the two units (a wave issues in order).  The operand
// reads run one group of four MFMAs ahead.
//
// issue_k / issue_v issue the step's HBM loads; they are called where their scalar address
// arithmetic runs in the shadow of LDS reads already issued and of MFMAs already queued.
//
// The slots read are at byte offsets K_IMM + k_off (K ring) and V_IMM + v_off (V ring, whose base is in v_rd); in the
// unrolled steady state the runtime parts are zero and the slot is an instruction immediate.
template <bool MASKED, int K_IMM, int V_IMM, typename IssueK, typename IssueV>
__device__ __forceinline__ void fused_step(int k_off, int v_off, const int (&k_rd)[8], const int (&v_rd)[4],
                                           const bf16x8 (&qreg)[8], f32x16& s_sm, f32x16& s_qk,
                                           const uint32_t (&pk_pv)[8], uint32_t (&pk_sm)[8], f32x16 (&acc)[4],
                                           float& m_run, float& l_run, float& alpha, float scale_log2,
                                           uint32_t vis, IssueK&& issue_k, IssueV&& issue_v) {
    const int a0 = v_off + v_rd[0], a1 = v_off + v_rd[1], a2 = v_off + v_rd[2], a3 = v_off + v_rd[3];
    u32x2 va[4][2], vb[4][2];
    u32x4 ka[4], kb[4];
    static_assert(K_IMM >= 0 && V_IMM >= 0 && K_IMM < 65536 && V_IMM + 6144 < 65536, "16-bit LDS offsets");
    SEER_TR8_ISSUE(va, a0, a1, a2, a3, V_IMM, V_IMM + 2048);
    SEER_TR8_ISSUE(vb, a0, a1, a2, a3, V_IMM + 4096, V_IMM + 6144);
    issue_k();
    rescale_if_moved(acc, alpha);
    if constexpr (MASKED) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (!((vis >> ((i >> 2) * 8 + (i & 3))) & 1u)) s_sm[i] = kNegInf;
    }
    SEER_TR8_WAIT(8, va);
    SEER_SCHED_FENCE();
    // ---- MFMAs 0..3: P.V on tokens 0..15 | row maximum
    const bf16x8 pb0 = as_bf16x8(u32x4{pk_pv[0], pk_pv[1], pk_pv[2], pk_pv[3]});
    float mx = kNegInf;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
        const bf16x8 v = as_bf16x8(u32x4{va[dt][0][0], va[dt][0][1], va[dt][1][0], va[dt][1][1]});
        acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v, pb0, acc[dt], 0, 0, 0);
        mx = fmaxf(fmaxf(mx, s_sm[4 * dt]), s_sm[4 * dt + 1]);
        mx = fmaxf(fmaxf(mx, s_sm[4 * dt + 2]), s_sm[4 * dt + 3]);
        SEER_PIN(mx);
        SEER_SCHED_FENCE();
    }
    {
        const int b0 = k_off + k_rd[0], b1 = k_off + k_rd[1], b2 = k_off + k_rd[2], b3 = k_off + k_rd[3];
        SEER_K4_ISSUE(ka, b0, b1, b2, b3, K_IMM);
    }
    issue_v();
    SEER_TR8_WAIT(4, vb);
    SEER_SCHED_FENCE();
    // ---- MFMAs 4..7: P.V on tokens 16..31 | exponent reference, first two pairs of probabilities
    const bf16x8 pb1 = as_bf16x8(u32x4{pk_pv[4], pk_pv[5], pk_pv[6], pk_pv[7]});
    float m_use = 0.f, psum = 0.f;
    // One pair of probabilities: scaled differences, exponentials, then the sum of the PREVIOUS pair (an
    // instruction that does not depend on the exponentials just issued, which need one more cycle before a
    // plain vector instruction may read them), then the packing of this pair.
    auto pair = [&](int i) __attribute__((always_inline)) {
        float p0 = fast_exp2(fmaf(s_sm[2 * i], scale_log2, -m_use));
        float p1 = fast_exp2(fmaf(s_sm[2 * i + 1], scale_log2, -m_use));
        asm volatile("" : "+v"(p0), "+v"(p1));
        if (i > 0) {
            psum = add_bf16_pair(pk_sm[i - 1], psum);
            SEER_PIN(psum);
        }
        pk_sm[i] = cvt_pk_bf16(p0, p1);
        SEER_PIN(pk_sm[i]);
    };
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
        const bf16x8 v = as_bf16x8(u32x4{vb[dt][0][0], vb[dt][0][1], vb[dt][1][0], vb[dt][1][1]});
        acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v, pb1, acc[dt], 0, 0, 0);
        if (dt == 0) {
            m_use = move_reference(mx, scale_log2, m_run, alpha);
            SEER_PIN(m_use);
            SEER_PIN(alpha);
            SEER_PIN(m_run);
        }
        if (dt == 2) pair(0);
        if (dt == 3) pair(1);
        SEER_SCHED_FENCE();
    }
    {
        const int b0 = k_off + k_rd[4], b1 = k_off + k_rd[5], b2 = k_off + k_rd[6], b3 = k_off + k_rd[7];
        SEER_K4_ISSUE(kb, b0, b1, b2, b3, K_IMM);
    }
    SEER_K4_WAIT(4, ka);
    SEER_SCHED_FENCE();
    // ---- MFMAs 8..15: scores of the next tile | the other six pairs
#pragma unroll
    for (int i = 0; i < 16; ++i) s_qk[i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        s_qk = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ka[kk]), qreg[kk], s_qk, 0, 0, 0);
        pair(2 + kk);
        SEER_SCHED_FENCE();
    }
    SEER_K4_WAIT(0, kb);
    SEER_SCHED_FENCE();
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        s_qk = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kb[kk]), qreg[4 + kk], s_qk, 0, 0, 0);
        if (kk < 2) pair(6 + kk);
        if (kk == 2) {
            psum = add_bf16_pair(pk_sm[7], psum);
            l_run = l_run * alpha + psum;
            SEER_PIN(l_run);
        }
        SEER_SCHED_FENCE();
    }
}

template <typename F, int... I>
__device__ __forceinline__ void for_each_index(F& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}

// STREAM: diagnostic variant that keeps the whole load path (plan, page lookups, direct-to-LDS loads,
// waits, barriers, partial-result writes) and leaves out the arithmetic.  Its time is what the memory
// system allows for exactly this access pattern and launch shape: the ceiling the kernel's
// bytes-per-second should be read against.  It writes "saw nothing" partials, so the output is zero.
// STREAM_PARTIALS: the partial results leave with non-temporal stores (see kStreamPartialsBelow).
// NH: helper waves (0 or 4) behind the NW main waves.  A row count just above a multiple of 32 (the multi-path
// tree on a group of four heads: 4 x 33 = 132 rows) would otherwise put a fifth wave with a handful of rows on the
// SIMD of wave 0; that wave runs the whole per-tile instruction stream whatever its row count, and with in-order
// issue it doubles the load of the one SIMD every step waits for.  Instead the NW = 4 main waves (one per SIMD)
// are joined by four helper waves (again one per SIMD) that serve the leftover rows TOGETHER: helper h takes
// the tiles u = h (mod 4) of a piece, each with a softmax state of its own, and the four states are merged
// through LDS at the end of the piece (in a fixed order, so the result does not depend on timing).  A helper
// scores and soft-maxes its tile at step u and multiplies by V at step u + 2, when that V tile has landed: a
// quarter of a wave's work per step on every SIMD instead of a whole wave's on one.  All eight waves issue loads.
template <int NW, int D, bool STREAM, bool STREAM_PARTIALS, int NH = 0>
__global__ __launch_bounds__((NW + NH) * kWave) __attribute__((amdgpu_waves_per_eu(NW + NH == 1 ? 1 : 2, 2)))
void attn_gqa128_kernel(AttnArgs a) {
    static_assert(NH == 0 || (NH == 4 && D >= 2), "helpers: four of them, and V tiles that land two steps after K");
    constexpr int NWT = NW + NH;                    // waves per workgroup
    constexpr int NT = NWT * kWave;
    constexpr int NSLOT = D + 1;                    // slots in the K ring and in the V ring
    constexpr int NL = Loaders<NWT>::kCount;        // waves that issue loads (the others have nothing to wait for)
    constexpr int CEIL = (8 + NL - 1) / NL;         // half-tile blocks of the busiest loading waves
    constexpr int FLOOR = 8 / NL;
    constexpr int REM = 8 % NL;                     // loaders below this index load CEIL blocks, the others FLOOR
    static_assert(D >= 1 && (D - 1) * 2 * CEIL < 64, "vmcnt range");

    // K ring, then V ring; at the end of a piece the helpers' states pass through the same memory
    constexpr int kMergeBytes = NH > 0 ? 4096 + (NH - 1) * 16 * kWave * 16 : 0;
    constexpr int kLdsBytes = 2 * NSLOT * kKBytes > kMergeBytes ? 2 * NSLOT * kKBytes : kMergeBytes;
    __shared__ __attribute__((aligned(1024))) unsigned char lds[kLdsBytes];
    constexpr int kVRing = NSLOT * kKBytes;

    // Workgroup ids are dealt round-robin to the 8 XCDs and dispatched in id order.  The grid is laid
    // out in groups of 8 stretches x Hkv heads so that the Hkv workgroups with the same stretch index
    // share XCD (id % 8) and dispatch round: the plan's per-index speed history relies on that.
    // The row blocks of a (stretch, head) are further workgroups with the same id % 8, so they share the XCD.
    int rest = blockIdx.x >> 3;
    const int kvh = rest % a.Hkv;
    rest /= a.Hkv;
    const int rb = rest % a.row_blocks;
    const int wg = (rest / a.row_blocks) * 8 + (blockIdx.x & 7);
    if (wg >= a.wgs_per_head) return;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int ln = lane & 31;
    const int lg = lane >> 5;
    const int l16 = lane >> 4;
    const int p16 = lane & 15;

    const int L = uniform_load(&a.header->tiles_per_wg);
    int b = uniform_load(a.wg_first + wg);
    if (b < 0) return;
    int g = uniform_load(L ? a.wg_start + wg : a.tile_off + b);
    const int g_end = uniform_load(L ? a.wg_start + wg + 1 : a.tile_off + b + 1);
    const int g_first = g;
    const uint64_t clock_begin = __builtin_amdgcn_s_memrealtime();
    bool bad_page = false;

    const unsigned char* __restrict__ kbase = static_cast<const unsigned char*>(a.k_pages);
    const unsigned char* __restrict__ vbase = static_cast<const unsigned char*>(a.v_pages);
    const int page_shift = __builtin_ctz(static_cast<unsigned>(a.P));              // pages hold 2^page_shift tokens
    const uint32_t page_bytes32 = static_cast<uint32_t>(a.Hkv) * a.P * kRowBytes;   // one page, all kv heads
    const size_t head_off = static_cast<size_t>(kvh) * a.P * kRowBytes;
    const int goff_k0 = l16 * kRowBytes + ((p16 ^ k_swz(l16)) << 4);
    const int goff_v = l16 * kRowBytes + ((p16 ^ v_swz(l16)) << 4);
    int k_rd[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) k_rd[kk] = ln * kRowBytes + (((2 * kk + lg) ^ k_swz(ln)) << 4);
    const int v_k = p16 >> 2, v_c4 = p16 & 3, v_dhalf = l16 & 1;
    int v_rd[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) {
        const int chunk = dt * 4 + v_dhalf * 2 + (v_c4 >> 1);
        // token lg*4 + k; the V ring's place behind the K ring is part of the lane address, so that the slot
        // offsets of both rings fit the 16-bit immediates of the LDS reads for rings of up to 8 slots
        v_rd[dt] = kVRing + (lg * 4 + v_k) * kRowBytes + ((chunk ^ v_swz(v_k)) << 4) + (v_c4 & 1) * 8;
    }

    // What a piece needs to know about its request comes from five small tables.  Read one after the other
    // (each value steers the next address or a branch) that is five dependent round trips to the L2 per
    // request boundary, several microseconds in which the workgroup has no tile in flight.  Instead one
    // vector load fetches all five (lane i reads word i), and it is issued a whole piece ahead, together
    // with the first 64 page ids of that next request: by the time a piece ends, the next one's plan words
    // and page ids are in registers.
    auto piece_words = [&](int bb) __attribute__((always_inline)) -> int {
        const int bc = min(bb, a.B - 1);
        const int32_t* ptr = a.tile_off + bc;
        if (lane == 1) ptr = a.tile_off + bc + 1;
        if (lane == 2) ptr = a.split_off + bc;
        if (lane == 3) ptr = (L ? a.req_first : a.split_off) + bc;
        if (lane == 4) ptr = a.ctx_len + bc;
        if (lane == 5) ptr = a.shared_tiles + bc;
        return *ptr;
    };
    auto first_pages = [&](int bb) __attribute__((always_inline)) -> int {
        return (a.block_table + static_cast<size_t>(min(bb, a.B - 1)) * a.max_pages)[min(lane, a.max_pages - 1)];
    };
    int pw = piece_words(b);
    int pg_ahead = 0;                 // the first 64 page ids of request b, if have_ahead
    bool have_ahead = false;

  for (; g < g_end; ++b) {
    const int t_lo = __builtin_amdgcn_readlane(pw, 0), t_hi = __builtin_amdgcn_readlane(pw, 1);
    const int item_idx = __builtin_amdgcn_readlane(pw, 2) + (L ? wg - __builtin_amdgcn_readlane(pw, 3) : 0);
    const int n = __builtin_amdgcn_readlane(pw, 4);
    const int shared_tiles = __builtin_amdgcn_readlane(pw, 5);
    const int pg_first = pg_ahead;
    const bool have_first = have_ahead;
    pw = piece_words(b + 1);          // in flight while this piece is worked on
    pg_ahead = first_pages(b + 1);
    have_ahead = b + 1 < a.B;
    if (t_hi == t_lo) continue;
    const int tok_begin = (g - t_lo) * kTile;
    const int tok_end = min(n, (min(g_end, t_hi) - t_lo) * kTile);
    g = t_hi;
    const int n0 = n - a.T;
    const int n_tiles = (tok_end - tok_begin + kTile - 1) / kTile;
    bare_barrier();                                // every wave is done with the previous piece's slots

    const int R = min(a.G * a.T, (rb + 1) * a.rows_per_block);     // rows of this row block end here
    const bool helper = NH > 0 && wave >= NW;                       // uniform for the wave
    const int r = rb * a.rows_per_block + (helper ? NW : wave) * 32 + ln;
    const bool row_ok = r < R;
    const int t = row_ok ? r / a.G : 0;
    const int hq = kvh * a.G + (row_ok ? r - t * a.G : 0);
    uint64_t word = 0;
    if (row_ok) {
        word = a.tree_mask ? a.tree_mask[static_cast<size_t>(b) * a.T + t]
                           : (t >= 63 ? ~0ull : ((1ull << (t + 1)) - 1));
    }
    // the query rows are requested here and awaited after the first tiles have been requested too
    bf16x8 qreg[8];
    u32x4 qv[8];
    {
        const u32x4* qp = reinterpret_cast<const u32x4*>(
            static_cast<const uint16_t*>(a.q) + ((static_cast<size_t>(b) * a.T + t) * a.Hq + hq) * kD + lg * 8);
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            qv[kk] = u32x4{0u, 0u, 0u, 0u};
            if (row_ok) qv[kk] = qp[kk * 2];
        }
    }

    f32x16 acc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[dt][i] = 0.f;
    float m_run = kNegInf, l_run = 0.f, alpha = 1.f;

    // page ids, 64 at a time (lane l holds logical page cache_base + l), handed out with v_readlane.
    // With 16-token pages a tile is one even-numbered page and its successor, and windows start at even
    // pages, so one window test covers both; with larger pages a tile is 32 rows inside one page.
    const int32_t* __restrict__ table = a.block_table + static_cast<size_t>(b) * a.max_pages;
    const int last_page = (n - 1) >> page_shift;
    auto in_pool = [&](int pg, int idx) __attribute__((always_inline)) -> int {
        if (pg < 0 || pg >= a.num_pages) {
            if (idx <= last_page) bad_page = true;
            pg = min(max(pg, 0), a.num_pages - 1);
        }
        return pg;
    };
    // a piece that starts at its request's first tile finds that window of page ids fetched ahead
    const bool window_ahead = have_first && tok_begin == 0;
    int cache_base = window_ahead ? 0 : -0x40000000;
    int pg_cache = window_ahead ? in_pool(pg_first, lane) : 0;
    auto page_pair = [&](int tb, size_t& p0, size_t& p1) __attribute__((always_inline)) {
        const int lp = tb >> page_shift;
        if (lp < cache_base || lp >= cache_base + kWave) {   // uniform
            cache_base = lp;
            const int idx = cache_base + lane;
            pg_cache = in_pool(table[min(idx, a.max_pages - 1)], idx);
        }
        const int i0 = __builtin_amdgcn_readfirstlane(lp - cache_base);
        const int i1 = a.P == kMinPage ? i0 + 1 : i0;
        const uint32_t g0 = __builtin_amdgcn_readlane(pg_cache, i0), g1 = __builtin_amdgcn_readlane(pg_cache, i1);
        const uint32_t in_page = static_cast<uint32_t>(tb & (a.P - 1));              // first row of the tile in its page
        p0 = static_cast<uint64_t>(g0) * page_bytes32 + head_off + in_page * kRowBytes;
        p1 = static_cast<uint64_t>(g1) * page_bytes32 + head_off + ((in_page + 16u) & (a.P - 1)) * kRowBytes;
    };

    // loads of step j: K tile j + D and V tile j + D - 2, where they exist.  The V tile sits in
    // the same pages of its pool as the K tile issued two steps earlier, whose offsets are kept.
    size_t pq0 = 0, pq1 = 0, pr0 = 0, pr1 = 0;     // page offsets of the K tiles of steps j - 1 and j - 2
    size_t pn0 = 0, pn1 = 0;
    // Tiles that a neighbouring request reads too (the plan's shared_tiles: a leading run of the request) are
    // loaded with the default cache policy, which keeps them in the memory-side cache for the repeats; all
    // other tiles are read once and stream past the caches.  The policy is an instruction immediate, so a
    // load site either streams or decides per tile with a scalar branch.
    const int keep_until = shared_tiles - tok_begin / kTile;   // tiles of this piece below this index are kept
    using StreamLoads = std::false_type;
    using CheckLoads = std::true_type;
    auto issue_k_at = [&](int kt, int slot_bytes, auto mode) __attribute__((always_inline)) {
        page_pair(tok_begin + kt * kTile, pn0, pn1);
        if (decltype(mode)::value && kt < keep_until)
            issue_half_tile<NWT, 0>(lds + slot_bytes, wave, pn0, pn1, kbase, goff_k0, true);
        else
            issue_half_tile<NWT>(lds + slot_bytes, wave, pn0, pn1, kbase, goff_k0, true);
    };
    auto issue_v_at = [&](int vt, int slot_bytes, auto mode) __attribute__((always_inline)) {
        if (decltype(mode)::value && vt < keep_until)
            issue_half_tile<NWT, 0>(lds + kVRing + slot_bytes, wave, pr0, pr1, vbase, goff_v, false);
        else
            issue_half_tile<NWT>(lds + kVRing + slot_bytes, wave, pr0, pr1, vbase, goff_v, false);
    };
    auto shift_pages = [&]() __attribute__((always_inline)) { pr0 = pq0, pr1 = pq1, pq0 = pn0, pq1 = pn1; };
    auto issue_k = [&](int j) __attribute__((always_inline)) {
        const int kt = j + D;
        if (kt < n_tiles) issue_k_at(kt, (kt % NSLOT) * kKBytes, CheckLoads{});
    };
    auto issue_v = [&](int j) __attribute__((always_inline)) {
        const int vt = j + D - 2;
        if (vt >= 0 && vt < n_tiles) issue_v_at(vt, (vt % NSLOT) * kKBytes, CheckLoads{});
        shift_pages();
    };
    auto issue_step = [&](int j) __attribute__((always_inline)) {
        issue_k(j);
        issue_v(j);
    };
    // The loads of step u - D have landed when at most the loads of the D - 1 steps after it are
    // outstanding.  That count is a compile-time number only while those steps all issued a full
    // K and V half tile; at the two ends of a piece wait for everything instead.
    auto wait_step = [&](int u) __attribute__((always_inline)) {
        const bool full = D > 1 && u >= 1 && u + D - 1 < n_tiles;
        if (full) {
            if (REM == 0 || wave - Loaders<NWT>::kFirst < REM) wait_vmcnt<(D - 1) * 2 * CEIL>();
            else wait_vmcnt<(D - 1) * 2 * FLOOR>();
        } else {
            wait_vmcnt<0>();
        }
    };
    // visibility bits of tile j's 32 tokens for this lane's row, shifted to the lane's token half
    auto vis_of = [&](int j) __attribute__((always_inline)) -> uint32_t {
        const int rel = tok_begin + j * kTile - n0;          // uniform; in (-32, 64) for a masked tile
        if (rel <= -kTile) return ~0u;                        // a tile of prefix tokens only
        const uint32_t vis = rel >= 0 ? static_cast<uint32_t>(word >> rel)
                                      : (static_cast<uint32_t>(word << (-rel)) | ((1u << (-rel)) - 1u));
        return vis >> (lg * 4);
    };
    auto k_off = [&](int j) __attribute__((always_inline)) -> int { return (j % NSLOT) * kKBytes; };
    auto v_off = [&](int j) __attribute__((always_inline)) -> int {
        return (j % NSLOT) * kKBytes;              // (v_rd holds the ring's base)
    };

#pragma unroll
    for (int j = -D; j < 0; ++j) issue_step(j);
    {
        // Pin the point where the query rows and the mask word must have returned to HERE, before the tile
        // loop: left to itself the compiler waits for them at their first use inside the loop, with a wait
        // that also drains the direct-to-LDS loads of the tiles in flight, on every iteration.
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            asm volatile("" : "+v"(qv[kk]));
            qreg[kk] = as_bf16x8(qv[kk]);
        }
        uint32_t w_lo = static_cast<uint32_t>(word), w_hi = static_cast<uint32_t>(word >> 32);
        asm volatile("" : "+v"(w_lo), "+v"(w_hi));
        word = (static_cast<uint64_t>(w_hi) << 32) | w_lo;
        if (a.T < 64) word &= (1ull << a.T) - 1;
    }

    f32x16 s_a, s_b;
    uint32_t pk_a[8], pk_b[8];
#pragma unroll
    for (int i = 0; i < 16; ++i) s_a[i] = s_b[i] = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) pk_a[i] = pk_b[i] = 0u;

    // Ragged last tile of a request: slots past the end hold whatever the page holds (NaN included), and
    // 0 * NaN must not reach the output: clear those V rows in LDS.  Every wave of the workgroup calls this at
    // step n_tiles + 1, after that step's barrier and before its P.V product.
    auto clear_ragged_tail = [&]() __attribute__((always_inline)) {
        const int tb = tok_begin + (n_tiles - 1) * kTile;
        if (tb + kTile > n) {
            unsigned char* vl = lds + kVRing + ((n_tiles - 1) % NSLOT) * kKBytes;
            const int first_bad = n - tb;
            int tid_here = tid;                    // (address computed here, not carried through the tile loop)
            asm volatile("" : "+v"(tid_here));
            for (int c = tid_here; c < kTile * 16; c += NT)
                if ((c >> 4) >= first_bad) *reinterpret_cast<u32x4*>(vl + c * 16) = u32x4{0u, 0u, 0u, 0u};
            __builtin_amdgcn_s_waitcnt(0xc07f);    // lgkmcnt(0): the clears are done
            bare_barrier();
        }
    };

  if (helper) {
    // A helper wave: the same waits, barriers and loads as the main waves, step for step; of the arithmetic,
    // the tiles u = h (mod NH) for the leftover rows, one phase per step so that no step is much longer than the
    // others: scores at step u (K tile u is in its slot during that step only), softmax at step u + 1, P.V at
    // step u + 2 (V tile u has landed by then and is overwritten after step u + 3's barrier).
    if constexpr (NH > 0) {
        const int h = wave - NW;
        // (the helpers' phases are dependent chains that otherwise wait behind the main wave of their SIMD, which the
        // issue arbiter prefers as the older wave, and every wave then waits for them at the barrier)
        __builtin_amdgcn_s_setprio(3);
        for (int u = 0; u <= n_tiles + 1; ++u) {
            wait_step(u);
            bare_barrier();
            if (u == n_tiles + 1) clear_ragged_tail();
            if (u <= n_tiles) issue_step(u);
            if constexpr (!STREAM) {
                if (u >= 2 && ((u - 2) & (NH - 1)) == h)
                    pipe_step<false, false, true>(lds, 0, v_off(u - 2), k_rd, v_rd, qreg, s_b, s_b, pk_a, pk_b, acc, m_run, l_run,
                                                  alpha, a.scale_log2, 0u);
                if (u >= 1 && u <= n_tiles && ((u - 1) & (NH - 1)) == h) {
                    if (tok_begin + u * kTile <= n0)          // a tile of prefix tokens only: nothing to mask
                        pipe_step<false, true, false, false>(lds, 0, 0, k_rd, v_rd, qreg, s_a, s_b, pk_b, pk_a, acc, m_run, l_run,
                                                             alpha, a.scale_log2, 0u);
                    else
                        pipe_step<false, true, false>(lds, 0, 0, k_rd, v_rd, qreg, s_a, s_b, pk_b, pk_a, acc, m_run, l_run, alpha,
                                                      a.scale_log2, vis_of(u - 1));
                }
                if (u < n_tiles && (u & (NH - 1)) == h)
                    pipe_step<true, false, false>(lds, k_off(u), 0, k_rd, v_rd, qreg, s_b, s_a, pk_b, pk_b, acc, m_run, l_run, alpha,
                                                  a.scale_log2, 0u);
            }
        }
    }
  } else {
    // step 0: scores of tile 0 -> s_a
    wait_step(0);
    bare_barrier();
    issue_step(0);
    if constexpr (!STREAM)
        pipe_step<true, false, false>(lds, k_off(0), 0, k_rd, v_rd, qreg, s_b, s_a, pk_b, pk_a, acc, m_run, l_run, alpha,
                                      a.scale_log2, 0u);
    // step 1: softmax of tile 0 (s_a -> pk_a), scores of tile 1 -> s_b
    wait_step(1);
    bare_barrier();
    issue_step(1);
    {
        const uint32_t vis = vis_of(0);
        if constexpr (!STREAM) {
            if (n_tiles > 1)
                pipe_step<true, true, false>(lds, k_off(1), 0, k_rd, v_rd, qreg, s_a, s_b, pk_b, pk_a, acc, m_run,
                                             l_run, alpha, a.scale_log2, vis);
            else
                pipe_step<false, true, false>(lds, 0, 0, k_rd, v_rd, qreg, s_a, s_b, pk_b, pk_a, acc, m_run, l_run,
                                              alpha, a.scale_log2, vis);
        }
    }
    // steps 2 .. n_tiles - 1: P.V of tile u-2 (pk_a), softmax of tile u-1 (s_b -> pk_b), scores of tile u -> s_a,
    // after which the two register sets have swapped roles.  Tiles are masked from some tile on
    // (the draft slots are the last T positions), so the steps split into an unmasked run, taken
    // two steps per iteration so that the role swap costs no register moves, and a short masked run.
    auto full_step = [&](auto masked, int u, f32x16& s_sm, f32x16& s_qk, uint32_t (&pk_pv)[8],
                         uint32_t (&pk_sm)[8]) __attribute__((always_inline)) {
        wait_step(u);
        bare_barrier();                        // all waves: loads of step u - D landed, step u - 1 computed
        if constexpr (STREAM) {
            issue_k(u);
            issue_v(u);
        } else {
            fused_step<decltype(masked)::value, 0, 0>(
                k_off(u), v_off(u - 2), k_rd, v_rd, qreg, s_sm, s_qk, pk_pv, pk_sm, acc, m_run, l_run, alpha,
                a.scale_log2, decltype(masked)::value ? vis_of(u - 1) : 0u,
                [&]() __attribute__((always_inline)) { issue_k(u); },
                [&]() __attribute__((always_inline)) { issue_v(u); });
        }
    };
    auto swap_roles = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 16; ++i) { const float x = s_a[i]; s_a[i] = s_b[i]; s_b[i] = x; }
#pragma unroll
        for (int i = 0; i < 8; ++i) { const uint32_t x = pk_a[i]; pk_a[i] = pk_b[i]; pk_b[i] = x; }
    };
    {
        const int first_masked = n0 > tok_begin ? (n0 - tok_begin) / kTile : 0;   // first tile with masked slots
        const int u_split = min(max(first_masked + 1, 2), n_tiles);
        int u = 2;
        // Steady state proper: groups of P steps in which every load exists, every wait count is
        // the compile-time one, and (u = 2 mod NSLOT at the start of a group) every ring slot is
        // known at compile time.
        constexpr int P = NSLOT % 2 == 0 ? NSLOT : 2 * NSLOT;
        auto steady_step = [&](auto ic, auto mode) __attribute__((always_inline)) {
            constexpr int I = decltype(ic)::value;
            constexpr int kReadSlot = (2 + I) % NSLOT, kVReadSlot = I % NSLOT;
            constexpr int kIssueSlot = (1 + I) % NSLOT, kVIssueSlot = (I + NSLOT - 1) % NSLOT;
            if (REM == 0 || wave - Loaders<NWT>::kFirst < REM) wait_vmcnt<(D - 1) * 2 * CEIL>();
            else wait_vmcnt<(D - 1) * 2 * FLOOR>();
            bare_barrier();
            const int uu = u + I;
            auto ik = [&]() __attribute__((always_inline)) { issue_k_at(uu + D, kIssueSlot * kKBytes, mode); };
            auto iv = [&]() __attribute__((always_inline)) {
                issue_v_at(uu + D - 2, kVIssueSlot * kKBytes, mode);
                shift_pages();
            };
            if constexpr (STREAM) {
                ik();
                iv();
            } else if constexpr (I % 2 == 0)
                fused_step<false, kReadSlot * kKBytes, kVReadSlot * kKBytes>(
                    0, 0, k_rd, v_rd, qreg, s_b, s_a, pk_a, pk_b, acc, m_run, l_run, alpha, a.scale_log2, 0u, ik, iv);
            else
                fused_step<false, kReadSlot * kKBytes, kVReadSlot * kKBytes>(
                    0, 0, k_rd, v_rd, qreg, s_a, s_b, pk_b, pk_a, acc, m_run, l_run, alpha, a.scale_log2, 0u, ik, iv);
        };
        auto steady_checking = [&](auto ic) __attribute__((always_inline)) { steady_step(ic, CheckLoads{}); };
        auto steady_streaming = [&](auto ic) __attribute__((always_inline)) { steady_step(ic, StreamLoads{}); };
        constexpr bool kUnrolled = NSLOT * kKBytes <= 65536;
        const int u_steady_end = min(u_split, n_tiles - D);
        // groups that may still load a kept tile (the oldest tile a group loads is V tile u + D - 2) decide per
        // tile; behind the kept run every load streams
        if constexpr (kUnrolled)
            for (; u + P <= u_steady_end && u + D - 2 < keep_until; u += P)
                for_each_index(steady_checking, std::make_integer_sequence<int, P>{});
        if constexpr (kUnrolled)
            for (; u + P <= u_steady_end; u += P) for_each_index(steady_streaming, std::make_integer_sequence<int, P>{});
        for (; u + 1 < u_split; u += 2) {
            full_step(std::false_type{}, u, s_b, s_a, pk_a, pk_b);
            full_step(std::false_type{}, u + 1, s_a, s_b, pk_b, pk_a);
        }
        if (u < u_split) {
            full_step(std::false_type{}, u, s_b, s_a, pk_a, pk_b);
            swap_roles();
            ++u;
        }
        for (; u < n_tiles; ++u) {
            full_step(std::true_type{}, u, s_b, s_a, pk_a, pk_b);
            swap_roles();
        }
    }
    // now: s_b = scores of the last tile (if n_tiles > 1), pk_a = probabilities of tile n_tiles - 2
    if (n_tiles > 1) {
        const int u = n_tiles;
        wait_step(u);
        bare_barrier();
        issue_step(u);
        if constexpr (!STREAM)
            pipe_step<false, true, true>(lds, 0, v_off(u - 2), k_rd, v_rd, qreg, s_b, s_a, pk_a, pk_b, acc, m_run, l_run,
                                         alpha, a.scale_log2, vis_of(u - 1));
#pragma unroll
        for (int i = 0; i < 8; ++i) pk_a[i] = pk_b[i];
    }
    {
        const int u = n_tiles + 1;
        wait_step(u);
        bare_barrier();
        clear_ragged_tail();
        if constexpr (!STREAM)
            pipe_step<false, false, true>(lds, 0, v_off(n_tiles - 1), k_rd, v_rd, qreg, s_b, s_a, pk_a, pk_b, acc, m_run,
                                          l_run, alpha, a.scale_log2, 0u);
    }
  }  // main waves

    // ---- partial result: (reference exponent, sum, unnormalised O) per row ------------
    float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
    bool stores = row_ok;                           // this lane's row leaves from this wave
    if constexpr (NH > 0) {
        // The helpers' four states of the leftover rows become one.  Every wave takes part in the barriers.
        // LDS (the ring is free once every wave has passed the first barrier): (m, l) of every helper lane,
        // then the scaled accumulators of helpers 1..3, sixteen 16-byte chunks per lane, chunk-major so that
        // a wave's access is one contiguous kilobyte.
        float* xml = reinterpret_cast<float*>(lds);                                    // [NH][64][2]
        unsigned char* xacc = lds + 4096;                                              // [NH - 1][16][64] x 16 bytes
        static_assert(NH * kWave * 2 * 4 <= 4096 && kMergeBytes <= kLdsBytes, "the merge area fits the ring's memory");
        const int h = wave - NW;
        bare_barrier();                              // every wave has read the piece's last tiles
        if (helper) {
            xml[(h * kWave + lane) * 2] = m_run;
            xml[(h * kWave + lane) * 2 + 1] = l_tot;
        }
        __builtin_amdgcn_s_waitcnt(0xc07f);
        bare_barrier();
        if (helper) {
            float mh[NH], lh[NH];
#pragma unroll
            for (int i = 0; i < NH; ++i) {
                mh[i] = xml[(i * kWave + lane) * 2];
                lh[i] = xml[(i * kWave + lane) * 2 + 1];
            }
            float M = mh[0];
#pragma unroll
            for (int i = 1; i < NH; ++i) M = fmaxf(M, mh[i]);
            float L = 0.f;
#pragma unroll
            for (int i = 0; i < NH; ++i) L += (mh[i] == kNegInf) ? 0.f : lh[i] * fast_exp2(mh[i] - M);   // fixed order
            const float f = (m_run == kNegInf) ? 0.f : fast_exp2(m_run - M);
            m_run = M;
            l_tot = L;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[dt][i] = (f == 0.f) ? 0.f : acc[dt][i] * f;
            if (h > 0) {
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                    for (int i4 = 0; i4 < 4; ++i4) {
                        const f32x4 v = {acc[dt][i4 * 4], acc[dt][i4 * 4 + 1], acc[dt][i4 * 4 + 2], acc[dt][i4 * 4 + 3]};
                        *reinterpret_cast<f32x4*>(xacc + (((h - 1) * 16 + dt * 4 + i4) * kWave + lane) * 16) = v;
                    }
            }
        }
        __builtin_amdgcn_s_waitcnt(0xc07f);
        bare_barrier();
        if (helper && h == 0) {
#pragma unroll
            for (int o = 0; o < NH - 1; ++o)            // helper 1, then 2, then 3: a fixed order of additions
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                    for (int i4 = 0; i4 < 4; ++i4) {
                        const f32x4 v = *reinterpret_cast<const f32x4*>(xacc + ((o * 16 + dt * 4 + i4) * kWave + lane) * 16);
#pragma unroll
                        for (int c = 0; c < 4; ++c) acc[dt][i4 * 4 + c] += v[c];
                    }
        }
        stores = row_ok && (!helper || h == 0);
    }
    if (stores && lg == 0) {
        const size_t prow = (static_cast<size_t>(item_idx) * a.T + t) * a.Hq + hq;
        a.part_ml[2 * prow] = m_run;
        a.part_ml[2 * prow + 1] = l_tot;
    }
    auto store_partial = [&](float* dst, const f32x4& v) __attribute__((always_inline)) {
        // (a compile-time choice: in two arms of a run-time branch the compiler folds the two stores of the
        // same value into one plain store)
        if constexpr (STREAM_PARTIALS) __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(dst));
        else *reinterpret_cast<f32x4*>(dst) = v;
    };
    if constexpr (NW <= 2 && NW * 16384 <= 2 * NSLOT * kKBytes) {
        // The accumulators hold, per lane, 16-byte pieces of a row that lie 32 bytes apart; written out as they
        // are, one store instruction touches 32 rows with 32 bytes each.  Through the ring (free now: 16 KB per
        // wave, 16-byte chunks XORed with the row so that neither side has bank conflicts) every store
        // instruction writes two whole rows of 512 bytes.  Worth 0.6 % of the kernel on the memory-bound
        // two-wave shape (many short pieces); nothing measurable with three waves and more, which keep the
        // direct stores.
        bare_barrier();                                  // every wave has read the last tiles
        unsigned char* st = lds + wave * 16384;
        // (the addresses below are computed here, from a copy of the lane index the compiler cannot see through:
        // hoisted out of the piece loop they would hold registers through the tile loop, which has none to spare)
        int ln_here = ln;
        asm volatile("" : "+v"(ln_here));
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const f32x4 v = {acc[dt][i4 * 4], acc[dt][i4 * 4 + 1], acc[dt][i4 * 4 + 2], acc[dt][i4 * 4 + 3]};
                const int c = dt * 8 + i4 * 2 + lg;
                *reinterpret_cast<f32x4*>(st + ln_here * 512 + ((c ^ ln_here) << 4)) = v;
            }
        const int first_row = rb * a.rows_per_block + wave * 32;
#pragma unroll 2
        for (int k = 0; k < 16; ++k) {                   // (not unrolled further: sixteen rows in flight spill registers)
            const int rr = 2 * k + lg;                   // row of the wave; this lane moves chunk ln of it
            const f32x4 v = *reinterpret_cast<const f32x4*>(st + rr * 512 + ((ln_here ^ rr) << 4));
            const int r2 = first_row + rr;
            if (r2 < R) {
                const int t2 = r2 / a.G;
                const int hq2 = kvh * a.G + (r2 - t2 * a.G);
                const size_t prow = (static_cast<size_t>(item_idx) * a.T + t2) * a.Hq + hq2;
                store_partial(a.part_acc + prow * kD + ln * 4, v);
            }
        }
    } else if (stores) {
        int lg_here = lg;                                // (as above)
        asm volatile("" : "+v"(lg_here));
        const size_t prow = (static_cast<size_t>(item_idx) * a.T + t) * a.Hq + hq;
        float* __restrict__ po = a.part_acc + prow * kD + lg_here * 4;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const f32x4 v = {acc[dt][i4 * 4], acc[dt][i4 * 4 + 1], acc[dt][i4 * 4 + 2], acc[dt][i4 * 4 + 3]};
                store_partial(po + dt * 32 + i4 * 8, v);
            }
    }
  }  // pieces of the stretch
    if (bad_page && lane == 0) atomicOr(&a.header->status, 2u);
    // speed history for the next call's plan: tiles streamed and time taken, by stretch index
    if (L && !a.fixed_split && tid == 0) {
        const uint64_t ticks = __builtin_amdgcn_s_memrealtime() - clock_begin;
        atomicAdd(a.fb_time + wg, static_cast<uint32_t>(ticks > 0xffffffu ? 0xffffffu : ticks));
        atomicAdd(a.fb_tiles + wg, static_cast<uint32_t>(g_end - g_first));
    }
}

bool gqa128_supports(const AttnArgs& a) {
    return a.Dqk == kD && a.Dv == kD && a.P >= kMinPage && a.P <= 1024 && (a.P & (a.P - 1)) == 0 &&
           a.v_pages != nullptr && a.Hkv <= 65535;
}

// Ring depth of the helper shape: two tiles in flight.  Its eight waves spend their time on operand reads and on
// each other, not on waiting for tiles (measured per wave on the multi-path batch: 50 of a step's 2000 clocks), and
// with three tiles in flight instead of two the kernel is 4 % slower (1.28 vs 1.23 ms; rings of 5 and 7: as 3).
constexpr int kHelperDepth = 2;

hipError_t launch_gqa128(const AttnArgs& a, hipStream_t stream) {
    const int nw = a.rows_per_block / 32;
    const dim3 grid(static_cast<unsigned>((a.wgs_per_head + 7) / 8) * 8u * static_cast<unsigned>(a.Hkv) *
                    static_cast<unsigned>(a.row_blocks));
    // four main waves and four helpers instead of five waves: 129 .. 144 query rows in a row block (a fifth wave
    // would hold at most half of its rows)
    if (gqa_block_uses_helpers(a.rows_per_block)) {
        const dim3 block(8 * kWave);
        if (a.stream_only && a.stream_partials) hipLaunchKernelGGL((attn_gqa128_kernel<4, kHelperDepth, true, true, 4>), grid, block, 0, stream, a);
        else if (a.stream_only) hipLaunchKernelGGL((attn_gqa128_kernel<4, kHelperDepth, true, false, 4>), grid, block, 0, stream, a);
        else if (a.stream_partials) hipLaunchKernelGGL((attn_gqa128_kernel<4, kHelperDepth, false, true, 4>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((attn_gqa128_kernel<4, kHelperDepth, false, false, 4>), grid, block, 0, stream, a);
        return hipGetLastError();
    }
    switch (nw) {
#define SEER_GQA_LAUNCH(NW_, STREAM_, PARTIALS_)                                                               \
    hipLaunchKernelGGL((attn_gqa128_kernel<NW_, gqa_pipe_depth(NW_), STREAM_, PARTIALS_>), grid, dim3(NW_ * kWave), 0, \
                       stream, a)
#define SEER_GQA_CASE(NW_)                                                                                     \
    case NW_:                                                                                                  \
        if (a.stream_only && a.stream_partials) SEER_GQA_LAUNCH(NW_, true, true);                              \
        else if (a.stream_only) SEER_GQA_LAUNCH(NW_, true, false);                                             \
        else if (a.stream_partials) SEER_GQA_LAUNCH(NW_, false, true);                                         \
        else SEER_GQA_LAUNCH(NW_, false, false);                                                               \
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
#undef SEER_GQA_LAUNCH
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace seer
