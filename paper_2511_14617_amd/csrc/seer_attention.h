// Internal declarations shared by the verify-attention sources: the split-K
// plan that lives at the head of the caller's workspace, and the launchers of
// the individual kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/seer_verify.h"

namespace seer {

// Split-K work is planned ON THE DEVICE from ctx_len (the host never sees the
// lengths, so it cannot size partitions without a synchronisation).
//
// Balanced ("stream") partitioning: per KV head, the 32-token tiles of all
// requests are laid end to end, request after request, and that line is cut
// into W stretches, one per workgroup.  W x Hkv is chosen to be what the GPU
// holds at once, so there is a single round of workgroups and every one of
// them streams about the same number of KV bytes, whatever the mix of lengths
// -- eight 100k-token stragglers and several hundred short requests both fill
// all 256 CUs.  A stretch that crosses a request boundary yields one partial
// result per request it touches; request b therefore owns
// n_parts(b) = last_wg(b) - first_wg(b) + 1 consecutive partial slots starting at
// split_off[b], and the combine kernel merges them.
//
// Stretch lengths follow the measured speed of each workgroup slot.  Workgroups
// that stream the same number of bytes do not finish together: on this part the
// eight XCDs differ by about 12 % in sustained gather bandwidth, and of two
// workgroups resident on one CU the one dispatched first is served first.  Both
// are properties of the workgroup's index (the grid is laid out so that the
// workgroups with the same stretch index w, one per KV head, share XCD and
// dispatch round), and stable from call to call.  So every partition workgroup
// adds its tiles and its duration (constant 100 MHz clock) to two counters of
// its stretch index in the workspace, and the next call's plan cuts the line in
// proportion to the smoothed tiles-per-time of each index (clamped to
// [3/4, 4/3] of the mean).  A workspace that holds no valid history (first use,
// other W) gives equal stretches; SEER_ATTN_FIXED_SPLIT always does.
struct PlanHeader {
    uint32_t status;     // bit 0: bad ctx_len somewhere; bit 1: page id out of range
    int32_t n_items;     // number of (request, stretch) pieces = partial slots in use
    int32_t tiles_per_wg;  // L; 0 = one workgroup per request (max_splits == 1)
    int32_t total_tiles;   // tiles per KV head over all requests
    uint32_t fb_magic;     // kFeedbackMagic once the speed history below the header is meaningful
    int32_t fb_w;          // W it was recorded for
};
constexpr uint32_t kFeedbackMagic = 0x5ee2fb01u;
constexpr int kMaxWgsPerHead = 1024;   // 256 CUs x 4 resident workgroups, one KV head

struct WorkItem {
    int32_t b;       // request
    int32_t begin;   // first logical KV position of the piece
    int32_t end;     // one past the last
    int32_t split;   // index of the piece inside the request
};

constexpr int kPlanTile = 32;          // tokens per scheduling tile
constexpr int kMinTilesPerWg = 4;      // do not cut finer than 128 tokens
constexpr int kDefaultMaxSplits = 256;
constexpr int kNumCU = 256;            // MI355X

struct WorkspaceLayout {
    int max_items;
    int wgs_per_head;    // W (balanced mode) or B (one workgroup per request)
    int max_splits;
    size_t off_header, off_split, off_tiles, off_first, off_start, off_reqfirst, off_shared, off_fb, off_items, off_ml, off_acc, total;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Ring depth D of the tiled GQA kernel (tiles in flight per workgroup while one is computed;
// the K ring and the V ring have D + 1 slots of 8 KB each), by waves per workgroup.  Two-wave
// workgroups run four to a CU and keep one tile in flight each; larger ones run at most two to a CU.
// Measured on the 8B- to 72B-class shapes: between depths 1 and 4 the time changes by a few per cent only.
constexpr int gqa_pipe_depth(int waves) { return waves <= 2 ? 1 : 3; }

// Partial results of the tiled D = 128 kernel are written with non-temporal stores while all of them are
// small: measured on the 8B-class shapes, the partition kernel of the grouped-rollout batch (28 MB of
// partials) is 2.7 % faster with them and the call 2 %, the long-tail batch (20 MB) does not care, and the
// multi-path batch (86 MB) loses 1 % of the call, because the combine kernel then fetches from DRAM what it
// would otherwise find in the memory-side cache.
constexpr size_t kStreamPartialsBelow = size_t{64} << 20;

// The tiled D = 128 kernel handles up to 256 query rows (8 waves) of a KV head per workgroup; a request
// with more rows per KV head (large groups of heads times a wide draft tree) is cut into row blocks of
// equal size, each a workgroup of its own walking the same stretch (placed on the same XCD, so all but
// the first find the tiles in that XCD's L2).
inline bool gqa_page_size_ok(int P) { return P >= 16 && P <= 1024 && (P & (P - 1)) == 0; }
inline int gqa_row_blocks(int rows) { return (rows + 255) / 256; }
// A row block of 129 .. 144 rows is served by four main waves plus four helper waves that share the leftover rows
// (see the kernel) instead of by a fifth wave; such a block keeps its exact row count.
inline bool gqa_block_uses_helpers(int rows_per_block) { return rows_per_block > 128 && rows_per_block <= 144; }
inline int gqa_rows_per_block(int rows) {
    const int nb = gqa_row_blocks(rows);
    const int per = (rows + nb - 1) / nb;
    return gqa_block_uses_helpers(per) ? per : (per + 31) / 32 * 32;
}
inline int gqa_waves_per_block(int rows_per_block) { return gqa_block_uses_helpers(rows_per_block) ? 8 : rows_per_block / 32; }

// Workgroups of the partition kernel that one CU holds at once, by kernel shape.
inline int resident_wgs_per_cu(const seer_attn_params& p) {
    const bool tiled = p.Dqk == 128 && p.Dv == 128 && gqa_page_size_ok(p.page_size) && !p.kv_shared_latent &&
                       !(p.flags & SEER_ATTN_GENERAL_KERNEL);
    if (!tiled) return 4;
    const int waves = gqa_waves_per_block(gqa_rows_per_block((p.Hq / p.Hkv) * p.T));   // one wave per 32 query rows
    const int by_waves = 8 / waves;                       // 2 waves per SIMD, 4 SIMDs
    const int depth = gqa_pipe_depth(waves);
    // 160 KB of LDS per CU, 16 KB per ring slot pair; five 32 KB workgroups would need all of it and
    // do not become resident together (measured: a fifth of the grid ran as a second round)
    const int by_lds = 159 / (16 * (depth + 1));
    return by_waves < 1 ? 1 : (by_waves < by_lds ? by_waves : by_lds);
}

// Host-only arithmetic; the plan kernel is given the same numbers.
inline WorkspaceLayout workspace_layout(const seer_attn_params& p) {
    WorkspaceLayout w{};
    w.max_splits = p.max_splits > 0 ? p.max_splits : kDefaultMaxSplits;
    if (w.max_splits == 1) {
        w.wgs_per_head = p.B;
        w.max_items = p.B;
    } else {
        const bool mla_tiled = p.Dqk == 576 && p.Dv == 512 && p.page_size >= 32 && gqa_page_size_ok(p.page_size) && p.kv_shared_latent &&
                               !(p.flags & SEER_ATTN_GENERAL_KERNEL);
        if (mla_tiled) {
            // one 4-wave workgroup per CU; a request's rows are cut into blocks of 128, and the
            // row-block workgroups of one stretch are launched as a group on one XCD (groups of 8 stretches)
            const int row_blocks = ((p.Hq / p.Hkv) * p.T + 127) / 128;
            w.wgs_per_head = 8 * (kNumCU / (8 * row_blocks * p.Hkv));
            if (w.wgs_per_head < 1) w.wgs_per_head = kNumCU / (row_blocks * p.Hkv);
        } else {
            const bool tiled = p.Dqk == 128 && p.Dv == 128 && gqa_page_size_ok(p.page_size) && !p.kv_shared_latent &&
                               !(p.flags & SEER_ATTN_GENERAL_KERNEL);
            const int row_blocks = tiled ? gqa_row_blocks((p.Hq / p.Hkv) * p.T) : 1;
            w.wgs_per_head = kNumCU * resident_wgs_per_cu(p) / (p.Hkv * row_blocks);
        }
        if (w.wgs_per_head < 1) w.wgs_per_head = 1;
        // a stretch adds one piece per request boundary it crosses: pieces <= W + B
        w.max_items = w.wgs_per_head + p.B;
    }
    const size_t rows = static_cast<size_t>(w.max_items) * p.T * p.Hq;
    const size_t per_b = sizeof(int32_t) * (static_cast<size_t>(p.B) + 1);
    w.off_header = 0;
    w.off_split = 256;
    w.off_tiles = align_up(w.off_split + per_b, 256);
    w.off_first = align_up(w.off_tiles + per_b, 256);
    const size_t per_w = sizeof(int32_t) * (static_cast<size_t>(w.wgs_per_head) + 1);
    w.off_start = align_up(w.off_first + per_w, 256);
    w.off_reqfirst = align_up(w.off_start + per_w, 256);
    w.off_shared = align_up(w.off_reqfirst + per_b, 256);
    w.off_fb = align_up(w.off_shared + per_b, 256);               // time[W], tiles[W], smoothed speed[W]
    w.off_items = align_up(w.off_fb + 3 * per_w, 256);
    w.off_ml = align_up(w.off_items + sizeof(WorkItem) * static_cast<size_t>(w.max_items), 256);
    w.off_acc = align_up(w.off_ml + 2 * sizeof(float) * rows, 256);
    w.total = align_up(w.off_acc + sizeof(float) * rows * p.Dv, 256);
    return w;
}

// Everything a kernel needs, by value.
struct AttnArgs {
    void* out;
    const void* q;
    const void* k_pages;
    const void* v_pages;     // nullptr: shared latent
    const int32_t* block_table;
    const int32_t* ctx_len;
    const uint64_t* tree_mask;
    PlanHeader* header;
    const int32_t* split_off;   // [B+1] first partial slot of each request
    const int32_t* tile_off;    // [B+1] first tile of each request on the per-head tile line
    const int32_t* wg_first;    // [wgs_per_head] request in which each workgroup's stretch starts, -1 = idle
    const int32_t* wg_start;    // [wgs_per_head + 1] first tile of each stretch on the tile line (balanced mode)
    const int32_t* req_first;   // [B] first stretch that touches each request (balanced mode)
    const int32_t* shared_tiles;  // [B] leading tiles of each request whose pages a neighbouring request maps too
    uint32_t* fb_time;          // [wgs_per_head] sum over KV heads of the workgroup's duration, 10 ns ticks
    uint32_t* fb_tiles;         // [wgs_per_head] sum over KV heads of the tiles it streamed
    float* fb_speed;            // [wgs_per_head] smoothed tiles per tick (owned by the plan kernel)
    int32_t fixed_split;        // 1: equal stretches, no history read or written
    int32_t stream_only;        // 1: the tiled D = 128 kernel only streams its tiles (diagnostic)
    int32_t stream_partials;    // 1: the tiled D = 128 kernel writes its partial results with non-temporal stores
    int32_t row_blocks, rows_per_block;   // tiled D = 128 kernel: workgroups per (stretch, KV head), rows of each
    const WorkItem* items;
    float* part_ml;             // [max_items][T][Hq][2]  (running max in log2 units, sum)
    float* part_acc;            // [max_items][T][Hq][Dv] unnormalised
    int32_t B, T, Hq, Hkv, G, Dqk, Dv, P, num_pages, max_pages, max_items, wgs_per_head;
    float scale_log2;           // scale * log2(e): scores are kept in base-2 units
};

hipError_t launch_plan(const AttnArgs& a, const WorkspaceLayout& w, hipStream_t stream);
hipError_t launch_general(const AttnArgs& a, hipStream_t stream);   // any supported shape
hipError_t launch_combine(const AttnArgs& a, hipStream_t stream);
bool general_supports(int Dqk, int Dv);
bool gqa128_supports(const AttnArgs& a);                            // D = 128, pages of 16..1024 tokens (power of two)
hipError_t launch_gqa128(const AttnArgs& a, hipStream_t stream);
bool mla_supports(const AttnArgs& a);                               // shared latent 576/512, pages of 32..1024 tokens
hipError_t launch_mla(const AttnArgs& a, hipStream_t stream);

}  // namespace seer
