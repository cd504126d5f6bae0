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
// lengths, so it cannot size partitions without a synchronisation).  The plan
// kernel cuts every request into partitions of about equal length such that
// the launch has enough workgroups to fill 256 CUs however the lengths are
// distributed -- a batch of a few 100k-token stragglers and a batch of several
// hundred short requests both end up with a few thousand workgroups.
struct PlanHeader {
    uint32_t status;     // bit 0: bad ctx_len somewhere; bit 1: page id out of range
    int32_t n_items;     // number of (request, partition) items
    int32_t part_len;    // nominal partition length in tokens
    int32_t reserved;
};

struct WorkItem {
    int32_t b;       // request
    int32_t begin;   // first logical KV position of the partition
    int32_t end;     // one past the last
    int32_t split;   // partition index inside the request
};

constexpr int kPartAlign = 256;        // partition lengths are multiples of this many tokens
constexpr int kDefaultMaxSplits = 256;
constexpr int kTargetWorkgroups = 2048;  // aimed-at (item x kv-head) workgroups per launch

struct WorkspaceLayout {
    int max_items;
    int target_items;    // (request, partition) items the plan aims for
    int max_splits;
    size_t off_header, off_split, off_items, off_ml, off_acc, total;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Host-only arithmetic; the plan kernel is given the same numbers.
inline WorkspaceLayout workspace_layout(const seer_attn_params& p) {
    WorkspaceLayout w{};
    w.max_splits = p.max_splits > 0 ? p.max_splits : kDefaultMaxSplits;
    w.target_items = kTargetWorkgroups / p.Hkv;
    if (w.target_items < 1) w.target_items = 1;
    // sum_b ceil(n_b / L) <= sum_b n_b / L + B <= target_items + B
    const int64_t bound = static_cast<int64_t>(w.target_items) + p.B;
    const int64_t cap = static_cast<int64_t>(p.B) * w.max_splits;
    w.max_items = static_cast<int>(bound < cap ? bound : cap);
    const size_t rows = static_cast<size_t>(w.max_items) * p.T * p.Hq;
    w.off_header = 0;
    w.off_split = 256;
    w.off_items = align_up(w.off_split + sizeof(int32_t) * (static_cast<size_t>(p.B) + 1), 256);
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
    const int32_t* split_off;   // [B+1]
    const WorkItem* items;
    float* part_ml;             // [max_items][T][Hq][2]  (running max in log2 units, sum)
    float* part_acc;            // [max_items][T][Hq][Dv] unnormalised
    int32_t B, T, Hq, Hkv, G, Dqk, Dv, P, num_pages, max_pages, max_items;
    float scale_log2;           // scale * log2(e): scores are kept in base-2 units
};

hipError_t launch_plan(const AttnArgs& a, const WorkspaceLayout& w, hipStream_t stream);
hipError_t launch_general(const AttnArgs& a, hipStream_t stream);   // any supported shape
hipError_t launch_combine(const AttnArgs& a, hipStream_t stream);
bool general_supports(int Dqk, int Dv);
bool gqa128_supports(const AttnArgs& a);                            // D = 128, 16-token pages, G*T <= 256
hipError_t launch_gqa128(const AttnArgs& a, hipStream_t stream);

}  // namespace seer
