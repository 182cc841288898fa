// Internal layout of bs_tilemap, shared by the host builder and the HIP launcher.
#pragma once
#include <cstdint>
#include <vector>

#include "blindsight.h"

namespace bs {

// Per-token code consumed by the kernel's element predicate:
//   bits 0..29  imgid (0 = text), bit 30 = sink key, bit 31 = text key.
constexpr uint32_t kCodeImgMask = 0x3fffffffu;
constexpr uint32_t kCodeSink = 1u << 30;
constexpr uint32_t kCodeText = 1u << 31;

// Half-open run of key tiles [begin, end) that all share one state.
struct TileRange {
    int32_t begin;
    int32_t end_state;  // (end << 1) | (1 if FULL, 0 if PARTIAL)
    int32_t end() const { return end_state >> 1; }
    bool full() const { return end_state & 1; }
};

struct ClassLists {
    std::vector<int64_t> row_ptr;     // M + 1 offsets into ranges
    std::vector<TileRange> ranges;
    std::vector<int32_t> row_tiles;   // visited tiles per query tile (scheduling weight)
    int64_t visited = 0, full = 0, partial = 0, allowed_pairs = 0, empty_rows = 0;
};

struct WorkItem { int32_t head, q_tile; };

// Work unit of the bf16 kernel: two (head, query tile) items that read the SAME KV head and walk
// one merged key-tile list, so a workgroup streams each K / V tile once for both.
//   item B is absent when head_b < 0.
struct PairItem {
    int32_t head_a, tile_a, head_b, tile_b;
    int32_t list_begin, list_end;  // entries of PairPlan::ranges
    int32_t n_tiles;               // key tiles in the merged list (scheduling weight)
    int32_t classes;               // head class of item A | head class of item B << 8
};

// Run of key tiles [begin, end) with one state per item: 0 skip, 1 partial, 2 full.
struct PairRange {
    int32_t begin;
    int32_t end_states;  // (end << 4) | (state_a << 2) | state_b
};

struct PairPlan {
    int32_t gqa_group = 0;  // the plan depends on which heads share a KV head ...
    uint64_t epoch = 0;     // ... and on the class vector (bs_tilemap::class_epoch when it was made)
    std::vector<PairRange> ranges;
    std::vector<PairItem> items;  // eight queues, one per XCD, each heaviest first
    int32_t queue_off[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};   // queue x = items[queue_off[x] .. queue_off[x + 1])
};

struct DeviceMap;  // defined by the HIP side

}  // namespace bs

// Pair up the work items for KV-sharing workgroups (host only; see PairItem).
void bs_plan_pairs(bs_tilemap *tm, int32_t gqa_group);
// The plain work list of the fp32 kernel: every (head, query tile), heaviest first (host only).
void bs_plan_work(bs_tilemap *tm);

struct bs_tilemap {
    int32_t L = 0, bm = 0, bn = 0, M = 0, N = 0, n_q_heads = 0, sink_len = 0;
    // Key tiles: ids [0, N0) are the prompt's keys in position order; with packed keys, ids
    // [N0, N) are compact tiles holding the free keys (text and sink keys) in position order.
    int32_t N0 = 0;
    bool packed = false;
    bool bidir = false;                    // image tokens also attend to the later tokens of their own image
    int32_t window = 0;                    // > 0: sliding window, keys with i - j >= window are masked
    int32_t q_begin = 0;                   // the query rows are positions q_begin .. L - 1 (q / out hold L - q_begin rows per head)
    bool intra_compact = false;            // packed: Intra-Image rows take their text keys from the compact tiles
    std::vector<int32_t> key_order;        // N * bn: position of each key-tile slot, -1 = none
    std::vector<int32_t> free_before;      // packed: L + 1, free keys at positions < t
    std::vector<int32_t> span_free_range;  // packed: 2 * (G + 1), compact slots [lo, hi) of the free keys inside span g (1-based)
    std::vector<bs_span> spans;
    std::vector<uint8_t> head_class;
    std::vector<int32_t> row_order;        // M * bm: position of each query-tile row, -1 = no row
    bool regrouped = false;                // row_order is not the natural order
    std::vector<uint32_t> code;            // L
    std::vector<uint64_t> text_bits;       // N: bit b of entry n = key n*bn + b is a text key (bn <= 64 only)
    std::vector<uint64_t> sink_bits;       // N: same for sink keys
    bs::ClassLists cls[4];
    uint64_t class_epoch = 1;              // bumped by bs_tilemap_rebind: work list, work units and their device copies are stale
    std::vector<bs::WorkItem> work;        // n_q_heads * M items, heaviest first; built on first use (work_epoch)
    uint64_t work_epoch = 0;
    bs::PairPlan pairs;                    // built on first use for a given gqa_group and class vector
    bs::DeviceMap *dev = nullptr;          // created lazily by bs_tilemap_upload
    void (*dev_free)(bs::DeviceMap *) = nullptr;
};
