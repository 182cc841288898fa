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

struct DeviceMap;  // defined by the HIP side

}  // namespace bs

struct bs_tilemap {
    int32_t L = 0, bm = 0, bn = 0, M = 0, N = 0, n_q_heads = 0, sink_len = 0;
    std::vector<bs_span> spans;
    std::vector<uint8_t> head_class;
    std::vector<uint32_t> code;            // L
    std::vector<uint64_t> text_bits;       // N: bit b of entry n = key n*bn + b is a text key (bn <= 64 only)
    std::vector<uint64_t> sink_bits;       // N: same for sink keys
    bs::ClassLists cls[4];
    std::vector<bs::WorkItem> work;        // n_q_heads * M items, heaviest first
    bs::DeviceMap *dev = nullptr;          // created lazily by bs_tilemap_upload
    void (*dev_free)(bs::DeviceMap *) = nullptr;
};
