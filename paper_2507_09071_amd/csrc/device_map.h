// Device-side copy of a tile map and the memory plumbing around it (internal to the library).
//
// A map has two parts on the device.  The PROMPT part depends on the span table and the map
// options only (token codes, row and key order, key bit masks, the four per-class range lists):
// it is uploaded once and serves every layer of the model.  The BINDING part depends on the class
// vector the map is bound to (and, for the bf16 kernel, on the GQA group size): the head classes
// and the work list or work units.  bs_tilemap_rebind only invalidates the binding part.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <memory>

#include "tilemap_internal.h"

namespace bs {

// Detail of the last failure on this thread, for bs_last_error().
extern thread_local char g_last_error[256];

// Records `what` and the HIP error string, clears HIP's sticky error, returns BS_ENOMEM or BS_EHIP.
int fail_hip(hipError_t e, const char *what);
// Records a plain message for bs_last_error() and returns `code`.
int fail_msg(int code, const char *what);

// An event that dies with its last owner (a map, or cached blocks that wait to be reused).
struct EventHolder {
    hipEvent_t ev = nullptr;
    ~EventHolder() { if (ev) (void)hipEventDestroy(ev); }
};

enum BindingKind : int32_t { kBindNone = 0, kBindWorkList = 1, kBindPairPlan = 2 };

struct DeviceMap {
    int device = -1;
    // ---- prompt part: one block, uploaded once
    void *blob = nullptr;
    size_t blob_cap = 0;
    const uint32_t *code = nullptr;       // [L] per-token code
    const int32_t *row_order = nullptr;   // [M * 128] position of each query-tile row, -1 = none
    const int32_t *key_order = nullptr;   // [N * 64] position of each key-tile slot, -1 = none
    const int32_t *free_before = nullptr; // packed: [L + 1]
    const int2 *span_free = nullptr;      // packed: [G + 1] compact slots of the free keys inside each image
    const uint64_t *text_bits = nullptr;  // [N] text keys of each key tile
    const uint64_t *sink_bits = nullptr;  // [N] sink keys of each key tile
    const int2 *span_range = nullptr;     // [G + 1] (start, end) by imgid; entry 0 unused
    const int32_t *row_ptr = nullptr;     // [4][M + 1] offsets into ranges
    const int2 *ranges = nullptr;         // concatenated over classes
    // ---- binding part: one block, uploaded again after a rebind / for another kind or group size
    void *bind_blob = nullptr;
    size_t bind_cap = 0;
    int32_t bind_kind = kBindNone;
    int32_t bind_G = 0;
    uint64_t bind_epoch = 0;              // class_epoch of the map the binding was made for
    const uint8_t *head_class = nullptr;  // [Hq]
    const int2 *work = nullptr;           // fp32 kernel: [n_work] (head, query tile)
    int32_t n_work = 0;
    const int4 *pair_items = nullptr;     // bf16 kernel: work units, two int4 each
    const int2 *pair_ranges = nullptr;
    int32_t n_pairs = 0;
    const int32_t *queue_off = nullptr;   // [9] the units of XCD x are pair_items[queue_off[x] .. queue_off[x + 1])
    int32_t *queue_ctr = nullptr;         // [8] next unit of each queue; cleared by the pre-pass of every call
    // ---- bf16 workspace: packed K tiles, then packed V^T tiles, of the last call
    void *vt_buf = nullptr;
    size_t vt_bytes = 0;
    hipStream_t last_stream = nullptr;    // stream of the most recent upload / launch (compared, never used)
    std::shared_ptr<EventHolder> last_use;   // recorded after the most recent upload / launch
};

// A device block of at least `bytes`, safe to use in work queued on `st` after this call.  Blocks
// come from a per-process cache of blocks that destroyed maps gave back (no hipMalloc / hipFree in
// a steady serving loop); the stream waits for the previous owner's last use.
hipError_t pool_acquire(int device, size_t bytes, hipStream_t st, void **out, size_t *cap_out);
// Hand a block back; `last_use` is the event after which nobody reads or writes it any more.
void pool_release(int device, void *ptr, size_t cap, const std::shared_ptr<EventHolder> &last_use);

// Host-to-device copies without blocking the host on the device: the caller fills a pinned buffer
// in place (staging_begin), the copy is queued on the caller's stream (staging_commit).
struct Staging {
    void *host = nullptr;
    int slot = -1;
};
hipError_t staging_begin(size_t bytes, Staging *out);
hipError_t staging_commit(const Staging &s, void *dst, size_t bytes, hipStream_t st);
void staging_abandon(const Staging &s);

// Upload the prompt part (once per map) / the binding part (when stale) on `st`; no host-side wait.
int upload_prompt_part(bs_tilemap *tm, hipStream_t st);
int upload_binding(bs_tilemap *tm, int32_t kind, int32_t gqa_group, hipStream_t st);
// Order work queued on `st` after the map's previous use if that was on another stream.
int order_after_last_use(DeviceMap *d, hipStream_t st);

void free_device_map(DeviceMap *d);

}  // namespace bs
