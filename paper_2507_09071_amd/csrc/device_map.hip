// Device memory for tile maps: block cache, pinned staging, upload of the two parts of a map.
//
// A serving loop builds a tile map per prompt and binds it to one class vector per layer.
// hipMalloc / hipFree per map would cost more than the pre-pass kernels and hipFree would drain
// the device, so the blocks a destroyed map held go back to a small per-process cache instead,
// tagged with an event recorded on the stream that last used them; the next owner's stream waits
// for that event before touching the block.  Host-to-device copies are assembled in place in a
// ring of pinned buffers and queued on the caller's stream, so nothing here blocks the host or
// drains the device once the cache is warm.  Cached blocks and pinned buffers are kept until the
// process ends.
#include "device_map.h"

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

namespace bs {

thread_local char g_last_error[256] = "";

int fail_hip(hipError_t e, const char *what)
{
    snprintf(g_last_error, sizeof g_last_error, "%s: %s (%d)", what, hipGetErrorString(e), (int)e);
    (void)hipGetLastError();
    return e == hipErrorOutOfMemory ? BS_ENOMEM : BS_EHIP;
}

int fail_msg(int code, const char *what)
{
    snprintf(g_last_error, sizeof g_last_error, "%s", what);
    return code;
}

namespace {

struct CachedBlock {
    int device;
    void *ptr;
    size_t cap;
    std::shared_ptr<EventHolder> released;   // last use of the block by its previous owner (may be null: never used)
};
struct StagingBuffer {
    void *host = nullptr;
    size_t cap = 0;
    hipEvent_t done = nullptr;   // the copy out of this buffer
    bool queued = false;         // a copy out of this buffer has been queued (done is recorded)
    bool in_use = false;         // a host thread is filling it
};
constexpr size_t kCacheMaxBlocks = 24;
constexpr int kStagingBuffers = 8;
std::mutex g_mem_mutex;
// never destroyed: at process exit the HIP runtime may already be gone
std::vector<CachedBlock> &g_cache = *new std::vector<CachedBlock>();
StagingBuffer g_staging[kStagingBuffers];
int g_staging_next = 0;
std::vector<void *> &g_outgrown = *new std::vector<void *>();   // pinned buffers replaced by larger ones

constexpr size_t kGranule = (size_t)1 << 20;
size_t round_up(size_t x, size_t g) { return (x + g - 1) / g * g; }

}  // namespace

hipError_t pool_acquire(int device, size_t bytes, hipStream_t st, void **out, size_t *cap_out)
{
    const size_t want = round_up(std::max<size_t>(bytes, 1), kGranule);
    {
        std::lock_guard<std::mutex> lock(g_mem_mutex);
        size_t best = g_cache.size();
        for (size_t i = 0; i < g_cache.size(); ++i)
            if (g_cache[i].device == device && g_cache[i].cap >= want && g_cache[i].cap <= 2 * want &&
                (best == g_cache.size() || g_cache[i].cap < g_cache[best].cap))
                best = i;
        if (best < g_cache.size()) {
            const CachedBlock b = g_cache[best];
            g_cache.erase(g_cache.begin() + best);
            const hipError_t e = b.released ? hipStreamWaitEvent(st, b.released->ev, 0) : hipSuccess;
            if (e != hipSuccess) { (void)hipFree(b.ptr); return e; }
            *out = b.ptr; *cap_out = b.cap;
            return hipSuccess;
        }
    }
    hipError_t e = hipMalloc(out, want);
    if (e == hipSuccess) *cap_out = want;
    return e;
}

void pool_release(int device, void *ptr, size_t cap, const std::shared_ptr<EventHolder> &last_use)
{
    if (!ptr) return;
    void *drop = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_mem_mutex);
        g_cache.push_back({device, ptr, cap, last_use});
        if (g_cache.size() > kCacheMaxBlocks) {   // drop the oldest block
            drop = g_cache.front().ptr;
            g_cache.erase(g_cache.begin());
        }
    }
    if (drop) (void)hipFree(drop);   // waits for the block's users; outside the lock
}

hipError_t staging_begin(size_t bytes, Staging *out)
{
    StagingBuffer *sb = nullptr;
    int slot = -1;
    hipEvent_t wait_for = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_mem_mutex);
        for (int i = 0; i < kStagingBuffers && !sb; ++i) {
            const int c = (g_staging_next + i) % kStagingBuffers;
            if (!g_staging[c].in_use) { sb = &g_staging[c]; slot = c; }
        }
        if (!sb) return hipErrorNotReady;   // more than kStagingBuffers host threads inside an upload
        g_staging_next = (slot + 1) % kStagingBuffers;
        sb->in_use = true;
        if (sb->queued) wait_for = sb->done;
    }
    // the copy that last read this buffer must be over (it was queued several uploads ago); the
    // wait happens outside the lock, the buffer is reserved by in_use
    hipError_t e = wait_for ? hipEventSynchronize(wait_for) : hipSuccess;
    if (e == hipSuccess && sb->cap < bytes) {
        // Grow in powers of two and keep the outgrown buffer (hipHostFree drains the device, which
        // would stall the caller behind every kernel it has queued): the buffers a slot has outgrown
        // add up to less than the one it holds.
        size_t cap = kGranule;
        while (cap < bytes) cap *= 2;
        void *grown = nullptr;
        e = hipHostMalloc(&grown, cap, hipHostMallocDefault);
        if (e == hipSuccess) {
            if (sb->host) {
                std::lock_guard<std::mutex> lock(g_mem_mutex);
                g_outgrown.push_back(sb->host);
            }
            sb->host = grown;
            sb->cap = cap;
        }
    }
    if (e == hipSuccess && !sb->done) {
        e = hipEventCreateWithFlags(&sb->done, hipEventDisableTiming);
        if (e != hipSuccess) sb->done = nullptr;
    }
    if (e != hipSuccess) {
        std::lock_guard<std::mutex> lock(g_mem_mutex);
        sb->in_use = false;
        return e;
    }
    out->host = sb->host;
    out->slot = slot;
    return hipSuccess;
}

hipError_t staging_commit(const Staging &s, void *dst, size_t bytes, hipStream_t st)
{
    StagingBuffer &sb = g_staging[s.slot];
    hipError_t e = bytes ? hipMemcpyAsync(dst, sb.host, bytes, hipMemcpyHostToDevice, st) : hipSuccess;
    if (e == hipSuccess) e = hipEventRecord(sb.done, st);
    std::lock_guard<std::mutex> lock(g_mem_mutex);
    sb.queued = (e == hipSuccess);
    sb.in_use = false;
    return e;
}

void staging_abandon(const Staging &s)
{
    if (s.slot < 0) return;
    std::lock_guard<std::mutex> lock(g_mem_mutex);
    g_staging[s.slot].in_use = false;
}

void free_device_map(DeviceMap *d)
{
    if (!d) return;
    int cur = -1;
    (void)hipGetDevice(&cur);
    if (d->device >= 0 && cur != d->device) (void)hipSetDevice(d->device);
    pool_release(d->device, d->blob, d->blob_cap, d->last_use);
    pool_release(d->device, d->bind_blob, d->bind_cap, d->last_use);
    pool_release(d->device, d->vt_buf, d->vt_bytes, d->last_use);
    if (cur >= 0 && cur != d->device) (void)hipSetDevice(cur);
    delete d;
}

int order_after_last_use(DeviceMap *d, hipStream_t st)
{
    if (d->last_stream == st) return BS_OK;
    // the buffers of the map were last written or read on another stream: order this call after that
    const hipError_t e = hipStreamWaitEvent(st, d->last_use->ev, 0);
    if (e != hipSuccess) return fail_hip(e, "hipStreamWaitEvent");
    d->last_stream = st;
    return BS_OK;
}

namespace {
size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
}

int upload_prompt_part(bs_tilemap *tm, hipStream_t st)
{
    if (!tm) return BS_EINVAL;
    if (tm->dev) return BS_OK;
    if (tm->bn > 64) return BS_EUNSUPPORTED;  // the per-tile key bit masks are 64 wide
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");

    const int64_t M1 = (int64_t)tm->M + 1;
    int64_t total_ranges = 0;
    for (int c = 0; c < 4; ++c) total_ranges += (int64_t)tm->cls[c].ranges.size();
    if (total_ranges >= INT32_MAX) return BS_EUNSUPPORTED;
    const size_t G1 = tm->spans.size() + 1;

    const size_t off_code = 0;
    const size_t off_rows = align256(off_code + (size_t)tm->L * 4);
    const size_t off_keys = align256(off_rows + tm->row_order.size() * 4);
    const size_t off_fbefore = align256(off_keys + tm->key_order.size() * 4);
    const size_t off_sfree = align256(off_fbefore + std::max<size_t>(tm->free_before.size(), 1) * 4);
    const size_t off_tbits = align256(off_sfree + std::max<size_t>(tm->span_free_range.size(), 2) * 4);
    const size_t off_sbits = align256(off_tbits + (size_t)tm->N * 8);
    const size_t off_spans = align256(off_sbits + (size_t)tm->N * 8);
    const size_t off_rowptr = align256(off_spans + G1 * 8);
    const size_t off_ranges = align256(off_rowptr + (size_t)(4 * M1) * 4);
    const size_t bytes = align256(off_ranges + (size_t)std::max<int64_t>(total_ranges, 1) * 8);

    DeviceMap *d = new (std::nothrow) DeviceMap();
    std::shared_ptr<EventHolder> holder;
    try {
        holder = std::make_shared<EventHolder>();
    } catch (const std::bad_alloc &) {
    }
    if (!d || !holder) { delete d; return BS_ENOMEM; }
    Staging sg;
    e = staging_begin(bytes, &sg);
    if (e != hipSuccess) { delete d; return fail_hip(e, "pinned staging buffer"); }
    unsigned char *host = static_cast<unsigned char *>(sg.host);
    std::memcpy(host + off_code, tm->code.data(), (size_t)tm->L * 4);
    std::memcpy(host + off_rows, tm->row_order.data(), tm->row_order.size() * 4);
    std::memcpy(host + off_keys, tm->key_order.data(), tm->key_order.size() * 4);
    if (!tm->free_before.empty()) std::memcpy(host + off_fbefore, tm->free_before.data(), tm->free_before.size() * 4);
    if (!tm->span_free_range.empty())
        std::memcpy(host + off_sfree, tm->span_free_range.data(), tm->span_free_range.size() * 4);
    else
        std::memset(host + off_sfree, 0, 8);
    std::memcpy(host + off_tbits, tm->text_bits.data(), (size_t)tm->N * 8);
    std::memcpy(host + off_sbits, tm->sink_bits.data(), (size_t)tm->N * 8);
    int2 *sp = reinterpret_cast<int2 *>(host + off_spans);
    sp[0] = make_int2(0, 0);
    for (size_t g = 0; g < tm->spans.size(); ++g) sp[g + 1] = make_int2(tm->spans[g].start, tm->spans[g].end);
    int32_t *rp = reinterpret_cast<int32_t *>(host + off_rowptr);
    int2 *rg = reinterpret_cast<int2 *>(host + off_ranges);
    int64_t base = 0;
    for (int c = 0; c < 4; ++c) {
        const ClassLists &cl = tm->cls[c];
        for (int64_t m = 0; m < M1; ++m) rp[c * M1 + m] = (int32_t)(base + cl.row_ptr[m]);
        static_assert(sizeof(TileRange) == sizeof(int2), "range lists are copied as they are");
        if (!cl.ranges.empty()) std::memcpy(rg + base, cl.ranges.data(), cl.ranges.size() * sizeof(TileRange));
        base += (int64_t)cl.ranges.size();
    }

    void *blob = nullptr;
    size_t blob_cap = 0;
    e = pool_acquire(dev, bytes, st, &blob, &blob_cap);
    if (e != hipSuccess) {
        staging_abandon(sg);
        delete d;
        return fail_hip(e, "hipMalloc(tile map)");
    }
    e = staging_commit(sg, blob, bytes, st);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&holder->ev, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventRecord(holder->ev, st);
    if (e != hipSuccess) {
        (void)hipFree(blob);
        delete d;
        return fail_hip(e, "hipMemcpyAsync(tile map)");
    }
    unsigned char *b = static_cast<unsigned char *>(blob);
    d->device = dev;
    d->blob = blob;
    d->blob_cap = blob_cap;
    d->last_stream = st;
    d->last_use = holder;
    d->code = reinterpret_cast<const uint32_t *>(b + off_code);
    d->row_order = reinterpret_cast<const int32_t *>(b + off_rows);
    d->key_order = reinterpret_cast<const int32_t *>(b + off_keys);
    d->free_before = reinterpret_cast<const int32_t *>(b + off_fbefore);
    d->span_free = reinterpret_cast<const int2 *>(b + off_sfree);
    d->text_bits = reinterpret_cast<const uint64_t *>(b + off_tbits);
    d->sink_bits = reinterpret_cast<const uint64_t *>(b + off_sbits);
    d->span_range = reinterpret_cast<const int2 *>(b + off_spans);
    d->row_ptr = reinterpret_cast<const int32_t *>(b + off_rowptr);
    d->ranges = reinterpret_cast<const int2 *>(b + off_ranges);
    tm->dev = d;
    tm->dev_free = free_device_map;
    return BS_OK;
}

int upload_binding(bs_tilemap *tm, int32_t kind, int32_t gqa_group, hipStream_t st)
{
    DeviceMap *d = tm->dev;
    if (!d) return BS_EINVAL;
    if (kind == kBindWorkList) gqa_group = 0;   // the work list does not depend on it
    if (d->bind_kind == kind && d->bind_G == gqa_group && d->bind_epoch == tm->class_epoch) return BS_OK;
    try {
        if (kind == kBindPairPlan) bs_plan_pairs(tm, gqa_group);
        else bs_plan_work(tm);
    } catch (const std::bad_alloc &) {
        return BS_ENOMEM;
    }
    const PairPlan &plan = tm->pairs;
    if (kind == kBindPairPlan && plan.ranges.size() >= (size_t)INT32_MAX) return BS_EUNSUPPORTED;
    const size_t n_heads = tm->head_class.size();
    const size_t off_class = 0;
    const size_t off_a = align256(off_class + n_heads);    // work list, or work units
    const size_t a_bytes = kind == kBindPairPlan ? plan.items.size() * sizeof(PairItem) : tm->work.size() * sizeof(WorkItem);
    const size_t off_b = align256(off_a + a_bytes);        // ranges of the work units
    const size_t b_bytes = kind == kBindPairPlan ? std::max<size_t>(plan.ranges.size(), 1) * sizeof(PairRange) : 0;
    const size_t off_q = align256(off_b + b_bytes);        // queue offsets [9], then queue counters [8]
    const size_t bytes = align256(off_q + 256);

    Staging sg;
    hipError_t e = staging_begin(bytes, &sg);
    if (e != hipSuccess) return fail_hip(e, "pinned staging buffer");
    unsigned char *host = static_cast<unsigned char *>(sg.host);
    std::memcpy(host + off_class, tm->head_class.data(), n_heads);
    if (kind == kBindPairPlan) {
        static_assert(sizeof(PairItem) == 2 * sizeof(int4) && sizeof(PairRange) == sizeof(int2), "copied as they are");
        std::memcpy(host + off_a, plan.items.data(), a_bytes);
        if (!plan.ranges.empty()) std::memcpy(host + off_b, plan.ranges.data(), plan.ranges.size() * sizeof(PairRange));
        std::memset(host + off_q, 0, 256);
        std::memcpy(host + off_q, plan.queue_off, sizeof plan.queue_off);
    } else {
        static_assert(sizeof(WorkItem) == sizeof(int2), "copied as it is");
        std::memcpy(host + off_a, tm->work.data(), a_bytes);
    }
    // a fresh block every time: kernels of an earlier binding may still be reading the old one,
    // which goes back to the cache behind the map's last-use event
    void *blob = nullptr;
    size_t cap = 0;
    e = pool_acquire(d->device, bytes, st, &blob, &cap);
    if (e != hipSuccess) {
        staging_abandon(sg);
        return fail_hip(e, "hipMalloc(work units)");
    }
    e = staging_commit(sg, blob, bytes, st);
    if (e != hipSuccess) {
        (void)hipFree(blob);
        return fail_hip(e, "hipMemcpyAsync(work units)");
    }
    if (d->bind_blob) {
        // the event object is shared with the cached block, and recorded again by later launches
        // of this map: the block then simply waits a little longer than it has to
        pool_release(d->device, d->bind_blob, d->bind_cap, d->last_use);
    }
    unsigned char *b = static_cast<unsigned char *>(blob);
    d->bind_blob = blob;
    d->bind_cap = cap;
    d->bind_kind = kind;
    d->bind_G = gqa_group;
    d->bind_epoch = tm->class_epoch;
    d->head_class = b + off_class;
    d->work = kind == kBindWorkList ? reinterpret_cast<const int2 *>(b + off_a) : nullptr;
    d->n_work = kind == kBindWorkList ? (int32_t)tm->work.size() : 0;
    d->pair_items = kind == kBindPairPlan ? reinterpret_cast<const int4 *>(b + off_a) : nullptr;
    d->pair_ranges = kind == kBindPairPlan ? reinterpret_cast<const int2 *>(b + off_b) : nullptr;
    d->n_pairs = kind == kBindPairPlan ? (int32_t)plan.items.size() : 0;
    d->queue_off = kind == kBindPairPlan ? reinterpret_cast<const int32_t *>(b + off_q) : nullptr;
    d->queue_ctr = kind == kBindPairPlan ? reinterpret_cast<int32_t *>(b + off_q + 64) : nullptr;
    return BS_OK;
}

}  // namespace bs
