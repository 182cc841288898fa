// Sparse causal prefill attention for gfx950 (MI355X): one flash-style pass over the key tiles
// the tile map lists for each (head, query tile).
//
// What is computed: paper Sec. 3.1 (softmax(QK^T * scale + mask) V) with the per-class masks of
// Sec. 3.2.  The tiled recurrence (running max, running sum, rescaled output) is the one of
// App. kernel Alg. 4-7; the four subroutines of Alg. 3 collapse into one loop because the tile
// map already says which key tiles a query tile visits and whether a visited tile needs the
// element predicate (PARTIAL) or not (FULL).  One softmax runs per row over the union of all
// visited keys, and the output is divided by the running sum at the end.
//
// Mapping to CDNA4:
//  * a workgroup of four 64-lane waves owns one 128-row query tile of one head; wave w owns
//    rows 32w..32w+31 and keeps its Q rows in registers for the whole pass;
//  * scores are produced transposed, S^T = K Q^T, with 32x32x16 bf16 MFMA tiles, so every lane
//    holds 16 keys of ONE query per 32-key block: row max / row sum are in-lane reductions plus
//    one exchange with the lane 32 apart (v_permlane32_swap);
//  * O^T = V^T P^T reuses the score registers, rounded to bf16, as the B operand;
//  * K and V tiles travel global -> LDS with 16-byte LDS-direct loads (no VGPR staging) into a
//    two-stage ring, one barrier per tile; rows are unpadded and XOR-swizzled so both the
//    128-bit K fragment reads and the 64-bit transposing V reads (ds_read_b64_tr_b16) are free
//    of bank conflicts;
//  * PARTIAL tiles build one 64-bit allowed-key word per lane from per-tile text/sink bit
//    masks, the query's own image range and the causal bound, then test one bit per score.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <new>
#include <type_traits>
#include <vector>

#include "tilemap_internal.h"

namespace bs {

// Detail of the last failure on this thread, for bs_last_error().
thread_local char g_last_error[256] = "";

static int fail_hip(hipError_t e, const char *what)
{
    snprintf(g_last_error, sizeof g_last_error, "%s: %s (%d)", what, hipGetErrorString(e), (int)e);
    (void)hipGetLastError();
    return e == hipErrorOutOfMemory ? BS_ENOMEM : BS_EHIP;
}

struct DeviceMap {
    int device = -1;
    void *blob = nullptr;                 // one allocation holding everything below
    const uint32_t *code = nullptr;       // [L] per-token code
    const uint64_t *text_bits = nullptr;  // [N] text keys of each key tile
    const uint64_t *sink_bits = nullptr;  // [N] sink keys of each key tile
    const int2 *span_range = nullptr;     // [G+1] (start, end) by imgid; entry 0 unused
    const int32_t *row_ptr = nullptr;     // [4][M+1] offsets into ranges
    const int32_t *row_tiles = nullptr;   // [4][M] visited key tiles per query tile
    const int2 *ranges = nullptr;         // concatenated over classes
    const int2 *work = nullptr;           // [n_work] (head, q_tile)
    const uint8_t *head_class = nullptr;  // [Hq]
    int32_t n_work = 0;
};

// Read-only tile-map arrays; passed as separate __restrict__ kernel parameters so that loads
// with wave-uniform addresses go through the scalar cache (they then never wait on the vector
// memory counter that tracks the in-flight LDS-direct loads).
struct KernelArgs {
    const void *q, *k, *v;
    void *out;
    int32_t L, M, G;
    float scale_log2e;  // scale * log2(e): softmax runs in the exp2 domain
};
#define BS_MAP_PARAMS                                                                              \
    const uint32_t *__restrict__ map_code, const uint64_t *__restrict__ map_text_bits,             \
        const uint64_t *__restrict__ map_sink_bits, const int2 *__restrict__ map_span_range,       \
        const int32_t *__restrict__ map_row_ptr, const int2 *__restrict__ map_ranges,              \
        const int2 *__restrict__ map_work, const uint8_t *__restrict__ map_head_class
#define BS_MAP_ARGS(d) (d)->code, (d)->text_bits, (d)->sink_bits, (d)->span_range, (d)->row_ptr, (d)->ranges, (d)->work, (d)->head_class

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kBlockM = 128, kBlockN = 64, kThreads = 256;

// Walks the key tiles of one (class, query tile): ranges of [begin, end) with a FULL flag.
struct TileWalker {
    const int2 *__restrict__ rg;
    int p, p_end, n, n_end;
    bool full;
    __device__ void load()
    {
        if (p < p_end) {
            // wave-uniform by construction; say so, so the loads go through the scalar cache
            const int2 r = rg[__builtin_amdgcn_readfirstlane(p)];
            n = __builtin_amdgcn_readfirstlane(r.x);
            n_end = __builtin_amdgcn_readfirstlane(r.y) >> 1;
            full = __builtin_amdgcn_readfirstlane(r.y) & 1;
        }
    }
    __device__ void init(const int2 *__restrict__ ranges, int begin, int end)
    {
        rg = ranges;
        p = __builtin_amdgcn_readfirstlane(begin);
        p_end = __builtin_amdgcn_readfirstlane(end);
        load();
    }
    __device__ bool valid() const { return p < p_end; }
    __device__ void next()
    {
        if (++n == n_end) { ++p; load(); }
    }
};

// What the lane's query may see (paper Sec. 3.2), in a form that is cheap to apply per tile.
struct QueryView {
    int32_t row;       // query position i
    int32_t own_lo;    // own image [own_lo, own_hi) if the class attends inside images, else empty
    int32_t own_hi;
    bool sees_all;     // text query or Dense head: every earlier key
    __device__ void init(const uint32_t *__restrict__ code, const int2 *__restrict__ span_range, int L, int cls, int32_t i)
    {
        row = i;
        const uint32_t qcode = i < L ? code[i] : kCodeText;
        sees_all = (qcode & kCodeText) || cls == BS_DENSE;
        own_lo = own_hi = 0;
        if (!sees_all && (cls & 2)) {
            const int2 sp = span_range[qcode & kCodeImgMask];
            own_lo = sp.x; own_hi = sp.y;
        }
    }
};

__device__ inline uint64_t bits_below(int x)  // bits [0, x), x in [0, 64]
{
    return x >= 64 ? ~0ull : ((1ull << x) - 1ull);
}

// Bit b set <=> key n0 + b is allowed for this lane's query.  tbits / sbits: text keys and
// (class-enabled) sink keys of the tile.
__device__ inline uint64_t allowed_keys(const QueryView &qv, uint64_t tbits, uint64_t sbits, int n0)
{
    const uint64_t base = qv.sees_all ? ~0ull : (tbits | sbits);
    const int lo = min(max(qv.own_lo - n0, 0), 64), hi = min(max(qv.own_hi - n0, 0), 64);
    const uint64_t own = bits_below(hi) & ~bits_below(lo);
    const int cz = min(max(qv.row - n0 + 1, 0), 64);  // causal: keys n0 .. row
    return (base | own) & bits_below(cz);
}

// Score block layout (two 32x32 MFMA C tiles): lane (hl = lane/32, col = lane%32) holds, for
// query col, keys 32*kb + 8*(v/4) + 4*hl + v%4, v = 0..15.
__device__ inline void apply_mask(floatx16 (&s)[2], uint64_t allowed, int hl)
{
    const uint32_t w[2] = {(uint32_t)allowed >> (4 * hl), (uint32_t)(allowed >> 32) >> (4 * hl)};
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const uint32_t bit = 1u << (8 * (v / 4) + (v % 4));
            s[kb][v] = (w[kb] & bit) ? s[kb][v] : -INFINITY;
        }
}

__device__ inline float max_across_halves(float x)
{
    // r[0] = (x.lo, x.lo), r[1] = (x.hi, x.hi): both halves see both values
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

__device__ inline float sum_across_halves(float x)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Online-softmax update (running max m, running sum l, rescale factor alpha; App. kernel
// Alg. 4) in the exp2 domain: p = exp2(s*c - m*c).  l is the lane's partial sum (its 32 keys);
// the halves are added once, in the epilogue.  MAY_BE_EMPTY guards rows with no allowed key
// so far (m = -inf), which only PARTIAL tiles can produce.
template <bool MAY_BE_EMPTY>
__device__ inline void softmax_block(floatx16 (&s)[2], float &m_run, float &l_run, float &alpha, float c)
{
    float mx = fmaxf(s[0][0], s[0][1]);
#pragma unroll
    for (int v = 2; v < 16; v += 2) mx = fmaxf(fmaxf(mx, s[0][v]), s[0][v + 1]);
#pragma unroll
    for (int v = 0; v < 16; v += 2) mx = fmaxf(fmaxf(mx, s[1][v]), s[1][v + 1]);
    mx = max_across_halves(mx);
    const float m_new = fmaxf(m_run, mx);
    const float m_use = (MAY_BE_EMPTY && m_new == -INFINITY) ? 0.f : m_new;
    const float mc = m_use * c;
    alpha = __builtin_amdgcn_exp2f(fmaf(m_run, c, -mc));  // m_run = -inf -> 0
    float sum0 = 0.f, sum1 = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const float p0 = __builtin_amdgcn_exp2f(fmaf(s[0][v], c, -mc));
        const float p1 = __builtin_amdgcn_exp2f(fmaf(s[1][v], c, -mc));
        s[0][v] = p0; s[1][v] = p1;
        sum0 += p0; sum1 += p1;
    }
    l_run = fmaf(l_run, alpha, sum0 + sum1);
    m_run = m_new;
}

typedef __attribute__((address_space(3))) void *lds_void_ptr;
typedef const __attribute__((address_space(1))) void *global_void_ptr;

// ------------------------------------------------------------------------------------ bf16
//
// LDS operand reads of the MFMA phase are issued through inline asm and waited for by hand
// (lds_wait<N>): the compiler would otherwise tie every LDS read to the LDS-direct loads that
// are in flight into the other ring slot and drain the vector-memory counter before it.

// 64-bit transposing LDS read: within each group of 16 lanes, lane i receives element i%4 of
// the 8-byte words addressed by lanes i/4, 4 + i/4, 8 + i/4, 12 + i/4.
template <int OFFSET>
__device__ inline void lds_read_tr16(shortx4 &dst, uint32_t addr)
{
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFFSET));
}

template <int OFFSET>
__device__ inline void lds_read_b128(bf16x8 &dst, uint32_t addr)
{
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFFSET));
}

// Wait until at most N LDS operations are outstanding.  The operands tie the wait to the
// registers it protects, so their consumers cannot be scheduled above it.
template <int N>
__device__ inline void lds_wait(shortx4 (&a)[8])
{
    asm volatile("s_waitcnt lgkmcnt(%8)"
                 : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7])
                 : "n"(N));
}
template <int N>
__device__ inline void lds_wait(bf16x8 (&a)[4])
{
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]) : "n"(N));
}

// LDS swizzles: row r of a tile stores its logical 16-byte chunk c at chunk c ^ f(r).
template <int D> __device__ inline int k_swizzle(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
template <int D> __device__ inline int v_swizzle(int row) { return D == 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2); }

constexpr int kPingPongThreads = 512;

// Optional phase timing (build with -DBS_PHASE_TIMING): wave 0 of every workgroup adds the
// cycles it spent in phase X, the barrier after X, phase Y and the barrier after Y.
#ifdef BS_PHASE_TIMING
__device__ unsigned long long g_phase_cycles[8];
__device__ inline unsigned long long bs_now(floatx16 &a, floatx16 &b, floatx16 &c)
{
    // the ties make the stamp wait for the MFMAs that produce these accumulators
    asm volatile("" : "+v"(a), "+v"(b), "+v"(c));
    unsigned long long t;
    asm volatile("s_memtime %0\n\ts_waitcnt lgkmcnt(0)" : "=s"(t));
    return t;
}
#define BS_T0() unsigned long long bs_acc[4] = {0, 0, 0, 0}; unsigned long long bs_t0 = bs_now(s[0], s[1], o[0])
#define BS_TICK(slot)                                                                  \
    do {                                                                               \
        const unsigned long long bs_t1 = bs_now(s[0], s[1], o[0]);                     \
        bs_acc[slot] += bs_t1 - bs_t0;                                                 \
        bs_t0 = bs_t1;                                                                 \
    } while (0)
#define BS_TFLUSH()                                                                    \
    do {                                                                               \
        if (tid == 0 || tid == 256)                                                    \
            for (int i = 0; i < 4; ++i) atomicAdd(&g_phase_cycles[i + 4 * (tid >> 8)], bs_acc[i]); \
    } while (0)
#else
#define BS_T0() do {} while (0)
#define BS_TICK(slot) do {} while (0)
#define BS_TFLUSH() do {} while (0)
#endif

template <int D>
constexpr int bf16_lds_bytes() { return 2 /*groups*/ * 4 /*2 K + 2 V slots*/ * kBlockN * D * 2; }

// One workgroup = two groups of four waves.  Each group owns one (head, query tile) work item
// and a private K/V ring (2 K slots + 2 V slots).  Per key tile a group runs two phases:
//   X (matrix):  O += P(k-1) V(k-1)  and  S(k) = K(k) Q^T        -- MFMA + LDS reads only
//   Y (vector):  mask, online softmax of S(k) -> P(k), rescale O  -- VALU only
// separated by workgroup barriers.  The second group starts half a step late, so on every SIMD
// one wave is in X while the other is in Y: the matrix pipe and the vector ALU stay busy
// together instead of the two waves queueing for the same unit.
template <int D>
__global__ __launch_bounds__(kPingPongThreads, 2) void attn_prefill_bf16(KernelArgs a, BS_MAP_PARAMS,
                                                                         const int32_t *__restrict__ map_row_tiles,
                                                                         int32_t n_work)
{
    constexpr int ROW = D * 2;            // bytes per K / V row in LDS
    constexpr int TILE = kBlockN * ROW;   // bytes per K or V tile
    constexpr int CPR = D / 8;            // 16-byte chunks per row
    constexpr int DMA_PER_THREAD = D / 32;  // LDS-direct loads per thread per matrix per tile
    constexpr int NDB = D / 32;           // 32-channel blocks of the output
    constexpr int NT = D / 16;            // 16-wide slices of the head dim
    extern __shared__ __align__(1024) unsigned char lds[];

    const int tid = threadIdx.x, lane = tid & 63, hl = lane >> 5, col = lane & 31;
    const int grp = __builtin_amdgcn_readfirstlane(tid >> 8);          // wave group 0 / 1
    const int wave = __builtin_amdgcn_readfirstlane((tid >> 6) & 3);   // wave within the group
    const int L = a.L;

    // this group's work item, and the step count both groups must agree on
    int my_tiles = 0, other_tiles = 0, head = 0, m = 0, cls = 0;
    {
        const int mine = 2 * blockIdx.x + grp, other = 2 * blockIdx.x + (grp ^ 1);
        if (mine < n_work) {
            const int2 it = map_work[mine];
            head = it.x; m = it.y; cls = map_head_class[head];
            my_tiles = map_row_tiles[cls * a.M + m];
        }
        if (other < n_work) {
            const int2 it = map_work[other];
            other_tiles = map_row_tiles[map_head_class[it.x] * a.M + it.y];
        }
    }
    const bool have_item = 2 * blockIdx.x + grp < n_work;
    // wave-uniform by construction; say so, so that addresses built from them stay scalar
    head = __builtin_amdgcn_readfirstlane(head);
    m = __builtin_amdgcn_readfirstlane(m);
    cls = __builtin_amdgcn_readfirstlane(cls);
    const int T = __builtin_amdgcn_readfirstlane(my_tiles);
    const int n_steps = (max(T, __builtin_amdgcn_readfirstlane(other_tiles)) + 2) & ~1;  // even, >= T + 1
    const int kvh = __builtin_amdgcn_readfirstlane(head / a.G);
    const int row = m * kBlockM + wave * 32 + col;

    const __bf16 *qh = reinterpret_cast<const __bf16 *>(a.q) + (size_t)head * L * D;
    const __bf16 *kh = reinterpret_cast<const __bf16 *>(a.k) + (size_t)kvh * L * D;
    const __bf16 *vh = reinterpret_cast<const __bf16 *>(a.v) + (size_t)kvh * L * D;

    // Q^T operand: lane holds Q[row][16t + 8hl .. +8] for every 16-wide slice t of the head dim.
    bf16x8 qreg[NT];
    {
        const int qrow = min(row, L - 1);  // rows past the end compute on a copy and are not stored
#pragma unroll
        for (int t = 0; t < NT; ++t)
            qreg[t] = *reinterpret_cast<const bf16x8 *>(qh + (size_t)qrow * D + 16 * t + 8 * hl);
    }
    QueryView qv;
    qv.init(map_code, map_span_range, L, cls, row);

    // LDS byte addresses of this lane's MFMA operand fragments inside the group's ring.
    //   ring layout: K slot 0, K slot 1, V slot 0, V slot 1 (TILE bytes each)
    //   K fragment t: row col (+32 kb), logical chunk 2t + hl
    //   V fragment (transposing read, per 16-lane group: 4 keys x 16 channels): lane j of the
    //   group addresses key j/4 of the group's 4 keys and channels 4(j%4)..+3 of its 16
    const uint32_t ring = (uint32_t)(uintptr_t)(lds_void_ptr)lds + grp * 4 * TILE;
    //   the swizzles only touch address bits that t (bits 5-7) and db (bits 6-7) also select,
    //   so fragment t / block db sits at the base address XOR (t << 5) / (db << 6)
    const uint32_t kaddr0 = ring + col * ROW + ((hl ^ k_swizzle<D>(col)) << 4);
    uint32_t vaddr0;
    {
        const int j = lane & 15, g16 = (lane >> 4) & 1, key = 4 * hl + (j >> 2);
        vaddr0 = ring + 2 * TILE + key * ROW + (((2 * g16 + ((j & 3) >> 1)) ^ v_swizzle<D>(key)) << 4) + 8 * (j & 1);
    }

    floatx16 o[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
    floatx16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
    bf16x8 pf[2][2];   // P^T of the previous tile as MFMA B operands
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) pf[i >> 1][i & 1][e] = (__bf16)0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // tile walkers: wk runs one tile ahead (K loads), wv names the tile of the current step
    TileWalker wk, wv;
    {
        const int rb = map_row_ptr[cls * (a.M + 1) + m], re = have_item ? map_row_ptr[cls * (a.M + 1) + m + 1] : rb;
        wk.init(map_ranges, rb, re);
        wv.init(map_ranges, rb, re);
    }

    // Start the LDS-direct loads of one K or V tile into a ring slot.  Each wave instruction
    // fills 1 KB of contiguous LDS (lane l -> bytes 16l..16l+15), i.e. 1024/ROW tile rows; the
    // swizzle is applied on the global side by choosing which chunk of the row a lane fetches.
    // Instruction r of wave w covers tile rows (4r + w) * RPI + lane / CPR; neither swizzle
    // depends on r, so one per-lane byte offset serves all r (the rest is scalar arithmetic).
    constexpr int RPI = 1024 / ROW;  // tile rows per wave instruction
    const int dma_row0 = wave * RPI + lane / CPR;
    const int dma_cp = lane % CPR;
    const uint32_t dma_off_k = dma_row0 * ROW + ((dma_cp ^ k_swizzle<D>(dma_row0)) << 4);
    const uint32_t dma_off_v = dma_row0 * ROW + ((dma_cp ^ v_swizzle<D>(dma_row0)) << 4);
    auto issue_tile = [&](const __bf16 *src, int n, int slot_byte, bool is_v) {
#ifdef BS_PROBE_SAME_TILE
        n = n & 7;
#endif
        const int n0 = n * kBlockN;
        const char *tile = reinterpret_cast<const char *>(src) + (size_t)n0 * ROW;
        unsigned char *dst0 = lds + grp * 4 * TILE + slot_byte + wave * 1024;
        if (n0 + kBlockN <= L) {
            const uint32_t off = is_v ? dma_off_v : dma_off_k;
#pragma unroll
            for (int r = 0; r < DMA_PER_THREAD; ++r)
                __builtin_amdgcn_global_load_lds((global_void_ptr)(tile + (off + r * 4 * 1024)),
                                                 (lds_void_ptr)(dst0 + r * 4 * 1024), 16, 0, 0);
        } else {
            // ragged last tile: rows past the end fetch the last row (masked by causality)
            const int last = L - 1 - n0;
#pragma unroll
            for (int r = 0; r < DMA_PER_THREAD; ++r) {
                const int trow = r * 4 * RPI + dma_row0;
                const int sw = is_v ? v_swizzle<D>(trow) : k_swizzle<D>(trow);
                const uint32_t off = min(trow, last) * ROW + ((dma_cp ^ sw) << 4);
                __builtin_amdgcn_global_load_lds((global_void_ptr)(tile + off),
                                                 (lds_void_ptr)(dst0 + r * 4 * 1024), 16, 0, 0);
            }
        }
    };

    // ---- phase X building blocks (PAR = parity of the step: K slot PAR, V slot PAR ^ 1) ----
    auto read_pv = [&](auto par, auto g, shortx4 (&dst)[8]) {
        constexpr int base = (decltype(par)::value ^ 1) * TILE + decltype(g)::value * 16 * ROW;
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
            lds_read_tr16<base>(dst[2 * db], vaddr0 ^ (db << 6));
            lds_read_tr16<base + 8 * ROW>(dst[2 * db + 1], vaddr0 ^ (db << 6));
        }
    };
    auto mul_pv = [&](auto g, shortx4 (&f)[8]) {
        constexpr int G = decltype(g)::value;
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
            const bf16x8 va = __builtin_bit_cast(bf16x8, __builtin_shufflevector(f[2 * db], f[2 * db + 1], 0, 1, 2, 3, 4, 5, 6, 7));
            o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pf[G >> 1][G & 1], o[db], 0, 0, 0);
        }
    };
    // S batch b covers head-dim slices 2b, 2b+1 for both 32-key blocks
    auto read_s = [&](auto par, auto b, bf16x8 (&dst)[4]) {
        constexpr int base = decltype(par)::value * TILE;
        constexpr int B = decltype(b)::value;
        lds_read_b128<base>(dst[0], kaddr0 ^ ((2 * B) << 5));
        lds_read_b128<base + 32 * ROW>(dst[1], kaddr0 ^ ((2 * B) << 5));
        lds_read_b128<base>(dst[2], kaddr0 ^ ((2 * B + 1) << 5));
        lds_read_b128<base + 32 * ROW>(dst[3], kaddr0 ^ ((2 * B + 1) << 5));
    };
    auto mul_s = [&](auto b, bf16x8 (&f)[4]) {
        constexpr int B = decltype(b)::value;
        if (B == 0) {
            const floatx16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[0], qreg[0], z, 0, 0, 0);
            s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[1], qreg[0], z, 0, 0, 0);
        } else {
            s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[0], qreg[2 * B], s[0], 0, 0, 0);
            s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[1], qreg[2 * B], s[1], 0, 0, 0);
        }
        s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[2], qreg[2 * B + 1], s[0], 0, 0, 0);
        s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[3], qreg[2 * B + 1], s[1], 0, 0, 0);
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;

    // Phase X of step k.  Always the same straight-line sequence, so the accumulators never
    // move between registers: before the first tile P is zero (the V slots were zero-filled),
    // after the last tile P is zero again and the scores it produces are ignored.  LDS reads
    // run one batch ahead of the MFMAs that consume them; each lds_wait<N> count is the number
    // of reads issued after the batch being waited for.  A batch's registers are refilled right
    // after the MFMAs that read them have issued (operands are read at issue, LDS data returns
    // later).
    auto phase_x = [&](auto par, int k) {
        // refill: K(k+1) -> K slot par^1 (last read in step k-1), V(k) -> V slot par (same)
        if (k + 1 < T) issue_tile(kh, wk.n, (decltype(par)::value ^ 1) * TILE, false);
        if (k < T) issue_tile(vh, wv.n, 2 * TILE + decltype(par)::value * TILE, true);
#ifdef BS_PROBE_NO_X
        return;
#endif
        shortx4 vf[8];
        bf16x8 kf[4];
        if constexpr (NDB < 4) {
#pragma unroll
            for (int i = 2 * NDB; i < 8; ++i) vf[i] = shortx4{0, 0, 0, 0};
        }
        if constexpr (D == 128) {
            read_pv(par, I0{}, vf); read_s(par, I0{}, kf);
            lds_wait<4>(vf); mul_pv(I0{}, vf); read_pv(par, I1{}, vf);
            lds_wait<8>(kf); mul_s(I0{}, kf); read_s(par, I1{}, kf);
            lds_wait<4>(vf); mul_pv(I1{}, vf); read_pv(par, I2{}, vf);
            lds_wait<8>(kf); mul_s(I1{}, kf); read_s(par, I2{}, kf);
            lds_wait<4>(vf); mul_pv(I2{}, vf); read_pv(par, I3{}, vf);
            lds_wait<8>(kf); mul_s(I2{}, kf); read_s(par, I3{}, kf);
            lds_wait<4>(vf); mul_pv(I3{}, vf);
            lds_wait<0>(kf); mul_s(I3{}, kf);
        } else {  // D == 64: PV batches hold 4 reads, S has 2 batches
            read_pv(par, I0{}, vf); read_s(par, I0{}, kf);
            lds_wait<4>(vf); mul_pv(I0{}, vf); read_pv(par, I1{}, vf);
            lds_wait<4>(kf); mul_s(I0{}, kf); read_s(par, I1{}, kf);
            lds_wait<4>(vf); mul_pv(I1{}, vf); read_pv(par, I2{}, vf);
            lds_wait<4>(kf); mul_s(I1{}, kf);
            lds_wait<0>(vf); mul_pv(I2{}, vf); read_pv(par, I3{}, vf);
            lds_wait<0>(vf); mul_pv(I3{}, vf);
        }
    };

    // Phase Y of step k: mask (PARTIAL tiles), online softmax, rescale O, round P to bf16.
    auto phase_y = [&](int k) {
#ifdef BS_PROBE_NO_Y
        if (k < T) wv.next();
        __builtin_amdgcn_s_waitcnt(0x0f70);
        return;
#endif
        if (k < T) {
            float alpha;
            if (wv.full) {
                softmax_block<false>(s, m_run, l_run, alpha, a.scale_log2e);
            } else {
                const int nu = __builtin_amdgcn_readfirstlane(wv.n);
                const uint64_t tb = map_text_bits[nu];
                const uint64_t sb = (cls & 1) ? map_sink_bits[nu] : 0ull;
                apply_mask(s, allowed_keys(qv, tb, sb, wv.n * kBlockN), hl);
                softmax_block<true>(s, m_run, l_run, alpha, a.scale_log2e);
            }
            if (__any(alpha != 1.f)) {
#pragma unroll
                for (int db = 0; db < NDB; ++db)
#pragma unroll
                    for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
            }
            // P^T as bf16 B operands: contraction slots e = 0..7 of MFMA (kb, t) are C values
            // v = 8t + e, i.e. keys 32kb + 16t + {4hl..4hl+3, 8+4hl..8+4hl+3}
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int e = 0; e < 8; ++e) pf[kb][t][e] = (__bf16)s[kb][8 * t + e];
            wv.next();
        } else if (k == T) {
            // past the last tile: phase X keeps running (the other group may have more tiles)
            // but must add nothing
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[i >> 1][i & 1][e] = (__bf16)0.f;
        }
        __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): the tiles requested in phase X have landed
    };

    // Zero the group's ring once: phase X reads every slot from its first step on, and stale
    // LDS bits could be NaN patterns (0 * NaN would poison the accumulators).
    {
        const uint4 z4 = make_uint4(0, 0, 0, 0);
        unsigned char *mine = lds + grp * 4 * TILE;
        for (int i = (tid & 255) * 16; i < 4 * TILE; i += 256 * 16) *reinterpret_cast<uint4 *>(mine + i) = z4;
    }
    __syncthreads();
    // prologue: K(0) into K slot 0
    if (T > 0) {
        issue_tile(kh, wk.n, 0, false);
        wk.next();
    }
    // Raw barriers: every LDS access of this kernel is an LDS-direct load (drained with vmcnt
    // at the end of phase Y) or an asm read (drained with lgkmcnt inside phase X), so no fence
    // is wanted here -- a fence would drain the loads already at the end of phase X.
    __builtin_amdgcn_s_waitcnt(0x0f70);
    __builtin_amdgcn_s_barrier();
    if (grp == 1) __builtin_amdgcn_s_barrier();  // second group runs half a step behind
    BS_T0();
    for (int k = 0; k < n_steps; k += 2) {
        phase_x(I0{}, k);
        if (k + 1 < T) wk.next();
        BS_TICK(0);
        __builtin_amdgcn_s_barrier();
        BS_TICK(1);
        phase_y(k);
        BS_TICK(2);
        __builtin_amdgcn_s_barrier();
        BS_TICK(3);
        phase_x(I1{}, k + 1);
        if (k + 2 < T) wk.next();
        BS_TICK(0);
        __builtin_amdgcn_s_barrier();
        BS_TICK(1);
        phase_y(k + 1);
        BS_TICK(2);
        __builtin_amdgcn_s_barrier();
        BS_TICK(3);
    }
    if (grp == 0) __builtin_amdgcn_s_barrier();  // same barrier count for every wave of the workgroup
    BS_TFLUSH();

    // epilogue: divide by the running sum, round, store.  Empty rows (l = 0) give zeros.
    const float l_tot = sum_across_halves(l_run);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    if (have_item && row < L) {
        __bf16 *orow = reinterpret_cast<__bf16 *>(a.out) + ((size_t)head * L + row) * D;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                bf16x4 w;
#pragma unroll
                for (int r = 0; r < 4; ++r) w[r] = (__bf16)(o[db][4 * g + r] * inv);
                *reinterpret_cast<bf16x4 *>(orow + 32 * db + 8 * g + 4 * hl) = w;
            }
    }
}

// ------------------------------------------------------------------------------------ fp32
// Same structure with fp32 MFMA (32x32x2) end to end; P stays fp32.  Parity path for fp32
// inputs, not tuned.  Dynamic LDS: K[64][D+1] floats, V[64][D+8] floats.

template <int D>
__global__ __launch_bounds__(kThreads, 1) void attn_prefill_f32(KernelArgs a, BS_MAP_PARAMS)
{
    constexpr int KS = D + 1, VS = D + 8;
    extern __shared__ __align__(16) unsigned char smem[];
    float *lds_k = reinterpret_cast<float *>(smem);
    float *lds_v = lds_k + kBlockN * KS;

    const int2 item = map_work[blockIdx.x];
    const int head = item.x, m = item.y;
    const int cls = map_head_class[head];
    const int kvh = head / a.G;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hl = lane >> 5, col = lane & 31;
    const int L = a.L;
    const int row = m * kBlockM + wave * 32 + col;

    const float *qh = reinterpret_cast<const float *>(a.q) + (size_t)head * L * D;
    const float *kh = reinterpret_cast<const float *>(a.k) + (size_t)kvh * L * D;
    const float *vh = reinterpret_cast<const float *>(a.v) + (size_t)kvh * L * D;

    float qreg[D / 2];  // Q[row][2t + hl]
    {
        const int qrow = min(row, L - 1);
#pragma unroll
        for (int t = 0; t < D / 2; ++t) qreg[t] = qh[(size_t)qrow * D + 2 * t + hl];
    }
    QueryView qv;
    qv.init(map_code, map_span_range, a.L, cls, row);

    floatx16 o[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    TileWalker tw;
    tw.init(map_ranges, map_row_ptr[cls * (a.M + 1) + m], map_row_ptr[cls * (a.M + 1) + m + 1]);

    for (; tw.valid(); tw.next()) {
        const int n0 = tw.n * kBlockN;
        __syncthreads();
        for (int idx = tid; idx < kBlockN * (D / 4); idx += kThreads) {
            const int key = idx / (D / 4), ch = idx % (D / 4);
            const int grow = min(n0 + key, L - 1);
            const floatx4 kk = *reinterpret_cast<const floatx4 *>(kh + (size_t)grow * D + ch * 4);
            const floatx4 vv = *reinterpret_cast<const floatx4 *>(vh + (size_t)grow * D + ch * 4);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                lds_k[key * KS + ch * 4 + r] = kk[r];
                lds_v[key * VS + ch * 4 + r] = vv[r];
            }
        }
        __syncthreads();

        floatx16 s[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
#pragma unroll
            for (int t = 0; t < D / 2; ++t)
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x2f32(lds_k[(32 * kb + col) * KS + 2 * t + hl], qreg[t], s[kb], 0, 0, 0);
        }
        float alpha;
        if (tw.full) {
            softmax_block<false>(s, m_run, l_run, alpha, a.scale_log2e);
        } else {
            const uint64_t tb = map_text_bits[tw.n];
            const uint64_t sb = (cls & 1) ? map_sink_bits[tw.n] : 0ull;
            apply_mask(s, allowed_keys(qv, tb, sb, n0), hl);
            softmax_block<true>(s, m_run, l_run, alpha, a.scale_log2e);
        }
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[db][v] *= alpha;

        // contraction slot hl of MFMA (kb, v) is key 32kb + 8(v/4) + 4hl + v%4
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = 32 * kb + 8 * (v / 4) + 4 * hl + (v % 4);
                    o[db] = __builtin_amdgcn_mfma_f32_32x32x2f32(lds_v[key * VS + 32 * db + col], s[kb][v], o[db], 0, 0, 0);
                }
    }

    const float l_tot = sum_across_halves(l_run);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    if (row < L) {
        float *orow = reinterpret_cast<float *>(a.out) + ((size_t)head * L + row) * D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                floatx4 w;
#pragma unroll
                for (int r = 0; r < 4; ++r) w[r] = o[db][4 * g + r] * inv;
                *reinterpret_cast<floatx4 *>(orow + 32 * db + 8 * g + 4 * hl) = w;
            }
    }
}

template <int D>
constexpr size_t f32_lds_bytes() { return (size_t)kBlockN * (D + 1) * 4 + (size_t)kBlockN * (D + 8) * 4; }

void free_device_map(DeviceMap *d)
{
    if (!d) return;
    if (d->blob) {
        int cur = -1;
        (void)hipGetDevice(&cur);
        if (cur != d->device) (void)hipSetDevice(d->device);
        (void)hipFree(d->blob);
        if (cur >= 0 && cur != d->device) (void)hipSetDevice(cur);
    }
    delete d;
}

}  // namespace bs

using bs::DeviceMap;

extern "C" int bs_tilemap_upload(bs_tilemap *tm)
{
    if (!tm) return BS_EINVAL;
    if (tm->dev) return BS_OK;
    if (tm->bn > 64) return BS_EUNSUPPORTED;  // the per-tile key bit masks are 64 wide
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return bs::fail_hip(e, "hipGetDevice");

    const int64_t M1 = (int64_t)tm->M + 1;
    int64_t total_ranges = 0;
    for (int c = 0; c < 4; ++c) total_ranges += (int64_t)tm->cls[c].ranges.size();
    if (total_ranges >= INT32_MAX) return BS_EUNSUPPORTED;
    const size_t G1 = tm->spans.size() + 1;

    auto align = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t off_code = 0;
    const size_t off_tbits = align(off_code + (size_t)tm->L * 4);
    const size_t off_sbits = align(off_tbits + (size_t)tm->N * 8);
    const size_t off_spans = align(off_sbits + (size_t)tm->N * 8);
    const size_t off_rowptr = align(off_spans + G1 * 8);
    const size_t off_rowtiles = align(off_rowptr + (size_t)(4 * M1) * 4);
    const size_t off_ranges = align(off_rowtiles + (size_t)(4 * tm->M) * 4);
    const size_t off_work = align(off_ranges + (size_t)std::max<int64_t>(total_ranges, 1) * 8);
    const size_t off_class = align(off_work + tm->work.size() * 8);
    const size_t bytes = align(off_class + tm->head_class.size());

    std::vector<unsigned char> host;
    DeviceMap *d = nullptr;
    try {
        host.assign(bytes, 0);
        d = new DeviceMap();
    } catch (const std::bad_alloc &) {
        return BS_ENOMEM;
    }
    std::memcpy(host.data() + off_code, tm->code.data(), (size_t)tm->L * 4);
    std::memcpy(host.data() + off_tbits, tm->text_bits.data(), (size_t)tm->N * 8);
    std::memcpy(host.data() + off_sbits, tm->sink_bits.data(), (size_t)tm->N * 8);
    int2 *sp = reinterpret_cast<int2 *>(host.data() + off_spans);
    sp[0] = make_int2(0, 0);
    for (size_t g = 0; g < tm->spans.size(); ++g) sp[g + 1] = make_int2(tm->spans[g].start, tm->spans[g].end);
    int32_t *rp = reinterpret_cast<int32_t *>(host.data() + off_rowptr);
    int32_t *rt = reinterpret_cast<int32_t *>(host.data() + off_rowtiles);
    int2 *rg = reinterpret_cast<int2 *>(host.data() + off_ranges);
    int64_t base = 0;
    for (int c = 0; c < 4; ++c) {
        const bs::ClassLists &cl = tm->cls[c];
        for (int64_t m = 0; m < M1; ++m) rp[c * M1 + m] = (int32_t)(base + cl.row_ptr[m]);
        for (int64_t m = 0; m < tm->M; ++m) rt[c * (int64_t)tm->M + m] = cl.row_tiles[m];
        for (size_t i = 0; i < cl.ranges.size(); ++i) rg[base + i] = make_int2(cl.ranges[i].begin, cl.ranges[i].end_state);
        base += (int64_t)cl.ranges.size();
    }
    int2 *wk = reinterpret_cast<int2 *>(host.data() + off_work);
    for (size_t i = 0; i < tm->work.size(); ++i) wk[i] = make_int2(tm->work[i].head, tm->work[i].q_tile);
    std::memcpy(host.data() + off_class, tm->head_class.data(), tm->head_class.size());

    void *blob = nullptr;
    e = hipMalloc(&blob, bytes);
    if (e != hipSuccess) {
        delete d;
        return bs::fail_hip(e, "hipMalloc(tile map)");
    }
    e = hipMemcpy(blob, host.data(), bytes, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        (void)hipFree(blob);
        delete d;
        return bs::fail_hip(e, "hipMemcpy(tile map)");
    }
    unsigned char *b = static_cast<unsigned char *>(blob);
    d->device = dev;
    d->blob = blob;
    d->code = reinterpret_cast<const uint32_t *>(b + off_code);
    d->text_bits = reinterpret_cast<const uint64_t *>(b + off_tbits);
    d->sink_bits = reinterpret_cast<const uint64_t *>(b + off_sbits);
    d->span_range = reinterpret_cast<const int2 *>(b + off_spans);
    d->row_ptr = reinterpret_cast<const int32_t *>(b + off_rowptr);
    d->row_tiles = reinterpret_cast<const int32_t *>(b + off_rowtiles);
    d->ranges = reinterpret_cast<const int2 *>(b + off_ranges);
    d->work = reinterpret_cast<const int2 *>(b + off_work);
    d->head_class = b + off_class;
    d->n_work = (int32_t)tm->work.size();
    tm->dev = d;
    tm->dev_free = bs::free_device_map;
    return BS_OK;
}

extern "C" int bs_attn_prefill(const void *q, const void *k, const void *v, void *out, bs_tilemap *tm,
                               int32_t dtype, int32_t n_q_heads, int32_t gqa_group, int32_t head_dim,
                               float scale, void *stream)
{
    if (!q || !k || !v || !out || !tm) return BS_EINVAL;
    if (n_q_heads <= 0 || gqa_group <= 0 || n_q_heads % gqa_group != 0) return BS_EINVAL;
    if (n_q_heads != tm->n_q_heads) return BS_EINVAL;
    if (!(scale > 0.f) || !(scale < INFINITY)) return BS_EINVAL;  // masking relies on -inf * scale = -inf
    if (tm->bm != bs::kBlockM || tm->bn != bs::kBlockN) return BS_EUNSUPPORTED;
    if (head_dim != 64 && head_dim != 128) return BS_EUNSUPPORTED;
    if (dtype != BS_BF16 && dtype != BS_F32) return BS_EUNSUPPORTED;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out) & 15) return BS_EINVAL;

    int rc = bs_tilemap_upload(tm);
    if (rc != BS_OK) return rc;
    const DeviceMap *d = tm->dev;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return bs::fail_hip(e, "hipGetDevice");
    if (dev != d->device) return BS_EINVAL;  // the map lives on another device

    bs::KernelArgs a;
    a.q = q; a.k = k; a.v = v; a.out = out;
    a.L = tm->L; a.M = tm->M; a.G = gqa_group;
    a.scale_log2e = scale * 1.4426950408889634f;

    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)d->n_work), block(bs::kThreads);
    if (dtype == BS_BF16) {
        // two work items per workgroup (one per wave group)
        const dim3 pgrid((unsigned)((d->n_work + 1) / 2)), pblock(bs::kPingPongThreads);
        if (head_dim == 128) {
            constexpr int lds = bs::bf16_lds_bytes<128>();
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(bs::attn_prefill_bf16<128>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, lds);
            if (e != hipSuccess) return bs::fail_hip(e, "hipFuncSetAttribute");
            hipLaunchKernelGGL(bs::attn_prefill_bf16<128>, pgrid, pblock, lds, st, a, BS_MAP_ARGS(d), d->row_tiles, d->n_work);
        } else {
            constexpr int lds = bs::bf16_lds_bytes<64>();
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(bs::attn_prefill_bf16<64>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, lds);
            if (e != hipSuccess) return bs::fail_hip(e, "hipFuncSetAttribute");
            hipLaunchKernelGGL(bs::attn_prefill_bf16<64>, pgrid, pblock, lds, st, a, BS_MAP_ARGS(d), d->row_tiles, d->n_work);
        }
    } else {
        if (head_dim == 128) {
            constexpr size_t lds = bs::f32_lds_bytes<128>();
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(bs::attn_prefill_f32<128>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return bs::fail_hip(e, "hipFuncSetAttribute");
            hipLaunchKernelGGL(bs::attn_prefill_f32<128>, grid, block, lds, st, a, BS_MAP_ARGS(d));
        } else {
            constexpr size_t lds = bs::f32_lds_bytes<64>();
            hipLaunchKernelGGL(bs::attn_prefill_f32<64>, grid, block, lds, st, a, BS_MAP_ARGS(d));
        }
    }
    e = hipGetLastError();
    if (e != hipSuccess) return bs::fail_hip(e, "kernel launch");
    return BS_OK;
}

extern "C" const char *bs_last_error(void) { return bs::g_last_error; }

#ifdef BS_PHASE_TIMING
extern "C" int bs_debug_phase_cycles(unsigned long long *out8, int reset)
{
    if (hipMemcpyFromSymbol(out8, HIP_SYMBOL(bs::g_phase_cycles), 64) != hipSuccess) return BS_EHIP;
    if (reset) {
        unsigned long long z[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (hipMemcpyToSymbol(HIP_SYMBOL(bs::g_phase_cycles), z, 64) != hipSuccess) return BS_EHIP;
    }
    return BS_OK;
}
#endif
