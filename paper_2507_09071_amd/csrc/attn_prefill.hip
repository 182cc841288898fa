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
// Mapping to CDNA4 (bf16 kernel):
//  * a workgroup of eight 64-lane waves owns one work unit: two (head, query tile) items that
//    read the same KV head, four waves each; wave w of a group owns rows 32w..32w+31 of its item
//    and keeps its Q rows in registers for the whole pass;
//  * the launch is one workgroup per CU; a workgroup stays resident and claims unit after unit from
//    the queue of the XCD it runs on (eight queues, filled by the host; see "Work distribution");
//  * scores are produced transposed, S^T = K Q^T, with 32x32x16 bf16 MFMA tiles, so every lane
//    holds 16 keys of ONE query per 32-key block: row max / row sum are in-lane reductions plus
//    one exchange with the lane 32 apart (v_permlane32_swap);
//  * O^T = V^T P^T reuses the probabilities, rounded to bf16, as the B operand; V^T comes from a
//    pre-pass that writes K and V^T per key tile in exactly the layout the LDS reads want;
//  * K and V^T tiles travel global -> LDS with 16-byte LDS-direct loads (no VGPR staging) into a
//    ring of 4 K + 4 V^T slots shared by the two groups; ONE barrier per key tile, placed so that
//    on every SIMD one wave runs its matrix phase while the other runs its vector phase;
//  * PARTIAL tiles build one 64-bit allowed-key word per lane from per-tile text/sink bit
//    masks, the query's own image range and the causal bound, then test one bit per score.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <type_traits>
#include <vector>

#include "device_map.h"
#include "tilemap_internal.h"

namespace bs {

// Read-only tile-map arrays; passed as separate __restrict__ kernel parameters so that loads
// with wave-uniform addresses go through the scalar cache (they then never wait on the vector
// memory counter that tracks the in-flight LDS-direct loads).
struct KernelArgs {
    const void *q, *k, *v;
    void *out;
    int32_t L, M, G;
    float scale_log2e;  // scale * log2(e): softmax runs in the exp2 domain
    int32_t n_prompt_tiles;   // key tiles that are the prompt in position order (compact tiles follow)
    int32_t packed, intra_compact;
    int32_t bidir;            // tokens of one image also see the later tokens of that image
    int32_t window;           // > 0: keys more than window - 1 positions before the query are masked
    int32_t q_begin;          // q / out hold the query positions q_begin .. L - 1, row r = position q_begin + r
};
#define BS_MAP_PARAMS                                                                              \
    const uint32_t *__restrict__ map_code, const uint64_t *__restrict__ map_text_bits,             \
        const uint64_t *__restrict__ map_sink_bits, const int2 *__restrict__ map_span_range,       \
        const int32_t *__restrict__ map_row_ptr, const int2 *__restrict__ map_ranges,              \
        const int2 *__restrict__ map_work, const uint8_t *__restrict__ map_head_class,             \
        const int32_t *__restrict__ map_row_order, const int32_t *__restrict__ map_key_order,      \
        const int32_t *__restrict__ map_free_before, const int2 *__restrict__ map_span_free
#define BS_MAP_ARGS(d) (d)->code, (d)->text_bits, (d)->sink_bits, (d)->span_range, (d)->row_ptr, (d)->ranges, (d)->work, (d)->head_class, (d)->row_order, (d)->key_order, (d)->free_before, (d)->span_free

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
        n = 0; n_end = 0; full = false;
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
// With packed keys (see the tile-map builder) an image query of a sparse class reads the free
// keys -- text and sink keys -- from compact tiles and only own-image keys from the prompt's
// tiles, so that every allowed pair is counted once.
struct QueryView {
    int32_t row;       // last visible position: the query's own (causal), the end of its image (bidirectional images)
    int32_t first;     // first visible position: 0, or the start of the query's sliding window
    int32_t own_lo;    // own image [own_lo, own_hi) if the class attends inside images, else empty
    int32_t own_hi;
    int32_t free_bound;  // packed: free keys at positions <= i (the visible compact slots are [0, free_bound))
    int32_t cfree_lo;    // packed, Intra-Image+Sink: compact slots of the free keys inside the own image
    int32_t cfree_hi;
    bool sees_all;     // text query or Dense head: every earlier key
    bool own_only;     // packed: in the prompt's tiles only own-image keys count for this query
    __device__ void init(const uint32_t *__restrict__ code, const int2 *__restrict__ span_range,
                         const int32_t *__restrict__ free_before, const int2 *__restrict__ span_free,
                         int L, int cls, int32_t i, bool packed, bool intra_compact, bool bidir, int32_t window)
    {
        row = i;
        first = window > 0 ? max(0, i - window + 1) : 0;
        const uint32_t qcode = i < L ? code[i] : kCodeText;
        sees_all = (qcode & kCodeText) || cls == BS_DENSE;
        own_lo = own_hi = 0;
        free_bound = cfree_lo = cfree_hi = 0;
        own_only = false;
        if (!(qcode & kCodeText) && (bidir || (cls & 2))) {
            const int2 sp = span_range[qcode & kCodeImgMask];
            // an image query that sees its whole image behaves, for every class, like the
            // image's last query under the causal mask; its image stays visible beyond a window
            if (bidir) { row = sp.y - 1; first = min(first, sp.x); }
            if (!sees_all && (cls & 2)) { own_lo = sp.x; own_hi = sp.y; }
        }
        if (packed && !sees_all && (cls != BS_INTRA || intra_compact)) {
            free_bound = free_before[row + 1];
            own_only = true;
            if (cls == BS_INTRA_SINK) {
                const int2 cr = span_free[qcode & kCodeImgMask];
                cfree_lo = cr.x; cfree_hi = cr.y;
            }
        }
    }
};

__device__ inline uint64_t bits_below(int x)  // bits [0, x), x in [0, 64]
{
    return x >= 64 ? ~0ull : ((1ull << x) - 1ull);
}
__device__ inline uint64_t bits_between(int lo, int hi)  // bits [lo, hi) clipped to [0, 64)
{
    return bits_below(min(max(hi, 0), 64)) & ~bits_below(min(max(lo, 0), 64));
}

// Bit b set <=> the key in slot b of key tile n is allowed for this lane's query.  tbits / sbits:
// text keys and sink keys of the tile; n_prompt: number of key tiles that are the prompt in
// position order (the tiles after them are compact tiles of free keys).
__device__ inline uint64_t allowed_keys(const QueryView &qv, int cls, uint64_t tbits, uint64_t sbits, int n, int n_prompt)
{
    if (n < n_prompt) {
        const int n0 = n * kBlockN;
        const uint64_t base = qv.sees_all ? ~0ull : (qv.own_only ? 0ull : (tbits | ((cls & 1) ? sbits : 0ull)));
        const uint64_t own = bits_between(qv.own_lo - n0, qv.own_hi - n0);
        return (base | own) & bits_between(qv.first - n0, qv.row - n0 + 1);   // keys first .. row
    }
    // compact tile: slots are free keys in position order, visible up to the row's bound
    const int s0 = (n - n_prompt) * kBlockN;
    const uint64_t base = qv.sees_all ? 0ull : ((cls & 1) ? ~0ull : tbits);   // Intra-Image: text keys only
    const uint64_t excl = bits_between(qv.cfree_lo - s0, qv.cfree_hi - s0);   // counted with the own image
    return base & ~excl & bits_below(min(max(qv.free_bound - s0, 0), 64));
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

// The same masking in two instructions per score, kept together so that the scheduler cannot
// hoist the 32 bit tests in front of the 32 selects (32 registers of pressure in a kernel that
// has none to spare): the allowed bit is spread over a word (0 / all ones) and a bit-field
// insert then keeps the score or takes -inf.
__device__ inline void apply_mask_tight(const floatx16 (&s)[2], floatx16 (&ms)[2], uint64_t allowed, int hl)
{
    const uint32_t w[2] = {(uint32_t)allowed >> (4 * hl), (uint32_t)(allowed >> 32) >> (4 * hl)};
    const float ninf = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            // out of place: the masked scores go to registers of their own, so the scores (in/out
            // operands of the matrix phase) are not copied first
            uint32_t t;
            float r;
            asm("v_bfe_i32 %1, %2, %3, 1\n\t"
                "v_bfi_b32 %0, %1, %4, %5"
                : "=v"(r), "=&v"(t)
                : "v"(w[kb]), "n"(8 * (v / 4) + (v % 4)), "v"(s[kb][v]), "v"(ninf));
            ms[kb][v] = r;
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

// Same update as softmax_block, but the scores are only read and the probabilities go straight
// into the bf16 B operands of the P.V MFMAs: contraction slot e of MFMA group (kb, t) is score
// v = 8t + e of block kb, i.e. key 32kb + 16t + {4hl..4hl+3, 8+4hl..8+4hl+3}[e].
//   MODE 0  FULL tile: every score counts.
//   MODE 1  row-uniform PARTIAL tile: a lane's query sees either all 64 keys or none (`drop`).
//           A dropped row keeps its running max and gets p = 0 through an infinite offset.
//   MODE 2  general PARTIAL tile: `s` already holds -inf at the masked positions.
// Fast path (FULL tiles): the probabilities are first formed against the reference point the row already
// has, without looking for the tile maximum.  Any reference gives the same quotient O / l as long as
// nothing overflows, so this is exact whenever the row sums of the tile stay below kFastLimit -- which
// they do on almost every tile after a row's first (scores of neighbouring tiles differ by a few units in
// the exp2 domain, not by 16).  A wave in which some lane's sum is too large, infinite or NaN (no reference
// yet: m = -inf) repeats the tile on the general path below, which moves the reference.  Returns whether
// alpha may differ from 1.
template <int MODE>
__device__ inline bool softmax_pack(const floatx16 (&s)[2], bf16x8 (&pf)[2][2], float &m_run, float &l_run,
                                    float &alpha, float c, bool drop)
{
    constexpr float kFastLimit = 65536.f;
    if constexpr (MODE == 0) {   // PARTIAL tiles keep the one path (no registers to spare for two)
        const float off = -(m_run * c);   // m = -inf: +inf, caught below
        float sum[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float pv = __builtin_amdgcn_exp2f(fmaf(s[kb][8 * t + e], c, off));
                    sum[e & 3] += pv;
                    pf[kb][t][e] = (__bf16)pv;
                }
        const float tile_sum = (sum[0] + sum[1]) + (sum[2] + sum[3]);
        if (!__any(!(tile_sum <= kFastLimit))) {
            l_run += tile_sum;
            alpha = 1.f;
            return false;
        }
    }
    // four independent max chains
    float mx[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) mx[i] = fmaxf(s[i >> 1][8 * (i & 1)], s[i >> 1][8 * (i & 1) + 1]);
#pragma unroll
    for (int v = 2; v < 8; v += 2)
#pragma unroll
        for (int i = 0; i < 4; ++i) mx[i] = fmaxf(fmaxf(mx[i], s[i >> 1][8 * (i & 1) + v]), s[i >> 1][8 * (i & 1) + v + 1]);
    float mxl = max_across_halves(fmaxf(fmaxf(mx[0], mx[1]), fmaxf(mx[2], mx[3])));
    if (MODE == 1) mxl = drop ? -INFINITY : mxl;
    // Lazy reference point: the running reference m only moves when the tile maximum exceeds it
    // by more than kLazyLog2 (in the exp2 domain), so p <= 2^kLazyLog2 instead of p <= 1.  The
    // result is the same quotient O / l; what changes is that alpha is exactly 1 on almost every
    // tile after the first few, and the rescaling of the 64 output accumulators is skipped.
    constexpr float kLazyLog2 = 8.f;
    const bool grow = fmaf(mxl, c, -(m_run * c)) > kLazyLog2;   // m_run = -inf, mxl finite: +inf > 8
    const float m_new = grow ? mxl : m_run;                     // both -inf: NaN > 8 is false
    const float m_use = (MODE != 0 && m_new == -INFINITY) ? 0.f : m_new;  // no key seen so far: p = 0
    const float mc = m_use * c;
    alpha = grow ? __builtin_amdgcn_exp2f(fmaf(m_run, c, -mc)) : 1.f;     // m_run = -inf -> 0
    const float off = (MODE == 1 && drop) ? -INFINITY : -mc;
    float sum[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float pv = __builtin_amdgcn_exp2f(fmaf(s[kb][8 * t + e], c, off));
                sum[e & 3] += pv;
                pf[kb][t][e] = (__bf16)pv;
            }
    l_run = fmaf(l_run, alpha, (sum[0] + sum[1]) + (sum[2] + sum[3]));
    m_run = m_new;
    return true;
}

typedef __attribute__((address_space(3))) void *lds_void_ptr;
typedef const __attribute__((address_space(1))) void *global_void_ptr;

// ------------------------------------------------------------------------------------ bf16
//
// LDS operand reads of the MFMA phase are issued through inline asm and waited for by hand
// (lds_wait<N>): the compiler would otherwise tie every LDS read to the LDS-direct loads that
// are in flight into the other ring slot and drain the vector-memory counter before it.

template <int OFFSET>
__device__ inline void lds_read_b128(bf16x8 &dst, uint32_t addr)
{
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFFSET));
}

// Wait until at most N LDS operations are outstanding.  The operands tie the wait to the
// registers it protects, so their consumers cannot be scheduled above it.
template <int N>
__device__ inline void lds_wait(bf16x8 (&a)[4])
{
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]) : "n"(N));
}

// The MFMAs of the matrix phase are asm as well: together with the asm reads and waits they
// form one chain of volatile statements, which the compiler keeps in program order, and the
// accumulator is an in/out operand, so it is updated in place (no copies of the 64 output
// registers).  The compiler does not see a matrix instruction here, so the wait states between
// the last MFMA writing an accumulator and the first vector instruction reading it are
// inserted by hand (mfma_drain) at the end of the chain.
__device__ inline void mfma_acc(floatx16 &c, const bf16x8 &a, const bf16x8 &b)
{
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
}
__device__ inline void mfma_set(floatx16 &c, const bf16x8 &a, const bf16x8 &b)   // c = a b
{
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(c) : "v"(a), "v"(b));
}
// 16 wait states: more than the 8 passes of a 32x32x16 MFMA plus the result write-back.
__device__ inline void mfma_drain(floatx16 &c0, floatx16 &c1)
{
    asm volatile("s_nop 15" : "+v"(c0), "+v"(c1));
}


// LDS tile layouts of the bf16 kernel (written by the pre-pass below, copied verbatim by the
// kernel's LDS-direct loads).  Both are "slice-major": everything an MFMA operand read selects
// at compile time (head-dim slice, key block, key group, channel block) is an immediate offset,
// and one per-lane base address serves all reads of a tile.
//   K tile   [D/16 slices t][64 keys][32 B]   32 B = channels 16t..16t+15 of one key, as two
//            16-byte halves h (channels 16t+8h..+7) stored at half h ^ ((key >> 3) & 1)
//   V^T tile [4 key groups g][D channels][32 B]   32 B = the 16 keys of group g of one channel,
//            as two halves h holding keys 16g + {4h..4h+3, 8+4h..8+4h+3} (the contraction slots
//            of lane half h), stored at half h ^ ((channel >> 3) & 1)
// A 128-bit read of 16 consecutive keys (channels) then touches every bank exactly once.
// The key of every tile slot comes from the map's key order (the prompt in position order, then
// the compact tiles of a packed map); slots without a key are zero-filled.
template <int D>
__device__ inline void pack_vt_tile(const __bf16 *__restrict__ v, __bf16 *__restrict__ vt,
                                    const int32_t *__restrict__ key_order, int L, int N, __bf16 *tile)
{
    constexpr int PAD = D + 2;  // odd word stride: the column gathers below spread over banks
    const int n = blockIdx.x, kvh = blockIdx.y, tid = threadIdx.x;
    const __bf16 *src = v + (size_t)kvh * L * D;
    for (int idx = tid; idx < kBlockN * (D / 8); idx += 256) {
        const int key = idx / (D / 8), ch = idx % (D / 8);
        const int pos = key_order[n * kBlockN + key];   // -1: the slot holds no key
        bf16x8 val;
#pragma unroll
        for (int e = 0; e < 8; ++e) val[e] = (__bf16)0.f;
        if (pos >= 0) val = *reinterpret_cast<const bf16x8 *>(src + (size_t)pos * D + ch * 8);
#pragma unroll
        for (int e = 0; e < 8; ++e) tile[key * PAD + ch * 8 + e] = val[e];
    }
    __syncthreads();
    __bf16 *dst = vt + ((size_t)kvh * N + n) * (size_t)(D * kBlockN);
    for (int idx = tid; idx < D * 8; idx += 256) {   // one 16-byte half per iteration
        const int hp = idx & 1, d = (idx >> 1) % D, g = idx / (2 * D);
        const int h = hp ^ ((d >> 3) & 1);
        bf16x8 val;
#pragma unroll
        for (int e = 0; e < 8; ++e) val[e] = tile[(16 * g + 8 * (e >> 2) + 4 * h + (e & 3)) * PAD + d];
        *reinterpret_cast<bf16x8 *>(dst + (size_t)idx * 8) = val;
    }
}

template <int D>
__device__ inline void pack_k_tile(const __bf16 *__restrict__ k, __bf16 *__restrict__ kp,
                                   const int32_t *__restrict__ key_order, int L, int N)
{
    const int n = blockIdx.x, kvh = blockIdx.y;
    const __bf16 *src = k + (size_t)kvh * L * D;
    __bf16 *dst = kp + ((size_t)kvh * N + n) * (size_t)(D * kBlockN);
    for (int idx = threadIdx.x; idx < kBlockN * (D / 8); idx += 256) {   // one 16-byte half per iteration
        const int hp = idx & 1, key = (idx >> 1) % kBlockN, t = idx / (2 * kBlockN);
        const int h = hp ^ ((key >> 3) & 1);
        const int pos = key_order[n * kBlockN + key];   // -1: the slot holds no key
        uint4 val = make_uint4(0, 0, 0, 0);
        if (pos >= 0) val = *reinterpret_cast<const uint4 *>(src + (size_t)pos * D + 16 * t + 8 * h);
        *reinterpret_cast<uint4 *>(dst + (size_t)idx * 8) = val;
    }
}

// The pre-pass of a bf16 call, one launch: grid (key tiles, KV heads, 2); z = 0 packs K, z = 1 packs V^T.
template <int D>
__global__ __launch_bounds__(256) void pack_kv_tiles(const __bf16 *__restrict__ k, const __bf16 *__restrict__ v,
                                                     __bf16 *__restrict__ kp, __bf16 *__restrict__ vt,
                                                     const int32_t *__restrict__ key_order, int L, int N,
                                                     int32_t *__restrict__ queue_ctr)
{
    __shared__ __bf16 tile[kBlockN * (D + 2)];
    // the attention kernel that follows starts on fresh unit queues
    if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x < 8) queue_ctr[threadIdx.x] = 0;
    if (blockIdx.z == 0) pack_k_tile<D>(k, kp, key_order, L, N);
    else pack_vt_tile<D>(v, vt, key_order, L, N, tile);
}

constexpr int kPingPongThreads = 512;

// Batch tags of the matrix phase: four operand reads + four MFMAs each.
template <int G> struct PvBatch { static constexpr int kind = 1, idx = G; static constexpr bool first = false; };            // O^T += V^T(group G) P^T(group G)
template <int B, bool FIRST> struct ScBatch { static constexpr int kind = 2, idx = B; static constexpr bool first = FIRST; }; // S += K(slices 2B, 2B+1) Q^T
struct NoBatch { static constexpr int kind = 0, idx = 0; static constexpr bool first = false; };

constexpr int kRing = 4;   // K slots = V^T slots of the LDS ring
template <int D>
constexpr int bf16_lds_bytes() { return 2 * kRing * kBlockN * D * 2 + 64; }   // ring, then the unit mailbox

// Walks the merged key-tile list of a work unit: runs of [begin, end) with a state per item.
struct PairWalker {
    const int2 *__restrict__ rg;
    int p, p_end, n, n_end, states;
    __device__ void load()
    {
        if (p < p_end) {
            const int2 r = rg[__builtin_amdgcn_readfirstlane(p)];
            n = __builtin_amdgcn_readfirstlane(r.x);
            n_end = __builtin_amdgcn_readfirstlane(r.y) >> 4;
            states = __builtin_amdgcn_readfirstlane(r.y) & 15;
        }
    }
    __device__ void init(const int2 *__restrict__ ranges, int begin, int end)
    {
        rg = ranges;
        n = 0; n_end = 0; states = 0;
        p = __builtin_amdgcn_readfirstlane(begin);
        p_end = __builtin_amdgcn_readfirstlane(end);
        load();
    }
    __device__ bool valid() const { return p < p_end; }
    __device__ void next()
    {
        if (++n == n_end) { ++p; load(); }
    }
    __device__ int state(int grp) const { return grp ? (states & 3) : (states >> 2); }  // 0 skip 1 partial 2 full
};

// One workgroup = two groups of four waves = one work unit: two (head, query tile) items that
// read the same KV head and walk one merged key-tile list (heads of a GQA group with the same
// class, or two neighbouring query tiles of one head), so each K / V^T tile is fetched ONCE for
// 256 query rows.  The tiles live in a shared ring of 4 K + 4 V^T slots.  Per key tile a group
// runs two phases:
//   X (matrix):  O += P(k-1) V(k-1)  and  S(k) = K(k) Q^T        -- MFMA + LDS reads only
//   Y (vector):  mask, online softmax of S(k) -> P(k), rescale O  -- VALU only
// and the workgroup meets at ONE barrier per tile, placed so that the two groups run the phases
// in opposite order between two barriers (X then Y / Y then X): on every SIMD one wave is in X
// while the other is in Y, and the matrix pipe and the vector ALU stay busy together instead
// of the two waves queueing for the same unit.
template <int D>
__global__ __launch_bounds__(kPingPongThreads, 2) void attn_prefill_bf16(
    KernelArgs a, const uint32_t *__restrict__ map_code, const uint64_t *__restrict__ map_text_bits,
    const uint64_t *__restrict__ map_sink_bits, const int2 *__restrict__ map_span_range,
    const int32_t *__restrict__ map_row_order,
    const int32_t *__restrict__ map_free_before, const int2 *__restrict__ map_span_free,
    const int4 *__restrict__ pair_items,
    const int2 *__restrict__ pair_ranges, const __bf16 *__restrict__ kp, const __bf16 *__restrict__ vt,
    int32_t n_k_tiles, int32_t *__restrict__ queue_ctr, const int32_t *__restrict__ queue_off)
{
    constexpr int ROW = D * 2;            // bytes per K row in LDS
    constexpr int TILE = kBlockN * ROW;   // bytes per K or V^T tile
    constexpr int DMA_PER_WAVE = D / 64;  // LDS-direct loads per wave per matrix per tile (8 waves)
    constexpr int NDB = D / 32;           // 32-channel blocks of the output
    constexpr int NT = D / 16;            // 16-wide slices of the head dim
    extern __shared__ __align__(1024) unsigned char lds[];   // K slots 0..3, then V^T slots 0..3

    const int tid = threadIdx.x, lane = tid & 63, hl = lane >> 5, col = lane & 31;
    const int grp = __builtin_amdgcn_readfirstlane(tid >> 8);          // wave group 0 / 1
    const int wave = __builtin_amdgcn_readfirstlane((tid >> 6) & 3);   // wave within the group
    const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);        // wave within the workgroup
    const int L = a.L;

    const int R = L - a.q_begin;   // query rows per head

    // ---- state of the work unit in progress (a workgroup takes units from its XCD's queue until
    // ---- the queues are empty; see the unit loop below)
    int head = 0, m = 0, T = 0, n_steps = 1, cls = 0;
    bool have_item = false;
    int row = 0;                    // the query position of this lane's row
    const char *kph = nullptr, *vth = nullptr;   // packed K / V^T tiles of the unit's KV head
    bf16x8 qreg[NT];                // Q^T operand: Q[row][16t + 8hl .. +8] for every 16-wide slice t
    QueryView qv;
    int list_begin = 0, list_end = 0;
    auto load_unit = [&](int unit) __attribute__((always_inline)) {
        const int4 it0 = pair_items[2 * unit], it1 = pair_items[2 * unit + 1];
        head = __builtin_amdgcn_readfirstlane(grp ? it0.z : it0.x);
        m = __builtin_amdgcn_readfirstlane(grp ? it0.w : it0.y);
        have_item = head >= 0;
        T = __builtin_amdgcn_readfirstlane(it1.z);            // key tiles in the merged list
        n_steps = T + 1;                                      // the last step only adds P(T-1) V(T-1)
        list_begin = __builtin_amdgcn_readfirstlane(it1.x);
        list_end = __builtin_amdgcn_readfirstlane(it1.y);
        const int hsafe = max(head, 0);
        cls = __builtin_amdgcn_readfirstlane((grp ? it1.w >> 8 : it1.w) & 3);   // head classes travel with the unit
        const int kvh = __builtin_amdgcn_readfirstlane(it0.x / a.G);            // both items share it
        // a tile slot without a row behaves like a row past the end of the prompt (computed on a
        // copy of the last row, never stored)
        const int row_slot = map_row_order[max(m, 0) * kBlockM + wave * 32 + col];
        row = row_slot < 0 ? L : row_slot;
        const __bf16 *qh = reinterpret_cast<const __bf16 *>(a.q) + (size_t)hsafe * R * D;
        // one TILE-byte block per key tile
        kph = reinterpret_cast<const char *>(kp + (size_t)kvh * n_k_tiles * (size_t)(D * kBlockN));
        vth = reinterpret_cast<const char *>(vt + (size_t)kvh * n_k_tiles * (size_t)(D * kBlockN));
        const int qrow = min(row, L - 1) - a.q_begin;  // rows past the end compute on a copy and are not stored
#pragma unroll
        for (int t = 0; t < NT; ++t)
            qreg[t] = *reinterpret_cast<const bf16x8 *>(qh + (size_t)qrow * D + 16 * t + 8 * hl);
        qv.init(map_code, map_span_range, map_free_before, map_span_free, L, cls, row, a.packed != 0, a.intra_compact != 0,
                a.bidir != 0, a.window);
    };

    // LDS byte address of this lane's MFMA operand fragments inside a K / V^T tile (see the
    // tile layouts above): key or channel `col`, half hl; slices, blocks and groups are
    // immediate offsets, the ring slot is added per step.
    const uint32_t ring = (uint32_t)(uintptr_t)(lds_void_ptr)lds;
    const uint32_t kaddr0 = ring + col * 32 + ((hl ^ ((col >> 3) & 1)) << 4);

    floatx16 o[NDB];
    floatx16 s[2];
    bf16x8 pf[2][2];   // P^T of the previous tile as MFMA B operands
    float m_run = -INFINITY, l_run = 0.f;
    // three walkers over the merged tile list: w0 names the tile of the current step (state),
    // w1 the next tile (V^T refill), w2 the one after (K refill)
    PairWalker w0, w1, w2, wt1, wt2;
    // Both groups fetch, in the barrier interval k, their shares of K(k+3) and V^T(k+2): the second group
    // at the end of its matrix phase k, the first group right behind barrier k, before its vector phase.
    constexpr int ahead = 1;
    auto reset_unit_state = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[i >> 1][i & 1][e] = (__bf16)0.f;
        m_run = -INFINITY;
        l_run = 0.f;
        w0.init(pair_ranges, list_begin, list_end);
        w1 = w0; if (w1.valid()) w1.next();
        wt1 = w1;                                              // tile 1 (prologue)
        if (ahead && w1.valid()) w1.next();
        w2 = w1; if (w2.valid()) w2.next();
        wt2 = wt1; if (wt2.valid()) wt2.next();                // tile 2 (prologue of the second group)
    };

    // LDS-direct loads of packed tiles into ring slots: straight TILE-byte copies.  Each wave
    // instruction moves 1 KB (lane l -> bytes 16l..16l+15); instruction r of wave w (0..7) covers
    // bytes (8r + w) KB .. +1 KB of the tile, so the eight waves together fetch a tile.  The instruction
    // takes its address as a scalar base (the tile, uniform) plus a vector offset that never changes, and
    // its LDS destination in M0: nothing of it goes through the vector ALU, which the other wave of the
    // SIMD keeps busy (asm: the compiler forms a 64-bit vector address with a vector add per load instead).
    const uint32_t dma_lane_off = wave8 * 1024 + lane * 16;
    auto dma = [&](int r, const char *tile, int slot_byte) __attribute__((always_inline)) {
        const uint32_t dst = ring + slot_byte + wave8 * 1024 + r * 8 * 1024;   // lane 0's 16 bytes
        const char *src = tile + r * 8 * 1024;
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                     :
                     : "v"(dma_lane_off), "s"(src), "s"(dst)
                     : "memory", "m0");
    };
    auto tile_ptr = [&](const char *base, int n) {
        return base + (size_t)min(n, n_k_tiles - 1) * TILE;  // a walker past its end names no tile
    };

    // ---- phase X building blocks (step k reads K slot k mod 4 and V^T slot (k - 1) mod 4) ----
    // A batch is four 128-bit operand reads feeding four MFMAs:
    //   PV batch g (D = 128): O^T block db += V^T(db, group g) . P^T(group g), db = 0..3
    //   S  batch b          : head-dim slices 2b, 2b+1 for both 32-key blocks
    uint32_t kbase = 0, vbase = 0;  // fragment base addresses inside the ring slots of this step
    // one operand read / one MFMA of a batch (element i = 0..3)
    auto read_one = [&](auto tag, auto ic, bf16x8 &dst) __attribute__((always_inline)) {
        using T = decltype(tag);
        constexpr int i = decltype(ic)::value;
        if constexpr (T::kind == 1) {
            if constexpr (i < NDB) lds_read_b128<T::idx * (D * 32) + i * 1024>(dst, vbase);   // channel block i
        } else if constexpr (T::kind == 2) {
            lds_read_b128<(2 * T::idx + (i >> 1)) * 2048 + (i & 1) * 1024>(dst, kbase);        // slice, key block
        }
    };
    auto mul_one = [&](auto tag, auto ic, const bf16x8 &f) __attribute__((always_inline)) {
        using T = decltype(tag);
        constexpr int i = decltype(ic)::value;
        if constexpr (T::kind == 1) {
            if constexpr (i < NDB) mfma_acc(o[i], f, pf[T::idx >> 1][T::idx & 1]);
        } else if constexpr (T::kind == 2) {
            if constexpr (T::first && i < 2) mfma_set(s[i & 1], f, qreg[2 * T::idx + (i >> 1)]);
            else mfma_acc(s[i & 1], f, qreg[2 * T::idx + (i >> 1)]);
        }
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;

    // Phase X of step k: O += P(k-1) V(k-1) and S(k) = K(k) Q^T.  Always the same straight-line
    // chain of asm statements: before the first tile P is zero (the ring was zero-filled), after
    // the last tile -- and on tiles this item skips -- P is zero again and the scores it
    // produces are ignored.  Operand reads run three batches ahead of the MFMAs that consume
    // them, in three rotating register sets; each lds_wait<N> count is the number of reads
    // issued after the batch waited for.  A register is refilled right after the MFMA that
    // read it has issued (operands are read at issue, LDS data returns later), so the reads
    // issue in the shadow of the MFMAs.
    // text / sink key bits of the tile w0 names (scalar registers, fetched one step ahead)
    uint64_t tb_cur = 0, sb_cur = 0;
    // Scalar bookkeeping between two vector phases: w0 moves on to the tile of the coming phase Y and
    // the key bit masks of that tile are requested.  It runs inside phase X, between two MFMA batches,
    // where the wave has issue slots to spare (every MFMA keeps the matrix pipe busy for 32 cycles).
    auto advance_tile = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_sched_barrier(0);
        w0.next();
        const int nn = min(__builtin_amdgcn_readfirstlane(w0.n), n_k_tiles - 1);
        tb_cur = map_text_bits[nn];
        sb_cur = map_sink_bits[nn];
        __builtin_amdgcn_sched_barrier(0);
    };
    const char *ksrc = nullptr, *vsrc = nullptr;   // tiles of the coming refill
    int Sk_dst = 0, Sv_dst = 0;                    // and their ring slots
    auto issue_refill = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int r = 0; r < DMA_PER_WAVE; ++r) dma(r, ksrc, Sk_dst * TILE);
#pragma unroll
        for (int r = 0; r < DMA_PER_WAVE; ++r) dma(r, vsrc, (kRing + Sv_dst) * TILE);
        __builtin_amdgcn_sched_barrier(0);
    };
    auto phase_x = [&](int S, bool advance, auto refill_here) __attribute__((always_inline)) {  // S = k mod 4; advance: k > 0
        auto ring = [](int x) { return x >= kRing ? x - kRing : x; };
        const int Sv = ring(S + kRing - 1);                          // V^T(k-1)
        Sk_dst = ring(ring(S + 2) + ahead); Sv_dst = ring(S + 1 + ahead);
        kbase = kaddr0 + S * TILE;
        vbase = kaddr0 + (kRing + Sv) * TILE;
        bf16x8 fa[4], fb[4], fc[4];
        if constexpr (NDB < 4) {
#pragma unroll
            for (int i = NDB; i < 4; ++i)
#pragma unroll
                for (int e = 0; e < 8; ++e) { fa[i][e] = (__bf16)0.f; fb[i][e] = (__bf16)0.f; fc[i][e] = (__bf16)0.f; }
        }
        // whole-batch reads of the pipeline head
        auto read_batch = [&](auto tag, bf16x8 (&f)[4]) __attribute__((always_inline)) {
            read_one(tag, I0{}, f[0]); read_one(tag, I1{}, f[1]);
            read_one(tag, I2{}, f[2]); read_one(tag, I3{}, f[3]);
        };
        // MFMA batch `cur` on fragment set f, each MFMA followed by the read that refills its
        // operand register for batch `nxt` (three batches ahead)
        auto batch = [&](auto cur, auto nxt, bf16x8 (&f)[4]) __attribute__((always_inline)) {
            mul_one(cur, I0{}, f[0]); read_one(nxt, I0{}, f[0]);
            mul_one(cur, I1{}, f[1]); read_one(nxt, I1{}, f[1]);
            mul_one(cur, I2{}, f[2]); read_one(nxt, I2{}, f[2]);
            mul_one(cur, I3{}, f[3]); read_one(nxt, I3{}, f[3]);
        };
        // The same with two reads behind each MFMA: the refill of its own register (batch `nxt`) and
        // one read of batch `mid` into the idle set g.
        auto batch2 = [&](auto cur, auto mid, bf16x8 (&g)[4], auto nxt, bf16x8 (&f)[4]) __attribute__((always_inline)) {
            mul_one(cur, I0{}, f[0]); read_one(mid, I0{}, g[0]); read_one(nxt, I0{}, f[0]);
            mul_one(cur, I1{}, f[1]); read_one(mid, I1{}, g[1]); read_one(nxt, I1{}, f[1]);
            mul_one(cur, I2{}, f[2]); read_one(mid, I2{}, g[2]); read_one(nxt, I2{}, f[2]);
            mul_one(cur, I3{}, f[3]); read_one(mid, I3{}, g[3]); read_one(nxt, I3{}, f[3]);
        };
        // Refill addresses: computed while the first operand reads are in flight.
        auto refill_prepare = [&]() __attribute__((always_inline)) {
            __builtin_amdgcn_sched_barrier(0);
            ksrc = tile_ptr(kph, w2.n);
            vsrc = tile_ptr(vth, w1.n);
            w1.next();
            w2.next();
            __builtin_amdgcn_sched_barrier(0);
        };
        if constexpr (D == 128) {
            // batch order: PV0 S0 PV1 S1 PV2 S2 PV3 S3, four reads / MFMAs each
            // Only two batches are read ahead of the first MFMA (the burst of all four waves of a group
            // costs every wave its share of the LDS time); the third goes out behind the first four
            // MFMAs together with their refills.
            read_batch(PvBatch<0>{}, fa); read_batch(ScBatch<0, true>{}, fb);
            refill_prepare();
            lds_wait<4>(fa); batch2(PvBatch<0>{}, PvBatch<1>{}, fc, ScBatch<1, false>{}, fa);
            lds_wait<8>(fb); batch(ScBatch<0, true>{}, PvBatch<2>{}, fb);
            lds_wait<5>(fc); batch(PvBatch<1>{}, ScBatch<2, false>{}, fc);   // behind the last PV1 read: one S1 read, four PV2
            lds_wait<8>(fa); batch(ScBatch<1, false>{}, PvBatch<3>{}, fa);
            if (advance) advance_tile();
            lds_wait<8>(fb); batch(PvBatch<2>{}, ScBatch<3, false>{}, fb);
            lds_wait<8>(fc); batch(ScBatch<2, false>{}, NoBatch{}, fc);
            lds_wait<4>(fa); batch(PvBatch<3>{}, NoBatch{}, fa);
            lds_wait<0>(fb); batch(ScBatch<3, false>{}, NoBatch{}, fb);
            mfma_drain(s[0], s[1]);   // the PV accumulators finished four MFMAs earlier
        } else {
            // D == 64: PV batches hold two reads / MFMAs, S has two batches of four
            read_batch(PvBatch<0>{}, fa); read_batch(ScBatch<0, true>{}, fb); read_batch(PvBatch<1>{}, fc);   // 2 + 4 + 2
            refill_prepare();
            lds_wait<6>(fa); batch(PvBatch<0>{}, PvBatch<2>{}, fa);                     // 4 2 | 2
            lds_wait<4>(fb); batch(ScBatch<0, true>{}, ScBatch<1, false>{}, fb);        // 2 2 | 4
            lds_wait<6>(fc); batch(PvBatch<1>{}, PvBatch<3>{}, fc);                     // 2 4 | 2
            if (advance) advance_tile();
            lds_wait<6>(fa); batch(PvBatch<2>{}, NoBatch{}, fa);
            lds_wait<2>(fb); batch(ScBatch<1, false>{}, NoBatch{}, fb);
            lds_wait<0>(fc); batch(PvBatch<3>{}, NoBatch{}, fc);
            mfma_drain(o[0], o[1]);   // the scores finished two MFMAs earlier
        }
        // Every LDS read and scalar load of the phase has returned (the last lds_wait was for zero): say so
        // in a form the compiler sees, or it waits for its own scalar loads in the middle of the next chain.
        __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
        // Refill: this wave's share of K(k+3) and V^T(k+2) into the slots of the tiles four steps older,
        // which nobody reads after barrier k.  Unconditional: past the end of the list a valid tile is
        // fetched again and never used.  An LDS-direct load issued while the other wave of the SIMD issues
        // matrix or vector instructions stalls this wave several times longer, so each group issues it in a
        // window in which its mate is quiet: the second group here, after its last MFMA, while the first
        // group waits for the head reads of its next matrix phase; the first group right behind the barrier
        // (see the step loop), while the second group waits for its head reads.
        if constexpr (decltype(refill_here)::value) issue_refill();
        // Wait for the loads issued one step ago (only this step's may stay in flight): after
        // the next barrier every wave has passed this wait, and the tile is read in the interval
        // that follows it.
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * DMA_PER_WAVE));
    };

    // Phase Y of step k: mask (PARTIAL tiles), online softmax, rescale O, round P to bf16.
    auto phase_y = [&](int k) __attribute__((always_inline)) {
        if (k < T) {
            // state of the tile for this group's item: 0 skip (only the other item wants the
            // tile), 1 partial, 2 full.  A skipped tile goes through the row-uniform path with
            // every row dropped (P = 0, running max and sum unchanged): rare, and one straight
            // code path keeps the register allocation of the loop simple.
            const int st = have_item ? w0.state(grp) : 0;
            float alpha;
            bool rescale;
            if (st == 2) {
                rescale = softmax_pack<0>(s, pf, m_run, l_run, alpha, a.scale_log2e, false);
            } else {
                const int nu = __builtin_amdgcn_readfirstlane(w0.n);
                uint64_t allowed = allowed_keys(qv, cls, tb_cur, sb_cur, nu, a.n_prompt_tiles);
                if (st == 0) allowed = 0ull;
                if (__all(allowed == 0ull || allowed == ~0ull)) {
                    // every query of the wave sees all 64 keys or none (e.g. a text row and an
                    // image row over keys of another image): no per-score work
                    rescale = softmax_pack<1>(s, pf, m_run, l_run, alpha, a.scale_log2e, allowed == 0ull);
                } else {
                    floatx16 ms[2];
                    apply_mask_tight(s, ms, allowed, hl);
                    rescale = softmax_pack<2>(ms, pf, m_run, l_run, alpha, a.scale_log2e, false);
                }
            }
            if (rescale && __any(alpha != 1.f)) {
#pragma unroll
                for (int db = 0; db < NDB; ++db)
#pragma unroll
                    for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
            }
        } else {
            // past the last tile: the final phase X adds P(T-1) V(T-1); steps after it (none
            // today) must add nothing
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[i >> 1][i & 1][e] = (__bf16)0.f;
        }
    };

    // Zero the ring once per workgroup: phase X reads every slot from its first step on, and stale LDS
    // bits could be NaN patterns (0 * NaN would poison the accumulators).  Between units the slots hold
    // tiles of the previous unit: finite values, which P = 0 wipes out just as well.
    {
        const uint4 z4 = make_uint4(0, 0, 0, 0);
        for (int i = tid * 16; i < 2 * kRing * TILE; i += kPingPongThreads * 16) *reinterpret_cast<uint4 *>(lds + i) = z4;
    }

    // ---- Work distribution.  The host deals the units (heaviest first) to eight queues, one per XCD,
    // so that units walking the same K / V^T tiles at about the same time share an L2.  A workgroup
    // reads the id of the XCD it runs on from the hardware register (it does not depend on the launch
    // order, which other streams can perturb) and claims the next unit of that queue with an atomic
    // counter; when the queue is empty it helps out on the next one.  The first wave takes the ticket
    // for the next unit two steps before the current one ends -- late, so that the units of a queue
    // start in queue order (units that start together walk the same tiles together and share them in
    // L2; a ticket taken a whole unit ahead was measured to cost half of that sharing), early enough
    // for the atomic to return under the last steps -- and passes the unit on through a mailbox behind
    // the ring.  Every wave reads the same mailbox entry, so the workgroup leaves the loop together.
    volatile int32_t *mailbox = reinterpret_cast<volatile int32_t *>(lds + 2 * kRing * TILE);
    int xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID, 0, 4)" : "=s"(xcc));
    xcc &= 7;
    // claims on queue q, then on the following ones: index of a unit, or -1 when all are empty
    auto claim_from = [&](int q0, int first_ticket) {
        int ticket = first_ticket;
        for (int t = 0; t < 8; ++t) {
            const int q = (q0 + t) & 7;
            const int begin = queue_off[q], len = queue_off[q + 1] - begin;
            if (t > 0) {
                ticket = len;
                if (len > 0) {
                    int r = 0;
                    if (lane == 0) r = atomicAdd(&queue_ctr[q], 1);
                    ticket = __builtin_amdgcn_readfirstlane(r);
                }
            }
            if (ticket < len) return begin + ticket;
        }
        return -1;
    };
    auto take_ticket = [&]() {   // one atomic on the own queue; lane 0's result counts
        int r = 0;
        if (lane == 0) r = atomicAdd(&queue_ctr[xcc], 1);
        return r;
    };
    // The same without waiting for the answer: lane 0 alone issues the atomic (asm, so that the compiler
    // does not wait for it on the spot) and the ticket is in lane 0 of the result once the vector-memory
    // counter has drained (ticket_wait).  Until then the register must not be read.
    auto take_ticket_async = [&]() __attribute__((always_inline)) {
        int r;
        unsigned long long save;
        int32_t *ctr = queue_ctr + xcc;
        const int one = 1;
        asm volatile("s_mov_b64 %[save], exec\n\t"
                     "s_mov_b64 exec, 1\n\t"
                     "global_atomic_add %[r], %[ptr], %[one], off sc0\n\t"
                     "s_mov_b64 exec, %[save]"
                     : [r] "=&v"(r), [save] "=&s"(save)
                     : [ptr] "v"(ctr), [one] "v"(one)
                     : "memory");
        return r;
    };
    auto ticket_wait = [&](int &ticket) __attribute__((always_inline)) {
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(ticket)::"memory");
    };
    if (wave8 == 0) {
        const int first = claim_from(xcc, __builtin_amdgcn_readfirstlane(take_ticket()));
        if (lane == 0) mailbox[0] = first;
    }
    __syncthreads();
    int unit = __builtin_amdgcn_readfirstlane(mailbox[0]);

    while (unit >= 0) {
        int next_ticket = 0;
        load_unit(unit);
        reset_unit_state();
        {
            const int nn = min(__builtin_amdgcn_readfirstlane(w0.n), n_k_tiles - 1);
            tb_cur = map_text_bits[nn];
            sb_cur = map_sink_bits[nn];
        }
        // prologue: K(0) -> K slot 0, K(1) -> K slot 1, V^T(0) -> V^T slot 0 (unconditional, clamped)
        {
            const char *k0 = tile_ptr(kph, w0.n), *k1 = tile_ptr(kph, wt1.n), *v0 = tile_ptr(vth, w0.n);
#pragma unroll
            for (int r = 0; r < DMA_PER_WAVE; ++r) dma(r, k0, 0);
#pragma unroll
            for (int r = 0; r < DMA_PER_WAVE; ++r) dma(r, k1, TILE);
#pragma unroll
            for (int r = 0; r < DMA_PER_WAVE; ++r) dma(r, v0, kRing * TILE);
            {
                const char *k2 = tile_ptr(kph, wt2.n), *v1 = tile_ptr(vth, wt1.n);
#pragma unroll
                for (int r = 0; r < DMA_PER_WAVE; ++r) dma(r, k2, 2 * TILE);
#pragma unroll
                for (int r = 0; r < DMA_PER_WAVE; ++r) dma(r, v1, (kRing + 1) * TILE);
            }
        }
        // Raw barriers: every LDS access of the loop is an LDS-direct load (drained with vmcnt
        // at the end of phase X) or an asm read (drained with lgkmcnt inside phase X), so no fence
        // is wanted there -- a fence would drain loads that are meant to stay in flight.
        __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): the first tiles
        __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the unit's scalar loads (none stays pending into the loop)
        __builtin_amdgcn_s_barrier();
        // ONE barrier per step.  Group 0 runs  X(k) | barrier | refill Y(k),  group 1  barrier | X(k) refill Y(k):
        // between two barriers group 0 does Y(k) then X(k+1) while group 1 does X(k) then Y(k), so
        // the waves of a SIMD are in opposite phases by program order but nothing holds them to a
        // half-step grid.  Between barrier k and k+1 the ring is read at K(k), K(k+1), V^T(k-1),
        // V^T(k) and written by both groups at K(k+3), V^T(k+2), whose slots (of K(k-1), V^T(k-2))
        // nobody reads after barrier k; at the end of every matrix phase a wave lets only its newest
        // loads stay in flight (vmcnt), so the loads of interval k have landed before barrier k + 2,
        // and the tiles are read from the interval after that barrier on: four slots each.
        if (grp == 0) {
            const int k_claim = max(n_steps - 2, 0);
            for (int k = 0, slot = 0; k < n_steps; ++k) {
                if (wave8 == 0 && k == k_claim) next_ticket = take_ticket_async();   // consumed after the loop
                phase_x(slot, k > 0, std::false_type{});
                __builtin_amdgcn_s_barrier();
                issue_refill();   // under the second group's head reads, before its chain starts
                phase_y(k);
                slot = slot == kRing - 1 ? 0 : slot + 1;
            }
        } else {
            for (int k = 0, slot = 0; k < n_steps; ++k) {
                __builtin_amdgcn_s_barrier();
                phase_x(slot, k > 0, std::true_type{});
                phase_y(k);
                slot = slot == kRing - 1 ? 0 : slot + 1;
            }
        }
        // End of the unit: the refills of its last steps (tiles nobody needs) must have landed
        // before the next unit's first tiles go into the same slots, and every wave must be done
        // reading the ring.  The ticket has returned by then as well.
        ticket_wait(next_ticket);            // vmcnt(0)
        if (wave8 == 0) {
            const int nxt = claim_from(xcc, __builtin_amdgcn_readfirstlane(next_ticket));
            if (lane == 0) mailbox[0] = nxt;
            __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the mailbox write is in LDS before the barrier
        }
        __builtin_amdgcn_s_barrier();
        const int next_unit = __builtin_amdgcn_readfirstlane(mailbox[0]);

        // epilogue: divide by the running sum, round, store.  Empty rows (l = 0) give zeros.  A lane holds
        // four channels of one row at a time (O^T accumulators), which would make every store instruction
        // touch 64 rows with 8 bytes each; the tile goes through LDS instead (the ring is free: every wave is
        // past the barrier above), 64 channels at a time in a wave-private patch, and leaves as 16-byte pieces
        // of 128-byte row segments.
        const float l_tot = sum_across_halves(l_run);
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        {
            constexpr int kStageRow = 128 + 16;                 // 64 channels, then the row's position
            unsigned char *stage = lds + wave8 * (32 * kStageRow);
            if (hl == 0) *reinterpret_cast<int32_t *>(stage + col * kStageRow + 128) = row;
#pragma unroll
            for (int half = 0; half < NDB / 2; ++half) {
#pragma unroll
                for (int dbl = 0; dbl < 2; ++dbl)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        bf16x4 w;
#pragma unroll
                        for (int r = 0; r < 4; ++r) w[r] = (__bf16)(o[2 * half + dbl][4 * g + r] * inv);
                        *reinterpret_cast<bf16x4 *>(stage + col * kStageRow + (32 * dbl + 8 * g + 4 * hl) * 2) = w;
                    }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int r = 8 * j + (lane >> 3), chunk = lane & 7;
                    const uint4 piece = *reinterpret_cast<const uint4 *>(stage + r * kStageRow + chunk * 16);
                    const int32_t pos = *reinterpret_cast<const int32_t *>(stage + r * kStageRow + 128);
                    if (have_item && pos < L) {
                        __bf16 *orow = reinterpret_cast<__bf16 *>(a.out) + ((size_t)head * R + (pos - a.q_begin)) * D;
                        *reinterpret_cast<uint4 *>(orow + 64 * half + chunk * 8) = piece;
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
        }
        // the patches lie in the ring: nobody loads the next unit's first tiles before every wave is done with its own
        __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
        unit = next_unit;
    }
}

// ------------------------------------------------------------------------------------ fp32
// Same structure with fp32 MFMA (32x32x2) end to end; P stays fp32.  Parity path for fp32
// inputs, not tuned: K / V tiles are gathered from the caller's arrays through key_order (no
// pre-pass).  Dynamic LDS: K[64][D+1] floats, V[64][D+8] floats.

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
    const int row_slot = map_row_order[m * kBlockM + wave * 32 + col];
    const int row = row_slot < 0 ? L : row_slot;

    const int R = L - a.q_begin;   // query rows per head
    const float *qh = reinterpret_cast<const float *>(a.q) + (size_t)head * R * D;
    const float *kh = reinterpret_cast<const float *>(a.k) + (size_t)kvh * L * D;
    const float *vh = reinterpret_cast<const float *>(a.v) + (size_t)kvh * L * D;

    float qreg[D / 2];  // Q[row][2t + hl]
    {
        const int qrow = min(row, L - 1) - a.q_begin;
#pragma unroll
        for (int t = 0; t < D / 2; ++t) qreg[t] = qh[(size_t)qrow * D + 2 * t + hl];
    }
    QueryView qv;
    qv.init(map_code, map_span_range, map_free_before, map_span_free, a.L, cls, row, a.packed != 0, a.intra_compact != 0,
            a.bidir != 0, a.window);

    floatx16 o[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    TileWalker tw;
    tw.init(map_ranges, map_row_ptr[cls * (a.M + 1) + m], map_row_ptr[cls * (a.M + 1) + m + 1]);

    for (; tw.valid(); tw.next()) {
        __syncthreads();
        for (int idx = tid; idx < kBlockN * (D / 4); idx += kThreads) {
            const int key = idx / (D / 4), ch = idx % (D / 4);
            // the key this slot of the tile holds (a compact tile of a packed map gathers free keys);
            // a slot without a key is masked below, any finite values will do for it
            const int grow = max(map_key_order[tw.n * kBlockN + key], 0);
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
            const uint64_t sb = map_sink_bits[tw.n];
            apply_mask(s, allowed_keys(qv, cls, tb, sb, tw.n, a.n_prompt_tiles), hl);
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
        float *orow = reinterpret_cast<float *>(a.out) + ((size_t)head * R + (row - a.q_begin)) * D;
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

}  // namespace bs

using bs::DeviceMap;

// ------------------------------------------------------------------------------------ launch

// Scratch of the entry point that allocates nothing (bs_attn_prefill_static): packed K tiles, then
// packed V^T tiles.  Every GPU the library runs on holds its own copy until the process ends.  In
// host code the name below is only a handle for hipGetSymbolAddress; kernels get the per-device
// address that call returns.
constexpr size_t kStaticScratchBytes = (size_t)BS_STATIC_SCRATCH_MIB << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_device_mutex;
void *g_scratch_ptr[kMaxDevices];       // device address of `scratch` on each device (looked up once)
bool g_attr_set[kMaxDevices];           // dynamic-LDS limits of the kernels raised on this device
int g_n_cus[kMaxDevices];               // compute units of the device

// Once per device, with that device current: the address of its copy of `scratch`, and the
// kernels' dynamic LDS limits.  Allocates nothing.
int device_setup(int dev, void **scratch_out, int *n_cus_out)
{
    if (dev < 0 || dev >= kMaxDevices) return bs::fail_msg(BS_EUNSUPPORTED, "device ordinal above 63");
    std::lock_guard<std::mutex> lock(g_device_mutex);
    hipError_t e;
    if (!g_attr_set[dev]) {
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(bs::attn_prefill_bf16<128>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, bs::bf16_lds_bytes<128>());
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(bs::attn_prefill_bf16<64>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, bs::bf16_lds_bytes<64>());
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(bs::attn_prefill_f32<128>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)bs::f32_lds_bytes<128>());
        if (e != hipSuccess) return bs::fail_hip(e, "hipFuncSetAttribute");
        int cus = 0;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess || cus <= 0) return bs::fail_hip(e, "hipDeviceGetAttribute(compute units)");
        g_n_cus[dev] = cus;
        g_attr_set[dev] = true;
    }
    if (n_cus_out) *n_cus_out = g_n_cus[dev];
    if (scratch_out) {
        if (!g_scratch_ptr[dev]) {
            void *ptr = nullptr;
            e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !ptr) return bs::fail_hip(e, "hipGetSymbolAddress(scratch)");
            g_scratch_ptr[dev] = ptr;
        }
        *scratch_out = g_scratch_ptr[dev];
    }
    return BS_OK;
}

int check_call(const void *q, const void *k, const void *v, void *out, const bs_tilemap *tm, int32_t dtype,
               int32_t n_q_heads, int32_t gqa_group, int32_t head_dim, float scale)
{
    if (!q || !k || !v || !out || !tm) return BS_EINVAL;
    if (n_q_heads <= 0 || gqa_group <= 0 || n_q_heads % gqa_group != 0) return BS_EINVAL;
    if (n_q_heads != tm->n_q_heads) return BS_EINVAL;
    if (!(scale > 0.f) || !(scale < INFINITY)) return BS_EINVAL;  // masking relies on -inf * scale = -inf
    if (tm->bm != bs::kBlockM || tm->bn != bs::kBlockN) return BS_EUNSUPPORTED;
    if (head_dim != 64 && head_dim != 128) return BS_EUNSUPPORTED;
    if (dtype != BS_BF16 && dtype != BS_F32) return BS_EUNSUPPORTED;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out) & 15) return BS_EINVAL;
    return BS_OK;
}

bs::KernelArgs kernel_args(const void *q, const void *k, const void *v, void *out, const bs_tilemap *tm,
                           int32_t gqa_group, float scale)
{
    bs::KernelArgs a;
    a.q = q; a.k = k; a.v = v; a.out = out;
    a.L = tm->L; a.M = tm->M; a.G = gqa_group;
    a.scale_log2e = scale * 1.4426950408889634f;
    a.n_prompt_tiles = tm->N0;
    a.packed = tm->packed;
    a.intra_compact = tm->intra_compact;
    a.bidir = tm->bidir;
    a.window = tm->window;
    a.q_begin = tm->q_begin;
    return a;
}

// Pre-pass (K and V^T into per-key-tile blocks of `workspace`) and the attention kernel.
template <int D>
void launch_bf16(const bs::KernelArgs &a, const bs_tilemap *tm, const DeviceMap *d, void *workspace, size_t pack_bytes,
                 int n_kv_heads, int n_cus, hipStream_t st, void *ev_main_start)
{
    __bf16 *kp = static_cast<__bf16 *>(workspace);
    __bf16 *vt = reinterpret_cast<__bf16 *>(static_cast<char *>(workspace) + pack_bytes);
    const dim3 tgrid((unsigned)tm->N, (unsigned)n_kv_heads, 2);
    // one workgroup per CU (128 KB of LDS each), which take the units from the queues until they are empty
    const dim3 pgrid((unsigned)std::min(d->n_pairs, n_cus)), pblock(bs::kPingPongThreads);
    hipLaunchKernelGGL(bs::pack_kv_tiles<D>, tgrid, dim3(256), 0, st, static_cast<const __bf16 *>(a.k),
                       static_cast<const __bf16 *>(a.v), kp, vt, d->key_order, tm->L, tm->N, d->queue_ctr);
    if (ev_main_start) (void)hipEventRecord(static_cast<hipEvent_t>(ev_main_start), st);
    hipLaunchKernelGGL(bs::attn_prefill_bf16<D>, pgrid, pblock, bs::bf16_lds_bytes<D>(), st, a, d->code, d->text_bits,
                       d->sink_bits, d->span_range, d->row_order, d->free_before, d->span_free, d->pair_items,
                       d->pair_ranges, kp, vt, tm->N, d->queue_ctr, d->queue_off);
}

size_t bf16_pack_bytes(const bs_tilemap *tm, int n_kv_heads, int head_dim)
{
    return (size_t)n_kv_heads * tm->N * (size_t)head_dim * bs::kBlockN * 2;   // one of the two halves (K, V^T)
}

}  // namespace

extern "C" int bs_tilemap_upload(bs_tilemap *tm)
{
    if (!tm) return BS_EINVAL;
    if (tm->dev) return BS_OK;
    const int rc = bs::upload_prompt_part(tm, nullptr);
    if (rc != BS_OK) return rc;
    const hipError_t e = hipStreamSynchronize(nullptr);   // this entry point promises a finished upload
    return e == hipSuccess ? BS_OK : bs::fail_hip(e, "hipStreamSynchronize");
}

extern "C" int bs_tilemap_prepare(bs_tilemap *tm, int32_t dtype, int32_t gqa_group, void *stream)
{
    if (!tm || gqa_group <= 0 || tm->n_q_heads % gqa_group != 0) return BS_EINVAL;
    if (dtype != BS_BF16 && dtype != BS_F32) return BS_EUNSUPPORTED;
    if (tm->bm != bs::kBlockM || tm->bn != bs::kBlockN) return BS_EUNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int rc = bs::upload_prompt_part(tm, st);
    if (rc != BS_OK) return rc;
    DeviceMap *d = tm->dev;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return bs::fail_hip(e, "hipGetDevice");
    if (dev != d->device) return BS_EINVAL;  // the map lives on another device
    void *unused = nullptr;
    if ((rc = device_setup(dev, &unused, nullptr)) != BS_OK) return rc;
    if ((rc = bs::order_after_last_use(d, st)) != BS_OK) return rc;
    rc = bs::upload_binding(tm, dtype == BS_BF16 ? bs::kBindPairPlan : bs::kBindWorkList, gqa_group, st);
    if (rc != BS_OK) return rc;
    e = hipEventRecord(d->last_use->ev, st);
    return e == hipSuccess ? BS_OK : bs::fail_hip(e, "hipEventRecord");
}

extern "C" int bs_attn_prefill(const void *q, const void *k, const void *v, void *out, bs_tilemap *tm,
                               int32_t dtype, int32_t n_q_heads, int32_t gqa_group, int32_t head_dim,
                               float scale, void *stream)
{
    return bs_attn_prefill_ex(q, k, v, out, tm, dtype, n_q_heads, gqa_group, head_dim, scale, stream, nullptr, nullptr);
}

extern "C" int bs_attn_prefill_ex(const void *q, const void *k, const void *v, void *out, bs_tilemap *tm,
                                  int32_t dtype, int32_t n_q_heads, int32_t gqa_group, int32_t head_dim,
                                  float scale, void *stream, void *ev_main_start, void *ev_main_stop)
{
    int rc = check_call(q, k, v, out, tm, dtype, n_q_heads, gqa_group, head_dim, scale);
    if (rc != BS_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if ((rc = bs::upload_prompt_part(tm, st)) != BS_OK) return rc;
    DeviceMap *d = tm->dev;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return bs::fail_hip(e, "hipGetDevice");
    if (dev != d->device) return BS_EINVAL;  // the map lives on another device
    int n_cus = 0;
    if ((rc = device_setup(dev, nullptr, &n_cus)) != BS_OK) return rc;
    if ((rc = bs::order_after_last_use(d, st)) != BS_OK) return rc;
    rc = bs::upload_binding(tm, dtype == BS_BF16 ? bs::kBindPairPlan : bs::kBindWorkList, gqa_group, st);
    if (rc != BS_OK) return rc;

    const bs::KernelArgs a = kernel_args(q, k, v, out, tm, gqa_group, scale);
    if (dtype == BS_BF16) {
        // workspace of the pre-pass: packed K tiles, then packed V^T tiles (owned by the map)
        const int n_kv_heads = n_q_heads / gqa_group;
        const size_t pack_bytes = bf16_pack_bytes(tm, n_kv_heads, head_dim);
        if (d->vt_bytes < 2 * pack_bytes) {
            bs::pool_release(dev, d->vt_buf, d->vt_bytes, d->last_use);
            d->vt_buf = nullptr; d->vt_bytes = 0;
            e = bs::pool_acquire(dev, 2 * pack_bytes, st, &d->vt_buf, &d->vt_bytes);
            if (e != hipSuccess) { d->vt_buf = nullptr; d->vt_bytes = 0; return bs::fail_hip(e, "hipMalloc(K / V^T workspace)"); }
        }
        if (head_dim == 128) launch_bf16<128>(a, tm, d, d->vt_buf, pack_bytes, n_kv_heads, n_cus, st, ev_main_start);
        else launch_bf16<64>(a, tm, d, d->vt_buf, pack_bytes, n_kv_heads, n_cus, st, ev_main_start);
    } else {
        if (ev_main_start) (void)hipEventRecord(static_cast<hipEvent_t>(ev_main_start), st);
        const dim3 grid((unsigned)d->n_work), block(bs::kThreads);
        if (head_dim == 128)
            hipLaunchKernelGGL(bs::attn_prefill_f32<128>, grid, block, bs::f32_lds_bytes<128>(), st, a, BS_MAP_ARGS(d));
        else
            hipLaunchKernelGGL(bs::attn_prefill_f32<64>, grid, block, bs::f32_lds_bytes<64>(), st, a, BS_MAP_ARGS(d));
    }
    e = hipGetLastError();
    if (e != hipSuccess) return bs::fail_hip(e, "kernel launch");
    if (ev_main_stop) (void)hipEventRecord(static_cast<hipEvent_t>(ev_main_stop), st);
    e = hipEventRecord(d->last_use->ev, st);
    if (e != hipSuccess) return bs::fail_hip(e, "hipEventRecord");
    return BS_OK;
}

extern "C" int64_t bs_static_scratch_bytes(void) { return (int64_t)kStaticScratchBytes; }

extern "C" int bs_attn_prefill_static(const void *q, const void *k, const void *v, void *out, bs_tilemap *tm,
                                      int32_t n_q_heads, int32_t gqa_group, int32_t head_dim, float scale, void *stream)
{
    int rc = check_call(q, k, v, out, tm, BS_BF16, n_q_heads, gqa_group, head_dim, scale);
    if (rc != BS_OK) return rc;
    DeviceMap *d = tm->dev;
    if (!d || d->bind_kind != bs::kBindPairPlan || d->bind_G != gqa_group || d->bind_epoch != tm->class_epoch)
        return bs::fail_msg(BS_EINVAL, "bs_attn_prefill_static: call bs_tilemap_prepare(tm, BS_BF16, gqa_group, stream) first "
                                       "(after every bs_tilemap_rebind); this entry point uploads and allocates nothing");
    const int n_kv_heads = n_q_heads / gqa_group;
    const size_t pack_bytes = bf16_pack_bytes(tm, n_kv_heads, head_dim);
    if (2 * pack_bytes > kStaticScratchBytes) {
        snprintf(bs::g_last_error, sizeof bs::g_last_error,
                 "bs_attn_prefill_static: packed K / V^T tiles need %zu bytes, the static scratch holds %zu "
                 "(n_kv_heads * key tiles * head_dim * 256 bytes); use bs_attn_prefill", 2 * pack_bytes, kStaticScratchBytes);
        return BS_EUNSUPPORTED;
    }
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return bs::fail_hip(e, "hipGetDevice");
    if (dev != d->device) return BS_EINVAL;  // the map lives on another device
    void *ws = nullptr;
    int n_cus = 0;
    if ((rc = device_setup(dev, &ws, &n_cus)) != BS_OK) return rc;   // looks the address up on the first call per device
    hipStream_t st = static_cast<hipStream_t>(stream);
    if ((rc = bs::order_after_last_use(d, st)) != BS_OK) return rc;
    const bs::KernelArgs a = kernel_args(q, k, v, out, tm, gqa_group, scale);
    // the pre-pass writes every slot of every tile it covers (keys, or zeros): nothing of the
    // previous call's contents is read
    if (head_dim == 128) launch_bf16<128>(a, tm, d, ws, pack_bytes, n_kv_heads, n_cus, st, nullptr);
    else launch_bf16<64>(a, tm, d, ws, pack_bytes, n_kv_heads, n_cus, st, nullptr);
    e = hipGetLastError();
    if (e != hipSuccess) return bs::fail_hip(e, "kernel launch");
    e = hipEventRecord(d->last_use->ev, st);
    if (e != hipSuccess) return bs::fail_hip(e, "hipEventRecord");
    return BS_OK;
}

extern "C" const char *bs_last_error(void) { return bs::g_last_error; }
