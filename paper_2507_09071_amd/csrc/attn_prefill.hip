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
// Mapping to CDNA4: a workgroup of four 64-lane waves owns one 128-row query tile of one head;
// wave w owns rows 32w..32w+31.  Scores are produced transposed, S^T = K Q^T, with 32x32 MFMA
// tiles so that every lane holds 16 keys of ONE query per 32-key block: row max / row sum are
// in-lane reductions plus a single exchange with the lane 32 apart.  O^T = V^T P^T reuses the
// score registers as the B operand after rounding to bf16; V is transposed on its way into LDS.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <new>
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
    void *blob = nullptr;            // one allocation holding everything below
    const uint32_t *code = nullptr;  // [L]
    const int32_t *row_ptr = nullptr;  // [4][M+1] offsets into ranges
    const int2 *ranges = nullptr;    // concatenated over classes
    const int2 *work = nullptr;      // [n_work] (head, q_tile)
    const uint8_t *head_class = nullptr;  // [Hq]
    int32_t n_work = 0;
};

struct KernelArgs {
    const void *q, *k, *v;
    void *out;
    const uint32_t *code;
    const int32_t *row_ptr;
    const int2 *ranges;
    const int2 *work;
    const uint8_t *head_class;
    int32_t L, M, G;
    float scale_log2e;  // scale * log2(e): softmax runs in the exp2 domain
};

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kBlockM = 128, kBlockN = 64, kThreads = 256;

// Walks the key tiles of one (class, query tile): ranges of [begin, end) with a FULL flag.
struct TileWalker {
    const int2 *rg;
    int p, p_end, n, n_end;
    bool full;
    __device__ void load()
    {
        if (p < p_end) {
            int2 r = rg[p];
            n = r.x; n_end = r.y >> 1; full = r.y & 1;
        }
    }
    __device__ void init(const int2 *ranges, int begin, int end) { rg = ranges; p = begin; p_end = end; load(); }
    __device__ bool valid() const { return p < p_end; }
    __device__ void next()
    {
        if (++n == n_end) { ++p; load(); }
    }
};

// Per-lane view of the query this lane's score column belongs to.
struct QueryPred {
    uint32_t kmask;  // key code bits that make a key visible regardless of image
    uint32_t img;    // image id that own-image keys must match (never matches when disabled)
    int32_t row;     // query position i
    __device__ void init(uint32_t qcode, int cls, int32_t i)
    {
        row = i;
        const bool sees_all = (qcode & kCodeText) || cls == BS_DENSE;
        kmask = sees_all ? 0xffffffffu : (kCodeText | ((cls & 1) ? kCodeSink : 0u));
        img = (!sees_all && (cls & 2)) ? (qcode & kCodeImgMask) : 0x7fffffffu;
    }
    __device__ bool allowed(uint32_t kcode, int32_t j) const
    {
        return j <= row && (((kcode & kmask) != 0u) || ((kcode & kCodeImgMask) == img));
    }
};

// Online-softmax update for one 32-query x 64-key score block held as two 32x32 C tiles.
// Lane (hl = lane/32, col = lane%32) holds, for query col, keys 32*kb + 8*(v/4) + 4*hl + v%4.
// On return s[][] holds p = exp2(s*c - m*c); m is the running max (raw score units), l the
// lane's partial running sum; alpha is the factor the output accumulators must be scaled by.
__device__ inline void softmax_block(floatx16 (&s)[2], float &m_run, float &l_run, float &alpha, float c)
{
    float mx = s[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[kb][v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;  // row fully masked so far: p = 0
    const float mc = m_use * c;
    alpha = exp2f(m_run * c - mc);  // m_run = -inf -> 0
    float sum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            float p = exp2f(fmaf(s[kb][v], c, -mc));
            s[kb][v] = p;
            sum += p;
        }
    l_run = l_run * alpha + sum;
    m_run = m_new;
}

// Apply the element predicate to a PARTIAL tile.  lds_code holds the 64 key codes of the tile.
__device__ inline void mask_block(floatx16 (&s)[2], const QueryPred &qp, const uint32_t *lds_code, int n0, int hl)
{
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int key = 32 * kb + 8 * g + 4 * hl;
            const uint4 kc = *reinterpret_cast<const uint4 *>(lds_code + key);
            const uint32_t kcs[4] = {kc.x, kc.y, kc.z, kc.w};
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (!qp.allowed(kcs[r], n0 + key + r)) s[kb][4 * g + r] = -INFINITY;
        }
}

// ------------------------------------------------------------------------------------ bf16

template <int D>
__global__ __launch_bounds__(kThreads, 2) void attn_prefill_bf16(KernelArgs a)
{
    constexpr int KS = D * 2 + 16;       // K row stride in LDS (bytes): 16 B pad kills bank conflicts
    constexpr int VS = kBlockN * 2 + 16; // V^T row stride in LDS (bytes)
    constexpr int KCH = D / 8;           // 16-byte chunks per K row
    constexpr int K_PER_THREAD = kBlockN * KCH / kThreads;
    __shared__ __align__(16) unsigned char lds_k[kBlockN * KS];
    __shared__ __align__(16) unsigned char lds_v[D * VS];
    __shared__ __align__(16) uint32_t lds_code[kBlockN];

    const int2 item = a.work[blockIdx.x];
    const int head = item.x, m = item.y;
    const int cls = a.head_class[head];
    const int kvh = head / a.G;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hl = lane >> 5, col = lane & 31;
    const int L = a.L;
    const int row = m * kBlockM + wave * 32 + col;

    const __bf16 *qh = reinterpret_cast<const __bf16 *>(a.q) + (size_t)head * L * D;
    const __bf16 *kh = reinterpret_cast<const __bf16 *>(a.k) + (size_t)kvh * L * D;
    const __bf16 *vh = reinterpret_cast<const __bf16 *>(a.v) + (size_t)kvh * L * D;

    // Q^T operand: lane holds Q[row][16t + 8hl .. +8] for every 16-wide slice t of the head dim.
    bf16x8 qreg[D / 16];
#pragma unroll
    for (int t = 0; t < D / 16; ++t) {
        uint4 raw = make_uint4(0, 0, 0, 0);
        if (row < L) raw = *reinterpret_cast<const uint4 *>(qh + (size_t)row * D + 16 * t + 8 * hl);
        qreg[t] = __builtin_bit_cast(bf16x8, raw);
    }
    QueryPred qp;
    qp.init(row < L ? a.code[row] : kCodeText, cls, row);

    floatx16 o[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    TileWalker tw;
    tw.init(a.ranges, a.row_ptr[cls * (a.M + 1) + m], a.row_ptr[cls * (a.M + 1) + m + 1]);

    // register staging of the next tile's K / V / codes (global -> regs -> LDS)
    uint4 kst[K_PER_THREAD];
    uint4 vst[4];
    uint32_t cst = 0;
    // V task of this thread: 4 consecutive keys (quad x) x 8 consecutive channels (group y)
    const int vx = (tid >> 2) & 15, vy = (tid & 3) + 4 * (tid >> 6);
    const bool v_task = vy < D / 8;

    auto fetch = [&](int n) {
        const int n0 = n * kBlockN;
#pragma unroll
        for (int r = 0; r < K_PER_THREAD; ++r) {
            const int idx = tid + kThreads * r, key = idx / KCH, ch = idx % KCH;
            kst[r] = make_uint4(0, 0, 0, 0);
            if (n0 + key < L) kst[r] = *reinterpret_cast<const uint4 *>(kh + (size_t)(n0 + key) * D + ch * 8);
        }
        if (v_task) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int key = 4 * vx + r;
                vst[r] = make_uint4(0, 0, 0, 0);
                if (n0 + key < L) vst[r] = *reinterpret_cast<const uint4 *>(vh + (size_t)(n0 + key) * D + vy * 8);
            }
        }
        if (tid < kBlockN) cst = (n0 + tid < L) ? a.code[n0 + tid] : 0u;
    };
    auto stage = [&]() {
#pragma unroll
        for (int r = 0; r < K_PER_THREAD; ++r) {
            const int idx = tid + kThreads * r, key = idx / KCH, ch = idx % KCH;
            *reinterpret_cast<uint4 *>(lds_k + key * KS + ch * 16) = kst[r];
        }
        if (v_task) {
            // 4 keys x 8 channels -> 8 channels x 4 keys; keys of a 16-group are laid out
            // [0..3, 8..11 | 4..7, 12..15] so each lane half reads its 8 MFMA slots as one 16 B word.
            const int colb = 32 * (vx >> 2) + 16 * (vx & 1) + 8 * ((vx & 3) >> 1);
            const uint32_t w[4][4] = {{vst[0].x, vst[0].y, vst[0].z, vst[0].w},
                                      {vst[1].x, vst[1].y, vst[1].z, vst[1].w},
                                      {vst[2].x, vst[2].y, vst[2].z, vst[2].w},
                                      {vst[3].x, vst[3].y, vst[3].z, vst[3].w}};
#pragma unroll
            for (int pr = 0; pr < 4; ++pr) {
                // channel 2pr (low halves) and 2pr+1 (high halves)
                uint2 lo, hi;
                lo.x = __builtin_amdgcn_perm(w[1][pr], w[0][pr], 0x05040100u);
                lo.y = __builtin_amdgcn_perm(w[3][pr], w[2][pr], 0x05040100u);
                hi.x = __builtin_amdgcn_perm(w[1][pr], w[0][pr], 0x07060302u);
                hi.y = __builtin_amdgcn_perm(w[3][pr], w[2][pr], 0x07060302u);
                *reinterpret_cast<uint2 *>(lds_v + (8 * vy + 2 * pr) * VS + colb) = lo;
                *reinterpret_cast<uint2 *>(lds_v + (8 * vy + 2 * pr + 1) * VS + colb) = hi;
            }
        }
        if (tid < kBlockN) lds_code[tid] = cst;
    };

    if (tw.valid()) fetch(tw.n);
    while (tw.valid()) {
        const int n = tw.n;
        const bool full = tw.full;
        __syncthreads();  // previous tile's LDS reads are done
        stage();
        __syncthreads();
        tw.next();
        if (tw.valid()) fetch(tw.n);  // in flight while this tile is computed

        // S^T = K Q^T
        floatx16 s[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
#pragma unroll
            for (int t = 0; t < D / 16; ++t) {
                const bf16x8 ka = *reinterpret_cast<const bf16x8 *>(lds_k + (32 * kb + col) * KS + (16 * t + 8 * hl) * 2);
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[t], s[kb], 0, 0, 0);
            }
        }
        if (!full) mask_block(s, qp, lds_code, n * kBlockN, hl);

        float alpha;
        softmax_block(s, m_run, l_run, alpha, a.scale_log2e);
        if (__any(alpha != 1.f)) {
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
        }

        // P^T as bf16 B operands: slots e of MFMA (kb, t) are C values v = 8t + e
        bf16x8 pf[2][2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[kb][t][e] = (__bf16)s[kb][8 * t + e];

        // O^T += V^T P^T
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const bf16x8 va = *reinterpret_cast<const bf16x8 *>(lds_v + (32 * db + col) * VS + 32 * (2 * kb + t) + 16 * hl);
                    o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pf[kb][t], o[db], 0, 0, 0);
                }
    }

    // epilogue: divide by the running sum, round, store.  Empty rows (l = 0) give zeros.
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    if (row < L) {
        __bf16 *orow = reinterpret_cast<__bf16 *>(a.out) + ((size_t)head * L + row) * D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
                bf16x4 w;
#pragma unroll
                for (int r = 0; r < 4; ++r) w[r] = (__bf16)(o[db][4 * g + r] * inv);
                *reinterpret_cast<bf16x4 *>(orow + 32 * db + 8 * g + 4 * hl) = w;
            }
    }
}

// ------------------------------------------------------------------------------------ fp32
// Same structure with fp32 MFMA (32x32x2) end to end; P stays fp32.  Parity path for fp32
// inputs, not tuned.  Dynamic LDS: K[64][D+1] floats, V[64][D+8] floats, 64 codes.

template <int D>
__global__ __launch_bounds__(kThreads, 1) void attn_prefill_f32(KernelArgs a)
{
    constexpr int KS = D + 1, VS = D + 8;
    extern __shared__ __align__(16) unsigned char smem[];
    float *lds_k = reinterpret_cast<float *>(smem);
    float *lds_v = lds_k + kBlockN * KS;
    uint32_t *lds_code = reinterpret_cast<uint32_t *>(lds_v + kBlockN * VS);

    const int2 item = a.work[blockIdx.x];
    const int head = item.x, m = item.y;
    const int cls = a.head_class[head];
    const int kvh = head / a.G;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hl = lane >> 5, col = lane & 31;
    const int L = a.L;
    const int row = m * kBlockM + wave * 32 + col;

    const float *qh = reinterpret_cast<const float *>(a.q) + (size_t)head * L * D;
    const float *kh = reinterpret_cast<const float *>(a.k) + (size_t)kvh * L * D;
    const float *vh = reinterpret_cast<const float *>(a.v) + (size_t)kvh * L * D;

    float qreg[D / 2];  // Q[row][2t + hl]
#pragma unroll
    for (int t = 0; t < D / 2; ++t) qreg[t] = row < L ? qh[(size_t)row * D + 2 * t + hl] : 0.f;
    QueryPred qp;
    qp.init(row < L ? a.code[row] : kCodeText, cls, row);

    floatx16 o[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    TileWalker tw;
    tw.init(a.ranges, a.row_ptr[cls * (a.M + 1) + m], a.row_ptr[cls * (a.M + 1) + m + 1]);

    for (; tw.valid(); tw.next()) {
        const int n0 = tw.n * kBlockN;
        __syncthreads();
        for (int idx = tid; idx < kBlockN * (D / 4); idx += kThreads) {
            const int key = idx / (D / 4), ch = idx % (D / 4);
            floatx4 kk = {0.f, 0.f, 0.f, 0.f}, vv = {0.f, 0.f, 0.f, 0.f};
            if (n0 + key < L) {
                kk = *reinterpret_cast<const floatx4 *>(kh + (size_t)(n0 + key) * D + ch * 4);
                vv = *reinterpret_cast<const floatx4 *>(vh + (size_t)(n0 + key) * D + ch * 4);
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                lds_k[key * KS + ch * 4 + r] = kk[r];
                lds_v[key * VS + ch * 4 + r] = vv[r];
            }
        }
        if (tid < kBlockN) lds_code[tid] = (n0 + tid < L) ? a.code[n0 + tid] : 0u;
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
        if (!tw.full) mask_block(s, qp, lds_code, n0, hl);

        float alpha;
        softmax_block(s, m_run, l_run, alpha, a.scale_log2e);
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

    const float l_tot = l_run + __shfl_xor(l_run, 32);
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
constexpr size_t f32_lds_bytes() { return (size_t)kBlockN * (D + 1) * 4 + (size_t)kBlockN * (D + 8) * 4 + kBlockN * 4; }

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
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return bs::fail_hip(e, "hipGetDevice");

    const int64_t M1 = (int64_t)tm->M + 1;
    int64_t total_ranges = 0;
    for (int c = 0; c < 4; ++c) total_ranges += (int64_t)tm->cls[c].ranges.size();
    if (total_ranges >= INT32_MAX) return BS_EUNSUPPORTED;

    auto align = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t off_code = 0;
    const size_t off_rowptr = align(off_code + (size_t)tm->L * 4);
    const size_t off_ranges = align(off_rowptr + (size_t)(4 * M1) * 4);
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
    int32_t *rp = reinterpret_cast<int32_t *>(host.data() + off_rowptr);
    int2 *rg = reinterpret_cast<int2 *>(host.data() + off_ranges);
    int64_t base = 0;
    for (int c = 0; c < 4; ++c) {
        const bs::ClassLists &cl = tm->cls[c];
        for (int64_t m = 0; m < M1; ++m) rp[c * M1 + m] = (int32_t)(base + cl.row_ptr[m]);
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
    d->row_ptr = reinterpret_cast<const int32_t *>(b + off_rowptr);
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
    a.code = d->code; a.row_ptr = d->row_ptr; a.ranges = d->ranges; a.work = d->work;
    a.head_class = d->head_class;
    a.L = tm->L; a.M = tm->M; a.G = gqa_group;
    a.scale_log2e = scale * 1.4426950408889634f;

    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)d->n_work), block(bs::kThreads);
    if (dtype == BS_BF16) {
        if (head_dim == 128) hipLaunchKernelGGL(bs::attn_prefill_bf16<128>, grid, block, 0, st, a);
        else hipLaunchKernelGGL(bs::attn_prefill_bf16<64>, grid, block, 0, st, a);
    } else {
        if (head_dim == 128) {
            constexpr size_t lds = bs::f32_lds_bytes<128>();
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(bs::attn_prefill_f32<128>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return bs::fail_hip(e, "hipFuncSetAttribute");
            hipLaunchKernelGGL(bs::attn_prefill_f32<128>, grid, block, lds, st, a);
        } else {
            constexpr size_t lds = bs::f32_lds_bytes<64>();
            hipLaunchKernelGGL(bs::attn_prefill_f32<64>, grid, block, lds, st, a);
        }
    }
    e = hipGetLastError();
    if (e != hipSuccess) return bs::fail_hip(e, "kernel launch");
    return BS_OK;
}

extern "C" const char *bs_last_error(void) { return bs::g_last_error; }
