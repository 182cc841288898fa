// Offline characterisation of attention heads on the GPU (paper Sec. 4, Alg. 1; Alg. 2 on the host).
//
// Alg. 1 compares, per head, the output of attention under each sparse mask with the output under
// the dense causal mask and keeps the first mask (Sink, Intra-Image, Intra-Image+Sink) whose
// normalised squared error is below alpha_layer.  Here the four outputs come from the library's
// own prefill kernel (ONE tile map of the prompt, bound in turn to "every head Dense / Sink /
// Intra-Image / Intra-Image+Sink"), the error is reduced
// by an HBM-bound kernel that reads both outputs once, and a last tiny kernel takes the decision
// in fp64.  Evaluating all three masks for every head instead of stopping at the first that
// passes gives the same head types (the stop only saves work, and the sparse runs are the cheap
// part next to the dense reference) and keeps the whole sequence free of host round trips.

#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <new>
#include <vector>

#include "blindsight.h"
#include "device_map.h"

namespace bs {

constexpr int kNmseThreads = 256;
constexpr int kNmseChunks = 256;   // workgroups per head

__device__ inline void widen8(const uint4 &raw, float (&f)[8])
{
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(w[i] << 16);
        f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}

__device__ inline double wave_sum(double x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

// sums[head] += (sum (a - r)^2, sum r^2) over the head's `n` elements; grid (kNmseChunks, heads).
// Differences of two bf16 (or fp32) values are formed in fp32 (fp64 for fp32 inputs) and squared
// and accumulated in fp64, so the result is the fp64 sum up to the order of the additions.
template <typename T>
__global__ __launch_bounds__(kNmseThreads) void head_sq_error(const T *__restrict__ a, const T *__restrict__ r,
                                                               int64_t n, double *__restrict__ sums)
{
    constexpr int kVec = 16 / sizeof(T);
    const int head = blockIdx.y;
    const T *ah = a + (int64_t)head * n;
    const T *rh = r + (int64_t)head * n;
    const int64_t n_vec = n / kVec;
    const int64_t per_chunk = (n_vec + kNmseChunks - 1) / kNmseChunks;
    const int64_t v0 = (int64_t)blockIdx.x * per_chunk;
    const int64_t v1 = v0 + per_chunk < n_vec ? v0 + per_chunk : n_vec;
    double err = 0.0, ref = 0.0;
#pragma unroll 4
    for (int64_t i = v0 + threadIdx.x; i < v1; i += kNmseThreads) {
        const uint4 ra = reinterpret_cast<const uint4 *>(ah)[i];
        const uint4 rr = reinterpret_cast<const uint4 *>(rh)[i];
        if constexpr (sizeof(T) == 2) {
            float fa[8], fr[8];
            widen8(ra, fa);
            widen8(rr, fr);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const double d = (double)(fa[e] - fr[e]), x = (double)fr[e];
                err += d * d;
                ref += x * x;
            }
        } else {
            const float fa[4] = {__uint_as_float(ra.x), __uint_as_float(ra.y), __uint_as_float(ra.z), __uint_as_float(ra.w)};
            const float fr[4] = {__uint_as_float(rr.x), __uint_as_float(rr.y), __uint_as_float(rr.z), __uint_as_float(rr.w)};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const double d = (double)fa[e] - (double)fr[e], x = (double)fr[e];
                err += d * d;
                ref += x * x;
            }
        }
    }
    if (blockIdx.x == kNmseChunks - 1) {   // ragged tail (n not a multiple of the vector width)
        for (int64_t i = n_vec * kVec + threadIdx.x; i < n; i += kNmseThreads) {
            double fa, fr;
            if constexpr (sizeof(T) == 2) {
                fa = (double)__uint_as_float((uint32_t)reinterpret_cast<const uint16_t *>(ah)[i] << 16);
                fr = (double)__uint_as_float((uint32_t)reinterpret_cast<const uint16_t *>(rh)[i] << 16);
            } else {
                fa = (double)ah[i];
                fr = (double)rh[i];
            }
            err += (fa - fr) * (fa - fr);
            ref += fr * fr;
        }
    }
    __shared__ double part[2][kNmseThreads / 64];
    err = wave_sum(err);
    ref = wave_sum(ref);
    if ((threadIdx.x & 63) == 0) {
        part[0][threadIdx.x >> 6] = err;
        part[1][threadIdx.x >> 6] = ref;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double e = 0.0, x = 0.0;
#pragma unroll
        for (int w = 0; w < kNmseThreads / 64; ++w) {
            e += part[0][w];
            x += part[1][w];
        }
        atomicAdd(&sums[2 * head], e);
        atomicAdd(&sums[2 * head + 1], x);
    }
}

__global__ void fill_zero(double *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0.0;
}

// Alg. 1's decision: sums [3][heads][2] -> nmse [3][heads], head_type [heads].
__global__ void select_head_type(const double *__restrict__ sums, int heads, double alpha,
                                 double *__restrict__ nmse, uint8_t *__restrict__ head_type)
{
    const int h = blockIdx.x * blockDim.x + threadIdx.x;
    if (h >= heads) return;
    uint8_t type = BS_DENSE;
    for (int m = 2; m >= 0; --m) {   // descending, so the earliest passing mask is what stays
        const double err = sums[(m * heads + h) * 2], ref = sums[(m * heads + h) * 2 + 1];
        const double e = ref == 0.0 ? (err == 0.0 ? 0.0 : INFINITY) : err / ref;
        nmse[m * heads + h] = e;
        if (e < alpha) type = (uint8_t)(m + 1);
    }
    head_type[h] = type;
}

static int launch_sq_error(const void *a, const void *r, int dtype, int heads, int64_t n, double *sums,
                           hipStream_t st)
{
    const dim3 grid(kNmseChunks, heads);
    if (dtype == BS_BF16)
        hipLaunchKernelGGL(head_sq_error<uint16_t>, grid, dim3(kNmseThreads), 0, st,
                           (const uint16_t *)a, (const uint16_t *)r, n, sums);
    else
        hipLaunchKernelGGL(head_sq_error<float>, grid, dim3(kNmseThreads), 0, st, (const float *)a,
                           (const float *)r, n, sums);
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? BS_OK : fail_hip(e, "head_sq_error launch");
}

// Device buffers of one characterisation, from the library's block cache; handed back on every way
// out (the caller has drained the stream by then, so the blocks are free for anyone at once).
struct Buffers {
    int device = -1;
    void *ref = nullptr, *cand = nullptr, *small = nullptr;   // small: sums [6 Hq], nmse [3 Hq], types [Hq]
    size_t ref_cap = 0, cand_cap = 0, small_cap = 0;
    ~Buffers()
    {
        pool_release(device, ref, ref_cap, nullptr);
        pool_release(device, cand, cand_cap, nullptr);
        pool_release(device, small, small_cap, nullptr);
    }
};

}  // namespace bs

extern "C" int bs_head_sq_error(const void *attn_mask, const void *attn_ref, int32_t dtype, int32_t n_heads,
                                int64_t elems_per_head, double *sums, void *stream)
{
    if (!attn_mask || !attn_ref || !sums || n_heads <= 0 || elems_per_head <= 0) return BS_EINVAL;
    if (dtype != BS_BF16 && dtype != BS_F32) return BS_EUNSUPPORTED;
    // the vector loads need each head's first element on a 16-byte boundary
    const int64_t elem = dtype == BS_BF16 ? 2 : 4;
    if (((uintptr_t)attn_mask | (uintptr_t)attn_ref) % 16 != 0 || (n_heads > 1 && elems_per_head * elem % 16 != 0))
        return BS_EUNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(bs::fill_zero, dim3((2 * n_heads + 255) / 256), dim3(256), 0, st, sums, 2 * n_heads);
    return bs::launch_sq_error(attn_mask, attn_ref, dtype, n_heads, elems_per_head, sums, st);
}

extern "C" int bs_characterize_prompt(const void *q, const void *k, const void *v, const bs_span *spans,
                                      int32_t n_spans, int32_t seq_len, int32_t sink_len, int32_t dtype,
                                      int32_t n_q_heads, int32_t gqa_group, int32_t head_dim, float scale,
                                      double alpha, uint32_t map_flags, const int32_t *sink_offsets,
                                      int32_t n_sink_offsets, int32_t window, uint8_t *head_type, double *nmse,
                                      void *stream)
{
    using namespace bs;
    if (!q || !k || !v || !head_type || n_q_heads <= 0 || seq_len <= 0 || head_dim <= 0 || !(alpha == alpha))
        return BS_EINVAL;
    if (dtype != BS_BF16 && dtype != BS_F32) return BS_EUNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    const int64_t per_head = (int64_t)seq_len * head_dim;
    const size_t out_bytes = (size_t)n_q_heads * per_head * (dtype == BS_BF16 ? 2 : 4);
    Buffers b;
    hipError_t e;
    if ((e = hipGetDevice(&b.device)) != hipSuccess) return fail_hip(e, "hipGetDevice");
    const size_t small_bytes = sizeof(double) * 9 * (size_t)n_q_heads + (size_t)n_q_heads;
    if ((e = pool_acquire(b.device, out_bytes, st, &b.ref, &b.ref_cap)) != hipSuccess) return fail_hip(e, "hipMalloc(reference output)");
    if ((e = pool_acquire(b.device, out_bytes, st, &b.cand, &b.cand_cap)) != hipSuccess) return fail_hip(e, "hipMalloc(masked output)");
    if ((e = pool_acquire(b.device, small_bytes, st, &b.small, &b.small_cap)) != hipSuccess) return fail_hip(e, "hipMalloc(sums)");
    double *sums = static_cast<double *>(b.small), *nmse_dev = sums + 6 * (size_t)n_q_heads;
    uint8_t *type_dev = reinterpret_cast<uint8_t *>(nmse_dev + 3 * (size_t)n_q_heads);

    int rc = BS_OK;
    hipLaunchKernelGGL(fill_zero, dim3((6 * n_q_heads + 255) / 256), dim3(256), 0, st, sums, 6 * n_q_heads);
    std::vector<uint8_t> cls;
    try {
        cls.assign(n_q_heads, (uint8_t)BS_DENSE);
    } catch (const std::bad_alloc &) {
        rc = BS_ENOMEM;
    }
    // one tile map of the prompt for the four runs: the per-class lists depend on the spans only
    bs_tilemap *tm = nullptr;
    if (rc == BS_OK)
        rc = bs_build_tilemap_model(spans, n_spans, seq_len, cls.data(), n_q_heads, sink_len, 128, 64, map_flags,
                                    sink_offsets, n_sink_offsets, window, &tm);
    for (int c = 0; c < 4 && rc == BS_OK; ++c) {   // Dense reference, then Sink, Intra-Image, Intra-Image+Sink
        std::fill(cls.begin(), cls.end(), (uint8_t)c);
        rc = bs_tilemap_rebind(tm, cls.data(), n_q_heads);
        if (rc == BS_OK)
            rc = bs_attn_prefill(q, k, v, c == 0 ? b.ref : b.cand, tm, dtype, n_q_heads, gqa_group, head_dim, scale, st);
        if (rc == BS_OK && c > 0)
            rc = launch_sq_error(b.cand, b.ref, dtype, n_q_heads, per_head, sums + (size_t)(c - 1) * 2 * n_q_heads, st);
    }
    bs_tilemap_destroy(tm);
    if (rc == BS_OK) {
        hipLaunchKernelGGL(select_head_type, dim3((n_q_heads + 63) / 64), dim3(64), 0, st, sums, n_q_heads, alpha,
                           nmse_dev, type_dev);
        if ((e = hipGetLastError()) != hipSuccess) rc = fail_hip(e, "select_head_type launch");
    }
    // the buffers are about to be handed back: wait for the queued work on every way out
    if ((e = hipStreamSynchronize(st)) != hipSuccess && rc == BS_OK) rc = fail_hip(e, "hipStreamSynchronize");
    if (rc != BS_OK) return rc;
    if ((e = hipMemcpy(head_type, type_dev, n_q_heads, hipMemcpyDeviceToHost)) != hipSuccess) return fail_hip(e, "hipMemcpy(head_type)");
    if (nmse && (e = hipMemcpy(nmse, nmse_dev, sizeof(double) * 3 * n_q_heads, hipMemcpyDeviceToHost)) != hipSuccess)
        return fail_hip(e, "hipMemcpy(nmse)");
    return BS_OK;
}

extern "C" int bs_aggregate_head_type(const double *fraction, double gamma_d, double gamma_s, double gamma_i)
{
    if (!fraction) return BS_EINVAL;
    if (fraction[BS_DENSE] > gamma_d) return BS_DENSE;
    if (fraction[BS_SINK] > gamma_s) return BS_SINK;
    if (fraction[BS_INTRA] > gamma_i) return BS_INTRA;
    return BS_INTRA_SINK;
}

extern "C" int bs_aggregate_layer(const uint8_t *head_types, int32_t n_prompts, int32_t n_q_heads, double gamma_d,
                                  double gamma_s, double gamma_i, uint8_t *head_class, double *fraction)
{
    if (!head_types || !head_class || n_prompts <= 0 || n_q_heads <= 0) return BS_EINVAL;
    for (int64_t i = 0; i < (int64_t)n_prompts * n_q_heads; ++i)
        if (head_types[i] > 3) return BS_EINVAL;
    for (int32_t h = 0; h < n_q_heads; ++h) {
        int64_t count[4] = {0, 0, 0, 0};
        for (int32_t p = 0; p < n_prompts; ++p) ++count[head_types[(int64_t)p * n_q_heads + h]];
        double f[4];
        for (int c = 0; c < 4; ++c) f[c] = (double)count[c] / (double)n_prompts;
        if (fraction)
            for (int c = 0; c < 4; ++c) fraction[4 * h + c] = f[c];
        head_class[h] = (uint8_t)bs_aggregate_head_type(f, gamma_d, gamma_s, gamma_i);
    }
    return BS_OK;
}

extern "C" double bs_alpha_layer(double alpha_first, double alpha_last, int32_t layer_idx, int32_t num_layers)
{
    if (num_layers <= 0 || layer_idx < 0 || layer_idx > num_layers) return NAN;
    return alpha_first + (alpha_last - alpha_first) * (double)layer_idx / (double)num_layers;
}
