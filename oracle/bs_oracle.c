/*
 * CPU oracle for masked causal prefill attention with per-head sparsity classes.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the sparse
 * prefill-attention path must compute.  It shares nothing with the HIP library: no header,
 * no helper, no table.  Only tests, the smoke check and the bench's CPU-baseline leg may
 * load it.
 *
 * What it states (paper sections in brackets):
 *   - attention = SoftMax(Q K^T * scale + Mask) V, causal in prefill            [Sec. 3.1]
 *   - the mask of each head class, from the positions of text and image tokens  [Sec. 3.2]
 *       Dense            : every earlier key
 *       Sink             : text keys and sink keys, no intra-image attention
 *       Intra-Image      : text keys and keys of the query's own image
 *       Intra-Image+Sink : union of the two
 *     and, for every class, a text query attends to all earlier tokens          [Sec. 3.2]
 *   - imgid[t] = 0 for text, g >= 1 for a token of image g; isimgsink marks the
 *     sink tokens                                                                [App. kernel, Notation]
 *   - the sink of an image is a prefix of that image                             [Sec. 6.1, mask generation]
 *   - model variant with non-causal attention inside an image (Gemma 3): the dense mask is the
 *     model's default mask [Sec. 2], here causal OR "query and key in the same image", and every
 *     sparse mask is its class pattern restricted to that dense mask; the sinks of such a model
 *     sit at a fixed list of offsets inside every image       [Sec. 6.1, App. "Attention Sink
 *     Positions in Gemma 3"].  Selected by img_bidir != 0 / a sink offset list.
 *   - layers whose default mask is a sliding window: the dense mask keeps only the `window`
 *     most recent keys of a query (i - j < window), for text queries too [App. kernel, "Dense
 *     Attention Subroutine": text queries follow the dense mask, causal or sliding window as per
 *     the original model]; the sparse masks live inside it.  With img_bidir the keys of the
 *     query's own image stay visible at any distance.  window <= 0: no window.
 *
 * Readings taken where the paper's pseudo-code is loose (Alg. 3-7):
 *   - the running sum l divides the output once at the end (the SoftMax of Sec. 3.1);
 *   - one softmax per row over the union of sink keys and own-image keys: a key that is
 *     both is counted once;
 *   - the class predicate applies element-wise in every tile, mixed text/image tiles included;
 *   - causality is on original token positions;
 *   - a row whose allowed set is empty yields zeros.
 *
 * Everything is fp64 from fp32 inputs (bf16 inputs are widened exactly by the caller).
 * Parity pins live in tests/test_oracle_pins.py.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { BSO_DENSE = 0, BSO_SINK = 1, BSO_INTRA = 2, BSO_INTRA_SINK = 3 };

/* spans: n_spans rows of (start, end, sink).  Fills imgid[L] and issink[L].
 * Returns 0, or a negative code naming the first violated rule. */
int bso_token_arrays(const int32_t *spans, int32_t n_spans, int32_t L, int32_t sink_len,
                     const int32_t *sink_offsets, int32_t n_offsets, int32_t *imgid, uint8_t *issink)
{
    if (L < 0 || n_spans < 0 || sink_len < 0 || sink_len > L || n_offsets < 0) return -1;
    for (int32_t o = 0; o < n_offsets; ++o)
        if (sink_offsets[o] < 0) return -4;
    int32_t prev_end = 0;
    for (int32_t g = 0; g < n_spans; ++g) {
        int32_t s = spans[3 * g], e = spans[3 * g + 1], k = spans[3 * g + 2];
        if (s < prev_end || e <= s || e > L) return -2;
        if (k < 0 || k > e - s) return -3;
        prev_end = e;
    }
    for (int32_t t = 0; t < L; ++t) {
        imgid[t] = 0;
        issink[t] = (uint8_t)(t < sink_len);
    }
    for (int32_t g = 0; g < n_spans; ++g) {
        int32_t s = spans[3 * g], e = spans[3 * g + 1], k = spans[3 * g + 2];
        for (int32_t t = s; t < e; ++t) {
            imgid[t] = g + 1;
            if (t - s < k) issink[t] = 1;
        }
        /* sinks at fixed offsets inside every image (offsets past the image's end are ignored) */
        for (int32_t o = 0; o < n_offsets; ++o)
            if (sink_offsets[o] < e - s) issink[s + sink_offsets[o]] = 1;
    }
    return 0;
}

/* May query i attend to key j in a head of class cls?  [Sec. 3.2]
 * img_bidir: tokens of one image also see the later tokens of that image (the model's dense mask). */
int bso_allowed(int cls, int32_t i, int32_t j, const int32_t *imgid, const uint8_t *issink, int img_bidir,
                int32_t window)
{
    /* the dense mask: causal, optionally windowed, optionally the whole own image */
    int causal = j <= i && (window <= 0 || i - j < window);
    if (!causal && !(img_bidir && imgid[i] != 0 && imgid[j] == imgid[i])) return 0;
    if (imgid[i] == 0) return 1;         /* text queries see all earlier tokens */
    if (cls == BSO_DENSE) return 1;
    if (imgid[j] == 0) return 1;         /* text keys stay visible: the vertical bands */
    if ((cls == BSO_SINK || cls == BSO_INTRA_SINK) && issink[j]) return 1;
    if ((cls == BSO_INTRA || cls == BSO_INTRA_SINK) && imgid[j] == imgid[i]) return 1;
    return 0;
}

/* Dense L x L bitmap (row-major, 1 = allowed).  Small prompts only. */
void bso_mask(int cls, int32_t L, const int32_t *imgid, const uint8_t *issink, int img_bidir, int32_t window,
              uint8_t *mask)
{
    for (int32_t i = 0; i < L; ++i)
        for (int32_t j = 0; j < L; ++j)
            mask[(size_t)i * L + j] = (uint8_t)bso_allowed(cls, i, j, imgid, issink, img_bidir, window);
}

/* Number of allowed (i, j) pairs, by enumeration. */
int64_t bso_pair_count(int cls, int32_t L, const int32_t *imgid, const uint8_t *issink, int img_bidir,
                       int32_t window)
{
    int64_t total = 0;
#pragma omp parallel for schedule(dynamic, 64) reduction(+ : total)
    for (int32_t i = 0; i < L; ++i) {
        int64_t c = 0;
        for (int32_t j = 0; j < L; ++j) c += bso_allowed(cls, i, j, imgid, issink, img_bidir, window);
        total += c;
    }
    return total;
}

/* The listed rows of the bitmap: mask is [n_rows][L].  For prompts too long for bso_mask. */
void bso_mask_rows(int cls, int32_t L, const int32_t *imgid, const uint8_t *issink, int img_bidir, int32_t window,
                   const int32_t *rows, int32_t n_rows, uint8_t *mask)
{
#pragma omp parallel for schedule(dynamic, 8)
    for (int32_t r = 0; r < n_rows; ++r)
        for (int32_t j = 0; j < L; ++j)
            mask[(size_t)r * L + j] = (uint8_t)bso_allowed(cls, rows[r], j, imgid, issink, img_bidir, window);
}

/* Number of allowed (i, j) pairs of the listed rows, by enumeration. */
int64_t bso_pair_count_rows(int cls, int32_t L, const int32_t *imgid, const uint8_t *issink, int img_bidir,
                            int32_t window, const int32_t *rows, int32_t n_rows)
{
    int64_t total = 0;
#pragma omp parallel for schedule(dynamic, 64) reduction(+ : total)
    for (int32_t r = 0; r < n_rows; ++r) {
        int64_t c = 0;
        for (int32_t j = 0; j < L; ++j) c += bso_allowed(cls, rows[r], j, imgid, issink, img_bidir, window);
        total += c;
    }
    return total;
}

/* Reduce the element mask to tile states for the listed query tiles.
 * Tile (m, n) covers rows [m*bm, m*bm+bm) x keys [n*bn, n*bn+bn); indices >= L count as
 * not allowed.  state: 0 = no element allowed, 2 = all bm*bn allowed, 1 = otherwise.
 * states is [n_qtiles][N], N = ceil(L / bn). */
void bso_tile_states(int cls, int32_t L, const int32_t *imgid, const uint8_t *issink, int img_bidir,
                     int32_t window, int32_t bm, int32_t bn, const int32_t *qtiles, int32_t n_qtiles,
                     uint8_t *states)
{
    int32_t N = (L + bn - 1) / bn;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t t = 0; t < n_qtiles; ++t) {
        int32_t m = qtiles[t];
        for (int32_t n = 0; n < N; ++n) {
            int64_t cnt = 0;
            for (int32_t i = m * bm; i < m * bm + bm; ++i) {
                if (i >= L) continue;
                for (int32_t j = n * bn; j < n * bn + bn; ++j) {
                    if (j >= L) continue;
                    cnt += bso_allowed(cls, i, j, imgid, issink, img_bidir, window);
                }
            }
            states[(size_t)t * N + n] = (uint8_t)(cnt == 0 ? 0 : (cnt == (int64_t)bm * bn ? 2 : 1));
        }
    }
}

/* The same reduction for query tiles given as explicit row lists (a tile map may group the
 * query rows in another order than their positions): rows is [n_qtiles][bm], entries < 0 or
 * >= L are slots without a row and count as not allowed, like positions past the end above. */
void bso_tile_states_rows(int cls, int32_t L, const int32_t *imgid, const uint8_t *issink, int img_bidir,
                          int32_t window, int32_t bm, int32_t bn, const int32_t *rows, int32_t n_qtiles,
                          uint8_t *states)
{
    int32_t N = (L + bn - 1) / bn;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t t = 0; t < n_qtiles; ++t) {
        for (int32_t n = 0; n < N; ++n) {
            int64_t cnt = 0;
            for (int32_t r = 0; r < bm; ++r) {
                int32_t i = rows[(size_t)t * bm + r];
                if (i < 0 || i >= L) continue;
                for (int32_t j = n * bn; j < n * bn + bn; ++j) {
                    if (j >= L) continue;
                    cnt += bso_allowed(cls, i, j, imgid, issink, img_bidir, window);
                }
            }
            states[(size_t)t * N + n] = (uint8_t)(cnt == 0 ? 0 : (cnt == (int64_t)bm * bn ? 2 : 1));
        }
    }
}

/* Masked softmax attention for the listed rows of every query head.
 *   q   [Hq][L][d], k, v [Hq/G][L][d] fp32;  query head h reads KV head h / G.
 *   rows: n_rows query positions (NULL = all L rows, n_rows ignored)
 *   out [Hq][n_rows][d] fp64
 * For each row: logits x_j = scale * <q_i, k_j> over the allowed set, m = max x_j,
 * out = sum_j exp(x_j - m) v_j / sum_j exp(x_j - m).  Empty allowed set -> zeros. */
int bso_attention(const float *q, const float *k, const float *v, int32_t Hq, int32_t G,
                  int32_t L, int32_t d, const uint8_t *head_class, const int32_t *imgid,
                  const uint8_t *issink, int img_bidir, int32_t window, double scale, const int32_t *rows, int32_t n_rows,
                  double *out)
{
    if (Hq <= 0 || G <= 0 || Hq % G || L <= 0 || d <= 0) return -1;
    if (!rows) n_rows = L;
    int64_t n_items = (int64_t)Hq * n_rows;
    int failed = 0;
#pragma omp parallel
    {
        double *x = (double *)malloc(sizeof(double) * (size_t)L);
        double *qi = (double *)malloc(sizeof(double) * (size_t)d);
        if (!x || !qi) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(dynamic, 8)
            for (int64_t it = 0; it < n_items; ++it) {
                int32_t h = (int32_t)(it / n_rows);
                int32_t r = (int32_t)(it % n_rows);
                int32_t i = rows ? rows[r] : r;
                int cls = head_class[h];
                const float *kh = k + (size_t)(h / G) * L * d;
                const float *vh = v + (size_t)(h / G) * L * d;
                const float *qrow = q + ((size_t)h * L + i) * d;
                double *o = out + (size_t)it * d;
                for (int32_t c = 0; c < d; ++c) { qi[c] = (double)qrow[c]; o[c] = 0.0; }

                double mx = -INFINITY;
                for (int32_t j = 0; j < L; ++j) {
                    if (!bso_allowed(cls, i, j, imgid, issink, img_bidir, window)) continue;
                    const float *kj = kh + (size_t)j * d;
                    double acc = 0.0;
#pragma omp simd reduction(+ : acc)
                    for (int32_t c = 0; c < d; ++c) acc += qi[c] * (double)kj[c];
                    x[j] = acc * scale;
                    if (x[j] > mx) mx = x[j];
                }
                if (mx == -INFINITY) continue; /* empty allowed set: zeros */
                double denom = 0.0;
                for (int32_t j = 0; j < L; ++j) {
                    if (!bso_allowed(cls, i, j, imgid, issink, img_bidir, window)) continue;
                    double p = exp(x[j] - mx);
                    denom += p;
                    const float *vj = vh + (size_t)j * d;
                    for (int32_t c = 0; c < d; ++c) o[c] += p * (double)vj[c];
                }
                for (int32_t c = 0; c < d; ++c) o[c] /= denom;
            }
        }
        free(x);
        free(qi);
    }
    return failed ? -2 : 0;
}

/* Threads the parallel regions above will use. */
#ifdef _OPENMP
#include <omp.h>
int bso_num_threads(void) { return omp_get_max_threads(); }
#else
int bso_num_threads(void) { return 1; }
#endif
