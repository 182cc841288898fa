/*
 * blindsight.h — C ABI of the MI355X sparse prefill-attention library.
 *
 * The library computes causal prefill attention over an interleaved text/image prompt in
 * which every query head carries one of four offline-assigned sparsity classes and the mask
 * follows from the prompt's image-span table alone (paper Sec. 3.2, Sec. 5, App. "BlindSight
 * Attention Kernel").  Two steps:
 *
 *   bs_build_tilemap   host, integer only: span table + class vector -> for every class and
 *                      every query tile the list of key tiles to run, each FULL (no masking
 *                      needed) or PARTIAL (element predicate needed); all other tiles are
 *                      skipped.  This replaces the paper kernel's per-tile metadata
 *                      (sink_end[M], first_image[M], the all/any(istext) tests of Alg. 3).
 *   bs_attn_prefill    device: one flash-style pass over the listed tiles (Alg. 3-7 folded
 *                      into one loop with a single running softmax per row).
 *
 * All functions return BS_OK (0) or a negative BS_E* code; nothing throws or aborts across
 * this boundary.  No function synchronises the device except where stated.
 */
#ifndef BLINDSIGHT_H
#define BLINDSIGHT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BS_OK            0
#define BS_EINVAL       (-1)  /* null pointer, negative size, malformed span table, bad class   */
#define BS_EUNSUPPORTED (-2)  /* tile size / head_dim / dtype the kernels do not implement      */
#define BS_ENOMEM       (-3)  /* host or device allocation failed                              */
#define BS_EHIP         (-4)  /* a HIP runtime call failed (no device, launch error, ...)      */

/* Head classes (paper Sec. 3.2; "headtype" in Alg. 3).  Bit 0 = sink keys visible,
 * bit 1 = own-image keys visible. */
typedef enum {
    BS_DENSE      = 0,  /* every earlier key                                        */
    BS_SINK       = 1,  /* text keys + sink keys                                    */
    BS_INTRA      = 2,  /* text keys + keys of the query's own image                */
    BS_INTRA_SINK = 3   /* union of the two                                         */
} bs_head_class;

/* Element types of q/k/v/out. */
#define BS_BF16 0
#define BS_F32  1

/* One image: tokens [start, end) of the prompt; its first `sink` tokens are sink keys
 * (paper Sec. 6.1 "Sparse Mask Generation": sinks sit at the start of an image).
 * Tokens outside every span are text (imgid = 0 in the paper's notation). */
typedef struct { int32_t start, end, sink; } bs_span;

typedef struct bs_tilemap bs_tilemap;   /* opaque; owns its host arrays and device buffers */

/*
 * Build the tile map of one prompt.
 *   spans        host pointer, n_spans rows sorted by start, non-overlapping, inside
 *                [0, seq_len), 0 <= sink <= end - start (may be NULL when n_spans == 0)
 *   seq_len      L > 0
 *   head_class   host pointer, n_q_heads values in 0..3
 *   sink_len     positions [0, sink_len) are sink keys too (0 <= sink_len <= L)
 *   block_m/n    query / key tile edge (the paper's block_m, block_n).  The builder accepts
 *                any positive sizes; the attention kernels need 128 x 64.
 *   out          receives the new map; untouched on failure.  Free with bs_tilemap_destroy.
 * Tile (m, n) covers queries [m*block_m, +block_m) x keys [n*block_n, +block_n); positions
 * >= L count as masked.  SKIP = no allowed pair, FULL = every pair allowed, else PARTIAL.
 * A pair (i, j) is allowed iff j <= i and ( query i is text, or class is Dense, or key j is
 * text, or (class has the sink bit and j is a sink key), or (class has the intra bit and
 * i, j belong to the same image) ).
 * Host only: needs no GPU.  Errors: BS_EINVAL, BS_ENOMEM.
 */
int bs_build_tilemap(const bs_span *spans, int32_t n_spans, int32_t seq_len,
                     const uint8_t *head_class, int32_t n_q_heads, int32_t sink_len,
                     int32_t block_m, int32_t block_n, bs_tilemap **out);

/*
 * Same, with options (flags = 0 is bs_build_tilemap):
 *   BS_MAP_REGROUP_ROWS   the query rows are taken in another order than their positions: all
 *       image rows first, then all text rows, each group in position order and padded to whole
 *       query tiles.  Why: a text query attends to every earlier token (Sec. 3.2), so a query
 *       tile that holds a single text row has to walk every causal key tile for every head
 *       class; with the text rows in tiles of their own, the image rows of the sparse classes
 *       keep their skipped tiles (the Q-side counterpart of the paper kernel's packing of
 *       sink keys, App. kernel "Notation").  Only the grouping of rows into work items changes:
 *       q, k, v, out keep their layout and the result is the same function of the inputs.
 *       n_q_tiles becomes ceil(image rows / block_m) + ceil(text rows / block_m); query tile m
 *       covers the rows bs_tilemap_row_order reports.  No effect on a prompt without text or
 *       without image tokens.
 * Errors: BS_EINVAL (also for unknown flag bits), BS_ENOMEM.
 */
#define BS_MAP_REGROUP_ROWS 1u
/*   BS_MAP_PACK_KEYS (implies BS_MAP_REGROUP_ROWS)   the map also gets compact key tiles: the free
 *       keys of the prompt -- text keys and sink keys, which are what an image query of a sparse
 *       class may see outside its own image -- gathered in position order into tiles of their
 *       own, after the prompt's key tiles (n_k_tiles counts both).  The paper's kernel permutes
 *       K / V so that text and sink keys are contiguous (App. kernel, "Attention Sink Subroutine",
 *       Alg. 6); here they are a second copy, written by the bf16 pre-pass, because text queries
 *       and Dense heads keep walking the prompt order.  An image-only query tile of a sparse
 *       class then walks the compact tiles up to its causal bound (Sink: every slot; Intra-Image:
 *       the text slots; Intra-Image+Sink: the slots outside its own image) plus, for the classes
 *       with the intra bit, the prompt tiles of its own image, in which only own-image keys count.
 *       Every allowed pair is still counted exactly once.  bs_tilemap_key_order reports the key
 *       of every tile slot.
 *       No effect on a prompt without images, without free keys, or made of free keys only. */
#define BS_MAP_PACK_KEYS 2u
/*   BS_MAP_BIDIR_IMAGES   model variant in which the tokens of one image attend to each other in
 *       both directions (Gemma 3; paper Sec. 2: the dense mask is the model's default mask; Sec. 6.1
 *       states that this model does not attend causally inside an image).  The causal condition j <= i of the pair
 *       rule above becomes "j <= i, or i and j belong to the same image", for every class: a sparse
 *       mask is its class pattern inside the model's dense mask.  An image query then sees exactly
 *       what the last query of its image sees under the causal rule, which is how the map and the
 *       kernels treat it.  Text queries are unchanged.  Combines with the other flags. */
#define BS_MAP_BIDIR_IMAGES 4u
int bs_build_tilemap_ex(const bs_span *spans, int32_t n_spans, int32_t seq_len,
                        const uint8_t *head_class, int32_t n_q_heads, int32_t sink_len,
                        int32_t block_m, int32_t block_n, uint32_t flags, bs_tilemap **out);

/*
 * Same, for models whose image sinks are not a prefix of the image: sink_offsets (host, n_sink_offsets
 * values >= 0, may be NULL when the count is 0) lists offsets inside an image; the token at
 * start + offset of EVERY image is a sink key as well (offsets at or past an image's length are ignored
 * for that image), in addition to the spans' `sink` prefixes and the sink_len prefix of the prompt.
 * Paper Sec. 6.1 and App. "Attention Sink Positions in Gemma 3": that model tokenises every image to
 * the same length and its sinks sit at fixed locations inside every image (the paper keeps the 10 % most
 * frequent locations found on its characterisation set; the list itself is the caller's input).
 * window > 0 makes the map one of a sliding-window layer: the layer's dense mask keeps, for every query
 * (text queries too) and every class, only the keys with i - j < window (paper App. kernel, "Dense
 * Attention Subroutine": text queries follow the model's own dense mask, which is causal or a sliding
 * window depending on the model; the sparse masks live inside the dense mask).  0 = no window; a window of seq_len or
 * more is no window.  With a window BS_MAP_PACK_KEYS acts as BS_MAP_REGROUP_ROWS (a windowed query tile
 * visits a handful of key tiles: there is nothing to pack).  Together with BS_MAP_BIDIR_IMAGES the keys of
 * the query's own image stay visible at any distance, also for images longer than the window: an image
 * query then sees its class pattern inside [min(window start, image start), image end).
 * Errors: as bs_build_tilemap_ex; BS_EINVAL for a negative offset, count or window.
 */
int bs_build_tilemap_model(const bs_span *spans, int32_t n_spans, int32_t seq_len,
                           const uint8_t *head_class, int32_t n_q_heads, int32_t sink_len,
                           int32_t block_m, int32_t block_n, uint32_t flags,
                           const int32_t *sink_offsets, int32_t n_sink_offsets, int32_t window,
                           bs_tilemap **out);

/*
 * Same, for a chunk of queries at the end of the prompt: the query rows are the positions q_begin .. seq_len - 1
 * only (0 <= q_begin < seq_len), attending to all seq_len keys under the same masks.  This is how the masks of
 * Sec. 3.2 carry over to chunked prefill and to decoding with the KV cache kept whole (the paper prunes no
 * KV entries, Sec. 6.1: its masks only drop attention pairs): the chunk's rows are rows of the same L x L mask.
 * With such a map, q and out of bs_attn_prefill hold seq_len - q_begin rows per head ([n_q_heads][seq_len -
 * q_begin][head_dim], row r = position q_begin + r); k and v hold all seq_len positions.  n_q_tiles counts the
 * tiles of those rows, bs_tilemap_row_order reports positions, allowed_pairs / empty_rows count those rows.
 * q_begin = 0 is bs_build_tilemap_model.  Errors: as bs_build_tilemap_model; BS_EINVAL for q_begin outside
 * [0, seq_len).
 */
int bs_build_tilemap_suffix(const bs_span *spans, int32_t n_spans, int32_t seq_len,
                            const uint8_t *head_class, int32_t n_q_heads, int32_t sink_len,
                            int32_t block_m, int32_t block_n, uint32_t flags,
                            const int32_t *sink_offsets, int32_t n_sink_offsets, int32_t window,
                            int32_t q_begin, bs_tilemap **out);

/* End of a map's life (the paper builds its mask metadata once per prompt, Sec. 5 "no runtime overhead";
 * so does a caller here, and destroys the map when the prompt's prefill is over).
 * Frees the host arrays; device buffers (if any) go back to a per-process cache of the library
 * and are handed to a later map only after the work queued with this map has finished (the
 * next owner's stream waits for an event recorded after this map's last call).  So a map may be
 * destroyed as soon as its last bs_attn_prefill has returned, without waiting for the stream,
 * and destroying it does not synchronise the device.  The cache keeps at most a few dozen
 * blocks until the process ends.  NULL is allowed. */
void bs_tilemap_destroy(bs_tilemap *tm);

/* Geometry of the map, in the paper's symbols (App. kernel, "Notation"): seq_len = L, n_q_tiles = M =
 * number of block_m-row query tiles, n_k_tiles = N = number of block_n-key tiles (compact tiles included).
 * Any output pointer may be NULL. */
int bs_tilemap_dims(const bs_tilemap *tm, int32_t *seq_len, int32_t *n_q_tiles,
                    int32_t *n_k_tiles, int32_t *n_q_heads);

/* rows[n_q_tiles * block_m] (host): the position of every row of every query tile, -1 where a
 * tile has no row (the last tile of the prompt, or of a group of regrouped rows). */
int bs_tilemap_row_order(const bs_tilemap *tm, int32_t *rows);

/* What the map options did (any pointer may be NULL): regrouped = the row order differs from the
 * position order; packed = compact key tiles exist; intra_compact = Intra-Image heads take their
 * text keys from the compact tiles (they keep the prompt's tiles when those hold the text keys in
 * fewer tiles, e.g. a few long images with little text between them). */
int bs_tilemap_layout(const bs_tilemap *tm, int32_t *regrouped, int32_t *packed, int32_t *intra_compact);

/* keys[n_k_tiles * block_n] (host, may be NULL): the position of the key in every slot of every
 * key tile, -1 where a tile has no key; n_prompt_tiles (may be NULL): how many of the tiles are
 * the prompt in position order (all of them unless the map was built with BS_MAP_PACK_KEYS). */
int bs_tilemap_key_order(const bs_tilemap *tm, int32_t *keys, int32_t *n_prompt_tiles);

/* The per-tile decision of the paper's kernel (App. kernel, Overview: fully masked tiles are skipped, tiles at
 * a mask boundary are masked element-wise) made explicit for the bit-exact check against the element-wise mask
 * of Sec. 3.2.  Expand the range lists of class `cls` for query tiles [q_tile_begin, +q_tile_count) into
 * states[q_tile_count][n_k_tiles] (host, row-major): 0 skip, 1 partial, 2 full. */
int bs_tilemap_tile_states(const bs_tilemap *tm, int32_t cls, int32_t q_tile_begin,
                           int32_t q_tile_count, uint8_t *states);

/* Per-class accounting behind the FLOP figures (the paper counts attention FLOPs per unmasked pair, App.
 * "FLOPs Reduction"; Sec. 3.2 defines which pairs a class keeps).  Any output pointer may be NULL:
 *   visited = full + partial tiles over all query tiles; allowed_pairs = number of allowed
 *   (i, j) pairs, from span geometry (the bench's "4 d FLOP per unmasked pair" counts these);
 *   empty_rows = query rows whose allowed set is empty (their output is zero);
 *   n_ranges = entries in the class's range list. */
int bs_tilemap_stats(const bs_tilemap *tm, int32_t cls, int64_t *visited, int64_t *full,
                     int64_t *partial, int64_t *allowed_pairs, int64_t *empty_rows,
                     int64_t *n_ranges);

/*
 * Plan (and check) the work units the bf16 kernel uses for `gqa_group` query heads per KV head:
 * pairs of (head, query tile) items that read the same KV head and walk one merged key-tile
 * list, so a workgroup streams every K / V tile once for two items.  Returns BS_OK only if
 * every (head, query tile) appears in exactly one unit and each unit's merged list reproduces
 * both items' tile states.  Outputs (may be NULL): number of units, key tiles summed over the
 * units' merged lists, and steps on which one of a unit's items has nothing to do.
 * Host only.  bs_attn_prefill plans by itself; this entry point is for tests and accounting.
 */
int bs_tilemap_pair_plan(bs_tilemap *tm, int32_t gqa_group, int64_t *n_units, int64_t *unit_tiles,
                         int64_t *skip_steps);

/*
 * Bind a built map to another class vector (paper Sec. 4: every layer of a model has its own offline-assigned
 * head classes, while the mask metadata depends on the prompt alone, Sec. 5): the four per-class tile lists,
 * token codes, row and key order -- everything bs_build_tilemap derived from the span table -- are kept,
 * on the host and on the device; only the work list / work units are planned again by the next
 * bs_attn_prefill (or bs_tilemap_prepare).  So a model builds ONE map per prompt and rebinds it per layer.
 *   head_class   host, n_q_heads values in 0..3 (n_q_heads may differ from the count the map was built with)
 * Host only, O(n_q_heads); binding the vector the map already has is free.  Stream order makes it safe to
 * rebind while kernels of the previous binding are still queued on the stream of the next call.
 * Errors: BS_EINVAL, BS_ENOMEM.
 */
int bs_tilemap_rebind(bs_tilemap *tm, const uint8_t *head_class, int32_t n_q_heads);

/*
 * Do, ahead of time, everything bs_attn_prefill would do on the first call with this map and these
 * arguments except the kernels: upload the prompt part (once per map), plan and upload the work list
 * (BS_F32) or the work units for `gqa_group` (BS_BF16) of the current class vector, raise the kernels'
 * dynamic-LDS limits and look up the address of the static scratch on the current device.  Enqueues
 * copies on `stream`, does not wait.  May allocate (block cache / hipMalloc, pinned staging).  After it,
 * bs_attn_prefill_static with the same map, class vector and gqa_group allocates nothing.
 * Errors: BS_EINVAL, BS_EUNSUPPORTED, BS_ENOMEM, BS_EHIP.
 */
int bs_tilemap_prepare(bs_tilemap *tm, int32_t dtype, int32_t gqa_group, void *stream);

/* Copy the map to the current HIP device and wait until the copy is done (default stream,
 * then hipStreamSynchronize on it).  Optional: bs_attn_prefill uploads on first use, on its own
 * stream and without waiting.  Not thread-safe against concurrent calls on the same map.
 * Errors: BS_EHIP, BS_ENOMEM. */
int bs_tilemap_upload(bs_tilemap *tm);

/*
 * Sparse causal prefill attention (paper Sec. 3.1 for the definition, App. kernel Alg. 3-7
 * for the tiled form):  for query head h with class head_class[h] and KV head h / gqa_group,
 *   out[h, i, :] = sum_j softmax_j( scale * <q[h,i], k[h/G,j]> over allowed j ) * v[h/G, j, :]
 * and zeros for a row with no allowed key.
 *   q, out   device pointers, [n_q_heads][L][head_dim], contiguous
 *   k, v     device pointers, [n_q_heads / gqa_group][L][head_dim], contiguous
 *   tm       map built for this prompt with block 128 x 64 and the same n_q_heads
 *   dtype    BS_BF16 (bf16 MFMA, fp32 accumulate, P rounded to bf16 before P.V) or
 *            BS_F32 (fp32 MFMA throughout)
 *   head_dim 64 or 128
 *   scale    finite and > 0 (1/sqrt(d_k) in the paper)
 *   stream   hipStream_t (NULL = default stream).  The call only enqueues work; the caller
 *            owns q/k/v/out and keeps them alive until the stream has drained.
 * bf16 path: a pre-pass first packs K and V into per-key-tile blocks (V transposed) in a
 * workspace the map owns (2 x the size of K, taken from the library's block cache or hipMalloc
 * on first use).  Calls that share a map share that workspace: the library orders a call after
 * the map's previous call when the stream changes, but two threads must not call with one map
 * at the same time.
 * The first call on a map uploads it: the arrays are staged through pinned host buffers and
 * copied on `stream`; the host does not wait for the device (it may wait for an upload queued
 * eight uploads earlier, whose staging buffer it reuses).
 * Errors: BS_EINVAL (null pointers, head counts that do not match), BS_EUNSUPPORTED,
 * BS_EHIP, BS_ENOMEM.  Nothing is launched on error.
 */
int bs_attn_prefill(const void *q, const void *k, const void *v, void *out, bs_tilemap *tm,
                    int32_t dtype, int32_t n_q_heads, int32_t gqa_group, int32_t head_dim,
                    float scale, void *stream);

/*
 * Same call, for profiling harnesses: if non-NULL, ev_main_start / ev_main_stop (hipEvent_t,
 * created by the caller with timing enabled) are recorded on `stream` immediately before and
 * after the attention kernel itself, i.e. excluding the bf16 path's K / V^T tile-pack pre-pass
 *.  hipEventElapsedTime between them is that kernel's duration.
 */
int bs_attn_prefill_ex(const void *q, const void *k, const void *v, void *out, bs_tilemap *tm,
                       int32_t dtype, int32_t n_q_heads, int32_t gqa_group, int32_t head_dim,
                       float scale, void *stream, void *ev_main_start, void *ev_main_stop);

/*
 * bs_attn_prefill (bf16) for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same kernels and same result as bs_attn_prefill with BS_BF16;
 * the packed K / V^T tiles of the pre-pass go to a static device array of BS_STATIC_SCRATCH_MIB MiB
 * inside the library (one copy per GPU, held until the process ends) instead of a workspace owned by the
 * map.  Calls no hipMalloc / hipFree, creates no events, uploads nothing.
 *   tm       must have been prepared: bs_tilemap_prepare(tm, BS_BF16, gqa_group, stream) after the build and
 *            after every bs_tilemap_rebind; BS_EINVAL otherwise (bs_last_error says so)
 *   limit    n_kv_heads * n_k_tiles * head_dim * 256 bytes (packed K plus packed V^T) must fit the scratch:
 *            BS_EUNSUPPORTED otherwise, nothing launched (96 MiB hold 4 KV heads x 768 key tiles of d = 128:
 *            a 40K-token prompt with its compact tiles)
 * Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (two streams, two
 * threads) race on it; calls queued on one stream are safe.  The pre-pass rewrites every tile slot it
 * uses, so nothing needs clearing between calls.
 * Other arguments and errors as bs_attn_prefill.
 */
#define BS_STATIC_SCRATCH_MIB 96
int bs_attn_prefill_static(const void *q, const void *k, const void *v, void *out, bs_tilemap *tm,
                           int32_t n_q_heads, int32_t gqa_group, int32_t head_dim, float scale, void *stream);

/* Size of that array in bytes. */
int64_t bs_static_scratch_bytes(void);

/*
 * Offline characterisation, prompt level (paper Sec. 4.1, Alg. 1), for all query heads of one layer:
 * the attention output under the dense causal mask is the reference; for the masks Sink,
 * Intra-Image, Intra-Image+Sink, in this order,
 *     NMSE = || Attn_mask - Attn_ref ||^2 / || Attn_ref ||^2      (over the head's [L, head_dim] output)
 * and the head takes the first mask with NMSE < alpha (strictly), Dense if none passes.
 *   q, k, v      device pointers, layouts as for bs_attn_prefill; spans / seq_len / sink_len as for
 *                bs_build_tilemap (host)
 *   alpha        the layer's threshold alpha_layer (the paper recommends 0.1 for Qwen-type models)
 *   map_flags    options for the tile map the call builds (BS_MAP_*); sink_offsets /
 *                n_sink_offsets / window as for bs_build_tilemap_model
 *   head_type    host, n_q_heads values out (bs_head_class)
 *   nmse         host, [3][n_q_heads] out, row m = mask m + 1; may be NULL.  All three masks are
 *                evaluated for every head (Alg. 1 stops at the first that passes, which only saves
 *                work: the head types are the same).  A reference of norm zero gives 0 if the masked
 *                output is zero as well, +inf otherwise.
 * The four outputs come from bs_attn_prefill in `dtype` (bf16: the outputs are rounded to bf16 before
 * they are compared, which puts a floor of about 1e-5 under the NMSE), the squared errors are
 * accumulated in fp64 and the decision is taken in fp64.
 * Builds ONE tile map of the prompt and binds it to the four class vectors in turn (bs_tilemap_rebind).  Takes
 * two output-sized device buffers from the library's block cache for the duration of the call (hipMalloc only
 * while the cache is cold; the blocks stay cached afterwards) and returns after `stream` has drained (this
 * is an offline routine).
 * Errors: as bs_build_tilemap_ex and bs_attn_prefill; nothing is written to head_type / nmse on error.
 */
int bs_characterize_prompt(const void *q, const void *k, const void *v, const bs_span *spans,
                           int32_t n_spans, int32_t seq_len, int32_t sink_len, int32_t dtype,
                           int32_t n_q_heads, int32_t gqa_group, int32_t head_dim, float scale,
                           double alpha, uint32_t map_flags, const int32_t *sink_offsets,
                           int32_t n_sink_offsets, int32_t window, uint8_t *head_type, double *nmse,
                           void *stream);

/*
 * The error measure of Alg. 1 on its own: for each of n_heads contiguous blocks of elems_per_head
 * elements, sums[2*h] = sum (attn_mask - attn_ref)^2 and sums[2*h+1] = sum attn_ref^2.
 *   attn_mask, attn_ref   device pointers, 16-byte aligned, dtype BS_BF16 or BS_F32
 *   sums                  device pointer, 2 * n_heads doubles (cleared by the call)
 * Enqueues on `stream` and does not wait.  The sums are accumulated in fp64; the order of the
 * additions across workgroups is not fixed (fp64 atomics), so the last bits may differ between runs.
 * Errors: BS_EINVAL; BS_EUNSUPPORTED (dtype, misaligned pointers, or several heads whose size in
 * bytes is not a multiple of 16); BS_EHIP.
 */
int bs_head_sq_error(const void *attn_mask, const void *attn_ref, int32_t dtype, int32_t n_heads,
                     int64_t elems_per_head, double *sums, void *stream);

/*
 * Offline characterisation, data-set level (paper Sec. 4.2, Alg. 2), for one head: fraction[c] is the
 * share of characterised prompts on which Alg. 1 chose class c (host, 4 values).  Returns Dense if
 * fraction[Dense] > gamma_d, else Sink if fraction[Sink] > gamma_s, else Intra-Image if
 * fraction[Intra-Image] > gamma_i, else Intra-Image+Sink (paper defaults gamma_d = 0.25, gamma_s = 0.6;
 * it names no value for gamma_i).  Host only.  Returns the class (0..3) or BS_EINVAL.
 */
int bs_aggregate_head_type(const double *fraction, double gamma_d, double gamma_s, double gamma_i);

/*
 * Alg. 2 for all heads of a layer, from the prompt-level results: head_types (host) is
 * [n_prompts][n_q_heads], one row per characterised prompt as bs_characterize_prompt returned it.
 * Counts, per head, the share of prompts that chose each class (the head_type_fraction of Alg. 2;
 * written to fraction[n_q_heads][4] if non-NULL) and applies bs_aggregate_head_type to it:
 * head_class[n_q_heads] (host) is the class vector to pass to bs_build_tilemap for this layer.
 * Host only.  Errors: BS_EINVAL (null pointers, non-positive counts, a type above 3).
 */
int bs_aggregate_layer(const uint8_t *head_types, int32_t n_prompts, int32_t n_q_heads, double gamma_d,
                       double gamma_s, double gamma_i, uint8_t *head_class, double *fraction);

/*
 * The layer threshold of Alg. 1 under the paper's linear schedule (App. "Impact of Linear alpha_layer
 * for Gemma 3"): alpha_first + (alpha_last - alpha_first) * layer_idx / num_layers, which keeps the
 * first layers denser.  The paper uses 0.005 .. 0.195 for Gemma 3 (12B), 0.001 .. 0.099 for Gemma 3 (4B)
 * and a fixed 0.1 (alpha_first = alpha_last) for the Qwen-type models.  Host only.  NaN for
 * num_layers <= 0 or layer_idx outside [0, num_layers].
 */
double bs_alpha_layer(double alpha_first, double alpha_last, int32_t layer_idx, int32_t num_layers);

/* Static description of an error code (error behaviour of this boundary; no passage of the paper). */
const char *bs_strerror(int code);

/* Detail of the most recent BS_EHIP / BS_ENOMEM failure on the calling thread (the HIP call
 * that failed and its error string); "" if none.  The pointer stays valid for the thread's life. */
const char *bs_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* BLINDSIGHT_H */
