// Host-side tile-map builder: span table + head classes -> per-class, per-query-tile lists of
// key-tile ranges (FULL / PARTIAL), by interval arithmetic on the span geometry.
//
// Mask definition: paper Sec. 3.2 (head classes; text queries see every earlier token; text
// keys stay visible to every class) and Sec. 3.1 (causal prefill).  The lists take the place
// of the paper kernel's sink_end[M] / first_image[M] arrays and its all/any(istext_m) dispatch
// (App. kernel, Notation and Alg. 3): a query tile that holds a text row walks every causal
// key tile, an image-only query tile walks only tiles that hold a text key, an enabled sink
// key, or a key of its own image.
#include <algorithm>
#include <climits>
#include <cstring>
#include <new>

#include "tilemap_internal.h"

namespace {

using bs::ClassLists;
using bs::TileRange;

// Rows [a, b) of the query tile lie in image g (0-based).  [ea, eb): the same rows by the last key
// position they may see (+1 for eb): themselves under the causal mask; with bidirectional images
// every row of image g sees up to the image's last token, as if it were that token's query.
struct Segment { int32_t g, a, b, ea, eb; };

struct Geometry {
    int32_t L, bm, bn, M, N;
    const std::vector<bs_span> *spans;
    std::vector<int32_t> n_text;       // L+1: text tokens in [0, t)
    std::vector<int32_t> n_free_sink;  // L+1: tokens in [0, t) that are text or sink
    std::vector<int32_t> last_text;    // L: largest text position <= t, or -1
    std::vector<int32_t> next_text;    // L+1: smallest text position >= t, or L
    std::vector<int32_t> next_free_sink;  // L+1: smallest (text or sink) position >= t, or L
    // per key tile, for classes without / with the sink bit: smallest n' >= n whose keys are
    // all free (text, or text/sink) and which is a complete tile; N if none
    std::vector<int32_t> next_allfree_tile[2];  // N+1 each
    // packed keys: compact tiles N .. N + Nc - 1 hold the free keys (text or sink) in position order
    bool packed = false, intra_compact = false;
    bool bidir = false;                // tokens of one image also see the later tokens of that image
    int32_t window = 0;                // > 0: a query at position i sees no key before i - window + 1
    int32_t Nc = 0, n_free = 0;
    // first key position a query at position i may see: the start of its window; with bidirectional
    // images the query's own image stays visible at any distance, so for an image token it is the
    // smaller of the window's start and the image's start (the visible keys stay one interval, and the
    // bound still grows with the position)
    std::vector<int32_t> first_visible;   // L entries when window > 0
    int32_t lo(int32_t i) const { return window > 0 ? first_visible[i] : 0; }
    std::vector<int32_t> ctext;        // n_free + 1: text keys among compact slots [0, s)

    const std::vector<int32_t> &free_count(int cls) const { return (cls & 1) ? n_free_sink : n_text; }
    const std::vector<int32_t> &next_free(int cls) const { return (cls & 1) ? next_free_sink : next_text; }
    const std::vector<int32_t> &next_allfree(int cls) const { return next_allfree_tile[cls & 1]; }
};

struct QueryTile {
    int32_t r0, r1;       // rows [r0, r1), clipped to L
    int32_t e0, e1;       // last visible key position of the first row, and of the last row + 1 (r0, r1 if causal)
    bool ragged;          // fewer than bm rows
    int32_t last_text;    // last text row inside, or -1
    std::vector<Segment> segs;
};

// Describe rows [r0, r1) of one query tile.  `ragged`: the tile holds fewer than bm rows (then
// no key tile can be FULL: the missing rows count as masked).  A query tile whose rows are
// not contiguous (regrouped order) is described run by run.
void describe_query_rows(const Geometry &G, int32_t r0, int32_t r1, bool ragged, QueryTile &qt)
{
    qt.r0 = r0;
    qt.r1 = r1;
    qt.ragged = ragged;
    int32_t lt = G.last_text[qt.r1 - 1];
    qt.last_text = (lt >= qt.r0) ? lt : -1;
    qt.segs.clear();
    const auto &sp = *G.spans;
    // first span whose end lies beyond r0
    size_t lo = std::upper_bound(sp.begin(), sp.end(), qt.r0,
                                 [](int32_t r, const bs_span &s) { return r < s.end; }) - sp.begin();
    for (size_t g = lo; g < sp.size() && sp[g].start < qt.r1; ++g) {
        const int32_t a = std::max(sp[g].start, qt.r0), b = std::min(sp[g].end, qt.r1);
        qt.segs.push_back({(int32_t)g, a, b, G.bidir ? sp[g].end - 1 : a, G.bidir ? sp[g].end : b});
    }
    // the visible range grows with the row position, so the first / last row bound the tile
    qt.e0 = (!qt.segs.empty() && qt.segs.front().a == qt.r0) ? qt.segs.front().ea : qt.r0;
    qt.e1 = (!qt.segs.empty() && qt.segs.back().b == qt.r1) ? qt.segs.back().eb : qt.r1;
}

// Exact state of tile (query tile qt, key tile n) for class cls: 0 skip, 1 partial, 2 full.
int tile_state(const Geometry &G, const QueryTile &qt, int cls, int32_t n)
{
    const int32_t c0 = n * G.bn, c1 = std::min(c0 + G.bn, G.L);
    if (c0 > qt.e1 - 1) return 0;  // beyond what the last row sees
    if (c1 - 1 < G.lo(qt.r0)) return 0;  // before the first row's window (and every later row's)
    const auto &sp = *G.spans;
    const auto &freec = G.free_count(cls);

    // Every row i sees the keys of its class pattern inside [lo(i), e(i)]; both ends grow with i, so
    // the rows of a run together see [lo(first), e(last)] and share [lo(last), e(first)].
    bool any = false;
    if (cls == BS_DENSE || qt.segs.empty()) {
        any = true;
    } else {
        // a text row at or after the tile's first key, close enough to see the tile's last key
        const int32_t t = G.next_text[std::max(qt.r0, c0)];
        if (t < qt.r1 && G.lo(t) <= c1 - 1) any = true;
        for (const Segment &s : qt.segs) {
            if (any) break;
            const int32_t lo = std::max(c0, G.lo(s.a)), hi = std::min(c1, s.eb);  // keys the segment's rows may see
            if (hi <= lo) continue;
            if (freec[hi] - freec[lo] > 0) { any = true; break; }
            if (cls & 2) {
                int32_t lo2 = std::max(lo, sp[s.g].start), hi2 = std::min(hi, sp[s.g].end);
                if (hi2 > lo2) { any = true; break; }
            }
        }
    }
    if (!any) return 0;

    bool all;
    if (qt.ragged || (c1 - c0) < G.bn || c1 - 1 > qt.e0 || c0 < G.lo(qt.r1 - 1)) {
        all = false;  // masked out-of-range positions, or the diagonal / the window's edge cuts through
    } else if (cls == BS_DENSE || qt.segs.empty()) {
        all = true;
    } else {
        int32_t nonfree = G.bn - (freec[c1] - freec[c0]);
        if (nonfree == 0) {
            all = true;
        } else if (!(cls & 2) || qt.segs.size() > 1) {
            all = false;  // a masked image key, or two images that cannot both own it
        } else {
            const bs_span &own = sp[qt.segs[0].g];
            int32_t lo2 = std::max(c0, own.start), hi2 = std::min(c1, own.end);
            int32_t nonfree_own = (hi2 > lo2) ? (hi2 - lo2) - (freec[hi2] - freec[lo2]) : 0;
            all = (nonfree_own == nonfree);
        }
    }
    return all ? 2 : 1;
}

// Key tiles that can hold an allowed pair for this query tile (a superset is fine; sorted, unique).
void candidate_tiles(const Geometry &G, const QueryTile &qt, int cls, std::vector<int32_t> &cand)
{
    cand.clear();
    const int32_t n_last = (qt.e1 - 1) / G.bn;
    if (cls == BS_DENSE || qt.last_text >= 0) {
        cand.resize(n_last + 1);
        for (int32_t n = 0; n <= n_last; ++n) cand[n] = n;
        return;
    }
    // image-only query tile of a sparse class: tiles with a free key (text / enabled sink) ...
    const auto &nf = G.next_free(cls);
    for (int32_t pos = 0; pos < qt.e1;) {
        int32_t j = nf[pos];
        if (j >= qt.e1) break;
        int32_t n = j / G.bn;
        cand.push_back(n);
        pos = (n + 1) * G.bn;
        if (pos > G.L) break;
    }
    // ... and tiles overlapping the part of an own image that lies at or before the tile's rows
    if (cls & 2) {
        const auto &sp = *G.spans;
        for (const Segment &s : qt.segs)
            for (int32_t n = sp[s.g].start / G.bn; n <= (s.eb - 1) / G.bn; ++n) cand.push_back(n);
        std::sort(cand.begin(), cand.end());
        cand.erase(std::unique(cand.begin(), cand.end()), cand.end());
    }
}

// Key-tile ranges (FULL / PARTIAL; skipped tiles are absent) of one run of contiguous query rows.
void build_run(const Geometry &G, int cls, const QueryTile &qt, std::vector<int32_t> &cand,
               std::vector<TileRange> &out)
{
    out.clear();
    int32_t run_begin = -1, run_end = -1, run_state = 0;
    auto flush = [&]() {
        if (run_begin >= 0) out.push_back({run_begin, (run_end << 1) | (run_state == 2)});
        run_begin = -1;
    };
    // append tiles [b, e) of one state (1 partial, 2 full), merging adjacent runs
    auto emit = [&](int32_t b, int32_t e, int st) {
        if (e <= b) return;
        if (run_begin >= 0 && b == run_end && st == run_state) {
            run_end = e;
        } else {
            flush();
            run_begin = b; run_end = e; run_state = st;
        }
    };
    const int32_t n_last = (qt.e1 - 1) / G.bn;
    // key tiles wholly within what the first row of a complete query tile sees can be FULL
    const int32_t n_full_limit = qt.ragged ? 0 : (qt.e0 + 1) / G.bn;

    if (G.window > 0) {
        // sliding window: few key tiles per query tile, each classified exactly
        for (int32_t n = G.lo(qt.r0) / G.bn; n <= n_last; ++n) {
            const int st = tile_state(G, qt, cls, n);
            if (st) emit(n, n + 1, st);
        }
    } else if (cls == BS_DENSE || qt.segs.empty()) {
        // every earlier key is visible: FULL below the diagonal, PARTIAL on it
        emit(0, n_full_limit, 2);
        emit(n_full_limit, n_last + 1, 1);
    } else if (qt.last_text >= 0) {
        // mixed text/image rows: every causal key tile up to the last text row is visited.
        // Only a few of them can differ from PARTIAL: all-free tiles and tiles overlapping an
        // own image (candidates for FULL), and the tiles past the last text row (may be SKIP).
        // Those are classified exactly; the rest are PARTIAL.
        cand.clear();
        const auto &naf = G.next_allfree(cls);
        for (int32_t n = naf[0]; n < n_full_limit; n = naf[n + 1]) cand.push_back(n);
        const auto &sp = *G.spans;
        for (const Segment &sg : qt.segs)
            for (int32_t n = sp[sg.g].start / G.bn; n <= (sg.eb - 1) / G.bn && n < n_full_limit; ++n) cand.push_back(n);
        for (int32_t n = qt.last_text / G.bn + 1; n <= n_last; ++n) cand.push_back(n);
        std::sort(cand.begin(), cand.end());
        cand.erase(std::unique(cand.begin(), cand.end()), cand.end());
        int32_t cur = 0;
        for (int32_t n : cand) {
            emit(cur, n, 1);
            const int st = tile_state(G, qt, cls, n);
            if (st) emit(n, n + 1, st);
            cur = n + 1;
        }
        emit(cur, qt.last_text / G.bn + 1, 1);
    } else {
        candidate_tiles(G, qt, cls, cand);
        for (int32_t n : cand) {
            const int st = tile_state(G, qt, cls, n);
            if (st) emit(n, n + 1, st);
        }
    }
    flush();
}

// Packed keys: range list of rows [a, b), all inside image g (0-based span index), for a sparse
// class.  Two parts, disjoint by construction:
// [a, b) are the rows by the last key position they may see (Segment::ea, eb).
//   own-image keys (classes with the intra bit): the prompt's own tiles over [start_g, b);
//     a pair (i, j) counts there iff start_g <= j <= i;
//   free keys: compact tiles; row i sees compact slot s iff s < free_before[i + 1] (the free
//     keys at positions <= i) and
//       Sink:             every such slot
//       Intra-Image:      the text slots
//       Intra-Image+Sink: every slot outside the image's own free keys (those are counted above).
void build_run_packed(const Geometry &G, int cls, int32_t g, int32_t a, int32_t b, bool ragged,
                      std::vector<TileRange> &out)
{
    out.clear();
    int32_t run_begin = -1, run_end = -1, run_state = 0;
    auto flush = [&]() {
        if (run_begin >= 0) out.push_back({run_begin, (run_end << 1) | (run_state == 2)});
        run_begin = -1;
    };
    auto emit = [&](int32_t bg, int32_t en, int st) {
        if (en <= bg || st == 0) return;
        if (run_begin >= 0 && bg == run_end && st == run_state) {
            run_end = en;
        } else {
            flush();
            run_begin = bg; run_end = en; run_state = st;
        }
    };
    const auto &sp = *G.spans;
    const auto &nfs = G.n_free_sink;
    if (cls & 2) {
        const int32_t s0 = sp[g].start;
        for (int32_t n = s0 / G.bn; n <= (b - 1) / G.bn; ++n) {
            const int32_t c0 = n * G.bn, c1 = c0 + G.bn;
            const bool full = !ragged && c0 >= s0 && c1 - 1 <= a && c1 <= G.L;
            emit(n, n + 1, full ? 2 : 1);
        }
    }
    const int32_t fb_min = nfs[a + 1], fb_max = nfs[b];   // visible free keys of the first / last row
    const int32_t own_lo = nfs[sp[g].start], own_hi = nfs[sp[g].end];
    const int32_t c_end = (fb_max + G.bn - 1) / G.bn;
    for (int32_t c = 0; c < c_end; ++c) {
        const int32_t s0 = c * G.bn, s1 = s0 + G.bn, vis = std::min(s1, fb_max);   // slots [s0, vis) are visible to the last row
        const bool below_all = !ragged && s1 <= fb_min;   // every slot visible to every row (implies a complete tile)
        int st;
        if (cls == BS_SINK) {
            st = below_all ? 2 : 1;
        } else if (cls == BS_INTRA) {
            const int32_t t = G.ctext[vis] - G.ctext[s0];
            st = t == 0 ? 0 : ((below_all && t == G.bn) ? 2 : 1);
        } else {
            const int32_t lo = std::max(s0, own_lo), hi = std::min(vis, own_hi);
            const int32_t own = hi > lo ? hi - lo : 0;
            st = own == vis - s0 ? 0 : ((below_all && own == 0) ? 2 : 1);
        }
        emit(G.N + c, G.N + c + 1, st);
    }
    flush();
}

// Union of two range lists of one query tile's runs.  A key tile is FULL for the tile only if
// it is FULL for every run; visited by some run and not FULL for all of them: PARTIAL.
// `a_runs` tells how many runs list a stands for (a tile absent from a is skipped by all of them).
void combine_runs(const std::vector<TileRange> &a, const std::vector<TileRange> &b, std::vector<TileRange> &out)
{
    out.clear();
    size_t ia = 0, ib = 0;
    int32_t pos = 0;
    auto push = [&](int32_t bg, int32_t en, bool full) {
        if (en <= bg) return;
        if (!out.empty() && out.back().end() == bg && out.back().full() == full) out.back().end_state = (en << 1) | full;
        else out.push_back({bg, (en << 1) | (int32_t)full});
    };
    while (ia < a.size() || ib < b.size()) {
        // state of a and b at `pos` and the next boundary
        int32_t next = INT32_MAX;
        int sa = 0, sb = 0;
        if (ia < a.size()) {
            if (a[ia].end() <= pos) { ++ia; continue; }
            if (a[ia].begin <= pos) { sa = a[ia].full() ? 2 : 1; next = std::min(next, a[ia].end()); }
            else next = std::min(next, a[ia].begin);
        }
        if (ib < b.size()) {
            if (b[ib].end() <= pos) { ++ib; continue; }
            if (b[ib].begin <= pos) { sb = b[ib].full() ? 2 : 1; next = std::min(next, b[ib].end()); }
            else next = std::min(next, b[ib].begin);
        }
        if (next == INT32_MAX) break;
        if (sa || sb) push(pos, next, sa == 2 && sb == 2);
        pos = next;
    }
}

void build_class(const Geometry &G, int cls, const std::vector<int32_t> &row_order, ClassLists &out)
{
    out.row_ptr.assign(G.M + 1, 0);
    out.row_tiles.assign(G.M, 0);
    out.ranges.clear();
    QueryTile qt;
    std::vector<int32_t> cand;
    std::vector<TileRange> run, seg_run, acc, tmp;
    for (int32_t m = 0; m < G.M; ++m) {
        // the tile's rows as runs of consecutive positions (one run in the natural order)
        const int32_t *rows = row_order.data() + (size_t)m * G.bm;
        int32_t n_rows = 0;
        while (n_rows < G.bm && rows[n_rows] >= 0) ++n_rows;
        const bool ragged = n_rows < G.bm;
        acc.clear();
        bool first = true;
        for (int32_t i = 0; i < n_rows;) {
            int32_t j = i + 1;
            while (j < n_rows && rows[j] == rows[j - 1] + 1) ++j;
            describe_query_rows(G, rows[i], rows[j - 1] + 1, ragged, qt);
            if (G.packed && cls != BS_DENSE && (cls != BS_INTRA || G.intra_compact) && qt.last_text < 0 && !qt.segs.empty()) {
                // image rows of a sparse class: one packed list per image the run touches
                // (two images can be adjacent without a text token between them)
                bool first_seg = true;
                for (const Segment &sg : qt.segs) {
                    build_run_packed(G, cls, sg.g, sg.ea, sg.eb, ragged, first_seg ? run : seg_run);
                    if (!first_seg) {
                        combine_runs(run, seg_run, tmp);
                        run.swap(tmp);
                    }
                    first_seg = false;
                }
            } else {
                build_run(G, cls, qt, cand, run);
            }
            if (first) {
                acc.swap(run);
                first = false;
            } else {
                combine_runs(acc, run, tmp);
                acc.swap(tmp);
            }
            i = j;
        }
        for (const TileRange &r : acc) {
            const int32_t len = r.end() - r.begin;
            out.row_tiles[m] += len;
            if (r.full()) out.full += len; else out.partial += len;
            out.ranges.push_back(r);
        }
        out.row_ptr[m + 1] = (int64_t)out.ranges.size();
    }
    out.visited = out.full + out.partial;
}

// Allowed pairs and empty rows per class, from prefix counts (no pair enumeration).
void count_pairs(const Geometry &G, const std::vector<uint32_t> &code, int32_t q_begin, ClassLists lists[4])
{
    const auto &sp = *G.spans;
    int64_t pairs[4] = {0, 0, 0, 0}, empty[4] = {0, 0, 0, 0};
    size_t g = 0;
    for (int32_t i = q_begin; i < G.L; ++i) {
        const int32_t lo = G.lo(i);   // first key position the row may see
        if (code[i] & bs::kCodeText) {
            for (int c = 0; c < 4; ++c) pairs[c] += i + 1 - lo;
            continue;
        }
        while (sp[g].end <= i) ++g;
        const int32_t e = G.bidir ? sp[g].end - 1 : i;   // last key position the row may see
        const int32_t s0 = std::max(sp[g].start, lo);    // first own-image key it may see
        const int64_t text = G.n_text[e + 1] - G.n_text[lo];
        const int64_t sink_img = G.n_free_sink[e + 1] - G.n_free_sink[lo] - text;  // image tokens that are sinks, in [lo, e]
        const int64_t own = e - s0 + 1;
        const int64_t own_sink = (G.n_free_sink[e + 1] - G.n_free_sink[s0]) - (G.n_text[e + 1] - G.n_text[s0]);
        const int64_t row[4] = {e + 1 - lo, text + sink_img, text + own, text + sink_img + own - own_sink};
        for (int c = 0; c < 4; ++c) {
            pairs[c] += row[c];
            if (row[c] == 0) ++empty[c];
        }
    }
    for (int c = 0; c < 4; ++c) { lists[c].allowed_pairs = pairs[c]; lists[c].empty_rows = empty[c]; }
}

bool spans_valid(const bs_span *spans, int32_t n, int32_t L)
{
    int32_t prev_end = 0;
    for (int32_t g = 0; g < n; ++g) {
        const bs_span &s = spans[g];
        if (s.start < prev_end || s.end <= s.start || s.end > L) return false;
        if (s.sink < 0 || s.sink > s.end - s.start) return false;
        prev_end = s.end;
    }
    return true;
}

}  // namespace

extern "C" int bs_build_tilemap(const bs_span *spans, int32_t n_spans, int32_t seq_len,
                                const uint8_t *head_class, int32_t n_q_heads, int32_t sink_len,
                                int32_t block_m, int32_t block_n, bs_tilemap **out)
{
    return bs_build_tilemap_ex(spans, n_spans, seq_len, head_class, n_q_heads, sink_len, block_m, block_n, 0, out);
}

extern "C" int bs_build_tilemap_ex(const bs_span *spans, int32_t n_spans, int32_t seq_len,
                                   const uint8_t *head_class, int32_t n_q_heads, int32_t sink_len,
                                   int32_t block_m, int32_t block_n, uint32_t flags, bs_tilemap **out)
{
    return bs_build_tilemap_model(spans, n_spans, seq_len, head_class, n_q_heads, sink_len, block_m, block_n, flags,
                                  nullptr, 0, 0, out);
}

extern "C" int bs_build_tilemap_model(const bs_span *spans, int32_t n_spans, int32_t seq_len,
                                      const uint8_t *head_class, int32_t n_q_heads, int32_t sink_len,
                                      int32_t block_m, int32_t block_n, uint32_t flags,
                                      const int32_t *sink_offsets, int32_t n_sink_offsets, int32_t window,
                                      bs_tilemap **out)
{
    return bs_build_tilemap_suffix(spans, n_spans, seq_len, head_class, n_q_heads, sink_len, block_m, block_n, flags,
                                   sink_offsets, n_sink_offsets, window, 0, out);
}

extern "C" int bs_build_tilemap_suffix(const bs_span *spans, int32_t n_spans, int32_t seq_len,
                                       const uint8_t *head_class, int32_t n_q_heads, int32_t sink_len,
                                       int32_t block_m, int32_t block_n, uint32_t flags,
                                       const int32_t *sink_offsets, int32_t n_sink_offsets, int32_t window,
                                       int32_t q_begin, bs_tilemap **out)
{
    if (q_begin < 0 || (seq_len > 0 && q_begin >= seq_len)) return BS_EINVAL;
    if (flags & ~(uint32_t)(BS_MAP_REGROUP_ROWS | BS_MAP_PACK_KEYS | BS_MAP_BIDIR_IMAGES)) return BS_EINVAL;
    if (window < 0) return BS_EINVAL;
    if (window >= seq_len) window = 0;   // every earlier key is inside the window
    if (window > 0 && (flags & BS_MAP_PACK_KEYS)) {
        // a windowed query tile visits a few key tiles only: nothing to pack; the rows stay regrouped
        flags = (flags & ~(uint32_t)BS_MAP_PACK_KEYS) | BS_MAP_REGROUP_ROWS;
    }
    if (n_sink_offsets < 0 || (n_sink_offsets > 0 && !sink_offsets)) return BS_EINVAL;
    for (int32_t o = 0; o < n_sink_offsets; ++o)
        if (sink_offsets[o] < 0) return BS_EINVAL;
    if (flags & BS_MAP_PACK_KEYS) flags |= BS_MAP_REGROUP_ROWS;   // packed lists exist for image-only query tiles
    if (!out || !head_class || n_q_heads <= 0 || seq_len <= 0 || n_spans < 0) return BS_EINVAL;
    if (n_spans > 0 && !spans) return BS_EINVAL;
    if (sink_len < 0 || sink_len > seq_len || block_m <= 0 || block_n <= 0) return BS_EINVAL;
    if ((int64_t)n_spans >= (int64_t)bs::kCodeImgMask) return BS_EINVAL;
    for (int32_t h = 0; h < n_q_heads; ++h)
        if (head_class[h] > 3) return BS_EINVAL;
    if (!spans_valid(spans, n_spans, seq_len)) return BS_EINVAL;

    bs_tilemap *tm = nullptr;
    try {
        tm = new bs_tilemap();
        const int32_t L = seq_len;
        tm->L = L; tm->bm = block_m; tm->bn = block_n; tm->sink_len = sink_len;
        tm->q_begin = q_begin;
        tm->N0 = tm->N = (L + block_n - 1) / block_n;
        tm->n_q_heads = n_q_heads;
        tm->spans.assign(spans, spans + n_spans);
        tm->head_class.assign(head_class, head_class + n_q_heads);

        // per-token codes
        tm->code.assign(L, bs::kCodeText);
        for (int32_t t = 0; t < sink_len; ++t) tm->code[t] |= bs::kCodeSink;
        for (int32_t g = 0; g < n_spans; ++g)
            for (int32_t t = spans[g].start; t < spans[g].end; ++t) {
                uint32_t c = (uint32_t)(g + 1);
                if (t - spans[g].start < spans[g].sink || t < sink_len) c |= bs::kCodeSink;
                tm->code[t] = c;
            }
        for (int32_t g = 0; g < n_spans; ++g)   // sinks at fixed offsets inside every image
            for (int32_t o = 0; o < n_sink_offsets; ++o)
                if (sink_offsets[o] < spans[g].end - spans[g].start) tm->code[spans[g].start + sink_offsets[o]] |= bs::kCodeSink;
        tm->bidir = (flags & BS_MAP_BIDIR_IMAGES) != 0 && n_spans > 0;

        // Key tiles: the prompt's keys in position order, then (packed) compact tiles with the
        // free keys -- text keys and sink keys, what an image query of a sparse class may see
        // outside its own image -- in position order.  The paper's kernel permutes K / V so that
        // these keys are contiguous (App. kernel, "Attention Sink Subroutine"); here they are a
        // second copy, because text queries and Dense heads keep walking the original order.
        std::vector<int32_t> free_pos;
        if (flags & BS_MAP_PACK_KEYS) {
            bool any_image = false;
            for (int32_t t = 0; t < L; ++t) {
                if (tm->code[t] & (bs::kCodeText | bs::kCodeSink)) free_pos.push_back(t);
                if (!(tm->code[t] & bs::kCodeText)) any_image = true;
            }
            if (any_image && !free_pos.empty() && free_pos.size() < (size_t)L) {
                tm->packed = true;
                tm->N = tm->N0 + (int32_t)((free_pos.size() + block_n - 1) / block_n);
            }
        }
        tm->key_order.assign((size_t)tm->N * block_n, -1);
        for (int32_t t = 0; t < L; ++t) tm->key_order[t] = t;
        if (tm->packed) std::copy(free_pos.begin(), free_pos.end(), tm->key_order.begin() + (size_t)tm->N0 * block_n);

        // per-key-tile bit masks for the kernel's 64-wide element predicate
        if (block_n <= 64) {
            tm->text_bits.assign(tm->N, 0);
            tm->sink_bits.assign(tm->N, 0);
            for (size_t slot = 0; slot < tm->key_order.size(); ++slot) {
                const int32_t t = tm->key_order[slot];
                if (t < 0) continue;
                const uint64_t bit = 1ull << (slot % block_n);
                if (tm->code[t] & bs::kCodeText) tm->text_bits[slot / block_n] |= bit;
                if (tm->code[t] & bs::kCodeSink) tm->sink_bits[slot / block_n] |= bit;
            }
        }

        // Order of the query rows.  Natural: tile m holds rows m*bm ... .  Regrouped: the image
        // rows first, then the text rows, each group in position order and padded to whole
        // tiles (-1).  A text row attends to every earlier token, so a tile that holds even one
        // walks every causal key tile for every class; gathered into tiles of their own, the
        // text rows stop costing the image rows of the sparse classes their skipped tiles.
        {
            const int64_t bm = block_m;
            const int64_t R = L - q_begin;                 // the query rows are positions q_begin .. L - 1
            std::vector<int32_t> img_rows, txt_rows;
            if (flags & BS_MAP_REGROUP_ROWS) {
                for (int32_t t = q_begin; t < L; ++t) ((tm->code[t] & bs::kCodeText) ? txt_rows : img_rows).push_back(t);
            }
            if (img_rows.empty() || txt_rows.empty()) {   // natural order (also: nothing to separate)
                tm->M = (int32_t)((R + bm - 1) / bm);
                tm->row_order.assign((size_t)tm->M * bm, -1);
                for (int64_t r = 0; r < R; ++r) tm->row_order[r] = (int32_t)(q_begin + r);
            } else {
                const int64_t m_img = ((int64_t)img_rows.size() + bm - 1) / bm, m_txt = ((int64_t)txt_rows.size() + bm - 1) / bm;
                tm->M = (int32_t)(m_img + m_txt);
                tm->row_order.assign((size_t)tm->M * bm, -1);
                std::copy(img_rows.begin(), img_rows.end(), tm->row_order.begin());
                std::copy(txt_rows.begin(), txt_rows.end(), tm->row_order.begin() + m_img * bm);
                tm->regrouped = true;
            }
        }

        Geometry G;
        G.L = L; G.bm = block_m; G.bn = block_n; G.M = tm->M; G.N = tm->N0; G.spans = &tm->spans;
        G.bidir = tm->bidir;
        G.window = tm->window = window;
        if (window > 0) {
            G.first_visible.resize(L);
            for (int32_t t = 0; t < L; ++t) G.first_visible[t] = std::max(0, t - window + 1);
            if (tm->bidir)
                for (int32_t g = 0; g < n_spans; ++g)
                    for (int32_t t = spans[g].start; t < spans[g].end; ++t)
                        G.first_visible[t] = std::min(G.first_visible[t], spans[g].start);
        }
        G.n_text.assign(L + 1, 0);
        G.n_free_sink.assign(L + 1, 0);
        G.last_text.assign(L, -1);
        G.next_text.assign(L + 1, L);
        G.next_free_sink.assign(L + 1, L);
        for (int32_t t = 0; t < L; ++t) {
            const bool text = tm->code[t] & bs::kCodeText;
            const bool fs = text || (tm->code[t] & bs::kCodeSink);
            G.n_text[t + 1] = G.n_text[t] + text;
            G.n_free_sink[t + 1] = G.n_free_sink[t] + fs;
            G.last_text[t] = text ? t : (t ? G.last_text[t - 1] : -1);
        }
        for (int32_t t = L - 1; t >= 0; --t) {
            const bool text = tm->code[t] & bs::kCodeText;
            const bool fs = text || (tm->code[t] & bs::kCodeSink);
            G.next_text[t] = text ? t : G.next_text[t + 1];
            G.next_free_sink[t] = fs ? t : G.next_free_sink[t + 1];
        }

        for (int b = 0; b < 2; ++b) {
            const std::vector<int32_t> &fc = b ? G.n_free_sink : G.n_text;
            G.next_allfree_tile[b].assign(tm->N0 + 1, tm->N0);
            for (int32_t n = tm->N0 - 1; n >= 0; --n) {
                const int32_t c0 = n * block_n, c1 = std::min(c0 + block_n, L);
                const bool allfree = (c1 - c0 == block_n) && (fc[c1] - fc[c0] == block_n);
                G.next_allfree_tile[b][n] = allfree ? n : G.next_allfree_tile[b][n + 1];
            }
        }
        if (tm->packed) {
            G.packed = true;
            G.n_free = (int32_t)free_pos.size();
            G.Nc = tm->N - tm->N0;
            G.ctext.assign(free_pos.size() + 1, 0);
            for (size_t s2 = 0; s2 < free_pos.size(); ++s2)
                G.ctext[s2 + 1] = G.ctext[s2] + ((tm->code[free_pos[s2]] & bs::kCodeText) ? 1 : 0);
            // what the kernel needs per row / per image: free keys before a position, and the
            // compact slots of the free keys that lie inside each image
            tm->free_before = G.n_free_sink;
            tm->span_free_range.assign(2 * ((size_t)n_spans + 1), 0);
            for (int32_t g = 0; g < n_spans; ++g) {
                tm->span_free_range[2 * (g + 1)] = G.n_free_sink[spans[g].start];
                tm->span_free_range[2 * (g + 1) + 1] = G.n_free_sink[spans[g].end];
            }
        }
        bool intra_close_call = false;
        if (tm->packed) {
            // Intra-Image rows need the text keys only.  Among the compact tiles they are mixed
            // with the sink keys; where text is rare (a few long images) the prompt's own tiles
            // hold it in fewer tiles.  Both lists are exact, so the choice is a matter of cost
            // only: count, for the last row of every image, the tiles with a text key either
            // way (prefix counts over the two tile spaces) and take the smaller total; a close
            // call is settled below by building both.
            std::vector<int32_t> prompt_tiles(tm->N0 + 1, 0), compact_tiles(G.Nc + 1, 0);
            for (int32_t n = 0; n < tm->N0; ++n) {
                const int32_t c0 = n * block_n, c1 = std::min(c0 + block_n, L);
                prompt_tiles[n + 1] = prompt_tiles[n] + (G.n_text[c1] - G.n_text[c0] > 0);
            }
            for (int32_t c = 0; c < G.Nc; ++c) {
                const int32_t s0 = c * block_n, s1 = std::min(s0 + block_n, G.n_free);
                compact_tiles[c + 1] = compact_tiles[c] + (G.ctext[s1] - G.ctext[s0] > 0);
            }
            int64_t cost_prompt = 0, cost_compact = 0;
            for (int32_t g = 0; g < n_spans; ++g) {
                const int64_t rows = spans[g].end - spans[g].start;
                cost_prompt += rows * prompt_tiles[(spans[g].end - 1) / block_n + 1];
                cost_compact += rows * compact_tiles[(G.n_free_sink[spans[g].end] + block_n - 1) / block_n];
            }
            G.intra_compact = tm->intra_compact = cost_compact < cost_prompt;
            intra_close_call = cost_compact * 4 >= cost_prompt * 3 && cost_prompt * 4 >= cost_compact * 3;
        }
        for (int c = 0; c < 4; ++c) build_class(G, c, tm->row_order, tm->cls[c]);
        if (intra_close_call) {
            // the estimate is within a quarter: build the other variant as well and keep the shorter list
            ClassLists alt;
            G.intra_compact = !G.intra_compact;
            build_class(G, BS_INTRA, tm->row_order, alt);
            if (alt.visited < tm->cls[BS_INTRA].visited) {
                tm->cls[BS_INTRA] = std::move(alt);
                tm->intra_compact = G.intra_compact;
            }
            G.intra_compact = tm->intra_compact;
        }
        count_pairs(G, tm->code, q_begin, tm->cls);

    } catch (const std::bad_alloc &) {
        delete tm;
        return BS_ENOMEM;
    }
    *out = tm;
    return BS_OK;
}

// Work list of the fp32 kernel: heaviest (head, query tile) first so the tail of the launch is
// short; ties keep one KV group's heads of a query tile next to each other.
void bs_plan_work(bs_tilemap *tm)
{
    if (tm->work_epoch == tm->class_epoch) return;
    const int32_t H = tm->n_q_heads;
    tm->work.resize((size_t)H * tm->M);
    size_t w = 0;
    for (int32_t h = 0; h < H; ++h)
        for (int32_t m = 0; m < tm->M; ++m) tm->work[w++] = {h, m};
    const bs_tilemap *t = tm;
    std::stable_sort(tm->work.begin(), tm->work.end(), [t](const bs::WorkItem &a, const bs::WorkItem &b) {
        int32_t ca = t->cls[t->head_class[a.head]].row_tiles[a.q_tile];
        int32_t cb = t->cls[t->head_class[b.head]].row_tiles[b.q_tile];
        if (ca != cb) return ca > cb;
        if (a.q_tile != b.q_tile) return a.q_tile > b.q_tile;
        return a.head < b.head;
    });
    tm->work_epoch = tm->class_epoch;
}

extern "C" int bs_tilemap_rebind(bs_tilemap *tm, const uint8_t *head_class, int32_t n_q_heads)
{
    if (!tm || !head_class || n_q_heads <= 0) return BS_EINVAL;
    for (int32_t h = 0; h < n_q_heads; ++h)
        if (head_class[h] > 3) return BS_EINVAL;
    if ((size_t)n_q_heads == tm->head_class.size() && std::equal(head_class, head_class + n_q_heads, tm->head_class.begin()))
        return BS_OK;   // same vector: the work units stay valid
    try {
        tm->head_class.assign(head_class, head_class + n_q_heads);
    } catch (const std::bad_alloc &) {
        return BS_ENOMEM;
    }
    tm->n_q_heads = n_q_heads;
    ++tm->class_epoch;
    return BS_OK;
}

// Pairing for the KV-sharing bf16 kernel.  Three rules, all exact (no approximation, only a
// different grouping of the same work), applied inside each KV group:
//   1. heads that carry the same class walk identical lists at the same query tile: pair them
//      two by two (no step is wasted);
//   2. heads left over with different classes may be paired at the same query tile: their lists
//      are merged and each run records the state for either item (a tile only one of them needs
//      is a SKIP step for the other).  Good when most query tiles mix text and image rows (then
//      both walk every causal tile anyway), bad when one class visits far more tiles;
//   3. a left-over head pairs its own query tiles 2j and 2j+1 the same way.
// Rule 2 is used for a pair of left-over heads only if it needs fewer steps than rule 3 for both.
void bs_plan_pairs(bs_tilemap *tm, int32_t G)
{
    bs::PairPlan &plan = tm->pairs;
    if (plan.gqa_group == G && plan.epoch == tm->class_epoch) return;
    plan.ranges.clear();
    plan.items.clear();
    const int32_t M = tm->M, H = tm->n_q_heads;

    // merged list of (class ca, row ma) and (class cb, row mb); cb < 0: item A alone
    struct Span2 { int32_t begin, end, tiles; };
    bool count_only = false;
    auto merged = [&](int ca, int32_t ma, int cb, int32_t mb) {
        const ClassLists &la = tm->cls[ca];
        const ClassLists &lb = tm->cls[cb < 0 ? ca : cb];
        int64_t pa = la.row_ptr[ma], ea = la.row_ptr[ma + 1];
        int64_t pb = cb < 0 ? 0 : lb.row_ptr[mb], eb = cb < 0 ? 0 : lb.row_ptr[mb + 1];
        Span2 out{(int32_t)plan.ranges.size(), 0, 0};
        int32_t cur = 0, rb = -1, re = -1, rs = 0;
        auto emit = [&](int32_t b, int32_t e, int sa, int sb) {
            if (e <= b || (sa == 0 && sb == 0)) return;
            out.tiles += e - b;
            const int st = (sa << 2) | sb;
            if (count_only) return;
            if (rb >= 0 && b == re && st == rs) { re = e; return; }
            if (rb >= 0) plan.ranges.push_back({rb, (re << 4) | rs});
            rb = b; re = e; rs = st;
        };
        while (pa < ea || pb < eb) {
            while (pa < ea && la.ranges[pa].end() <= cur) ++pa;
            while (pb < eb && lb.ranges[pb].end() <= cur) ++pb;
            if (pa >= ea && pb >= eb) break;
            const bool in_a = pa < ea && la.ranges[pa].begin <= cur;
            const bool in_b = pb < eb && lb.ranges[pb].begin <= cur;
            int32_t nxt = INT32_MAX;  // next boundary after cur
            if (pa < ea) nxt = std::min(nxt, in_a ? la.ranges[pa].end() : la.ranges[pa].begin);
            if (pb < eb) nxt = std::min(nxt, in_b ? lb.ranges[pb].end() : lb.ranges[pb].begin);
            emit(cur, nxt, in_a ? (la.ranges[pa].full() ? 2 : 1) : 0, in_b ? (lb.ranges[pb].full() ? 2 : 1) : 0);
            cur = nxt;
        }
        if (rb >= 0) plan.ranges.push_back({rb, (re << 4) | rs});
        out.end = (int32_t)plan.ranges.size();
        return out;
    };
    // lists shared by many units are made once: key (ca, cb or 4 for "alone"/same row pair kind, row)
    std::vector<Span2> cache_same[4], cache_cross[4][4], cache_rows[4], cache_alone[4];
    auto cached = [&](std::vector<Span2> &tab, int32_t idx, int32_t size, auto make) -> const Span2 & {
        if (tab.empty()) tab.assign(size, Span2{-1, -1, 0});
        if (tab[idx].begin < 0) tab[idx] = make();
        return tab[idx];
    };

    // total steps of rule 2 for a class pair / of rule 3 for a class, over all query tiles
    int64_t cross_total[4][4], rows_total[4];
    for (int a = 0; a < 4; ++a) { rows_total[a] = -1; for (int b = 0; b < 4; ++b) cross_total[a][b] = -1; }
    auto cross_cost = [&](int ca, int cb) {
        if (cross_total[ca][cb] < 0) {
            count_only = true;
            int64_t t = 0;
            for (int32_t m = 0; m < M; ++m) t += merged(ca, m, cb, m).tiles;
            count_only = false;
            cross_total[ca][cb] = cross_total[cb][ca] = t;
        }
        return cross_total[ca][cb];
    };
    auto rows_cost = [&](int c) {
        if (rows_total[c] < 0) {
            count_only = true;
            int64_t t = 0;
            for (int32_t j = 0; 2 * j < M; ++j)
                t += (2 * j + 1 < M) ? merged(c, 2 * j, c, 2 * j + 1).tiles : merged(c, 2 * j, -1, 0).tiles;
            count_only = false;
            rows_total[c] = t;
        }
        return rows_total[c];
    };

    std::vector<int32_t> byclass[4], rest, solo;
    for (int32_t kv = 0; kv < H / G; ++kv) {
        for (int c = 0; c < 4; ++c) byclass[c].clear();
        for (int32_t h = kv * G; h < (kv + 1) * G; ++h) byclass[tm->head_class[h]].push_back(h);
        rest.clear();
        for (int c = 0; c < 4; ++c) {
            size_t i = 0;
            for (; i + 1 < byclass[c].size(); i += 2)  // rule 1
                for (int32_t m = 0; m < M; ++m) {
                    const Span2 &sp = cached(cache_same[c], m, M, [&] { return merged(c, m, c, m); });
                    plan.items.push_back({byclass[c][i], m, byclass[c][i + 1], m, sp.begin, sp.end, sp.tiles, 0});
                }
            if (i < byclass[c].size()) rest.push_back(byclass[c][i]);
        }
        // rule 2 where it saves steps over rule 3: repeatedly take the pair with the best saving
        solo.clear();
        while (rest.size() >= 2) {
            int64_t best = 0;
            size_t bi = 0, bj = 0;
            for (size_t i = 0; i < rest.size(); ++i)
                for (size_t j = i + 1; j < rest.size(); ++j) {
                    const int ca = tm->head_class[rest[i]], cb = tm->head_class[rest[j]];
                    const int64_t saving = rows_cost(ca) + rows_cost(cb) - cross_cost(ca, cb);
                    if (saving > best) { best = saving; bi = i; bj = j; }
                }
            if (best <= 0) break;
            const int32_t ha = rest[bi], hb = rest[bj];
            const int ca = tm->head_class[ha], cb = tm->head_class[hb];
            for (int32_t m = 0; m < M; ++m) {
                const Span2 &sp = cached(cache_cross[ca][cb], m, M, [&] { return merged(ca, m, cb, m); });
                plan.items.push_back({ha, m, hb, m, sp.begin, sp.end, sp.tiles, 0});
            }
            rest.erase(rest.begin() + bj);
            rest.erase(rest.begin() + bi);
        }
        for (int32_t h : rest) {  // rule 3
            const int c = tm->head_class[h];
            for (int32_t j = 0; 2 * j < M; ++j) {
                if (2 * j + 1 < M) {
                    const Span2 &sp = cached(cache_rows[c], j, (M + 1) / 2, [&] { return merged(c, 2 * j, c, 2 * j + 1); });
                    plan.items.push_back({h, 2 * j, h, 2 * j + 1, sp.begin, sp.end, sp.tiles, 0});
                } else {
                    const Span2 &sp = cached(cache_alone[c], 0, 1, [&] { return merged(c, 2 * j, -1, 0); });
                    plan.items.push_back({h, 2 * j, -1, 0, sp.begin, sp.end, sp.tiles, 0});
                }
            }
        }
    }
    // Queue order.  Heaviest units first (longest-processing-time rule), but in coarse cost
    // buckets inside which units of one KV head stay together, walking the same tiles at about
    // the same time.  The sorted list is then dealt to eight queues, one per XCD (each XCD has its
    // own L2), in blocks of kXcdBlock consecutive units: the units of a block run side by side on
    // one XCD and find each other's K / V^T tiles in its L2.  The kernel's workgroups take the
    // units of their XCD's queue in this order (plan.queue_off delimits the queues in plan.items).
    // Block size: 8 for a few thousand units (a bigger block costs load balance at the tail),
    // 16 for tens of thousands (measured on the 36K and 300K workloads).
    // Bucket width: 32 tiles for up to four KV heads.  With more KV heads a 32-tile bucket holds about one
    // block of each head, neighbours in a queue read different heads and the L2s share less: the width
    // grows with the square of the head count (measured: 16 KV heads at 300K tokens gain 2-3 % from 512-
    // 1024 tiles, 8 KV heads at 140K 0.3-1 % from 256-1024, 4 KV heads lose 0.2-0.5 % with anything above
    // 32), but never so wide that the heaviest-first order loses its grip on the tail (a workgroup's
    // share of the steps / 64).
    constexpr int32_t kXcds = 8;
    int32_t cost_bucket = 32;
    {
        int64_t total = 0;
        for (const bs::PairItem &it : plan.items) total += it.n_tiles;
        const int64_t n_kv = std::max<int64_t>(1, (int64_t)tm->head_class.size() / std::max(G, 1));
        const int64_t for_locality = 32 * std::max<int64_t>(1, n_kv / 4) * std::max<int64_t>(1, n_kv / 4);
        const int64_t for_balance = total / 256 / 64;                     // 256 workgroups
        cost_bucket = (int32_t)std::max<int64_t>(32, std::min(for_locality, for_balance) / 32 * 32);
    }
    const int32_t kXcdBlock = std::min<int64_t>(16, std::max<int64_t>(8, (int64_t)plan.items.size() / 2048));
    std::stable_sort(plan.items.begin(), plan.items.end(), [G, cost_bucket](const bs::PairItem &a, const bs::PairItem &b) {
        const int32_t ba = a.n_tiles / cost_bucket, bb = b.n_tiles / cost_bucket;
        if (ba != bb) return ba > bb;
        const int32_t ka = a.head_a / G, kb = b.head_a / G;
        if (ka != kb) return ka < kb;
        return a.n_tiles > b.n_tiles;
    });
    {
        const size_t n = plan.items.size();
        std::vector<bs::PairItem> queues[kXcds];
        for (size_t p = 0; p < n; ++p) queues[(p / kXcdBlock) % kXcds].push_back(plan.items[p]);
        plan.items.clear();
        for (int x = 0; x < kXcds; ++x) {
            plan.queue_off[x] = (int32_t)plan.items.size();
            plan.items.insert(plan.items.end(), queues[x].begin(), queues[x].end());
        }
        plan.queue_off[kXcds] = (int32_t)plan.items.size();
    }
    for (bs::PairItem &it : plan.items)
        it.classes = tm->head_class[it.head_a] | (it.head_b >= 0 ? tm->head_class[it.head_b] << 8 : 0);
    plan.gqa_group = G;
    plan.epoch = tm->class_epoch;
}

extern "C" int bs_tilemap_pair_plan(bs_tilemap *tm, int32_t gqa_group, int64_t *n_units, int64_t *unit_tiles,
                                    int64_t *skip_steps)
{
    if (!tm || gqa_group <= 0 || tm->n_q_heads % gqa_group != 0) return BS_EINVAL;
    try {
        bs_plan_pairs(tm, gqa_group);
        // check the plan against the per-class lists it was derived from
        const bs::PairPlan &plan = tm->pairs;
        std::vector<uint8_t> want_a(tm->N), want_b(tm->N), got_a(tm->N), got_b(tm->N);
        std::vector<int32_t> seen((size_t)tm->n_q_heads * tm->M, 0);
        int64_t tiles = 0, skips = 0;
        for (const bs::PairItem &it : plan.items) {
            if (it.head_a < 0 || it.head_a >= tm->n_q_heads || it.tile_a < 0 || it.tile_a >= tm->M) return BS_EINVAL;
            if (it.head_b >= tm->n_q_heads || (it.head_b >= 0 && (it.tile_b < 0 || it.tile_b >= tm->M))) return BS_EINVAL;
            if (it.head_b >= 0 && it.head_b / gqa_group != it.head_a / gqa_group) return BS_EINVAL;
            ++seen[(size_t)it.head_a * tm->M + it.tile_a];
            if (it.head_b >= 0) ++seen[(size_t)it.head_b * tm->M + it.tile_b];
            std::fill(got_a.begin(), got_a.end(), 0);
            std::fill(got_b.begin(), got_b.end(), 0);
            int32_t prev_end = 0, n_tiles = 0;
            for (int32_t p = it.list_begin; p < it.list_end; ++p) {
                const bs::PairRange &r = plan.ranges[p];
                const int32_t e = r.end_states >> 4, sa = (r.end_states >> 2) & 3, sb = r.end_states & 3;
                if (r.begin < prev_end || e <= r.begin || e > tm->N || (sa == 0 && sb == 0) || sa == 3 || sb == 3) return BS_EINVAL;
                for (int32_t n = r.begin; n < e; ++n) { got_a[n] = (uint8_t)sa; got_b[n] = (uint8_t)sb; }
                skips += (int64_t)(e - r.begin) * ((sa == 0) + (sb == 0 && it.head_b >= 0));
                n_tiles += e - r.begin;
                prev_end = e;
            }
            if (n_tiles != it.n_tiles) return BS_EINVAL;
            tiles += n_tiles;
            if (bs_tilemap_tile_states(tm, tm->head_class[it.head_a], it.tile_a, 1, want_a.data()) != BS_OK) return BS_EINVAL;
            if (want_a != got_a) return BS_EINVAL;
            if (it.head_b >= 0) {
                if (bs_tilemap_tile_states(tm, tm->head_class[it.head_b], it.tile_b, 1, want_b.data()) != BS_OK) return BS_EINVAL;
                if (want_b != got_b) return BS_EINVAL;
            }
        }
        for (int32_t v : seen)
            if (v != 1) return BS_EINVAL;  // every (head, query tile) exactly once
        if (n_units) *n_units = (int64_t)plan.items.size();
        if (unit_tiles) *unit_tiles = tiles;
        if (skip_steps) *skip_steps = skips;
    } catch (const std::bad_alloc &) {
        return BS_ENOMEM;
    }
    return BS_OK;
}

extern "C" void bs_tilemap_destroy(bs_tilemap *tm)
{
    if (!tm) return;
    if (tm->dev && tm->dev_free) tm->dev_free(tm->dev);
    delete tm;
}

extern "C" int bs_tilemap_dims(const bs_tilemap *tm, int32_t *seq_len, int32_t *n_q_tiles,
                               int32_t *n_k_tiles, int32_t *n_q_heads)
{
    if (!tm) return BS_EINVAL;
    if (seq_len) *seq_len = tm->L;
    if (n_q_tiles) *n_q_tiles = tm->M;
    if (n_k_tiles) *n_k_tiles = tm->N;
    if (n_q_heads) *n_q_heads = tm->n_q_heads;
    return BS_OK;
}

extern "C" int bs_tilemap_row_order(const bs_tilemap *tm, int32_t *rows)
{
    if (!tm || !rows) return BS_EINVAL;
    std::memcpy(rows, tm->row_order.data(), tm->row_order.size() * sizeof(int32_t));
    return BS_OK;
}

extern "C" int bs_tilemap_layout(const bs_tilemap *tm, int32_t *regrouped, int32_t *packed, int32_t *intra_compact)
{
    if (!tm) return BS_EINVAL;
    if (regrouped) *regrouped = tm->regrouped;
    if (packed) *packed = tm->packed;
    if (intra_compact) *intra_compact = tm->intra_compact;
    return BS_OK;
}

extern "C" int bs_tilemap_key_order(const bs_tilemap *tm, int32_t *keys, int32_t *n_prompt_tiles)
{
    if (!tm) return BS_EINVAL;
    if (keys) std::memcpy(keys, tm->key_order.data(), tm->key_order.size() * sizeof(int32_t));
    if (n_prompt_tiles) *n_prompt_tiles = tm->N0;
    return BS_OK;
}

extern "C" int bs_tilemap_tile_states(const bs_tilemap *tm, int32_t cls, int32_t q_tile_begin,
                                      int32_t q_tile_count, uint8_t *states)
{
    if (!tm || !states || cls < 0 || cls > 3 || q_tile_begin < 0 || q_tile_count < 0 ||
        (int64_t)q_tile_begin + q_tile_count > tm->M)
        return BS_EINVAL;
    const ClassLists &cl = tm->cls[cls];
    std::memset(states, 0, (size_t)q_tile_count * tm->N);
    for (int32_t r = 0; r < q_tile_count; ++r) {
        uint8_t *row = states + (size_t)r * tm->N;
        for (int64_t p = cl.row_ptr[q_tile_begin + r]; p < cl.row_ptr[q_tile_begin + r + 1]; ++p) {
            const TileRange &rg = cl.ranges[p];
            for (int32_t n = rg.begin; n < rg.end(); ++n) row[n] = rg.full() ? 2 : 1;
        }
    }
    return BS_OK;
}

extern "C" int bs_tilemap_stats(const bs_tilemap *tm, int32_t cls, int64_t *visited, int64_t *full,
                                int64_t *partial, int64_t *allowed_pairs, int64_t *empty_rows,
                                int64_t *n_ranges)
{
    if (!tm || cls < 0 || cls > 3) return BS_EINVAL;
    const ClassLists &cl = tm->cls[cls];
    if (visited) *visited = cl.visited;
    if (full) *full = cl.full;
    if (partial) *partial = cl.partial;
    if (allowed_pairs) *allowed_pairs = cl.allowed_pairs;
    if (empty_rows) *empty_rows = cl.empty_rows;
    if (n_ranges) *n_ranges = (int64_t)cl.ranges.size();
    return BS_OK;
}

extern "C" const char *bs_strerror(int code)
{
    switch (code) {
        case BS_OK: return "ok";
        case BS_EINVAL: return "invalid argument";
        case BS_EUNSUPPORTED: return "unsupported tile size, head_dim or dtype";
        case BS_ENOMEM: return "out of memory";
        case BS_EHIP: return "HIP runtime error";
        default: return "unknown error";
    }
}
