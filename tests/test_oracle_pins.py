"""Pins for the CPU oracle: each test checks the oracle against something other than itself —
hand-derived bitmaps (tests/golden/), a library attention routine, closed forms, invariants.

Paper passages: Sec. 3.1 (attention definition, causal prefill), Sec. 3.2 (head classes;
text tokens attend to all previous tokens), App. kernel Alg. 4 (online-softmax recurrence),
App. D.2 remark that Intra-Image+Sink masks are a superset of the other two.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as W
from golden_masks import all_fixtures, full_fixtures, load, load_full

D, S, I, IS = 0, 1, 2, 3


def np_token_arrays(spans, L, sink_len, offsets=()):
    """Independent (numpy slicing) construction of imgid / issink from the span table;
    offsets: in-image offsets that are sink keys in every image as well."""
    imgid = np.zeros(L, dtype=np.int32)
    issink = np.zeros(L, dtype=np.uint8)
    issink[:sink_len] = 1
    for g, (s, e, k) in enumerate(np.asarray(spans).reshape(-1, 3)):
        imgid[s:e] = g + 1
        issink[s:s + k] = 1
        for o in offsets or ():
            if o < e - s:
                issink[s + o] = 1
    return imgid, issink


def small_prompt(seed=0, classes=(D, S, I, IS), n_kv=2, d=16, dtype="f32", sink_len=3):
    rng = np.random.default_rng(seed)
    runs = [("T", int(rng.integers(0, 9)))]
    for _ in range(int(rng.integers(2, 6))):
        runs.append(("I", int(rng.integers(1, 70))))
        runs.append(("T", int(rng.integers(0, 12))))
    return W.custom_prompt(runs, classes, n_kv, d, dtype=dtype, sink_len=sink_len,
                           name=f"small{seed}")


# ----------------------------------------------------------------------------- mask predicate

@pytest.mark.parametrize("path", all_fixtures())
def test_mask_matches_hand_derived_bitmaps(path):
    L, spans, sink_len, expected = load(path)
    imgid, issink = oracle.token_arrays(spans, L, sink_len)
    for cls, want in expected.items():
        got = oracle.mask(cls, imgid, issink)
        assert np.array_equal(got, want), f"{path} class {cls}\n{got}\n{want}"


def test_token_arrays_match_numpy_slicing():
    for seed in range(5):
        p = small_prompt(seed)
        a, b = oracle.token_arrays(p.spans, p.seq_len, p.sink_len)
        c, d_ = np_token_arrays(p.spans, p.seq_len, p.sink_len)
        assert np.array_equal(a, c) and np.array_equal(b, d_)


@pytest.mark.parametrize("bad", [
    [(0, 0, 0)], [(5, 3, 0)], [(0, 4, 5)], [(0, 4, -1)], [(0, 40, 0)], [(4, 8, 0), (6, 9, 0)],
    [(4, 8, 0), (0, 2, 0)],
])
def test_token_arrays_reject_bad_spans(bad):
    with pytest.raises(ValueError):
        oracle.token_arrays(np.asarray(bad, dtype=np.int32), 32, 0)


def test_mask_set_identities():
    """IS = I u S; every class within Dense; Dense = lower triangle; text rows equal in all classes."""
    for seed in range(6):
        p = small_prompt(seed, sink_len=seed % 3)
        imgid, issink = oracle.token_arrays(p.spans, p.seq_len, p.sink_len)
        m = [oracle.mask(c, imgid, issink).astype(bool) for c in range(4)]
        L = p.seq_len
        assert np.array_equal(m[D], np.tril(np.ones((L, L), dtype=bool)))
        assert np.array_equal(m[IS], m[I] | m[S])
        for c in (S, I, IS):
            assert not (m[c] & ~m[D]).any()
            assert np.array_equal(m[c][imgid == 0], m[D][imgid == 0])
            # text keys are visible to every query (vertical bands)
            assert np.array_equal(m[c][:, imgid == 0], m[D][:, imgid == 0])
        # Intra-Image heads never cross images; Sink heads never see a non-sink image key
        ii, jj = np.nonzero(m[I])
        cross = (imgid[ii] > 0) & (imgid[jj] > 0) & (imgid[ii] != imgid[jj])
        assert not cross.any()
        ii, jj = np.nonzero(m[S])
        bad = (imgid[ii] > 0) & (imgid[jj] > 0) & (issink[jj] == 0)
        assert not bad.any()


def closed_form_pair_counts(spans, L, sink_len, offsets=(), bidir=False):
    """Pair counts per class from prefix sums over the span table (no per-pair enumeration).
    bidir: an image row sees up to the last token of its image (non-causal attention inside an image)."""
    imgid, issink = np_token_arrays(spans, L, sink_len, offsets)
    text = imgid == 0
    text_cum = np.cumsum(text)                       # text keys in [0..i]
    snt = (issink == 1) & ~text
    snt_cum = np.cumsum(snt)                         # sink-and-image keys in [0..i]
    idx = np.arange(L)
    start = np.zeros(L, dtype=np.int64)
    last = idx.copy()                                # last key position a row may see
    for s, e, _ in np.asarray(spans).reshape(-1, 3):
        start[s:e] = s
        if bidir:
            last[s:e] = e - 1
    own = last - start + 1                           # own-image keys in [start..last]
    snt_before = np.where(start > 0, snt_cum[np.maximum(start - 1, 0)], 0)
    own_sink = snt_cum[last] - snt_before            # of which sinks
    per_row = {D: last + 1, S: text_cum[last] + snt_cum[last], I: text_cum[last] + own,
               IS: text_cum[last] + snt_cum[last] + own - own_sink}
    return {c: int(np.where(text, idx + 1, r).sum()) for c, r in per_row.items()}


def test_pair_counts_match_closed_form():
    for seed in range(6):
        p = small_prompt(seed, sink_len=2 * (seed % 2))
        imgid, issink = oracle.token_arrays(p.spans, p.seq_len, p.sink_len)
        want = closed_form_pair_counts(p.spans, p.seq_len, p.sink_len)
        for c in range(4):
            assert oracle.pair_count(c, imgid, issink) == want[c]
            assert int(oracle.mask(c, imgid, issink).sum()) == want[c]
    p = W.tiny_config("paper10")
    imgid, issink = oracle.token_arrays(p.spans, p.seq_len, p.sink_len)
    want = closed_form_pair_counts(p.spans, p.seq_len, p.sink_len)
    for c in range(4):
        assert oracle.pair_count(c, imgid, issink) == want[c]
    # images that attend in both directions, sinks at in-image offsets
    for seed in range(6):
        p = small_prompt(seed + 20, sink_len=seed % 3)
        offsets = [0, 4, 11, 40][: 1 + seed % 4]
        imgid, issink = oracle.token_arrays(p.spans, p.seq_len, p.sink_len, offsets)
        for bidir in (False, True):
            want = closed_form_pair_counts(p.spans, p.seq_len, p.sink_len, offsets, bidir)
            for c in range(4):
                assert oracle.pair_count(c, imgid, issink, bidir) == want[c]
                assert int(oracle.mask(c, imgid, issink, bidir).sum()) == want[c]


def test_row_subsets_of_the_bitmap_and_of_the_pair_count():
    """mask_rows / pair_count_rows are the listed rows of the full bitmap (itself pinned to the hand-derived ones)."""
    for seed in range(4):
        p = small_prompt(seed + 30, sink_len=seed)
        offsets = [2, 9] if seed % 2 else None
        imgid, issink = oracle.token_arrays(p.spans, p.seq_len, p.sink_len, offsets)
        rows = np.random.default_rng(seed).permutation(p.seq_len)[: max(1, p.seq_len // 3)].astype(np.int32)
        for c in range(4):
            for bidir, window in ((False, 0), (True, 0), (False, 7), (True, 5)):
                full = oracle.mask(c, imgid, issink, bidir, window)
                assert np.array_equal(oracle.mask_rows(c, imgid, issink, rows, bidir, window), full[rows])
                assert oracle.pair_count_rows(c, imgid, issink, rows, bidir, window) == int(full[rows].sum())
                assert oracle.pair_count_rows(c, imgid, issink, np.arange(p.seq_len), bidir, window) == int(full.sum())


def test_tile_states_from_bitmap():
    """The tile reduction equals a numpy block reduction of the dense bitmap (out-of-range = masked)."""
    for seed, (bm, bn) in enumerate([(8, 4), (16, 8), (128, 64), (4, 4)]):
        p = small_prompt(seed)
        imgid, issink = oracle.token_arrays(p.spans, p.seq_len, p.sink_len)
        L = p.seq_len
        M, N = -(-L // bm), -(-L // bn)
        for c in range(4):
            full = np.zeros((M * bm, N * bn), dtype=np.int64)
            full[:L, :L] = oracle.mask(c, imgid, issink)
            cnt = full.reshape(M, bm, N, bn).sum(axis=(1, 3))
            want = np.where(cnt == 0, 0, np.where(cnt == bm * bn, 2, 1)).astype(np.uint8)
            got = oracle.tile_states(c, imgid, issink, bm, bn)
            assert np.array_equal(got, want)
            sub = np.array([M - 1, 0], dtype=np.int32)
            assert np.array_equal(oracle.tile_states(c, imgid, issink, bm, bn, sub), want[sub])


def test_tile_states_for_row_lists_from_bitmap():
    """Tile states of query tiles given as row lists: numpy gather + reduction of the bitmap.
    The natural order reproduces the contiguous reduction; a shuffled order and tiles with
    missing rows (slots of -1) are checked too."""
    rng = np.random.default_rng(7)
    for seed, (bm, bn) in enumerate([(8, 4), (16, 8), (4, 4)]):
        p = small_prompt(seed)
        imgid, issink = oracle.token_arrays(p.spans, p.seq_len, p.sink_len)
        L = p.seq_len
        M, N = -(-L // bm), -(-L // bn)
        natural = np.full(M * bm, -1, dtype=np.int32)
        natural[:L] = np.arange(L)
        shuffled = natural.copy()
        rng.shuffle(shuffled)
        for c in range(4):
            bitmap = np.zeros((L + 1, N * bn), dtype=np.int64)   # row L: "no row"
            bitmap[:L, :L] = oracle.mask(c, imgid, issink)
            for order in (natural, shuffled):
                rows = order.reshape(M, bm)
                cnt = bitmap[np.where(rows < 0, L, rows)].reshape(M, bm, N, bn).sum(axis=(1, 3))
                want = np.where(cnt == 0, 0, np.where(cnt == bm * bn, 2, 1)).astype(np.uint8)
                assert np.array_equal(oracle.tile_states_rows(c, imgid, issink, rows, bn), want)
            assert np.array_equal(oracle.tile_states_rows(c, imgid, issink, natural.reshape(M, bm), bn),
                                  oracle.tile_states(c, imgid, issink, bm, bn))


# ----------------------------------------------------------------------------- softmax . V numerics

def sdpa_fp64(q, k, v, G, scale, mask=None):
    """Library attention on CPU in fp64: causal when mask is None, else an explicit boolean mask."""
    qt, kt, vt = (torch.from_numpy(np.asarray(x, dtype=np.float64)) for x in (q, k, v))
    kt = kt.repeat_interleave(G, dim=0)
    vt = vt.repeat_interleave(G, dim=0)
    if mask is None:
        o = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, is_causal=True, scale=scale)
    else:
        o = torch.nn.functional.scaled_dot_product_attention(
            qt, kt, vt, attn_mask=torch.from_numpy(mask.astype(bool)), scale=scale)
    return o.numpy()


def test_all_dense_equals_library_causal_attention():
    p = W.custom_prompt([("T", 7), ("I", 300), ("T", 5), ("I", 211), ("T", 40)], [D] * 6, 2, 32,
                        dtype="f32", scale=0.31)
    q, k, v = (t.numpy() for t in W.make_qkv(p, 3))
    got = oracle.attention_for_prompt(p, q, k, v)
    want = sdpa_fp64(q, k, v, p.gqa_group, p.scale)
    assert np.abs(got - want).max() < 1e-12


def test_tiny_config_dense_head_equals_library_causal_attention():
    p = W.tiny_config("paper10")
    q, k, v = (t.numpy() for t in W.make_qkv(p, 0))
    got = oracle.attention_for_prompt(p, q, k, v)
    want = sdpa_fp64(q, k, v, p.gqa_group, p.scale)
    assert p.head_class[0] == D
    assert np.abs(got[0] - want[0]).max() < 1e-11
    assert np.abs(got[1] - want[1]).max() > 1e-3      # the sparse head really differs


def test_sparse_classes_equal_library_attention_with_explicit_mask():
    """Checks the numerics (scale, GQA head mapping, operand order) for every class; the mask
    itself is pinned by the bitmap / identity / perturbation tests."""
    p = W.custom_prompt([("T", 5), ("I", 90), ("T", 3), ("I", 120), ("I", 40), ("T", 9)],
                        [D, S, I, IS, IS, I, S, D], 4, 24, dtype="f32", sink_len=2, scale=0.4)
    q, k, v = (t.numpy() for t in W.make_qkv(p, 1))
    imgid, issink = np_token_arrays(p.spans, p.seq_len, p.sink_len)
    got = oracle.attention_for_prompt(p, q, k, v)
    for h, c in enumerate(p.head_class):
        m = oracle.mask(int(c), imgid, issink)
        assert m.any(axis=1).all()
        want = sdpa_fp64(q[h:h + 1], k[h // 2:h // 2 + 1], v[h // 2:h // 2 + 1], 1, p.scale, m[None])
        assert np.abs(got[h] - want[0]).max() < 1e-12, h


def test_rows_sum_to_one_and_empty_rows_are_zero():
    # first image has no sink and no text before it: Sink-head rows there are empty
    p = W.custom_prompt([("I", 20), ("T", 4), ("I", 30)], [S, I, IS, D], 1, 8, dtype="f32",
                        sink_mode="prefix")
    q, k, v = (t.numpy() for t in W.make_qkv(p, 2))
    v1 = np.ones_like(v)
    o = oracle.attention_for_prompt(p, q, k, v1)
    imgid, issink = oracle.token_arrays(p.spans, p.seq_len, p.sink_len)
    for h, c in enumerate(p.head_class):
        nonempty = oracle.mask(int(c), imgid, issink).any(axis=1)
        assert np.allclose(o[h][nonempty], 1.0, atol=1e-13)
        assert np.all(o[h][~nonempty] == 0.0)
    assert (~oracle.mask(S, imgid, issink).any(axis=1)).sum() == 20


def test_key_shift_invariance():
    p = small_prompt(4, d=16)
    q, k, v = (t.numpy().astype(np.float64) for t in W.make_qkv(p, 4))
    c = np.random.default_rng(0).standard_normal(16)
    # exactly representable inputs keep the fp32 interface exact
    q, k, v, c = (np.round(x * 64) / 64 for x in (q, k, v, c))
    a = oracle.attention_for_prompt(p, q, k, v)
    b = oracle.attention_for_prompt(p, q, k + c, v)
    assert np.abs(a - b).max() < 1e-11


def test_row_subset_equals_full():
    p = small_prompt(5)
    q, k, v = (t.numpy() for t in W.make_qkv(p, 5))
    full = oracle.attention_for_prompt(p, q, k, v)
    rows = np.array([p.seq_len - 1, 0, 7, 7, 3], dtype=np.int32)
    sub = oracle.attention_for_prompt(p, q, k, v, rows)
    assert np.array_equal(sub, full[:, rows])


# ----------------------------------------------------------------------------- mask seen through the output

def test_perturbation_invariances():
    runs = [("T", 6), ("I", 50), ("T", 4), ("I", 60), ("T", 3), ("I", 40), ("T", 5)]
    p = W.custom_prompt(runs, [I, S, IS, D], 1, 16, dtype="f32", sink_len=0, span_sink=5)
    q, k, v = (t.numpy() for t in W.make_qkv(p, 6))
    base = oracle.attention_for_prompt(p, q, k, v)
    (s1, e1, _), (s2, e2, k2), (s3, e3, _) = (tuple(int(x) for x in r) for r in p.spans)
    rng = np.random.default_rng(1)

    def perturbed(lo, hi):
        kk, vv = k.copy(), v.copy()
        kk[:, lo:hi] = rng.standard_normal(kk[:, lo:hi].shape)
        vv[:, lo:hi] = rng.standard_normal(vv[:, lo:hi].shape)
        return oracle.attention_for_prompt(p, q, kk, vv)

    rows2 = np.arange(s2, e2)
    # other images' keys (non-sink part for the sink classes) do not matter to image 2's queries
    o = perturbed(s1, e1)
    assert np.array_equal(o[0][rows2], base[0][rows2])                  # Intra: whole image 1
    o = perturbed(s1 + 5, e1)
    assert np.array_equal(o[1][rows2], base[1][rows2])                  # Sink: non-sink part of image 1
    assert np.array_equal(o[2][rows2], base[2][rows2])                  # Intra+Sink likewise
    assert np.abs(o[3][rows2] - base[3][rows2]).max() > 1e-6            # Dense notices
    # the sink part of image 1 matters to Sink and Intra+Sink, not to Intra
    o = perturbed(s1, s1 + 5)
    assert np.array_equal(o[0][rows2], base[0][rows2])
    assert np.abs(o[1][rows2] - base[1][rows2]).max() > 1e-6
    assert np.abs(o[2][rows2] - base[2][rows2]).max() > 1e-6
    # a Sink head ignores the non-sink keys of the query's own image
    o = perturbed(s2 + 5, e2)
    assert np.array_equal(o[1][rows2], base[1][rows2])
    late = np.arange(s2 + 6, e2)
    assert np.abs(o[0][late] - base[0][late]).max() > 1e-6
    # earlier text matters to everyone; later tokens to no one (causality)
    o = perturbed(e1, s2)
    for h in range(4):
        assert np.abs(o[h][rows2] - base[h][rows2]).max() > 1e-6
    o = perturbed(e2, p.seq_len)
    for h in range(4):
        assert np.array_equal(o[h][: e2], base[h][: e2])


def uniform_attention_closed_form_heads(p, v):
    """With q = 0 every allowed key gets the same weight: out[h, i] = mean of v over the allowed
    set of row i, from per-category prefix sums of v (O(L d) per head, no pair enumeration).
    Yields (h, out[h]) head by head, so that a 300K-token prompt needs one head's array at a time.
    Covers the model variant with non-causal images (a row then sees up to the last token of its
    image) and sinks at in-image offsets; no sliding window."""
    assert not p.window
    L = p.seq_len
    imgid, issink = np_token_arrays(p.spans, L, p.sink_len, p.sink_offsets)
    text = imgid == 0
    snt = (issink == 1) & ~text
    start = np.zeros(L, dtype=np.int64)
    idx = np.arange(L)
    last = idx.copy()                # last key position a row may see
    for s, e, _ in p.spans:
        start[s:e] = s
        if p.img_bidir:
            last[s:e] = e - 1

    def csum(w):  # inclusive prefix sums with a leading zero row
        out = np.zeros((L + 1,) + w.shape[1:])
        np.cumsum(w, axis=0, out=out[1:])
        return out

    # three disjoint key categories: text, image sinks, other image tokens
    cats = (text, snt, ~text & ~snt)
    cnt = [csum(sel.astype(np.float64)[:, None]) for sel in cats]
    acc, acc_kv = None, -1
    img_rows = np.flatnonzero(~text)
    hi_t, hi_i, lo_i = idx[text] + 1, last[img_rows] + 1, start[img_rows]
    for h, c in enumerate(p.head_class):
        if h // p.gqa_group != acc_kv:   # prefix sums of this KV head's values, shared by its query heads
            acc_kv = h // p.gqa_group
            vh = np.asarray(v[acc_kv], dtype=np.float64)
            acc = [csum(np.where(sel[:, None], vh, 0.0)) for sel in cats]
        num = np.empty((L, vh.shape[1]))
        den = np.empty((L, 1))
        for tab, dst in ((acc, num), (cnt, den)):
            dst[text] = tab[0][hi_t] + tab[1][hi_t] + tab[2][hi_t]          # text rows: every key up to the row
            if c == D:
                dst[img_rows] = tab[0][hi_i] + tab[1][hi_i] + tab[2][hi_i]
                continue
            r = tab[0][hi_i].copy()                                          # text keys up to the last visible position
            if c in (S, IS):
                r += tab[1][hi_i]                                            # image sinks anywhere before it
            if c == I:
                r += tab[1][hi_i] - tab[1][lo_i]                             # own image: its sinks ...
            if c in (I, IS):
                r += tab[2][hi_i] - tab[2][lo_i]                             # ... and its other tokens
            dst[img_rows] = r
        yield h, np.where(den > 0, num / np.maximum(den, 1), 0.0)


def uniform_attention_closed_form(p, v):
    """All heads of uniform_attention_closed_form_heads at once: [n_q_heads, L, d]."""
    out = np.zeros((p.n_q_heads, p.seq_len, v.shape[-1]))
    for h, o in uniform_attention_closed_form_heads(p, v):
        out[h] = o
    return out


def test_uniform_attention_closed_form():
    for seed in range(4):
        p = small_prompt(seed + 10, classes=(D, S, I, IS), n_kv=2, sink_len=seed)
        q, k, v = (t.numpy() for t in W.make_qkv(p, seed))
        got = oracle.attention_for_prompt(p, np.zeros_like(q), k, v)
        want = uniform_attention_closed_form(p, v)
        assert np.abs(got - want).max() < 1e-12
    p = W.tiny_config("paper10").with_classes([S, I])
    q, k, v = (t.numpy() for t in W.make_qkv(p, 0))
    got = oracle.attention_for_prompt(p, np.zeros_like(q), k, v)
    assert np.abs(got - uniform_attention_closed_form(p, v)).max() < 1e-12
    # non-causal images and sinks at in-image offsets
    p = W.custom_prompt([("T", 5), ("I", 40), ("T", 3), ("I", 61), ("I", 17), ("T", 9)], [D, S, I, IS], 2, 16,
                        dtype="f32", sink_len=2, img_bidir=True, sink_offsets=(0, 7, 33))
    q, k, v = (t.numpy() for t in W.make_qkv(p, 3))
    got = oracle.attention_for_prompt(p, np.zeros_like(q), k, v)
    assert np.abs(got - uniform_attention_closed_form(p, v)).max() < 1e-12


# ----------------------------------------------------------------------------- tiled recurrence

def tiled_online_softmax(q, k, v, mask, scale, bm, bn):
    """fp64 re-statement of the flash recurrence (running max, running sum, rescaled output;
    App. kernel Alg. 4) with a final division by the running sum."""
    L, d = q.shape
    out = np.zeros((L, d))
    for m0 in range(0, L, bm):
        rows = slice(m0, min(m0 + bm, L))
        nr = rows.stop - rows.start
        acc = np.zeros((nr, d))
        l = np.zeros(nr)
        mx = np.full(nr, -np.inf)
        for n0 in range(0, rows.stop, bn):
            cols = slice(n0, min(n0 + bn, L))
            s = (q[rows] @ k[cols].T) * scale
            s = np.where(mask[rows, cols] > 0, s, -np.inf)
            mx_n = s.max(axis=1)
            new = np.maximum(mx, mx_n)
            safe = np.where(np.isinf(new), 0.0, new)
            pmat = np.exp(s - safe[:, None])
            alpha = np.exp(np.where(np.isinf(mx), -np.inf, mx - safe))
            l = alpha * l + pmat.sum(axis=1)
            acc = alpha[:, None] * acc + pmat @ v[cols]
            mx = new
        out[rows] = np.where(l[:, None] > 0, acc / np.where(l > 0, l, 1.0)[:, None], 0.0)
    return out


@pytest.mark.parametrize("bm,bn", [(128, 64), (16, 8)])
def test_tile_size_independence(bm, bn):
    p = W.custom_prompt([("T", 9), ("I", 150), ("T", 2), ("I", 77), ("T", 20)], [D, S, I, IS], 2, 16,
                        dtype="f32", sink_len=4)
    q, k, v = (t.numpy().astype(np.float64) for t in W.make_qkv(p, 8))
    k[0, 0] *= 8.0
    imgid, issink = oracle.token_arrays(p.spans, p.seq_len, p.sink_len)
    got = oracle.attention_for_prompt(p, q, k, v)
    for h, c in enumerate(p.head_class):
        m = oracle.mask(int(c), imgid, issink)
        want = tiled_online_softmax(q[h], k[h // 2], v[h // 2], m, p.scale, bm, bn)
        assert np.abs(got[h] - want).max() < 1e-12


# ----------------------------------------------------------------------------- non-causal images, offset sinks

@pytest.mark.parametrize("path", full_fixtures())
def test_bidirectional_and_offset_sink_masks_match_hand_derived_bitmaps(path):
    L, spans, sink_len, offsets, bidir, expected, window = load_full(path)
    imgid, issink = oracle.token_arrays(spans, L, sink_len, offsets)
    assert len(expected) == 4
    for cls, want in expected.items():
        got = oracle.mask(cls, imgid, issink, bidir, window)
        assert np.array_equal(got, want), f"{path} class {cls}\n{got}\n{want}"


def test_offset_sinks_match_numpy_construction():
    spans = np.array([(3, 20, 2), (20, 27, 0), (40, 90, 5)], dtype=np.int32)
    offsets = [0, 6, 9, 30, 49, 200]
    imgid, issink = oracle.token_arrays(spans, 100, 1, offsets)
    want_id, want_sink = np_token_arrays(spans, 100, 1)
    for s, e, _ in spans:
        for o in offsets:
            if o < e - s:
                want_sink[s + o] = 1
    assert np.array_equal(imgid, want_id) and np.array_equal(issink, want_sink)
    assert issink[26] == 1 and issink[29] == 0 and issink[89] == 1   # offset 6 of image 2; 9 is past its end
    with pytest.raises(ValueError):
        oracle.token_arrays(spans, 100, 1, [-1])


def test_bidirectional_mask_is_the_causal_mask_plus_later_keys_of_the_own_image():
    """The dense mask gains exactly the pairs (i, j > i) inside one image; a sparse class keeps of
    them what its pattern allows: own-image keys for the intra classes, sink keys for Sink."""
    for seed in range(6):
        p = small_prompt(seed)
        imgid, issink = oracle.token_arrays(p.spans, p.seq_len, p.sink_len, [1, 5, 17])
        L = p.seq_len
        ii, jj = np.meshgrid(np.arange(L), np.arange(L), indexing="ij")
        later_own = (jj > ii) & (imgid[ii] == imgid[jj]) & (imgid[ii] > 0)
        for cls in (D, S, I, IS):
            causal = oracle.mask(cls, imgid, issink, False).astype(bool)
            bidir = oracle.mask(cls, imgid, issink, True).astype(bool)
            extra = later_own & (issink[jj] == 1) if cls == S else later_own
            assert np.array_equal(bidir, causal | extra), (seed, cls)
            assert oracle.pair_count(cls, imgid, issink, True) == int((causal | extra).sum())
        # closed form for the dense mask: the lower triangle plus len (len - 1) / 2 per image
        lens = p.spans[:, 1] - p.spans[:, 0]
        assert oracle.pair_count(D, imgid, issink, True) == L * (L + 1) // 2 + int((lens * (lens - 1) // 2).sum())


def test_bidirectional_attention_equals_library_attention_with_explicit_mask():
    p = W.custom_prompt([("T", 5), ("I", 90), ("T", 3), ("I", 120), ("I", 40), ("T", 9)],
                        [D, S, I, IS, IS, I, S, D], 4, 24, dtype="f32", sink_len=2, scale=0.4,
                        img_bidir=True, sink_offsets=(0, 7, 33, 100))
    q, k, v = (t.numpy() for t in W.make_qkv(p, 1))
    imgid, issink = oracle.token_arrays(p.spans, p.seq_len, p.sink_len, p.sink_offsets)
    got = oracle.attention_for_prompt(p, q, k, v)
    L = p.seq_len
    # the model's own dense mask, written out: lower triangle OR same-image block
    block = (imgid[:, None] == imgid[None, :]) & (imgid[:, None] > 0)
    dense = np.tril(np.ones((L, L), dtype=bool)) | block
    want = sdpa_fp64(q[0:1], k[0:1], v[0:1], 1, p.scale, dense[None])
    assert np.abs(got[0] - want[0]).max() < 1e-12
    for h, c in enumerate(p.head_class):
        m = oracle.mask(int(c), imgid, issink, True)
        want = sdpa_fp64(q[h:h + 1], k[h // 2:h // 2 + 1], v[h // 2:h // 2 + 1], 1, p.scale, m[None])
        assert np.abs(got[h] - want[0]).max() < 1e-12, h
    # and a row subset goes through the same loop
    rows = np.array([0, 5, 6, 94, 95, 100, 217, L - 1], dtype=np.int32)
    sub = oracle.attention_for_prompt(p, q, k, v, rows)
    assert np.array_equal(sub, got[:, rows])


# ----------------------------------------------------------------------------- sliding window

def test_window_mask_is_the_plain_mask_inside_the_band():
    for seed in range(6):
        p = small_prompt(seed)
        imgid, issink = oracle.token_arrays(p.spans, p.seq_len, p.sink_len, [2, 9])
        L = p.seq_len
        ii, jj = np.meshgrid(np.arange(L), np.arange(L), indexing="ij")
        own = (imgid[ii] == imgid[jj]) & (imgid[ii] > 0)
        for window in (1, 2, 7, 33, L, L + 5):
            band = (ii - jj < window)
            for bidir in (False, True):
                keep = band | own if bidir else band
                for cls in (D, S, I, IS):
                    plain = oracle.mask(cls, imgid, issink, bidir, 0).astype(bool)
                    got = oracle.mask(cls, imgid, issink, bidir, window).astype(bool)
                    assert np.array_equal(got, plain & keep), (seed, window, bidir, cls)
                    assert oracle.pair_count(cls, imgid, issink, bidir, window) == int((plain & keep).sum())
            if window >= L:
                assert np.array_equal(oracle.mask(IS, imgid, issink, False, window), oracle.mask(IS, imgid, issink))
        # closed form, causal dense mask: row i keeps min(i + 1, window) keys
        assert oracle.pair_count(D, imgid, issink, False, 7) == sum(min(i + 1, 7) for i in range(L))


def test_window_attention_equals_library_attention_with_explicit_mask():
    p = W.custom_prompt([("T", 5), ("I", 90), ("T", 3), ("I", 120), ("I", 40), ("T", 9)],
                        [D, S, I, IS, IS, I, S, D], 4, 24, dtype="f32", sink_len=2, scale=0.4, window=50)
    q, k, v = (t.numpy() for t in W.make_qkv(p, 1))
    imgid, issink = oracle.token_arrays(p.spans, p.seq_len, p.sink_len)
    got = oracle.attention_for_prompt(p, q, k, v)
    L = p.seq_len
    band = np.tril(np.ones((L, L), dtype=bool)) & ~np.tril(np.ones((L, L), dtype=bool), -50)   # the textbook band
    want = sdpa_fp64(q[0:1], k[0:1], v[0:1], 1, p.scale, band[None])
    assert np.abs(got[0] - want[0]).max() < 1e-12
    empty = 0
    for h, c in enumerate(p.head_class):
        m = oracle.mask(int(c), imgid, issink, False, 50).astype(bool)
        rows = np.flatnonzero(m.any(axis=1))
        empty += L - len(rows)
        want = sdpa_fp64(q[h:h + 1, rows], k[h // 2:h // 2 + 1], v[h // 2:h // 2 + 1], 1, p.scale, m[None, rows])
        assert np.abs(got[h][rows] - want[0]).max() < 1e-12, h
        assert (got[h][~m.any(axis=1)] == 0).all()
    assert empty > 0   # Sink-class rows deep inside an image see nothing within the window
