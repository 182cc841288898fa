"""Tile maps whose query rows are the last positions of the prompt only (chunked prefill, decoding with the
whole KV cache): the same masks (paper Sec. 3.2; the method prunes no KV entries, Sec. 6.1), restricted to
rows q_begin .. L - 1.  Bit-exact against the oracle's element mask reduced over the map's own row lists."""
import ctypes

import numpy as np
import pytest

import oracle
import paper_2507_09071_amd as bs
import workloads as W
from paper_2507_09071_amd import binding
from test_tilemap_model import random_layout


def check_suffix(spans, L, sink_len, bm, bn, q_begin, flags=0, bidir=False, offsets=None, window=0, q_tiles=None, pairs=True):
    f = flags | (bs.BS_MAP_BIDIR_IMAGES if bidir else 0)
    tm = bs.bs_build_tilemap(spans, L, np.zeros(1, np.uint8), sink_len, bm, bn, flags=f, sink_offsets=offsets,
                             window=window, q_begin=q_begin)
    imgid, issink = oracle.token_arrays(spans, L, sink_len, offsets)
    rows = tm.row_order(bm)
    flat = rows[rows >= 0]
    assert np.array_equal(np.sort(flat), np.arange(q_begin, L))            # exactly the chunk's positions
    lay = tm.layout()
    if lay["regrouped"]:
        img = flat[imgid[flat] > 0]
        assert np.array_equal(flat[: len(img)], img) and np.array_equal(img, np.sort(img))   # image rows first, in order
        assert np.array_equal(flat[len(img):], np.sort(flat[len(img):]))
    else:
        assert np.array_equal(flat, np.arange(q_begin, L))
    assert tm.n_k_tiles >= -(-L // bn)                                        # every key of the prompt stays a key
    sel = np.arange(tm.n_q_tiles) if q_tiles is None else np.asarray(q_tiles)
    keys, n0 = tm.key_order(bn)
    for c in range(4):
        if lay["packed"]:
            continue   # packed lists are checked pair by pair in test_packed_suffix below
        want = oracle.tile_states_rows(c, imgid, issink, rows[sel], bn, bidir, window)
        got = np.stack([tm.tile_states(c, int(m), 1)[0] for m in sel])
        assert np.array_equal(got, want), (c, np.argwhere(got != want)[:5])
        if pairs:
            assert tm.stats(c)["allowed_pairs"] == oracle.pair_count_rows(c, imgid, issink, np.arange(q_begin, L), bidir, window)
            if L <= 2048:
                m = oracle.mask(c, imgid, issink, bidir, window)[q_begin:]
                assert tm.stats(c)["empty_rows"] == int((~m.any(axis=1)).sum())
    return tm


@pytest.mark.parametrize("seed", range(40))
def test_random_prompts_every_option(seed):
    L, spans, offsets, sink_len, bm, bn = random_layout(700 + seed)
    if not L:
        return
    rng = np.random.default_rng(seed)
    for q_begin in sorted({0, L - 1, int(rng.integers(0, L)), int(rng.integers(0, L))}):
        for flags in (0, bs.BS_MAP_REGROUP_ROWS):
            check_suffix(spans, L, sink_len, bm, bn, q_begin, flags)
            check_suffix(spans, L, sink_len, bm, bn, q_begin, flags, bidir=True, offsets=offsets)
            w = int(rng.integers(1, max(2, L // 2)))
            check_suffix(spans, L, sink_len, bm, bn, q_begin, flags, window=w)
            check_suffix(spans, L, sink_len, bm, bn, q_begin, flags, bidir=True, offsets=offsets, window=w)


@pytest.mark.parametrize("seed", range(20))
def test_packed_suffix(seed):
    """Packed keys with a chunk of query rows: every allowed pair of the chunk's rows exactly once over the
    two key-tile spaces, tile states from the oracle's bitmap."""
    from test_tilemap import packed_expectation
    L, spans, offsets, sink_len, bm, bn = random_layout(800 + seed)
    if not L:
        return
    rng = np.random.default_rng(seed)
    for bidir in (False, True):
        q_begin = int(rng.integers(0, L))
        tm = bs.bs_build_tilemap(spans, L, np.zeros(1, np.uint8), sink_len, bm, bn,
                                 flags=bs.BS_MAP_PACK_KEYS | (bs.BS_MAP_BIDIR_IMAGES if bidir else 0),
                                 sink_offsets=offsets if bidir else None, q_begin=q_begin)
        imgid, issink = oracle.token_arrays(spans, L, sink_len, offsets if bidir else None)
        rows = tm.row_order(bm)
        assert np.array_equal(np.sort(rows[rows >= 0]), np.arange(q_begin, L))
        keys, n0 = tm.key_order(bn)
        lay = tm.layout()
        for c in range(4):
            mask = oracle.mask(c, imgid, issink, bidir)
            got = tm.tile_states(c)
            want = np.zeros_like(got)
            for m in range(tm.n_q_tiles):
                total = 0
                for n in range(tm.n_k_tiles):
                    e = packed_expectation(c, rows[m], keys[n], n < n0, mask, imgid, lay["packed"], lay["intra_compact"])
                    cnt = int(e.sum())
                    total += cnt
                    want[m, n] = 0 if cnt == 0 else (2 if cnt == bm * bn else 1)
                valid = rows[m][rows[m] >= 0]
                assert total == int(mask[valid].sum()), (c, m)
            assert np.array_equal(got, want), (c, np.argwhere(got != want)[:5])
            assert tm.stats(c)["allowed_pairs"] == int(mask[q_begin:].sum())
        tm.pair_plan(1)


def test_kernel_tile_size_chunks_of_config2():
    p = W.config(2)
    for q_begin in (p.seq_len - 1, p.seq_len - 2048, p.seq_len // 2 + 77):
        probe = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len, flags=bs.BS_MAP_REGROUP_ROWS, q_begin=q_begin)
        sel = sorted({0, probe.n_q_tiles // 2, probe.n_q_tiles - 1})
        tm = check_suffix(p.spans, p.seq_len, p.sink_len, 128, 64, q_begin, bs.BS_MAP_REGROUP_ROWS, q_tiles=sel,
                          pairs=(q_begin > p.seq_len - 4096))
        assert tm.n_q_tiles <= -(-(p.seq_len - q_begin) // 128) + 1
        tm2 = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len, flags=bs.BS_MAP_PACK_KEYS, q_begin=q_begin)
        tm2.pair_plan(p.gqa_group)


def test_bad_q_begin_is_rejected():
    lib = binding.load_library()
    sp = (binding._Span * 1)(binding._Span(2, 9, 0))
    hc = (ctypes.c_uint8 * 1)(0)
    out = ctypes.c_void_p()
    for q_begin in (-1, 20, 21):
        assert lib.bs_build_tilemap_suffix(sp, 1, 20, hc, 1, 0, 4, 4, 0, None, 0, 0, q_begin, ctypes.byref(out)) == -1
    assert lib.bs_build_tilemap_suffix(sp, 1, 20, hc, 1, 0, 4, 4, 0, None, 0, 0, 19, ctypes.byref(out)) == 0
    lib.bs_tilemap_destroy(out)
