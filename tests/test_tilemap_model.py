"""Tile maps of the model variant with non-causal attention inside an image and sinks at fixed
in-image offsets (paper Sec. 6.1, App. "Attention Sink Positions in Gemma 3"): bit-exact against the
oracle's element mask reduced to tiles, for the three map layouts."""
import ctypes

import numpy as np
import pytest

import oracle
import paper_2507_09071_amd as bs
import workloads as W
from golden_masks import full_fixtures, load_full
from paper_2507_09071_amd import binding
from test_tilemap import check_against_oracle, check_packed, check_regrouped


def random_layout(seed, equal_images=False):
    rng = np.random.default_rng(1300 + seed)
    runs = []
    n_img = int(rng.integers(1, 8))
    size = int(rng.integers(3, 40))
    for _ in range(n_img):
        runs.append(("T", int(rng.integers(0, 14))))
        runs.append(("I", size if equal_images else int(rng.integers(1, 40))))
        if rng.random() < 0.3:
            runs.append(("I", size if equal_images else int(rng.integers(1, 20))))
    runs.append(("T", int(rng.integers(0, 10))))
    L, spans = W.layout_from_runs(runs, "prefix", [0, 0, 2][seed % 3])
    offsets = sorted(set(int(o) for o in rng.integers(0, 40, size=int(rng.integers(0, 6)))))
    sink_len = int(rng.integers(0, min(L, 6) + 1)) if L else 0
    bm, bn = [(8, 4), (16, 8), (4, 4), (8, 16), (32, 16)][seed % 5]
    return L, spans, offsets, sink_len, bm, bn


@pytest.mark.parametrize("path", [p for p in full_fixtures() if "window" not in p])   # those: test_tilemap_window.py
@pytest.mark.parametrize("bm,bn", [(1, 1), (2, 2), (4, 2), (3, 5)])
def test_golden_prompts(path, bm, bn):
    L, spans, sink_len, offsets, bidir, _, window = load_full(path)
    assert window == 0
    check_against_oracle(spans, L, sink_len, bm, bn, bidir=bidir, offsets=offsets)
    check_regrouped(spans, L, sink_len, bm, bn, bidir=bidir, offsets=offsets)
    check_packed(spans, L, sink_len, bm, bn, bidir=bidir, offsets=offsets)


@pytest.mark.parametrize("seed", range(30))
@pytest.mark.parametrize("bidir", [True, False])
def test_random_prompts_natural_order(seed, bidir):
    L, spans, offsets, sink_len, bm, bn = random_layout(seed, equal_images=seed % 2 == 0)
    if L:
        check_against_oracle(spans, L, sink_len, bm, bn, bidir=bidir, offsets=offsets)


@pytest.mark.parametrize("seed", range(30))
def test_random_prompts_regrouped(seed):
    L, spans, offsets, sink_len, bm, bn = random_layout(100 + seed, equal_images=seed % 2 == 0)
    if L:
        check_regrouped(spans, L, sink_len, bm, bn, bidir=True, offsets=offsets)


@pytest.mark.parametrize("seed", range(30))
@pytest.mark.parametrize("bidir", [True, False])
def test_random_prompts_packed(seed, bidir):
    L, spans, offsets, sink_len, bm, bn = random_layout(200 + seed, equal_images=seed % 2 == 0)
    if L:
        check_packed(spans, L, sink_len, bm, bn, bidir=bidir, offsets=offsets)


def test_kernel_tile_size_sampled_tiles_of_the_gemma_like_config():
    p = W.gemma3_bidir_config(0, n_images=60)
    q_tiles = W.sample_q_tiles(p, 128, n_random=4, seed=1, max_tiles=10)
    check_against_oracle(p.spans, p.seq_len, p.sink_len, 128, 64, q_tiles, bidir=True, offsets=p.sink_offsets)
    tm = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len, 128, 64,
                             flags=bs.BS_MAP_PACK_KEYS | bs.BS_MAP_BIDIR_IMAGES, sink_offsets=p.sink_offsets)
    sel = np.unique(np.concatenate([[0, tm.n_q_tiles - 1], np.arange(0, tm.n_q_tiles, 17)]))
    check_regrouped(p.spans, p.seq_len, p.sink_len, 128, 64, q_tiles=sel, bidir=True, offsets=p.sink_offsets)
    plan = tm.pair_plan(p.gqa_group)
    assert plan["n_units"] > 0


def test_bidirectional_map_visits_at_least_the_causal_tiles():
    p = W.gemma3_bidir_config(1, n_images=20)
    a = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len, 128, 64, sink_offsets=p.sink_offsets)
    b = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len, 128, 64, flags=bs.BS_MAP_BIDIR_IMAGES,
                            sink_offsets=p.sink_offsets)
    for c in range(4):
        sa, sb = a.tile_states(c), b.tile_states(c)
        assert (sb >= sa).all()
        assert b.stats(c)["allowed_pairs"] > a.stats(c)["allowed_pairs"]


def test_model_entry_point_rejects_bad_arguments():
    lib = binding.load_library()
    sp = (binding._Span * 1)(binding._Span(2, 9, 0))
    hc = (ctypes.c_uint8 * 1)(0)
    out = ctypes.c_void_p()
    off = (ctypes.c_int32 * 2)(1, -3)
    f = lambda flags, o, n: lib.bs_build_tilemap_model(sp, 1, 20, hc, 1, 0, 4, 4, flags, o, n, 0, ctypes.byref(out))
    assert f(0, off, 2) == -1          # negative offset
    assert f(0, None, 1) == -1         # count without a list
    assert f(0, off, -1) == -1
    assert f(8, None, 0) == -1         # unknown flag
    assert f(4, off, 1) == 0 and out.value
    lib.bs_tilemap_destroy(out)
