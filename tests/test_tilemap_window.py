"""Tile maps of sliding-window layers (paper App. kernel, "Dense Attention Subroutine": the dense mask
is causal or a sliding window as in the original model): bit-exact against the oracle's element mask."""
import ctypes

import numpy as np
import pytest

import oracle
import paper_2507_09071_amd as bs
import workloads as W
from golden_masks import full_fixtures, load_full
from paper_2507_09071_amd import binding
from test_tilemap import check_against_oracle, check_packed, check_regrouped
from test_tilemap_model import random_layout


@pytest.mark.parametrize("path", [p for p in full_fixtures() if "window" in p])
@pytest.mark.parametrize("bm,bn", [(1, 1), (2, 2), (4, 2), (3, 5)])
def test_golden_prompts(path, bm, bn):
    L, spans, sink_len, offsets, bidir, _, window = load_full(path)
    check_against_oracle(spans, L, sink_len, bm, bn, bidir=bidir, offsets=offsets, window=window)
    check_regrouped(spans, L, sink_len, bm, bn, bidir=bidir, offsets=offsets, window=window)


@pytest.mark.parametrize("seed", range(40))
def test_random_prompts_causal_images(seed):
    L, spans, offsets, sink_len, bm, bn = random_layout(300 + seed)
    if not L:
        return
    rng = np.random.default_rng(seed)
    for window in (1, int(rng.integers(2, 12)), int(rng.integers(12, 60)), L - 1):
        if window < 1:
            continue
        check_against_oracle(spans, L, sink_len, bm, bn, offsets=offsets, window=window)
        check_regrouped(spans, L, sink_len, bm, bn, offsets=offsets, window=window)


@pytest.mark.parametrize("seed", range(30))
def test_random_prompts_bidirectional_images(seed):
    L, spans, offsets, sink_len, bm, bn = random_layout(400 + seed, equal_images=seed % 2 == 0)
    if not L or not len(spans):
        return
    longest = int((spans[:, 1] - spans[:, 0]).max())
    rng = np.random.default_rng(seed)
    # windows shorter than the longest image too: the own image stays visible beyond the window
    for window in (1, max(1, longest // 3), max(1, longest - 1), longest, longest + int(rng.integers(1, 30))):
        if window >= L:
            continue
        check_against_oracle(spans, L, sink_len, bm, bn, bidir=True, offsets=offsets, window=window)
        check_regrouped(spans, L, sink_len, bm, bn, bidir=True, offsets=offsets, window=window)


def test_window_of_the_whole_prompt_is_no_window_and_pack_flag_regroups():
    L, spans, offsets, sink_len, bm, bn = random_layout(7)
    hc = np.zeros(1, np.uint8)
    a = bs.bs_build_tilemap(spans, L, hc, sink_len, bm, bn)
    for window in (L, L + 3):
        b = bs.bs_build_tilemap(spans, L, hc, sink_len, bm, bn, window=window)
        for c in range(4):
            assert np.array_equal(a.tile_states(c), b.tile_states(c)) and a.stats(c) == b.stats(c)
    tm = check_regrouped(spans, L, sink_len, bm, bn, window=5, flags=bs.BS_MAP_PACK_KEYS)
    lay = tm.layout()
    assert lay["regrouped"] and not lay["packed"]


def test_kernel_tile_size_window_1024_sampled():
    p = W.gemma3_bidir_config(0, n_images=60)
    q_tiles = W.sample_q_tiles(p, 128, n_random=4, seed=2, max_tiles=10)
    check_against_oracle(p.spans, p.seq_len, p.sink_len, 128, 64, q_tiles, bidir=True, offsets=p.sink_offsets, window=1024)
    p2 = W.config(2)
    q_tiles = W.sample_q_tiles(p2, 128, n_random=4, seed=3, max_tiles=10)
    tm = check_against_oracle(p2.spans, p2.seq_len, p2.sink_len, 128, 64, q_tiles, window=4096)
    # a windowed layer visits at most window / 64 + 3 key tiles per query tile
    dense = tm.stats(0)
    assert dense["visited"] <= tm.n_q_tiles * (4096 // 64 + 3)


def test_negative_window_is_rejected():
    lib = binding.load_library()
    sp = (binding._Span * 1)(binding._Span(2, 9, 0))
    hc = (ctypes.c_uint8 * 1)(0)
    out = ctypes.c_void_p()
    assert lib.bs_build_tilemap_model(sp, 1, 20, hc, 1, 0, 4, 4, 0, None, 0, -1, ctypes.byref(out)) == -1
    for window in (6, 7):   # an image of 7 tokens that attends in both directions: longer than the window, and not
        assert lib.bs_build_tilemap_model(sp, 1, 20, hc, 1, 0, 4, 4, 4, None, 0, window, ctypes.byref(out)) == 0
        lib.bs_tilemap_destroy(out)


@pytest.mark.parametrize("seed", range(24))
def test_all_options_together_on_random_prompts(seed):
    """Every combination of map layout, image attention rule, offset sinks and window on one random
    prompt each: the maps stay bit-exact against the oracle."""
    rng = np.random.default_rng(7000 + seed)
    L, spans, offsets, sink_len, bm, bn = random_layout(500 + seed, equal_images=seed % 3 == 0)
    if not L:
        return
    longest = int((spans[:, 1] - spans[:, 0]).max()) if len(spans) else 1
    for bidir in (False, True):
        for window in (0, max(longest, int(rng.integers(1, 50)))):
            if window >= L:
                window = 0
            check_against_oracle(spans, L, sink_len, bm, bn, bidir=bidir, offsets=offsets, window=window)
            check_regrouped(spans, L, sink_len, bm, bn, bidir=bidir, offsets=offsets, window=window,
                            flags=bs.BS_MAP_PACK_KEYS if window else None)
            if not window:
                check_packed(spans, L, sink_len, bm, bn, bidir=bidir, offsets=offsets)
