"""Host logic of the library: the tile map must equal the oracle's element-wise mask reduced to
tiles, bit for bit (SKIP / PARTIAL / FULL), and its pair counts must equal the oracle's
enumeration.  Mask definition: paper Sec. 3.2; per-tile metadata: App. kernel, Notation."""
import ctypes
import re
import os

import numpy as np
import pytest

import oracle
import workloads as W
import paper_2507_09071_amd as bs
from paper_2507_09071_amd import binding
from golden_masks import all_fixtures, load

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def model_flags(bidir):
    return bs.BS_MAP_BIDIR_IMAGES if bidir else 0


def check_against_oracle(spans, L, sink_len, bm, bn, q_tiles=None, pairs=True, bidir=False, offsets=None, window=0):
    tm = bs.bs_build_tilemap(spans, L, np.zeros(1, np.uint8), sink_len, bm, bn, flags=model_flags(bidir),
                             sink_offsets=offsets, window=window)
    imgid, issink = oracle.token_arrays(spans, L, sink_len, offsets)
    for c in range(4):
        if q_tiles is None:
            want = oracle.tile_states(c, imgid, issink, bm, bn, None, bidir, window)
            got = tm.tile_states(c)
        else:
            want = oracle.tile_states(c, imgid, issink, bm, bn, q_tiles, bidir, window)
            got = np.stack([tm.tile_states(c, int(m), 1)[0] for m in q_tiles])
        assert np.array_equal(got, want), (c, np.argwhere(got != want)[:5])
        st = tm.stats(c)
        if q_tiles is None:
            assert st["visited"] == int((want > 0).sum())
            assert st["full"] == int((want == 2).sum())
            assert st["partial"] == int((want == 1).sum())
        if pairs:
            assert st["allowed_pairs"] == oracle.pair_count(c, imgid, issink, bidir, window)
            m = None
            if L <= 2048:
                m = oracle.mask(c, imgid, issink, bidir, window)
                assert st["empty_rows"] == int((~m.any(axis=1)).sum())
    return tm


@pytest.mark.parametrize("path", all_fixtures())
@pytest.mark.parametrize("bm,bn", [(1, 1), (2, 2), (4, 2), (3, 5)])
def test_golden_prompts_small_tiles(path, bm, bn):
    L, spans, sink_len, _ = load(path)
    check_against_oracle(spans, L, sink_len, bm, bn)


@pytest.mark.parametrize("seed", range(40))
def test_random_prompts_small_tiles(seed):
    rng = np.random.default_rng(seed)
    runs = []
    for _ in range(int(rng.integers(1, 8))):
        runs.append(("T", int(rng.integers(0, 14))))
        runs.append(("I", int(rng.integers(1, 40))))
        if rng.random() < 0.3:   # adjacent images, no text between
            runs.append(("I", int(rng.integers(1, 20))))
    runs.append(("T", int(rng.integers(0, 10))))
    mode = ["prefix", "paper10"][seed % 2]
    span_sink = [None, None, 3, 1000][seed % 4]
    L, spans = W.layout_from_runs(runs, mode, span_sink)
    if L == 0:
        return
    sink_len = int(rng.integers(0, min(L, 12) + 1))
    bm, bn = [(8, 4), (16, 8), (4, 4), (8, 16), (32, 16)][seed % 5]
    check_against_oracle(spans, L, sink_len, bm, bn)


@pytest.mark.parametrize("mode,span_sink", [("prefix", None), ("paper10", None), ("prefix", 32), ("prefix", 256)])
def test_tiny_config_full(mode, span_sink):
    p = W.tiny_config(mode, span_sink)
    check_against_oracle(p.spans, p.seq_len, p.sink_len, 128, 64)


def test_text_only_and_image_only_prompts():
    check_against_oracle(np.zeros((0, 3), np.int32), 300, 0, 128, 64)
    check_against_oracle(np.array([[0, 300, 0]], np.int32), 300, 0, 128, 64)
    check_against_oracle(np.array([[0, 300, 30]], np.int32), 300, 0, 128, 64)
    check_against_oracle(np.array([[0, 300, 300]], np.int32), 300, 300, 128, 64)
    check_against_oracle(np.array([[0, 1, 0], [1, 2, 1], [2, 3, 0]], np.int32), 3, 0, 128, 64)


@pytest.mark.parametrize("cfg", [2, 3, 4, 5])
def test_large_configs_sampled_query_tiles(cfg):
    p = W.config(cfg, seed=0, sink_mode="paper10", target_len=W.STRESS_LENGTHS[1])
    q_tiles = W.sample_q_tiles(p, 128, n_random=4, seed=cfg, max_tiles=14)
    tm = check_against_oracle(p.spans, p.seq_len, p.sink_len, 128, 64, q_tiles, pairs=(cfg in (2, 5)))
    assert tm.n_q_tiles == -(-p.seq_len // 128) and tm.n_k_tiles == -(-p.seq_len // 64)


def test_config2_prefix_mode_full_map():
    p = W.config(2, seed=1, sink_mode="prefix")
    check_against_oracle(p.spans, p.seq_len, p.sink_len, 128, 64)


def test_states_do_not_depend_on_head_classes():
    p = W.config(2)
    a = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len)
    b = bs.bs_build_tilemap(p.spans, p.seq_len, np.zeros_like(p.head_class), p.sink_len)
    for c in range(4):
        assert np.array_equal(a.tile_states(c, 100, 20), b.tile_states(c, 100, 20))
        assert a.stats(c) == b.stats(c)


# ------------------------------------------------------------------------- regrouped query rows

def check_regrouped(spans, L, sink_len, bm, bn, hc=None, q_tiles=None, bidir=False, offsets=None, window=0,
                    flags=None, pairs=True):
    """Map built with BS_MAP_REGROUP_ROWS against the oracle's reduction over the map's own row lists."""
    hc = np.zeros(1, np.uint8) if hc is None else hc
    tm = bs.bs_build_tilemap(spans, L, hc, sink_len, bm, bn,
                             flags=(bs.BS_MAP_REGROUP_ROWS if flags is None else flags) | model_flags(bidir),
                             sink_offsets=offsets, window=window)
    imgid, issink = oracle.token_arrays(spans, L, sink_len, offsets)
    rows = tm.row_order(bm)
    # a permutation of the positions, image rows first, each group in position order
    flat = rows[rows >= 0]
    assert np.array_equal(np.sort(flat), np.arange(L))
    n_img = int((imgid > 0).sum())
    if 0 < n_img < L:
        m_img = -(-n_img // bm)
        img_part, txt_part = rows[:m_img].ravel(), rows[m_img:].ravel()
        assert np.array_equal(img_part[img_part >= 0], np.flatnonzero(imgid > 0))
        assert np.array_equal(txt_part[txt_part >= 0], np.flatnonzero(imgid == 0))
        assert (img_part[:n_img] >= 0).all() and (img_part[n_img:] < 0).all()
        assert tm.n_q_tiles == m_img + -(-(L - n_img) // bm)
    else:
        assert np.array_equal(rows.ravel()[:L], np.arange(L))
    sel = np.arange(tm.n_q_tiles) if q_tiles is None else np.asarray(q_tiles)
    for c in range(4):
        want = oracle.tile_states_rows(c, imgid, issink, rows[sel], bn, bidir, window)
        got = tm.tile_states(c) if q_tiles is None else np.stack([tm.tile_states(c, int(m), 1)[0] for m in sel])
        assert np.array_equal(got, want), (c, np.argwhere(got != want)[:5])
        st = tm.stats(c)
        if q_tiles is None:
            assert st["visited"] == int((want > 0).sum()) and st["full"] == int((want == 2).sum())
        if pairs:   # by enumeration: quadratic in the prompt length
            assert st["allowed_pairs"] == oracle.pair_count(c, imgid, issink, bidir, window)   # the grouping changes no pair
    return tm


@pytest.mark.parametrize("seed", range(30))
def test_regrouped_random_prompts_small_tiles(seed):
    rng = np.random.default_rng(500 + seed)
    runs = []
    for _ in range(int(rng.integers(1, 8))):
        runs.append(("T", int(rng.integers(0, 14))))
        runs.append(("I", int(rng.integers(1, 40))))
        if rng.random() < 0.3:
            runs.append(("I", int(rng.integers(1, 20))))
    runs.append(("T", int(rng.integers(0, 10))))
    L, spans = W.layout_from_runs(runs, ["prefix", "paper10"][seed % 2], [None, None, 3, 1000][seed % 4])
    if L == 0:
        return
    bm, bn = [(8, 4), (16, 8), (4, 4), (8, 16), (32, 16)][seed % 5]
    check_regrouped(spans, L, int(rng.integers(0, min(L, 12) + 1)), bm, bn)


@pytest.mark.parametrize("path", all_fixtures())
def test_regrouped_golden_prompts(path):
    L, spans, sink_len, _ = load(path)
    check_regrouped(spans, L, sink_len, 4, 2)


def test_regrouped_single_text_tokens_between_images():
    """Worst case for the number of runs in a text tile: every text row is its own run."""
    runs = [("T", 1)]
    for _ in range(40):
        runs += [("I", 9), ("T", 1)]
    L, spans = W.layout_from_runs(runs, "paper10")
    check_regrouped(spans, L, 0, 16, 8)
    check_regrouped(spans, L, 3, 128, 64)


@pytest.mark.parametrize("cfg", [2, 4])
def test_regrouped_large_configs_sampled(cfg):
    p = W.config(cfg)
    probe = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len, flags=bs.BS_MAP_REGROUP_ROWS)
    M = probe.n_q_tiles
    n_img_tiles = -(-int(sum(e - s for s, e, _ in p.spans)) // 128)
    sel = sorted({0, 1, n_img_tiles // 2, n_img_tiles - 1, n_img_tiles, M - 1})   # both groups and their ragged ends
    tm = check_regrouped(p.spans, p.seq_len, p.sink_len, 128, 64, p.head_class, sel, pairs=(cfg == 2))
    tm.pair_plan(p.gqa_group)   # validates every unit against the per-class lists
    # the point of the grouping: the sparse classes visit fewer key tiles than in the natural order
    nat = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len)
    for c in (1, 2, 3):
        assert tm.stats(c)["visited"] < nat.stats(c)["visited"]
        assert tm.stats(c)["allowed_pairs"] == nat.stats(c)["allowed_pairs"]   # the grouping changes no pair


def test_regroup_flag_without_effect_and_bad_flags():
    L, spans = W.layout_from_runs([("T", 100)], "paper10")
    a = bs.bs_build_tilemap(spans, L, np.zeros(2, np.uint8), 0, flags=bs.BS_MAP_REGROUP_ROWS)
    b = bs.bs_build_tilemap(spans, L, np.zeros(2, np.uint8), 0)
    assert np.array_equal(a.row_order(), b.row_order())
    for c in range(4):
        assert np.array_equal(a.tile_states(c), b.tile_states(c))
    with pytest.raises(bs.BlindsightError):
        bs.bs_build_tilemap(spans, L, np.zeros(2, np.uint8), 0, flags=8)


# ------------------------------------------------------------------------- packed keys

def packed_expectation(c, rows, keys, in_prompt_space, mask, imgid, packed=True, intra_compact=True):
    """Allowed pairs of query rows x key slots of one tile of a packed map, from the oracle's
    bitmap: text rows and Dense heads use the prompt's tiles with the plain predicate; an image
    row of a sparse class counts own-image keys in the prompt's tiles and everything else it
    may see in the compact tiles."""
    i = rows[rows >= 0][:, None]
    j = keys[keys >= 0][None, :]
    if i.size == 0 or j.size == 0:
        return np.zeros((i.shape[0], j.shape[1]), dtype=bool)
    allowed = mask[i, j].astype(bool)
    if not packed:
        return allowed
    plain = (imgid[i] == 0) | (c == 0) | (c == 2 and not intra_compact)
    own = (imgid[i] == imgid[j]) & bool(c & 2)
    if in_prompt_space:
        return np.where(plain, allowed, allowed & own)
    return np.where(plain, False, allowed & ~own)


def check_packed(spans, L, sink_len, bm, bn, bidir=False, offsets=None):
    tm = bs.bs_build_tilemap(spans, L, np.zeros(1, np.uint8), sink_len, bm, bn,
                             flags=bs.BS_MAP_PACK_KEYS | model_flags(bidir), sink_offsets=offsets)
    imgid, issink = oracle.token_arrays(spans, L, sink_len, offsets)
    rows = tm.row_order(bm)
    keys, n0 = tm.key_order(bn)
    assert np.array_equal(keys[:n0].ravel()[:L], np.arange(L)) and (keys[:n0].ravel()[L:] < 0).all()
    free = np.flatnonzero((imgid == 0) | (issink == 1))
    packed = n0 < tm.n_k_tiles
    lay = tm.layout()
    assert lay["packed"] == packed and (lay["regrouped"] or not packed or (imgid > 0).all())   # regrouped, or no text rows
    if packed:
        comp = keys[n0:].ravel()
        assert np.array_equal(comp[comp >= 0], free) and (comp[:len(free)] >= 0).all()
    else:
        assert len(free) in (0, L) or (imgid == 0).all()
    for c in range(4):
        mask = oracle.mask(c, imgid, issink, bidir)
        got = tm.tile_states(c)
        want = np.zeros_like(got)
        for m in range(tm.n_q_tiles):
            total = 0
            for n in range(tm.n_k_tiles):
                e = packed_expectation(c, rows[m], keys[n], n < n0, mask, imgid, packed, lay["intra_compact"])
                cnt = int(e.sum())
                total += cnt
                want[m, n] = 0 if cnt == 0 else (2 if cnt == bm * bn else 1)
            valid = rows[m][rows[m] >= 0]
            assert total == int(mask[valid].sum()), (c, m)      # every allowed pair exactly once
        assert np.array_equal(got, want), (c, np.argwhere(got != want)[:5], got[got != want][:5], want[got != want][:5])
        assert tm.stats(c)["allowed_pairs"] == oracle.pair_count(c, imgid, issink, bidir)
    return tm


@pytest.mark.parametrize("seed", range(30))
def test_packed_random_prompts_small_tiles(seed):
    rng = np.random.default_rng(900 + seed)
    runs = []
    for _ in range(int(rng.integers(1, 8))):
        runs.append(("T", int(rng.integers(0, 14))))
        runs.append(("I", int(rng.integers(1, 40))))
        if rng.random() < 0.3:
            runs.append(("I", int(rng.integers(1, 20))))
    runs.append(("T", int(rng.integers(0, 10))))
    L, spans = W.layout_from_runs(runs, ["prefix", "paper10"][seed % 2], [None, None, 3, 1000][seed % 4])
    if L == 0:
        return
    bm, bn = [(8, 4), (16, 8), (4, 4), (8, 16), (32, 16)][seed % 5]
    check_packed(spans, L, int(rng.integers(0, min(L, 12) + 1)), bm, bn)


@pytest.mark.parametrize("path", all_fixtures())
def test_packed_golden_prompts(path):
    L, spans, sink_len, _ = load(path)
    check_packed(spans, L, sink_len, 4, 2)


def test_packed_kernel_tile_size_and_plan():
    runs = [("T", 30)]
    for i in range(12):
        runs += [("I", 150 + 37 * (i % 4)), ("T", 1 + 5 * (i % 3))]
    L, spans = W.layout_from_runs(runs, "paper10")
    tm = check_packed(spans, L, 9, 128, 64)
    hc = np.array([0, 1, 2, 3, 3, 1], dtype=np.uint8)
    tm2 = bs.bs_build_tilemap(spans, L, hc, 9, flags=bs.BS_MAP_PACK_KEYS)
    tm2.pair_plan(2)
    tm2.pair_plan(3)
    reg = bs.bs_build_tilemap(spans, L, hc, 9, flags=bs.BS_MAP_REGROUP_ROWS)
    for c in (1, 3):
        assert tm2.stats(c)["visited"] <= reg.stats(c)["visited"]


def check_packed_sampled(p, q_tiles, bm=128, bn=64):
    """Packed map of a long prompt at the kernel's tile size against the oracle, on sampled query tiles of the
    map's own row order: every (query tile, key tile) state from the oracle's bitmap rows, and every allowed
    pair of those rows counted exactly once over the two key-tile spaces."""
    from test_oracle_pins import closed_form_pair_counts
    flags = bs.BS_MAP_PACK_KEYS | model_flags(p.img_bidir)
    tm = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len, bm, bn, flags=flags,
                             sink_offsets=p.sink_offsets or None)
    L = p.seq_len
    imgid, issink = oracle.token_arrays(p.spans, L, p.sink_len, p.sink_offsets or None)
    rows_all = tm.row_order(bm)
    keys, n0 = tm.key_order(bn)
    lay = tm.layout()
    assert lay["packed"] and lay["regrouped"] and n0 == -(-L // bn)
    free = np.flatnonzero((imgid == 0) | (issink == 1))
    comp = keys[n0:].ravel()
    assert np.array_equal(comp[comp >= 0], free) and (comp[:len(free)] >= 0).all()
    nc = tm.n_k_tiles - n0
    for c in range(4):
        plain_class = c == 0 or (c == 2 and not lay["intra_compact"])
        for m in q_tiles:
            rows = rows_all[int(m)]
            valid = rows[rows >= 0]
            allowed = oracle.mask_rows(c, imgid, issink, valid, p.img_bidir).astype(bool)      # [rows, L]
            plain = (imgid[valid] == 0) | plain_class
            own = (imgid[valid][:, None] == imgid[None, :]) & bool(c & 2)
            in_prompt = np.where(plain[:, None], allowed, allowed & own)
            in_compact = np.where(plain[:, None], False, allowed & ~own)[:, free]
            assert int(in_prompt.sum()) + int(in_compact.sum()) == int(allowed.sum()), (c, m)   # each pair once
            cnt_p = np.pad(in_prompt, ((0, 0), (0, n0 * bn - L))).reshape(len(valid), n0, bn).sum(axis=(0, 2))
            cnt_c = np.pad(in_compact, ((0, 0), (0, nc * bn - len(free)))).reshape(len(valid), nc, bn).sum(axis=(0, 2))
            cnt = np.concatenate([cnt_p, cnt_c])
            want = np.where(cnt == 0, 0, np.where(cnt == bm * bn, 2, 1)).astype(np.uint8)
            got = tm.tile_states(c, int(m), 1)[0]
            assert np.array_equal(got, want), (p.name, c, int(m), np.flatnonzero(got != want)[:5])
    # the numerator of every TFLOP/s figure: allowed pairs per class against the test-side closed form
    want = closed_form_pair_counts(p.spans, L, p.sink_len, p.sink_offsets, p.img_bidir)
    for c in range(4):
        assert tm.stats(c)["allowed_pairs"] == want[c], (p.name, c)
    tm.pair_plan(p.gqa_group)   # validates every work unit against the per-class lists
    return tm


def packed_sample_tiles(tm, p, n_random, seed):
    """Query tiles of a packed map worth checking: the ends of the image group and of the text group, tiles
    around the start / end of a few images (in the image group rows are image tokens in position order), random."""
    rng = np.random.default_rng([17, seed])
    n_img = int(sum(e - s for s, e, _ in p.spans))
    m_img = -(-n_img // 128)
    picks = {0, m_img - 1, m_img, tm.n_q_tiles - 1}
    lens = np.cumsum([0] + [int(e - s) for s, e, _ in p.spans])
    for g in rng.choice(len(p.spans), size=min(3, len(p.spans)), replace=False):
        picks.update({int(lens[g]) // 128, max(0, int(lens[g + 1]) - 1) // 128})
    picks.update(int(t) for t in rng.integers(0, tm.n_q_tiles, size=n_random))
    return sorted(picks)


@pytest.mark.parametrize("cfg,target", [(2, None), (3, None), (4, None), (6, None), (5, 36864), (5, 153600), (5, 307200)])
def test_packed_large_configs_states_and_pair_counts(cfg, target):
    p = W.config(cfg, target_len=target)
    probe = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len, flags=bs.BS_MAP_PACK_KEYS | model_flags(p.img_bidir),
                                sink_offsets=p.sink_offsets or None)
    check_packed_sampled(p, packed_sample_tiles(probe, p, n_random=2, seed=cfg))


@pytest.mark.parametrize("cfg,target", [(3, None), (4, None), (6, None), (5, 153600), (5, 307200)])
def test_natural_map_pair_counts_long_configs(cfg, target):
    """allowed_pairs of the long prompts, where enumeration is out of reach: against the test-side closed form
    (itself pinned to the oracle's enumeration on small prompts)."""
    from test_oracle_pins import closed_form_pair_counts
    p = W.config(cfg, target_len=target)
    tm = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len, flags=model_flags(p.img_bidir),
                             sink_offsets=p.sink_offsets or None)
    want = closed_form_pair_counts(p.spans, p.seq_len, p.sink_len, p.sink_offsets, p.img_bidir)
    for c in range(4):
        assert tm.stats(c)["allowed_pairs"] == want[c]


@pytest.mark.parametrize("cfg", [2, 4])
def test_packed_large_configs_fewer_tiles(cfg):
    p = W.config(cfg)
    reg = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len, flags=bs.BS_MAP_REGROUP_ROWS)
    pk = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len, flags=bs.BS_MAP_PACK_KEYS)
    pk.pair_plan(p.gqa_group)
    assert pk.stats(0) == reg.stats(0) or pk.stats(0)["visited"] == reg.stats(0)["visited"]
    for c in (1, 2, 3):
        if c == 2 and not pk.layout()["intra_compact"]:
            assert pk.stats(c)["visited"] == reg.stats(c)["visited"]   # kept its plain lists
        else:
            assert pk.stats(c)["visited"] < reg.stats(c)["visited"]
        assert pk.stats(c)["allowed_pairs"] == reg.stats(c)["allowed_pairs"]


# ------------------------------------------------------------------------- work units (KV-sharing pairs)

@pytest.mark.parametrize("seed", range(12))
def test_pair_plan_random_prompts(seed):
    rng = np.random.default_rng(100 + seed)
    runs = [("T", int(rng.integers(0, 200)))]
    for _ in range(int(rng.integers(1, 7))):
        runs += [("I", int(rng.integers(1, 900))), ("T", int(rng.integers(0, 70)))]
    G = [1, 2, 3, 7][seed % 4]
    n_kv = [1, 2, 3][seed % 3]
    hc = rng.integers(0, 4, size=G * n_kv).astype(np.uint8)
    L, spans = W.layout_from_runs(runs, "paper10")
    if L == 0:
        return
    tm = bs.bs_build_tilemap(spans, L, hc, int(rng.integers(0, min(L, 40) + 1)))
    plan = tm.pair_plan(G)          # BS_OK only if the plan reproduces every item's tile states
    per_class = [tm.stats(c) for c in range(4)]
    item_tiles = sum(per_class[int(c)]["visited"] for c in hc)
    n_items = len(hc) * tm.n_q_tiles
    assert n_items / 2 <= plan["n_units"] <= n_items
    # every item's tiles are covered; a unit step serves one or two items
    assert plan["unit_tiles"] * 2 - plan["skip_steps"] - (2 * plan["n_units"] - n_items) * 0 >= item_tiles
    assert plan["unit_tiles"] <= item_tiles
    # planning again for another group size replaces the plan
    if len(hc) % 2 == 0:
        tm.pair_plan(2)
    tm.pair_plan(G)


@pytest.mark.parametrize("cfg", [1, 2, 5])
def test_pair_plan_configs(cfg):
    p = W.config(cfg)
    tm = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len)
    plan = tm.pair_plan(p.gqa_group)
    per_class = [tm.stats(c) for c in range(4)]
    item_tiles = sum(per_class[int(c)]["visited"] for c in p.head_class)
    assert item_tiles / 2 <= plan["unit_tiles"] <= item_tiles
    with pytest.raises(bs.BlindsightError):
        tm.pair_plan(5 if p.n_q_heads % 5 else 0)


# ------------------------------------------------------------------------- one map per prompt, one class vector per layer

def test_rebind_keeps_the_lists_and_replans_the_units():
    p = W.config(2)
    tm = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len, flags=bs.BS_MAP_PACK_KEYS)
    before = [(tm.stats(c), tm.tile_states(c, 50, 8)) for c in range(4)]
    plan_a = tm.pair_plan(p.gqa_group)
    rng = np.random.default_rng(3)
    for _ in range(3):
        hc = rng.integers(0, 4, size=p.n_q_heads).astype(np.uint8)
        tm.rebind(hc)
        fresh = bs.bs_build_tilemap(p.spans, p.seq_len, hc, p.sink_len, flags=bs.BS_MAP_PACK_KEYS)
        assert tm.pair_plan(p.gqa_group) == fresh.pair_plan(p.gqa_group)    # validated unit by unit inside the call
        for c in range(4):
            assert tm.stats(c) == before[c][0] and np.array_equal(tm.tile_states(c, 50, 8), before[c][1])
    tm.rebind(p.head_class)
    assert tm.pair_plan(p.gqa_group) == plan_a
    # another head count (same prompt, a layer with fewer heads)
    tm.rebind(np.array([0, 1, 2, 3, 3, 2, 1, 0], dtype=np.uint8))
    assert tm.n_q_heads == 8
    assert tm.pair_plan(2)["n_units"] == 4 * tm.n_q_tiles
    with pytest.raises(bs.BlindsightError):
        tm.rebind(np.array([0, 4], dtype=np.uint8))
    with pytest.raises(bs.BlindsightError):
        tm.rebind(np.zeros(0, dtype=np.uint8))
    assert tm.n_q_heads == 8


# ------------------------------------------------------------------------- error behaviour

def _raw_build(spans, n_spans, L, hc, nh, sink_len, bm, bn, out):
    return binding.load_library().bs_build_tilemap(spans, n_spans, L, hc, nh, sink_len, bm, bn, out)


def test_build_rejects_bad_arguments():
    lib = binding.load_library()
    hc = (ctypes.c_uint8 * 2)(0, 3)
    sp = (binding._Span * 2)(binding._Span(0, 4, 1), binding._Span(6, 9, 0))
    out = ctypes.c_void_p()
    ok = lambda: _raw_build(sp, 2, 16, hc, 2, 0, 128, 64, ctypes.byref(out))
    assert ok() == 0
    lib.bs_tilemap_destroy(out)
    out = ctypes.c_void_p()
    EINVAL = -1
    assert _raw_build(sp, 2, 16, hc, 2, 0, 128, 64, None) == EINVAL
    assert _raw_build(None, 2, 16, hc, 2, 0, 128, 64, ctypes.byref(out)) == EINVAL
    assert _raw_build(sp, 2, 16, None, 2, 0, 128, 64, ctypes.byref(out)) == EINVAL
    assert _raw_build(sp, 2, 0, hc, 2, 0, 128, 64, ctypes.byref(out)) == EINVAL
    assert _raw_build(sp, 2, 8, hc, 2, 0, 128, 64, ctypes.byref(out)) == EINVAL      # span beyond L
    assert _raw_build(sp, 2, 16, hc, 2, 17, 128, 64, ctypes.byref(out)) == EINVAL    # sink_len > L
    assert _raw_build(sp, 2, 16, hc, 2, -1, 128, 64, ctypes.byref(out)) == EINVAL
    assert _raw_build(sp, 2, 16, hc, 2, 0, 0, 64, ctypes.byref(out)) == EINVAL
    assert _raw_build(sp, 2, 16, hc, 0, 0, 128, 64, ctypes.byref(out)) == EINVAL
    bad_cls = (ctypes.c_uint8 * 2)(0, 4)
    assert _raw_build(sp, 2, 16, bad_cls, 2, 0, 128, 64, ctypes.byref(out)) == EINVAL
    for a, b in [((4, 4, 0), (6, 9, 0)), ((0, 7, 0), (6, 9, 0)), ((6, 9, 0), (0, 4, 0)),
                 ((0, 4, 5), (6, 9, 0)), ((0, 4, -1), (6, 9, 0))]:
        bad = (binding._Span * 2)(binding._Span(*a), binding._Span(*b))
        assert _raw_build(bad, 2, 16, hc, 2, 0, 128, 64, ctypes.byref(out)) == EINVAL
    assert out.value is None     # untouched on failure
    with pytest.raises(bs.BlindsightError):
        bs.bs_build_tilemap([(0, 99, 0)], 16, [0])


def test_introspection_rejects_bad_arguments():
    lib = binding.load_library()
    tm = bs.bs_build_tilemap([(2, 9, 1)], 300, [0, 1])
    buf = (ctypes.c_uint8 * (tm.n_q_tiles * tm.n_k_tiles))()
    assert lib.bs_tilemap_tile_states(tm.handle, 4, 0, 1, buf) == -1
    assert lib.bs_tilemap_tile_states(tm.handle, 0, 0, tm.n_q_tiles + 1, buf) == -1
    assert lib.bs_tilemap_tile_states(tm.handle, 0, -1, 1, buf) == -1
    assert lib.bs_tilemap_tile_states(tm.handle, 0, 0, 1, None) == -1
    assert lib.bs_tilemap_stats(None, 0, None, None, None, None, None, None) == -1
    assert lib.bs_tilemap_stats(tm.handle, 7, None, None, None, None, None, None) == -1
    assert lib.bs_tilemap_stats(tm.handle, 0, None, None, None, None, None, None) == 0
    assert lib.bs_tilemap_dims(None, None, None, None, None) == -1
    lib.bs_tilemap_destroy(None)
    for code in (0, -1, -2, -3, -4, -99):
        assert isinstance(lib.bs_strerror(code), bytes) and lib.bs_strerror(code)


def test_attn_prefill_argument_checks_need_no_gpu():
    """Argument validation happens before any HIP call."""
    lib = binding.load_library()
    tm = bs.bs_build_tilemap([(2, 9, 1)], 300, [0, 1])
    small = bs.bs_build_tilemap([(2, 9, 1)], 300, [0, 1], 0, 64, 64)
    one = ctypes.c_void_p(256)
    f = lambda *a: lib.bs_attn_prefill(*a)
    assert f(None, one, one, one, tm.handle, 0, 2, 2, 128, 0.1, None) == -1
    assert f(one, one, one, one, None, 0, 2, 2, 128, 0.1, None) == -1
    assert f(one, one, one, one, tm.handle, 0, 3, 2, 128, 0.1, None) == -1      # heads % group
    assert f(one, one, one, one, tm.handle, 0, 4, 2, 128, 0.1, None) == -1      # map built for 2 heads
    assert f(one, one, one, one, tm.handle, 0, 2, 2, 128, 0.0, None) == -1      # scale must be > 0
    assert f(one, one, one, one, tm.handle, 0, 2, 2, 96, 0.1, None) == -2
    assert f(one, one, one, one, tm.handle, 5, 2, 2, 128, 0.1, None) == -2
    assert f(one, one, one, one, small.handle, 0, 2, 2, 128, 0.1, None) == -2   # 64x64 map
    assert f(ctypes.c_void_p(260), one, one, one, tm.handle, 0, 2, 2, 128, 0.1, None) == -1  # alignment


def test_static_entry_point_rejects_an_unprepared_map_without_touching_the_gpu():
    lib = binding.load_library()
    tm = bs.bs_build_tilemap([(2, 9, 1)], 300, [0, 1])
    one = ctypes.c_void_p(256)
    assert lib.bs_attn_prefill_static(one, one, one, one, tm.handle, 2, 2, 128, 0.1, None) == -1
    assert b"bs_tilemap_prepare" in lib.bs_last_error()
    assert lib.bs_attn_prefill_static(None, one, one, one, tm.handle, 2, 2, 128, 0.1, None) == -1
    assert lib.bs_attn_prefill_static(one, one, one, one, tm.handle, 2, 2, 96, 0.1, None) == -2
    assert lib.bs_static_scratch_bytes() == 96 << 20


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "blindsight.h")).read()
    declared = set(re.findall(r"\b(bs_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    lib = ctypes.CDLL(bs.library_path())
    for name in declared:
        assert getattr(lib, name) is not None
