"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, element by element.
Tolerances: bf16 inputs max-abs 2e-2 and relative-L2 5e-3; fp32 configuration 1e-5."""
import numpy as np
import pytest
import torch

import paper_2507_09071_amd as bs
import workloads as W
from gpu_util import assert_close, errors, oracle_rows, rows_of_tiles, run_prefill
from test_oracle_pins import uniform_attention_closed_form, uniform_attention_closed_form_heads

pytestmark = pytest.mark.gpu
D, S, I, IS = 0, 1, 2, 3
DEV = "cuda:0"


def full_parity(p, seed=0, what=None, flags=0):
    q, k, v = W.make_qkv(p, seed, DEV)
    out, tm = run_prefill(p, q, k, v, flags=flags)
    want = oracle_rows(p, q, k, v)
    print(what or p.name, "L", p.seq_len, flush=True)
    res = []
    for h in range(p.n_q_heads):
        res.append(assert_close(out[h].float().cpu().numpy(), want[h], p.dtype, f"{p.name} head {h} class {p.head_class[h]}"))
    return res


@pytest.mark.parametrize("mode,span_sink", [("prefix", None), ("paper10", None), ("prefix", 32)])
def test_config1_tiny_fp32(mode, span_sink):
    p = W.tiny_config(mode, span_sink)
    full_parity(p)
    full_parity(p.with_classes([S, I]), seed=1)


RUNS_A = [("T", 37), ("I", 300), ("T", 5), ("I", 451), ("T", 9), ("I", 130), ("I", 77), ("T", 61)]


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 128), ("f32", 64)])
def test_small_prompt_all_classes_sharp_values(dtype, d):
    # q, k ~ N(0,1): logits of order 1..4 sigma, so the running max really moves
    p = W.custom_prompt(RUNS_A, [D, S, I, IS, IS, I, S, D], 4, d, dtype=dtype, sink_len=5,
                        name=f"small-{dtype}-d{d}", value_recipe={"std": 1.0, "first_key_scale": 4.0})
    full_parity(p, seed=3)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_small_prompt_config_like_values(dtype):
    p = W.custom_prompt(RUNS_A, [IS, D, S, I], 2, 128, dtype=dtype, sink_len=37, sink_mode="paper10",
                        value_recipe={"std": 1.0 / np.sqrt(128), "outlier_frac": 0.02, "outlier_scale": 6.0})
    full_parity(p, seed=4)


@pytest.mark.parametrize("L", [1, 31, 64, 127, 128, 129, 192, 256, 1000])
def test_ragged_lengths(L):
    n_img = max(1, L // 3)
    runs = [("T", (L - n_img) // 2), ("I", n_img), ("T", L - n_img - (L - n_img) // 2)]
    p = W.custom_prompt(runs, [D, S, I, IS], 2, 128, dtype="bf16", sink_len=0, name=f"ragged{L}")
    assert p.seq_len == L
    full_parity(p, seed=L)
    p32 = W.custom_prompt(runs, [IS, D], 1, 64, dtype="f32", sink_len=1, name=f"ragged{L}-f32")
    full_parity(p32, seed=L)


def test_text_only_and_image_only():
    full_parity(W.custom_prompt([("T", 333)], [D, S, I, IS], 4, 128, name="text-only"))
    full_parity(W.custom_prompt([("I", 333)], [D, S, I, IS], 1, 128, name="image-only"))
    full_parity(W.custom_prompt([("I", 333)], [D, S, I, IS], 1, 128, sink_mode="prefix", sink_len=0,
                                name="image-only-nosink"))


def test_empty_rows_give_zeros():
    # image first, no sink anywhere: Sink-head image rows of the first image have no allowed key
    p = W.custom_prompt([("I", 200), ("T", 10), ("I", 150)], [S, IS], 1, 128, sink_mode="prefix",
                        name="empty-rows")
    q, k, v = W.make_qkv(p, 0, DEV)
    out, tm = run_prefill(p, q, k, v)
    assert tm.stats(S)["empty_rows"] == 200
    assert torch.all(out[0, :200] == 0)
    want = oracle_rows(p, q, k, v)
    for h in range(2):
        assert_close(out[h].float().cpu().numpy(), want[h], "bf16", f"head {h}")


def test_many_small_images():
    rng = np.random.default_rng(5)
    runs = [("T", 3)]
    for _ in range(40):
        runs += [("I", int(rng.integers(1, 90))), ("T", int(rng.integers(0, 6)))]
    p = W.custom_prompt(runs, [S, I, IS, D, I, IS], 3, 128, sink_len=2, name="many-small")
    full_parity(p, seed=6)


def test_rows_sum_to_one_and_uniform_closed_form_config2():
    """Properties that hold at any size, on every row of the 36K configuration."""
    p = W.config(2)
    q, k, v = W.make_qkv(p, 0, DEV)
    out, tm = run_prefill(p, q, k, torch.ones_like(v), None)
    assert torch.all((out.float() - 1.0).abs() <= 2 ** -8), "rows do not sum to one"
    out0, _ = run_prefill(p, torch.zeros_like(q), k, v, tm)
    want = uniform_attention_closed_form(p, v.float().cpu().numpy())
    for h in range(p.n_q_heads):
        assert_close(out0[h].float().cpu().numpy(), want[h], "bf16", f"uniform head {h}")


def sampled_parity(p, seed, n_random, max_tiles, row_step, flags=0):
    q, k, v = W.make_qkv(p, seed, DEV)
    out, tm = run_prefill(p, q, k, v, flags=flags)
    tiles = W.sample_q_tiles(p, 128, n_random=n_random, seed=seed, max_tiles=max_tiles)
    rows = rows_of_tiles(p, tiles, row_step)
    print(p.name, "L", p.seq_len, "rows checked", len(rows), flush=True)
    want = oracle_rows(p, q.float().cpu().numpy(), k.float().cpu().numpy(), v.float().cpu().numpy(), rows)
    got = out[:, torch.from_numpy(rows).long().to(out.device)].float().cpu().numpy()
    worst = (0.0, 0.0)
    for h in range(p.n_q_heads):
        e = assert_close(got[h], want[h], p.dtype, f"{p.name} head {h} class {p.head_class[h]}")
        worst = (max(worst[0], e[0]), max(worst[1], e[1]))
    print("worst max_abs %.3e rel_l2 %.3e" % worst, flush=True)
    return out, tm


@pytest.mark.parametrize("sink_mode", ["paper10", "prefix"])
def test_config2_sampled_rows(sink_mode):
    sampled_parity(W.config(2, 0, sink_mode), 0, n_random=4, max_tiles=12, row_step=4)


def test_config2_all_dense_sampled_rows():
    sampled_parity(W.config(2).all_dense(), 1, n_random=2, max_tiles=6, row_step=8)


def test_config3_sampled_rows():
    sampled_parity(W.config(3), 0, n_random=2, max_tiles=8, row_step=16)


def test_config4_sampled_rows():
    sampled_parity(W.config(4), 0, n_random=2, max_tiles=8, row_step=32)


# --- regrouped query rows (BS_MAP_REGROUP_ROWS): same function of the inputs, other work items

@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 128)])
def test_regrouped_small_prompt_all_classes(dtype, d):
    p = W.custom_prompt(RUNS_A, [D, S, I, IS, IS, I, S, D], 4, d, dtype=dtype, sink_len=5,
                        name=f"regrouped-{dtype}-d{d}", value_recipe={"std": 1.0, "first_key_scale": 4.0})
    full_parity(p, seed=5, flags=bs.BS_MAP_REGROUP_ROWS)


def test_regrouped_many_small_images_and_single_text_tokens():
    runs = [("T", 3)]
    for i in range(30):
        runs += [("I", 40 + 7 * (i % 5)), ("T", 1 + (i % 3))]
    p = W.custom_prompt(runs, [S, I, IS, D], 2, 128, dtype="bf16", sink_len=2, name="regrouped-many")
    full_parity(p, seed=6, flags=bs.BS_MAP_REGROUP_ROWS)


def test_regrouped_matches_natural_order_bitwise_on_text_only():
    p = W.custom_prompt([("T", 700)], [D, S, I, IS], 2, 128, dtype="bf16")
    q, k, v = W.make_qkv(p, 7, DEV)
    a, _ = run_prefill(p, q, k, v)
    b, _ = run_prefill(p, q, k, v, flags=bs.BS_MAP_REGROUP_ROWS)
    assert torch.equal(a, b)


@pytest.mark.parametrize("cfg", [2, 4])
def test_regrouped_configs_sampled_rows(cfg):
    sampled_parity(W.config(cfg), 0, n_random=3, max_tiles=10, row_step=[0, 0, 4, 16, 32][cfg],
                   flags=bs.BS_MAP_REGROUP_ROWS)


# --- packed keys (BS_MAP_PACK_KEYS): compact tiles of text and sink keys for the sparse classes

@pytest.mark.parametrize("d", [128, 64])
def test_packed_small_prompt_all_classes(d):
    p = W.custom_prompt(RUNS_A, [D, S, I, IS, IS, I, S, D], 4, d, dtype="bf16", sink_len=5,
                        name=f"packed-d{d}", value_recipe={"std": 1.0, "first_key_scale": 4.0})
    full_parity(p, seed=8, flags=bs.BS_MAP_PACK_KEYS)


def test_packed_many_small_images():
    runs = [("T", 3)]
    for i in range(40):
        runs += [("I", 40 + 7 * (i % 5)), ("T", 1 + (i % 3))]
        if i % 7 == 3:
            runs += [("I", 33)]          # two images without text between them
    p = W.custom_prompt(runs, [S, I, IS, D, IS, S], 3, 128, dtype="bf16", sink_len=2, name="packed-many")
    full_parity(p, seed=9, flags=bs.BS_MAP_PACK_KEYS)


def test_packed_long_images_prefix_sinks():
    p = W.custom_prompt([("T", 70), ("I", 900), ("T", 3), ("I", 1300), ("T", 40)], [IS, S, I, D], 2, 128,
                        dtype="bf16", sink_len=37, sink_mode="prefix", name="packed-long")
    full_parity(p, seed=10, flags=bs.BS_MAP_PACK_KEYS)


@pytest.mark.parametrize("d", [64, 128])
def test_packed_fp32(d):
    p = W.custom_prompt(RUNS_A, [D, S, I, IS, I, IS], 2, d, dtype="f32", sink_len=5, name=f"packed-f32-d{d}",
                        value_recipe={"std": 1.0, "first_key_scale": 4.0})
    full_parity(p, seed=1, flags=bs.BS_MAP_PACK_KEYS)


@pytest.mark.parametrize("cfg", [2, 4])
def test_packed_configs_sampled_rows(cfg):
    sampled_parity(W.config(cfg), 0, n_random=3, max_tiles=10, row_step=[0, 0, 4, 16, 32][cfg],
                   flags=bs.BS_MAP_PACK_KEYS)


# --- the layout the bench times (packed keys) on the long prompts: sampled rows against the oracle, and the
# --- two properties that hold at any size on EVERY row

@pytest.mark.parametrize("cfg,target,row_step", [(3, None, 16), (5, 36864, 8), (5, 73728, 16), (5, 153600, 16),
                                                  (5, 307200, 32), (6, None, 32)])
def test_packed_long_configs_sampled_rows(cfg, target, row_step):
    sampled_parity(W.config(cfg, target_len=target), 0, n_random=2, max_tiles=8, row_step=row_step,
                   flags=bs.BS_MAP_PACK_KEYS)


def all_rows_closed_forms(p, flags, seed=0, channel_step=1):
    """V = 1 gives 1 on every row with a visible key (the weights of a row sum to one), and q = 0 gives the
    mean of V over the row's allowed set, which a closed form from prefix sums states for every row in
    O(L d): the mask of every row of every head, at any prompt length.  channel_step > 1 compares every
    channel_step-th channel only (a wrong allowed set shows in every channel; the host side of this test is
    a few fp64 passes over [L, d] per head)."""
    q, k, v = W.make_qkv(p, seed, DEV)
    ones = torch.ones_like(v)
    out, tm = run_prefill(p, q, k, ones, flags=flags)
    empty = sum(tm.stats(int(c))["empty_rows"] for c in p.head_class)
    assert int((out == 0).all(dim=-1).sum()) == empty               # rows without a visible key give zeros
    nonzero = out.float()[(out != 0).any(dim=-1)]
    assert torch.all((nonzero - 1.0).abs() <= 2 ** -8), "rows do not sum to one"
    del out, ones, nonzero
    q.zero_()
    out0, _ = run_prefill(p, q, k, v, tm)
    vn = v[..., ::channel_step].float().cpu().numpy()
    worst = (0.0, 0.0)
    for h, want in uniform_attention_closed_form_heads(p, vn):
        e = assert_close(out0[h][:, ::channel_step].float().cpu().numpy(), want, "bf16", f"{p.name} uniform head {h} class {p.head_class[h]}")
        worst = (max(worst[0], e[0]), max(worst[1], e[1]))
    print(p.name, "all rows: worst max_abs %.3e rel_l2 %.3e" % worst, flush=True)


@pytest.mark.parametrize("cfg,target", [(2, None), (3, None), (4, None), (5, 307200), (6, None)])
def test_packed_all_rows_sum_to_one_and_uniform_closed_form(cfg, target):
    all_rows_closed_forms(W.config(cfg, target_len=target), bs.BS_MAP_PACK_KEYS, channel_step=1 if cfg == 2 else 4)


def test_natural_map_all_rows_closed_forms_300k():
    all_rows_closed_forms(W.config(5, target_len=307200), 0, channel_step=4)


def test_config5_stress_72k_sampled_rows():
    sampled_parity(W.config(5, target_len=W.STRESS_LENGTHS[1]), 0, n_random=2, max_tiles=8, row_step=16)


def test_determinism_and_tilemap_reuse():
    p = W.config(2)
    q, k, v = W.make_qkv(p, 2, DEV)
    a, tm = run_prefill(p, q, k, v)
    b, _ = run_prefill(p, q, k, v, tm)
    assert torch.equal(a, b)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        c, _ = run_prefill(p, q, k, v, tm, s.cuda_stream)
    assert torch.equal(a, c)


def test_map_recycling_without_synchronisation():
    """A serving loop: one map per prompt, destroyed right after its launch was queued, no
    device synchronisation in between.  The library recycles the device blocks of destroyed
    maps; every result must still match the oracle (sizes go down and up again, and the
    second half runs on another stream)."""
    lengths = [900, 300, 1500, 128, 700, 1500]
    prompts = [W.custom_prompt([("T", 16)] + [("I", max(32, L // 4)), ("T", 8)] * 3 + [("T", L // 8)],
                               [D, S, I, IS], n_kv_heads=2, head_dim=128, dtype="bf16", sink_len=7)
               for L in lengths]
    data = [W.make_qkv(p, 10 + i, DEV) for i, p in enumerate(prompts)]
    outs = [torch.full_like(q, float("nan")) for q, _, _ in data]
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    for i, (p, (q, k, v)) in enumerate(zip(prompts, data)):
        st = torch.cuda.current_stream() if i < 3 else side
        tm = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len, 128, 64)
        bs.bs_attn_prefill(q, k, v, outs[i], tm, bs.BS_BF16, p.n_q_heads, p.gqa_group, p.head_dim, p.scale,
                           st.cuda_stream)
        tm.close()   # destroyed while its kernels may still be queued or running
    torch.cuda.synchronize()
    for i, (p, (q, k, v)) in enumerate(zip(prompts, data)):
        want = oracle_rows(p, q, k, v)
        for h in range(p.n_q_heads):
            assert_close(outs[i][h].float().cpu().numpy(), want[h], "bf16", f"prompt {i} head {h}")


def test_one_map_per_prompt_rebound_per_layer_without_synchronisation():
    """A model's prefill: ONE tile map of the prompt, bound to each layer's class vector in turn, the
    launches queued back to back on one stream (the re-planned work units of layer l + 1 are uploaded
    while layer l's kernels still run).  Every layer's output against the oracle; both dtypes."""
    rng = np.random.default_rng(11)
    for dtype, d, tol in (("bf16", 128, "bf16"), ("f32", 64, "f32")):
        base = W.custom_prompt([("T", 33), ("I", 420), ("T", 6), ("I", 515), ("I", 90), ("T", 40)], [D, S, I, IS, IS, I], 3, d,
                               dtype=dtype, sink_len=33, name=f"layers-{dtype}")
        layers = [base.head_class] + [rng.integers(0, 4, size=base.n_q_heads).astype(np.uint8) for _ in range(3)]
        layers.append(np.zeros(base.n_q_heads, np.uint8))
        q, k, v = W.make_qkv(base, 12, DEV)
        tm = bs.bs_build_tilemap(base.spans, base.seq_len, layers[0], base.sink_len, 128, 64, flags=bs.BS_MAP_PACK_KEYS)
        outs = [torch.full_like(q, float("nan")) for _ in layers]
        st = torch.cuda.current_stream().cuda_stream
        dt = bs.BS_BF16 if dtype == "bf16" else bs.BS_F32
        for hc, o in zip(layers, outs):
            tm.rebind(hc)
            bs.bs_attn_prefill(q, k, v, o, tm, dt, base.n_q_heads, base.gqa_group, base.head_dim, base.scale, st)
        torch.cuda.synchronize()
        for li, (hc, o) in enumerate(zip(layers, outs)):
            want = oracle_rows(base.with_classes(hc), q, k, v)
            for h in range(base.n_q_heads):
                assert_close(o[h].float().cpu().numpy(), want[h], tol, f"{dtype} layer {li} head {h} class {hc[h]}")


def test_two_streams_one_map_and_two_maps_side_by_side():
    """Streams of equal priority.  (1) One map used alternately on two streams, re-bound in between: the
    library orders every use behind the previous one, so each call must give what the same binding gives
    on one stream.  (2) Two prompts with a map each, queued on two streams at the same time: their kernels
    may overlap on the device and share nothing but the library's block cache."""
    p = W.config(2)
    q, k, v = W.make_qkv(p, 5, DEV)
    rolled = np.roll(p.head_class, 3)
    ref_a, tm = run_prefill(p, q, k, v, flags=bs.BS_MAP_PACK_KEYS)
    tm.rebind(rolled)
    ref_b, _ = run_prefill(p.with_classes(rolled), q, k, v, tm)
    assert not torch.equal(ref_a, ref_b)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    outs = [torch.full_like(q, float("nan")) for _ in range(6)]
    torch.cuda.synchronize()
    for i, o in enumerate(outs):
        st = (s1, s2)[i % 2]
        tm.rebind(p.head_class if i % 3 == 0 else rolled)
        bs.bs_attn_prefill(q, k, v, o, tm, bs.BS_BF16, p.n_q_heads, p.gqa_group, p.head_dim, p.scale, st.cuda_stream)
    torch.cuda.synchronize()
    for i, o in enumerate(outs):
        assert torch.equal(o, ref_a if i % 3 == 0 else ref_b), f"call {i}"

    p2 = W.config(5, target_len=W.STRESS_LENGTHS[0])
    q2, k2, v2 = W.make_qkv(p2, 6, DEV)
    ref_2, tm2 = run_prefill(p2, q2, k2, v2, flags=bs.BS_MAP_PACK_KEYS)
    tm.rebind(p.head_class)
    o1 = [torch.full_like(q, float("nan")) for _ in range(3)]
    o2 = [torch.full_like(q2, float("nan")) for _ in range(3)]
    torch.cuda.synchronize()
    for a, b in zip(o1, o2):
        bs.bs_attn_prefill(q, k, v, a, tm, bs.BS_BF16, p.n_q_heads, p.gqa_group, p.head_dim, p.scale, s1.cuda_stream)
        bs.bs_attn_prefill(q2, k2, v2, b, tm2, bs.BS_BF16, p2.n_q_heads, p2.gqa_group, p2.head_dim, p2.scale,
                           s2.cuda_stream)
    torch.cuda.synchronize()
    for a, b in zip(o1, o2):
        assert torch.equal(a, ref_a) and torch.equal(b, ref_2)


@pytest.mark.parametrize("rise", [0.02, 0.35, 4.0, -0.35])
def test_scores_that_drift_along_the_keys(rise):
    """Scores that rise (or fall) steadily with the key position, on top of the usual noise: `rise` is
    the step per key in the exp2 domain, i.e. 1.3, 22 and 256 per key tile.  The kernel's softmax first
    tries a tile against the reference point the row already has and only looks for the tile maximum
    when a row sum passes its limit or overflows: the small rise stays on that path, the middle one
    passes the limit on every tile, the large one overflows fp32 within a tile (the general path must
    take over and rescale), the falling one underflows against a reference set by the first tile.
    All classes, both map layouts."""
    d = 128
    p = W.custom_prompt([("T", 40), ("I", 700), ("T", 9), ("I", 900), ("T", 30), ("I", 260), ("T", 77)],
                        [D, S, I, IS, D, IS], n_kv_heads=2, head_dim=d, dtype="bf16", sink_len=16,
                        name=f"drift{rise}", value_recipe={"std": 1.0})
    q, k, v = W.make_qkv(p, 21, DEV)
    # channel 0 carries the drift: q[.., 0] = 8, k[j, 0] = j * step, so that scale * log2(e) * 8 * step = rise
    step = rise / (8.0 * p.scale * 1.4426950408889634)
    q[:, :, 0] = 8.0
    k[:, :, 0] = (torch.arange(p.seq_len, device=DEV, dtype=torch.float32) * step).to(k.dtype)[None, :]
    for flags in (0, bs.BS_MAP_PACK_KEYS):
        out, _ = run_prefill(p, q, k, v, flags=flags)
        want = oracle_rows(p, q, k, v)
        for h in range(p.n_q_heads):
            assert_close(out[h].float().cpu().numpy(), want[h], "bf16", f"rise {rise} flags {flags} head {h} class {p.head_class[h]}")
