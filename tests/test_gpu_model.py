"""GPU parity of the model variant with non-causal attention inside an image and sinks at fixed
in-image offsets (paper Sec. 6.1, App. "Attention Sink Positions in Gemma 3") against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2507_09071_amd as bs
import workloads as W
from oracle import characterize as C
from dataclasses import replace

from gpu_util import assert_close, oracle_rows
from test_gpu_parity import RUNS_A, full_parity, sampled_parity

pytestmark = pytest.mark.gpu
D, S, I, IS = 0, 1, 2, 3
DEV = "cuda:0"
OFFSETS = (0, 3, 64, 65, 129, 299, 400)


@pytest.mark.parametrize("dtype,d,flags", [("f32", 64, 0), ("f32", 128, bs.BS_MAP_REGROUP_ROWS), ("f32", 64, bs.BS_MAP_PACK_KEYS), ("bf16", 128, 0),
                                           ("bf16", 64, bs.BS_MAP_REGROUP_ROWS), ("bf16", 128, bs.BS_MAP_PACK_KEYS),
                                           ("bf16", 64, bs.BS_MAP_PACK_KEYS)])
def test_bidirectional_small_prompt_all_classes(dtype, d, flags):
    p = W.custom_prompt(RUNS_A, [D, S, I, IS, IS, I, S, D], 4, d, dtype=dtype, sink_len=5, span_sink=0,
                        name=f"bidir-{dtype}-d{d}-f{flags}", value_recipe={"std": 1.0, "first_key_scale": 4.0},
                        img_bidir=True, sink_offsets=OFFSETS)
    full_parity(p, seed=11, flags=flags)


@pytest.mark.parametrize("flags", [0, bs.BS_MAP_PACK_KEYS])
def test_offset_sinks_with_causal_images(flags):
    p = W.custom_prompt(RUNS_A, [S, IS, I, D], 2, 128, dtype="bf16", sink_len=0, span_sink=0,
                        name=f"offset-sinks-causal-f{flags}", sink_offsets=OFFSETS)
    full_parity(p, seed=12, flags=flags)


@pytest.mark.parametrize("flags", [0, bs.BS_MAP_PACK_KEYS])
def test_bidirectional_equal_small_images(flags):
    """Many images of one size with little text between them, image first, two adjacent images:
    the layout of the Gemma-like workload in small."""
    runs = []
    for i in range(30):
        runs += [("I", 96), ("T", 1 + (i % 4))]
        if i % 9 == 4:
            runs += [("I", 96)]
    p = W.custom_prompt(runs, [S, I, IS, D, IS, S], 3, 128, dtype="bf16", sink_len=0, span_sink=0,
                        name=f"bidir-equal-f{flags}", img_bidir=True, sink_offsets=(5, 17, 18, 70, 95))
    full_parity(p, seed=13, flags=flags)


def test_bidirectional_ragged_image_at_the_end():
    p = W.custom_prompt([("T", 10), ("I", 500), ("T", 2), ("I", 333)], [D, IS, S, I], 2, 128, dtype="bf16",
                        span_sink=0, name="bidir-tail", img_bidir=True, sink_offsets=(1, 2, 300))
    assert p.seq_len % 128 != 0
    full_parity(p, seed=14, flags=bs.BS_MAP_PACK_KEYS)
    full_parity(p, seed=14, flags=0)


def test_gemma_like_config_sampled_rows():
    p = W.gemma3_bidir_config(0)
    sampled_parity(p, 0, n_random=3, max_tiles=10, row_step=32, flags=bs.BS_MAP_PACK_KEYS)


def test_characterisation_with_bidirectional_images():
    kinds = ["dense", "sink", "intra", "intra_sink"] * 2
    runs = [("T", 40), ("I", 256), ("T", 12), ("I", 256), ("T", 20), ("I", 256), ("T", 17)]
    offs = (3, 50, 51, 200)
    p = W.custom_prompt(runs, [0] * 8, 2, 64, dtype="bf16", span_sink=0, img_bidir=True, sink_offsets=offs)
    q, k, v = W.make_planted_qkv(p, kinds, seed=5, device=DEV)
    got_type, got = bs.bs_characterize_prompt(q, k, v, p.spans, p.seq_len, p.sink_len, bs.BS_BF16, 8, 4, 64, p.scale,
                                              0.1, bs.BS_MAP_PACK_KEYS | bs.BS_MAP_BIDIR_IMAGES,
                                              torch.cuda.current_stream().cuda_stream, sink_offsets=offs)
    imgid, issink = oracle.token_arrays(p.spans, p.seq_len, p.sink_len, offs)
    f = lambda t: t.float().cpu().numpy()
    _, want = C.characterize_prompt(f(q), f(k), f(v), imgid, issink, p.scale, 0.0, True)
    want_type, _ = C.characterize_prompt(f(q), f(k), f(v), imgid, issink, p.scale, 0.1, True)
    tol = 5e-3 * (2 + 2 * np.sqrt(want)) / (1 - 5e-3)
    assert (np.abs(np.sqrt(got) - np.sqrt(want)) <= tol).all(), (got, want)
    clear = np.abs(np.sqrt(want) - np.sqrt(0.1)) > tol
    for h in range(8):
        if clear[:, h].all():
            assert got_type[h] == want_type[h], (h, got[:, h], want[:, h])
    assert clear.all(axis=0).sum() >= 6


# --- sliding-window layers

@pytest.mark.parametrize("dtype,d,flags,window", [("f32", 64, 0, 100), ("bf16", 128, 0, 100), ("bf16", 64, bs.BS_MAP_REGROUP_ROWS, 37),
                                                  ("bf16", 128, bs.BS_MAP_PACK_KEYS, 200), ("bf16", 128, 0, 1),
                                                  ("f32", 128, bs.BS_MAP_REGROUP_ROWS, 64)])
def test_window_small_prompt_all_classes(dtype, d, flags, window):
    p = W.custom_prompt(RUNS_A, [D, S, I, IS, IS, I, S, D], 4, d, dtype=dtype, sink_len=5,
                        name=f"window{window}-{dtype}-d{d}-f{flags}", value_recipe={"std": 1.0, "first_key_scale": 4.0},
                        window=window)
    full_parity(p, seed=21, flags=flags)


def test_window_with_bidirectional_images():
    runs = []
    for i in range(24):
        runs += [("I", 96), ("T", 1 + (i % 4))]
    for window in (96, 250):
        p = W.custom_prompt(runs, [S, I, IS, D, IS, S], 3, 128, dtype="bf16", sink_len=0, span_sink=0,
                            name=f"bidir-window{window}", img_bidir=True, sink_offsets=(5, 17, 18, 70, 95), window=window)
        full_parity(p, seed=22, flags=bs.BS_MAP_REGROUP_ROWS)


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("f32", 64)])
def test_window_shorter_than_bidirectional_images(dtype, d):
    """The query's own image stays visible beyond the window (the model's dense mask keeps it): images of 300
    and 700 tokens against windows of 64, 150 and 400."""
    runs = [("T", 20), ("I", 300), ("T", 9), ("I", 700), ("I", 120), ("T", 30), ("I", 300), ("T", 11)]
    for window in (64, 150, 400):
        p = W.custom_prompt(runs, [S, I, IS, D, IS, S, I, D], 4, d, dtype=dtype, sink_len=3, span_sink=0,
                            name=f"bidir-long-window{window}-{dtype}-d{d}", value_recipe={"std": 1.0, "first_key_scale": 3.0},
                            img_bidir=True, sink_offsets=(0, 5, 64, 130, 299, 650), window=window)
        full_parity(p, seed=23, flags=bs.BS_MAP_REGROUP_ROWS)


def test_window_1024_on_the_gemma_like_config_sampled_rows():
    p = replace(W.gemma3_bidir_config(0), window=1024, name="cfg6-window1024")
    sampled_parity(p, 0, n_random=3, max_tiles=10, row_step=8, flags=bs.BS_MAP_REGROUP_ROWS)


def test_window_4096_on_config2_sampled_rows():
    p = replace(W.config(2), window=4096, name="cfg2-window4096")
    sampled_parity(p, 0, n_random=3, max_tiles=10, row_step=4, flags=bs.BS_MAP_PACK_KEYS)


# --- every option combined, random small prompts

@pytest.mark.parametrize("seed", range(16))
def test_random_prompts_random_options(seed):
    rng = np.random.default_rng(9100 + seed)
    runs = [("T", int(rng.integers(0, 50)))]
    size = int(rng.integers(40, 400))
    equal = bool(rng.integers(0, 2))
    for _ in range(int(rng.integers(1, 7))):
        runs.append(("I", size if equal else int(rng.integers(20, 500))))
        if rng.random() < 0.85:
            runs.append(("T", int(rng.integers(1, 40))))
    if sum(n for _, n in runs) == 0:
        runs = [("T", 5)]
    dtype = ["bf16", "bf16", "f32"][seed % 3]
    d = [128, 64][(seed // 3) % 2]
    n_kv = int(rng.integers(1, 3))
    G = int(rng.integers(1, 4))
    classes = rng.integers(0, 4, size=n_kv * G)
    bidir = bool(rng.integers(0, 2))
    longest = max(n for kind, n in runs if kind == "I")
    window = [0, 0, int(rng.integers(longest, longest + 300)), int(rng.integers(1, 200))][int(rng.integers(0, 4))]
    offsets = tuple(sorted(set(int(o) for o in rng.integers(0, 300, size=int(rng.integers(0, 8))))))
    flags = [0, bs.BS_MAP_REGROUP_ROWS, bs.BS_MAP_PACK_KEYS][int(rng.integers(0, 3))]
    p = W.custom_prompt(runs, classes, n_kv, d, dtype=dtype, sink_len=int(rng.integers(0, 8)),
                        sink_mode=["paper10", "prefix"][int(rng.integers(0, 2))], span_sink=[None, 0, 7][int(rng.integers(0, 3))],
                        name=f"rand{seed}-{dtype}-d{d}-f{flags}-w{window}-b{int(bidir)}",
                        value_recipe={"std": 1.0, "first_key_scale": 3.0}, img_bidir=bidir, sink_offsets=offsets, window=window)
    full_parity(p, seed=seed, flags=flags)


# --- a chunk of queries at the end of the prompt (chunked prefill, decoding): same masks, rows q_begin .. L - 1

def suffix_parity(p, q_begin, seed, flags, row_step=1):
    q, k, v = W.make_qkv(p, seed, DEV)
    f = flags | (bs.BS_MAP_BIDIR_IMAGES if p.img_bidir else 0)
    tm = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len, 128, 64, flags=f,
                             sink_offsets=p.sink_offsets or None, window=p.window, q_begin=q_begin)
    qs = q[:, q_begin:].contiguous()
    out = torch.full_like(qs, float("nan"))
    dt = bs.BS_BF16 if p.dtype == "bf16" else bs.BS_F32
    print(p.name, "L", p.seq_len, "q_begin", q_begin, flush=True)
    bs.bs_attn_prefill(qs, k, v, out, tm, dt, p.n_q_heads, p.gqa_group, p.head_dim, p.scale,
                       torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([np.arange(q_begin, p.seq_len, row_step), [p.seq_len - 1]])).astype(np.int32)
    want = oracle_rows(p, q.float().cpu().numpy(), k.float().cpu().numpy(), v.float().cpu().numpy(), rows)
    got = out[:, torch.from_numpy(rows - q_begin).long().to(out.device)].float().cpu().numpy()
    for h in range(p.n_q_heads):
        assert_close(got[h], want[h], p.dtype, f"{p.name} q_begin {q_begin} head {h} class {p.head_class[h]}")


@pytest.mark.parametrize("dtype,d,flags", [("bf16", 128, 0), ("bf16", 64, bs.BS_MAP_REGROUP_ROWS), ("bf16", 128, bs.BS_MAP_PACK_KEYS),
                                           ("f32", 64, bs.BS_MAP_PACK_KEYS), ("f32", 128, 0)])
def test_suffix_queries_small_prompt(dtype, d, flags):
    p = W.custom_prompt(RUNS_A, [D, S, I, IS, IS, I, S, D], 4, d, dtype=dtype, sink_len=5,
                        name=f"suffix-{dtype}-d{d}-f{flags}", value_recipe={"std": 1.0, "first_key_scale": 4.0})
    for q_begin in (p.seq_len - 1, p.seq_len - 130, 400, 37):   # one decode row; inside the last text run; inside images
        suffix_parity(p, q_begin, 31, flags)


def test_suffix_queries_with_model_options():
    runs = [("T", 20), ("I", 300), ("T", 9), ("I", 700), ("I", 120), ("T", 30), ("I", 300), ("T", 11)]
    p = W.custom_prompt(runs, [S, I, IS, D, IS, S, I, D], 4, 128, dtype="bf16", sink_len=3, span_sink=0, name="suffix-bidir-window",
                        value_recipe={"std": 1.0, "first_key_scale": 3.0}, img_bidir=True, sink_offsets=(0, 5, 64, 130, 299, 650),
                        window=150)
    for q_begin in (p.seq_len - 1, 1200, 333):
        suffix_parity(p, q_begin, 32, bs.BS_MAP_REGROUP_ROWS)
    suffix_parity(replace(p, window=0), 777, 33, bs.BS_MAP_PACK_KEYS)


@pytest.mark.parametrize("chunk", [1, 2048])
def test_suffix_queries_config2(chunk):
    p = W.config(2)
    suffix_parity(p, p.seq_len - chunk, 0, bs.BS_MAP_PACK_KEYS, row_step=16)
