"""Seeded synthetic prompt layouts and Q/K/V tensors for the sparse prefill-attention path.

This module is shared by the CPU oracle's tests and by the HIP path's tests and
bench.  It holds *no* arithmetic of the method: it only draws the inputs — the
image-span table, the per-head class vector, and random Q/K/V — in the shapes of
the multi-image prompts the paper evaluates on (Sec. 6.1 set-up, App. "FLOPs
Reduction": 1,280-5,120 tokens per image for Qwen-type models, small fixed-size
images for Gemma 3; Sec. 5.1: the first 10 % of every image is its sink).

Head classes are encoded as in the paper's four categories (Sec. 3.2):
0 Dense, 1 Sink, 2 Intra-Image, 3 Intra-Image+Sink.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace

import numpy as np

DENSE, SINK, INTRA, INTRA_SINK = 0, 1, 2, 3
CLASS_NAMES = ("dense", "sink", "intra", "intra_sink")


@dataclass
class Prompt:
    """One synthetic prefill problem: geometry only, no tensors."""

    name: str
    seq_len: int
    spans: np.ndarray          # int32 [G, 3]: (start, end, sink) per image, sorted, disjoint
    sink_len: int              # global sink: prompt positions [0, sink_len)
    head_class: np.ndarray     # uint8 [n_q_heads]
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str                 # "bf16" | "f32"
    scale: float
    value_recipe: dict = field(default_factory=dict)
    img_bidir: bool = False    # tokens of one image also attend to the later tokens of that image
    sink_offsets: tuple = ()   # offsets inside every image that are sink keys too
    window: int = 0            # > 0: sliding-window layer, a query sees keys with i - j < window

    @property
    def gqa_group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def all_dense(self) -> "Prompt":
        return replace(self, name=self.name + "/all-dense",
                       head_class=np.zeros_like(self.head_class))

    def with_classes(self, classes) -> "Prompt":
        hc = np.asarray(classes, dtype=np.uint8)
        assert hc.shape == self.head_class.shape
        return replace(self, head_class=hc)


def ten_percent_sink(length: int) -> int:
    """Bench rule for 'the sink of an image is 10 % of its length': ceil(len/10), at least 1."""
    return max(1, (int(length) + 9) // 10)


def layout_from_runs(runs, sink_mode: str = "paper10", span_sink=None):
    """runs: sequence of ('T'|'I', length).  Returns (seq_len, spans[G,3]).

    sink_mode 'prefix'  -> every span's sink count is 0 (only the global prefix is a sink)
              'paper10' -> every span's sink count is ceil(len/10)
    span_sink (int)     -> overrides with a fixed per-span count (clipped to the span length)
    """
    pos = 0
    spans = []
    for kind, n in runs:
        n = int(n)
        if n <= 0:
            continue
        if kind == "I":
            if span_sink is not None:
                s = min(int(span_sink), n)
            elif sink_mode == "paper10":
                s = ten_percent_sink(n)
            elif sink_mode == "prefix":
                s = 0
            else:
                raise ValueError(f"unknown sink_mode {sink_mode!r}")
            spans.append((pos, pos + n, s))
        elif kind != "T":
            raise ValueError(kind)
        pos += n
    return pos, np.asarray(spans, dtype=np.int32).reshape(-1, 3)


def _class_vector(rng, counts):
    v = np.concatenate([np.full(c, k, dtype=np.uint8) for k, c in enumerate(counts)])
    rng.shuffle(v)
    return v


def _first_text_len(runs):
    return int(runs[0][1]) if runs and runs[0][0] == "T" else 0


def tiny_config(sink_mode: str = "prefix", span_sink=None) -> Prompt:
    """Config 1: fp32, 2 query heads on 1 KV head, d=64, 1,136 tokens."""
    runs = [("T", 32)]
    for g in range(4):
        runs.append(("I", 256))
        runs.append(("T", 16 if g < 3 else 32))
    L, spans = layout_from_runs(runs, sink_mode, span_sink)
    assert L == 1136
    return Prompt(name=f"cfg1-tiny-f32/{sink_mode if span_sink is None else 'sink%d' % span_sink}",
                  seq_len=L, spans=spans, sink_len=32,
                  head_class=np.array([DENSE, INTRA_SINK], dtype=np.uint8),
                  n_q_heads=2, n_kv_heads=1, head_dim=64, dtype="f32", scale=1.0 / 8.0,
                  value_recipe={"std": 1.0, "first_key_scale": 8.0})


def qwen2vl_7b_config(seed: int = 0, sink_mode: str = "paper10") -> Prompt:
    """Config 2: 28/4 heads, d=128, bf16, ~36-40K tokens, 16 images of 1,024-3,600 tokens."""
    rng = np.random.default_rng([2, seed])
    runs = [("T", 64)]
    for _ in range(16):
        runs.append(("I", rng.integers(1024, 3601)))
        runs.append(("T", rng.integers(8, 65)))
    L, spans = layout_from_runs(runs, sink_mode)
    return Prompt(name=f"cfg2-qwen2vl7b-36k/{sink_mode}/seed{seed}", seq_len=L, spans=spans,
                  sink_len=_first_text_len(runs), head_class=_class_vector(rng, (7, 7, 7, 7)),
                  n_q_heads=28, n_kv_heads=4, head_dim=128, dtype="bf16",
                  scale=1.0 / math.sqrt(128),
                  value_recipe={"std": 1.0 / math.sqrt(128), "outlier_frac": 0.01, "outlier_scale": 6.0})


def qwen25vl_32b_config(seed: int = 0, sink_mode: str = "paper10") -> Prompt:
    """Config 3: 40/8 heads, d=128, bf16, 48 images of 1,600-4,096 tokens (~140K tokens)."""
    rng = np.random.default_rng([3, seed])
    runs = [("T", rng.integers(16, 129))]
    for _ in range(48):
        runs.append(("I", rng.integers(1600, 4097)))
        runs.append(("T", rng.integers(16, 129)))
    L, spans = layout_from_runs(runs, sink_mode)
    return Prompt(name=f"cfg3-qwen25vl32b-128k/{sink_mode}/seed{seed}", seq_len=L, spans=spans,
                  sink_len=_first_text_len(runs), head_class=_class_vector(rng, (4, 8, 16, 12)),
                  n_q_heads=40, n_kv_heads=8, head_dim=128, dtype="bf16",
                  scale=1.0 / math.sqrt(128),
                  value_recipe={"std": 1.0 / math.sqrt(128), "outlier_frac": 0.01, "outlier_scale": 6.0})


def gemma3_27b_config(seed: int = 0, sink_mode: str = "paper10") -> Prompt:
    """Config 4: 32/16 heads, d=128, bf16, 1,100 images of 256 tokens (~300K tokens)."""
    rng = np.random.default_rng([4, seed])
    runs = [("T", rng.integers(4, 33))]
    for _ in range(1100):
        runs.append(("I", 256))
        runs.append(("T", rng.integers(4, 33)))
    L, spans = layout_from_runs(runs, sink_mode)
    return Prompt(name=f"cfg4-gemma3-27b-300k/{sink_mode}/seed{seed}", seq_len=L, spans=spans,
                  sink_len=_first_text_len(runs), head_class=_class_vector(rng, (5, 5, 11, 11)),
                  n_q_heads=32, n_kv_heads=16, head_dim=128, dtype="bf16",
                  scale=1.0 / math.sqrt(128),
                  value_recipe={"std": 1.0 / math.sqrt(128), "first_key_scale": 8.0})


def gemma3_bidir_config(seed: int = 0, n_images: int = 1100) -> Prompt:
    """Config 4 as the Gemma 3 models actually attend (Sec. 6.1): every image has 256 tokens that
    attend to each other in both directions, and the sinks sit at a fixed list of offsets inside
    every image.  The paper took the 10 % most frequent sink positions found on its
    characterisation data set; that list is not available, a seeded draw of 26 offsets stands in."""
    rng = np.random.default_rng([6, seed])
    runs = [("T", rng.integers(4, 33))]
    for _ in range(n_images):
        runs.append(("I", 256))
        runs.append(("T", rng.integers(4, 33)))
    L, spans = layout_from_runs(runs, "prefix", 0)
    offsets = tuple(int(o) for o in np.sort(rng.choice(256, size=26, replace=False)))
    return Prompt(name=f"cfg4-gemma3-27b-bidir-{n_images}img/offset-sinks/seed{seed}", seq_len=L, spans=spans,
                  sink_len=_first_text_len(runs), head_class=_class_vector(rng, (5, 5, 11, 11)),
                  n_q_heads=32, n_kv_heads=16, head_dim=128, dtype="bf16",
                  scale=1.0 / math.sqrt(128),
                  value_recipe={"std": 1.0 / math.sqrt(128), "first_key_scale": 8.0},
                  img_bidir=True, sink_offsets=offsets)


STRESS_LENGTHS = (36864, 73728, 153600, 307200)


def stress_config(target_len: int, seed: int = 0, sink_mode: str = "paper10") -> Prompt:
    """Config 5: Qwen2-VL-7B head shape, image sizes log-uniform in [64, 8192], given target length."""
    rng = np.random.default_rng([5, seed, int(target_len)])
    runs = [("T", 64)]
    pos = 64
    while pos < target_len:
        n = int(round(math.exp(rng.uniform(math.log(64), math.log(8192)))))
        t = int(rng.integers(8, 65))
        room = target_len - pos - t
        if room < 64:
            # not enough room for a minimum-size image plus its trailing text: end with text
            runs.append(("T", target_len - pos))
            pos = target_len
            break
        n = min(n, room)
        runs.append(("I", n))
        runs.append(("T", t))
        pos += n + t
    L, spans = layout_from_runs(runs, sink_mode)
    assert L == target_len, (L, target_len)
    return Prompt(name=f"cfg5-stress-{target_len}/{sink_mode}/seed{seed}", seq_len=L, spans=spans,
                  sink_len=64, head_class=_class_vector(rng, (7, 7, 7, 7)),
                  n_q_heads=28, n_kv_heads=4, head_dim=128, dtype="bf16",
                  scale=1.0 / math.sqrt(128),
                  value_recipe={"std": 1.0 / math.sqrt(128), "outlier_frac": 0.01, "outlier_scale": 6.0})


def config(idx: int, seed: int = 0, sink_mode: str = "paper10", target_len: int | None = None) -> Prompt:
    """The five workload families, numbered 1..5 in the order the baseline lists them; 6 is family 4
    with the Gemma 3 attention rules (non-causal inside an image, sinks at fixed in-image offsets)."""
    if idx == 1:
        return tiny_config(sink_mode)
    if idx == 2:
        return qwen2vl_7b_config(seed, sink_mode)
    if idx == 3:
        return qwen25vl_32b_config(seed, sink_mode)
    if idx == 4:
        return gemma3_27b_config(seed, sink_mode)
    if idx == 5:
        return stress_config(target_len or STRESS_LENGTHS[0], seed, sink_mode)
    if idx == 6:
        return gemma3_bidir_config(seed)
    raise ValueError(idx)


def custom_prompt(runs, head_class, n_kv_heads, head_dim, dtype="bf16", sink_len=0,
                  sink_mode="paper10", span_sink=None, scale=None, name="custom",
                  value_recipe=None, img_bidir=False, sink_offsets=(), window=0) -> Prompt:
    """Small hand-shaped prompts for tests."""
    L, spans = layout_from_runs(runs, sink_mode, span_sink)
    hc = np.asarray(head_class, dtype=np.uint8)
    return Prompt(name=name, seq_len=L, spans=spans, sink_len=sink_len, head_class=hc,
                  n_q_heads=len(hc), n_kv_heads=n_kv_heads, head_dim=head_dim, dtype=dtype,
                  scale=(1.0 / math.sqrt(head_dim)) if scale is None else scale,
                  value_recipe=value_recipe or {"std": 1.0}, img_bidir=bool(img_bidir),
                  sink_offsets=tuple(int(o) for o in sink_offsets), window=int(window))


def make_qkv(p: Prompt, seed: int = 0, device: str = "cpu"):
    """Draw q [Hq,L,d], k, v [Hkv,L,d] as torch tensors of the prompt's dtype on `device`.

    Values: N(0, std^2); optionally the first token's key scaled (an artificial sink), and a
    fraction of (kv head, channel) key columns scaled up as outlier channels.
    """
    import torch

    rec = p.value_recipe
    std = float(rec.get("std", 1.0))
    dt = {"bf16": torch.bfloat16, "f32": torch.float32}[p.dtype]
    g = torch.Generator(device=device)
    g.manual_seed(1000003 * int(seed) + 17)

    def draw(h):
        out = torch.empty((h, p.seq_len, p.head_dim), dtype=dt, device=device)
        for i in range(h):  # one head at a time bounds the fp32 staging buffer
            out[i] = (torch.randn((p.seq_len, p.head_dim), generator=g, device=device,
                                  dtype=torch.float32) * std).to(dt)
        return out

    q = draw(p.n_q_heads)
    k = draw(p.n_kv_heads)
    v = draw(p.n_kv_heads)
    if "first_key_scale" in rec:
        k[:, 0, :] = (k[:, 0, :].float() * float(rec["first_key_scale"])).to(dt)
    if rec.get("outlier_frac", 0.0) > 0.0:
        n_out = int(round(rec["outlier_frac"] * p.n_kv_heads * p.head_dim))
        rng = np.random.default_rng([77, seed])
        flat = rng.choice(p.n_kv_heads * p.head_dim, size=n_out, replace=False)
        for f in flat:
            h, c = divmod(int(f), p.head_dim)
            k[h, :, c] = (k[h, :, c].float() * float(rec["outlier_scale"])).to(dt)
    return q, k, v


def sample_q_tiles(p: Prompt, block_m: int = 128, n_random: int = 6, seed: int = 0,
                   max_tiles: int = 24) -> np.ndarray:
    """Pick query tiles worth checking one by one: first, last (ragged), tiles that straddle the
    start or the end of an image, a tile just inside an image, and a few random ones."""
    M = -(-p.seq_len // block_m)
    picks = {0, M - 1}
    rng = np.random.default_rng([91, seed])
    G = len(p.spans)
    if G:
        chosen = rng.choice(G, size=min(G, 4), replace=False)
        for gi in chosen:
            s, e, _ = (int(x) for x in p.spans[gi])
            picks.update({s // block_m, (e - 1) // block_m, min(M - 1, s // block_m + 1)})
        picks.add(int(p.spans[-1][0]) // block_m)
        picks.add((int(p.spans[-1][1]) - 1) // block_m)
    for t in rng.integers(0, M, size=n_random):
        picks.add(int(t))
    picks = sorted(picks)
    if len(picks) > max_tiles:
        keep = {0, M - 1}
        rest = [t for t in picks if t not in keep]
        idx = rng.choice(len(rest), size=max_tiles - 2, replace=False)
        picks = sorted(keep | {rest[i] for i in idx})
    return np.asarray(picks, dtype=np.int32)


HEAD_KINDS = ("dense", "sink", "intra", "intra_sink")


def make_planted_qkv(p: Prompt, head_kinds, seed: int = 0, boost: float = 30.0, noise: float = 0.5,
                     device: str = "cpu"):
    """Q/K/V in which each query head has a planted attention habit, as inputs for the offline
    characterisation (Alg. 1): a test needs heads for which the sparse masks matter differently.

    Keys: noise, plus a direction `s` on every sink key (prefix sink and image sinks) and a direction
    `u_g` on the other keys of image g (the directions are orthonormal while images + 1 <= head_dim,
    then reused cyclically).  Queries of head h, by head_kinds[h]:
      "dense"       noise only (attention spread over every earlier key)
      "sink"        + s on every row
      "intra"       + u_g on the rows of image g
      "intra_sink"  + s on every row and + u_g on the rows of image g
    with lengths chosen so that a matching query/key pair scores `boost` logits above the rest.
    V is N(0, 1).  Returns torch tensors of the prompt's dtype: q [Hq,L,d], k, v [Hkv,L,d].
    """
    import torch

    kinds = list(head_kinds)
    assert len(kinds) == p.n_q_heads and all(kd in HEAD_KINDS for kd in kinds)
    L, d = p.seq_len, p.head_dim
    dt = {"bf16": torch.bfloat16, "f32": torch.float32}[p.dtype]
    rng = np.random.default_rng([4241, seed])
    basis, _ = np.linalg.qr(rng.standard_normal((d, d)))
    beta = math.sqrt(boost / p.scale)
    img = np.zeros(L, dtype=np.int64)        # 0 text, g + 1 inside image g
    sink = np.zeros(L, dtype=bool)
    sink[:p.sink_len] = True
    for g, (s0, e0, sk) in enumerate(np.asarray(p.spans).reshape(-1, 3)):
        img[s0:e0] = g + 1
        sink[s0:s0 + sk] = True
        for o in p.sink_offsets:
            if o < e0 - s0:
                sink[s0 + o] = True
    direction = np.zeros((L, d))
    in_img = img > 0
    direction[in_img] = basis[1 + (img[in_img] - 1) % (d - 1)]
    s_dir = basis[0]
    key_plant = np.where(sink[:, None], s_dir[None, :], direction) * beta
    key_plant[~sink & ~in_img] = 0.0
    g = torch.Generator(device="cpu")
    g.manual_seed(1000003 * int(seed) + 4241)

    def randn(h, std):
        return torch.randn((h, L, d), generator=g, dtype=torch.float32) * std

    k = randn(p.n_kv_heads, noise) + torch.from_numpy(key_plant).float()[None]
    v = randn(p.n_kv_heads, 1.0)
    q = randn(p.n_q_heads, noise)
    s_t = torch.from_numpy(s_dir * beta).float()
    u_t = torch.from_numpy(direction * beta).float()
    for h, kd in enumerate(kinds):
        if kd in ("sink", "intra_sink"):
            q[h] += s_t[None, :]
        if kd in ("intra", "intra_sink"):
            q[h] += u_t
    return q.to(dt).to(device), k.to(dt).to(device), v.to(dt).to(device)
