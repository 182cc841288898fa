"""Pins of the characterisation oracle (oracle/characterize.py; paper Sec. 4, Alg. 1 and Alg. 2)
against what the algorithm and the mathematics fix: closed forms of the error measure, prompts
whose answer follows from the mask definition alone, and a brute-force evaluation with explicit
mask matrices on a tiny prompt."""
import math

import numpy as np
import pytest

import oracle
import workloads as W
from oracle import characterize as C

D, S, I, IS = oracle.DENSE, oracle.SINK, oracle.INTRA, oracle.INTRA_SINK


def test_nmse_closed_forms():
    rng = np.random.default_rng(0)
    r = rng.standard_normal((37, 8))
    assert C.nmse(r, r) == 0.0
    assert C.nmse(np.zeros_like(r), r) == pytest.approx(1.0, rel=1e-15)
    for c in (0.5, -0.25, 2.0):  # scaled copy: error c^2, whatever the reference is
        assert C.nmse((1.0 + c) * r, r) == pytest.approx(c * c, rel=1e-12)
    # one changed element: its squared change over the reference's energy
    a = r.copy()
    a[5, 3] += 3.0
    assert C.nmse(a, r) == pytest.approx(9.0 / float((r ** 2).sum()), rel=1e-12)
    # the reference normalises, not the candidate
    assert C.nmse(3.0 * r, r) == pytest.approx(4.0, rel=1e-12)
    assert C.nmse(r, 3.0 * r) == pytest.approx(4.0 / 9.0, rel=1e-12)


def test_nmse_zero_reference_reading():
    z = np.zeros((4, 4))
    assert C.nmse(z, z) == 0.0
    assert C.nmse(np.ones((4, 4)), z) == math.inf


def constant_v_case():
    # image of 50 tokens first, no sinks anywhere: under the Sink mask its rows see no key at all
    p = W.custom_prompt([("I", 50), ("T", 10), ("I", 30), ("T", 6)], [0, 0], 1, 8, dtype="f32",
                        span_sink=0)
    rng = np.random.default_rng(3)
    L, d = p.seq_len, p.head_dim
    q = rng.standard_normal((2, L, d)).astype(np.float32)
    k = rng.standard_normal((1, L, d)).astype(np.float32)
    v = np.tile(rng.standard_normal((1, 1, d)).astype(np.float32), (1, L, 1))
    imgid, issink = oracle.token_arrays(p.spans, L, p.sink_len)
    return p, q, k, v, imgid, issink


def test_constant_values_error_is_the_share_of_empty_rows():
    """With the same value vector on every key a softmax average returns it whatever the mask, so
    the only error is a row whose mask is empty (output zero): NMSE = empty rows / L."""
    p, q, k, v, imgid, issink = constant_v_case()
    L = p.seq_len
    ht, e = C.characterize_prompt(q, k, v, imgid, issink, p.scale, alpha=0.0)  # nothing passes
    assert list(ht) == [D, D]
    assert e[0] == pytest.approx([50 / L, 50 / L], rel=1e-12)   # Sink: first image's rows are empty
    assert e[1] == pytest.approx([0.0, 0.0], abs=1e-24)          # Intra-Image: every row sees itself
    assert e[2] == pytest.approx([0.0, 0.0], abs=1e-24)


def test_order_break_and_strict_threshold():
    p, q, k, v, imgid, issink = constant_v_case()
    L = p.seq_len
    # Sink fails (50/96 >= 0.1), Intra-Image passes and ends the search
    ht, e = C.characterize_prompt(q, k, v, imgid, issink, p.scale, alpha=0.1)
    assert list(ht) == [I, I]
    assert np.isnan(e[2]).all() and not np.isnan(e[:2]).any()
    # a looser threshold takes the cheaper Sink pattern first
    ht, e = C.characterize_prompt(q, k, v, imgid, issink, p.scale, alpha=0.6)
    assert list(ht) == [S, S] and np.isnan(e[1:]).all()
    # strictly below: a threshold equal to the Sink error does not pass it
    ht, _ = C.characterize_prompt(q, k, v, imgid, issink, p.scale, alpha=float(e[0, 0]))
    assert ht[0] == I


def test_prompt_without_images_takes_the_first_pattern():
    p = W.custom_prompt([("T", 70)], [0, 0, 0], 1, 8, dtype="f32")
    rng = np.random.default_rng(5)
    q = rng.standard_normal((3, 70, 8)).astype(np.float32)
    k = rng.standard_normal((1, 70, 8)).astype(np.float32)
    v = rng.standard_normal((1, 70, 8)).astype(np.float32)
    imgid, issink = oracle.token_arrays(p.spans, 70, 0)
    ht, e = C.characterize_prompt(q, k, v, imgid, issink, p.scale, alpha=1e-30)
    assert list(ht) == [S, S, S] and (e[0] == 0.0).all()
    ht, _ = C.characterize_prompt(q, k, v, imgid, issink, p.scale, alpha=0.0)
    assert list(ht) == [D, D, D]


def test_against_explicit_mask_matrices_with_grouped_heads():
    """Tiny prompt, two KV heads with different keys: every head's errors recomputed with the
    textbook masked softmax over the full mask matrix (pins the head -> KV head mapping, the
    reference being the Dense mask, and the order of the three candidates)."""
    p = W.custom_prompt([("T", 5), ("I", 21), ("T", 3), ("I", 17), ("T", 4)], [0] * 4, 2, 8,
                        dtype="f32", sink_len=2)
    rng = np.random.default_rng(11)
    L, d = p.seq_len, p.head_dim
    q = rng.standard_normal((4, L, d)).astype(np.float32) * 2
    k = rng.standard_normal((2, L, d)).astype(np.float32) * 2
    v = rng.standard_normal((2, L, d)).astype(np.float32)
    imgid, issink = oracle.token_arrays(p.spans, L, p.sink_len)
    _, e = C.characterize_prompt(q, k, v, imgid, issink, p.scale, alpha=0.0)

    def textbook(h, cls):
        m = oracle.mask(cls, imgid, issink).astype(bool)
        s = (q[h].astype(np.float64) @ k[h // 2].astype(np.float64).T) * p.scale
        s = np.where(m, s, -np.inf)
        w = np.exp(s - s.max(axis=1, keepdims=True))
        return (w / w.sum(axis=1, keepdims=True)) @ v[h // 2].astype(np.float64)

    for h in range(4):
        ref = textbook(h, D)
        for mi, cls in enumerate((S, I, IS)):
            out = textbook(h, cls)
            want = ((out - ref) ** 2).sum() / (ref ** 2).sum()
            assert e[mi, h] == pytest.approx(want, rel=1e-9), (h, cls)
    assert e.min() > 1e-3  # the case is not degenerate


def test_planted_heads_are_recovered():
    kinds = ["dense", "sink", "intra", "intra_sink"] * 2
    p = W.custom_prompt([("T", 40), ("I", 300), ("T", 12), ("I", 260), ("T", 20), ("I", 333), ("T", 17)],
                        [0] * 8, 2, 64, dtype="f32")
    q, k, v = W.make_planted_qkv(p, kinds, seed=0)
    imgid, issink = oracle.token_arrays(p.spans, p.seq_len, p.sink_len)
    ht, _ = C.characterize_prompt(q.numpy(), k.numpy(), v.numpy(), imgid, issink, p.scale, alpha=0.1)
    assert list(ht) == [D, S, I, IS] * 2


def test_aggregation_rules():
    g = dict(gamma_d=0.25, gamma_s=0.6, gamma_i=0.6)
    assert C.aggregate([0.26, 0.74, 0.0, 0.0], **g) == D          # Dense share wins first
    assert C.aggregate([0.25, 0.75, 0.0, 0.0], **g) == S          # "exceeds" is strict
    assert C.aggregate([0.0, 0.6, 0.4, 0.0], **g) == IS           # 0.6 does not exceed 0.6; neither does 0.4
    assert C.aggregate([0.1, 0.2, 0.7, 0.0], **g) == I
    assert C.aggregate([0.1, 0.3, 0.3, 0.3], **g) == IS           # no dominant sparse pattern
    assert C.aggregate([0.0, 0.0, 0.0, 1.0], **g) == IS
    assert C.aggregate([1.0, 0.0, 0.0, 0.0], **g) == D


def test_head_type_fraction_counts_prompts():
    t = np.array([[0, 1, 3], [0, 2, 3], [1, 2, 3], [0, 2, 1]])
    f = C.head_type_fraction(t)
    assert f.shape == (3, 4)
    assert list(f[0]) == [0.75, 0.25, 0.0, 0.0]
    assert list(f[1]) == [0.0, 0.25, 0.75, 0.0]
    assert list(f[2]) == [0.0, 0.25, 0.0, 0.75]
    assert np.allclose(f.sum(axis=1), 1.0)
