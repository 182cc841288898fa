"""CPU oracle of the offline characterisation (paper Sec. 4, Alg. 1 and Alg. 2), fp64 numpy.

TEST INFRASTRUCTURE ONLY, like the rest of this package: the product path never imports it.

Alg. 1 (prompt level, one attention head): the dense causal output is the reference; the three
sparse masks are tried in the order Sink, Intra-Image, Intra-Image+Sink; the first whose
normalised squared error against the reference is strictly below alpha_layer is the head's type;
if none is, the head stays Dense.  Later masks are not evaluated once one has passed.

Alg. 2 (data-set level, one head): from the fractions of prompts that chose each type: Dense if the
Dense fraction exceeds gamma_d, else Sink if the Sink fraction exceeds gamma_s, else Intra-Image if
that fraction exceeds gamma_i, else Intra-Image+Sink.

Readings where the paper is silent:
  * the norms are Frobenius norms over the head's whole [L, d] output;
  * a reference of norm zero gives NMSE 0 if the masked output is zero too, +inf otherwise;
  * gamma_i has no recommended value in the paper; callers pass it (the tests use gamma_s's).
"""
from __future__ import annotations

import numpy as np

from . import DENSE, SINK, INTRA, INTRA_SINK, attention

MASK_ORDER = (SINK, INTRA, INTRA_SINK)  # Alg. 1: cheapest pattern first


def nmse(attn_mask: np.ndarray, attn_ref: np.ndarray) -> float:
    """||attn_mask - attn_ref||^2 / ||attn_ref||^2 for one head (Alg. 1)."""
    a = np.asarray(attn_mask, dtype=np.float64)
    r = np.asarray(attn_ref, dtype=np.float64)
    assert a.shape == r.shape
    diff = a - r
    num = float(np.sum(diff * diff))
    den = float(np.sum(r * r))
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / den


def characterize_prompt(q, k, v, imgid, issink, scale: float, alpha: float, img_bidir: bool = False,
                        window: int = 0):
    """Alg. 1 for every query head of one layer.

    q [Hq, L, d], k / v [Hkv, L, d] float32 arrays.  Returns (head_type uint8 [Hq],
    nmse float64 [3, Hq]) with nmse[m, h] = NaN where mask MASK_ORDER[m] was not evaluated for
    head h because an earlier one had passed.
    """
    q = np.asarray(q, dtype=np.float32)
    Hq = q.shape[0]
    Hkv = k.shape[0]
    G = Hq // Hkv
    head_type = np.full(Hq, DENSE, dtype=np.uint8)
    errs = np.full((3, Hq), np.nan, dtype=np.float64)
    for h in range(Hq):
        kv = h // G

        def attn(cls):
            return attention(q[h:h + 1], k[kv:kv + 1], v[kv:kv + 1], np.array([cls], dtype=np.uint8),
                             imgid, issink, scale, None, img_bidir, window)[0]

        attn_ref = attn(DENSE)
        for m, cls in enumerate(MASK_ORDER):
            attn_mask = attn(cls)
            errs[m, h] = nmse(attn_mask, attn_ref)
            if errs[m, h] < alpha:
                head_type[h] = cls
                break
    return head_type, errs


def head_type_fraction(head_types) -> np.ndarray:
    """[n_prompts, Hq] head types (one row per characterised prompt) -> [Hq, 4] fractions."""
    t = np.asarray(head_types)
    assert t.ndim == 2 and t.shape[0] > 0
    out = np.zeros((t.shape[1], 4), dtype=np.float64)
    for c in (DENSE, SINK, INTRA, INTRA_SINK):
        out[:, c] = (t == c).sum(axis=0) / t.shape[0]
    return out


def aggregate(fraction, gamma_d: float, gamma_s: float, gamma_i: float) -> int:
    """Alg. 2 for one head; fraction[c] = share of prompts that chose class c."""
    if fraction[DENSE] > gamma_d:
        return DENSE
    if fraction[SINK] > gamma_s:
        return SINK
    if fraction[INTRA] > gamma_i:
        return INTRA
    return INTRA_SINK
