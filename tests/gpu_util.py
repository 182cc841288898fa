"""Helpers for the GPU parity tests: run the HIP path through the C ABI, compare with the oracle."""
import numpy as np
import torch

import oracle
import paper_2507_09071_amd as bs

BF16_MAX_ABS, BF16_REL_L2 = 2e-2, 5e-3     # tolerance for bf16 inputs
F32_TOL = 1e-5                              # max-abs and relative-L2 for the fp32 configuration


def run_prefill(p, q, k, v, tm=None, stream=None, flags=0):
    """Launch bs_attn_prefill on the tensors' device; returns (out, tilemap)."""
    assert q.is_cuda and q.is_contiguous() and k.is_contiguous() and v.is_contiguous()
    if tm is None:
        if getattr(p, "img_bidir", False):
            flags |= bs.BS_MAP_BIDIR_IMAGES
        tm = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len, 128, 64, flags=flags,
                                 sink_offsets=getattr(p, "sink_offsets", None) or None,
                                 window=int(getattr(p, "window", 0)))
    out = torch.full_like(q, float("nan"))
    dt = bs.BS_BF16 if q.dtype == torch.bfloat16 else bs.BS_F32
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    bs.bs_attn_prefill(q, k, v, out, tm, dt, p.n_q_heads, p.gqa_group, p.head_dim, p.scale, st)
    torch.cuda.synchronize()
    return out, tm


def errors(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape
    assert np.isfinite(got).all(), "non-finite output"
    max_abs = float(np.abs(got - want).max()) if got.size else 0.0
    denom = float(np.sqrt((want ** 2).sum()))
    rel = float(np.sqrt(((got - want) ** 2).sum()) / denom) if denom > 0 else max_abs
    return max_abs, rel


def assert_close(got, want, dtype, what=""):
    max_abs, rel = errors(got, want)
    if dtype == "f32":
        assert max_abs <= F32_TOL and rel <= F32_TOL, f"{what}: max_abs {max_abs:.3e} rel_l2 {rel:.3e}"
    else:
        assert max_abs <= BF16_MAX_ABS and rel <= BF16_REL_L2, f"{what}: max_abs {max_abs:.3e} rel_l2 {rel:.3e}"
    return max_abs, rel


def oracle_rows(p, q, k, v, rows=None):
    return oracle.attention_for_prompt(p, q, k, v, rows)


def rows_of_tiles(p, q_tiles, step=1):
    rows = []
    for m in q_tiles:
        lo, hi = int(m) * 128, min(int(m) * 128 + 128, p.seq_len)
        rows.extend(range(lo, hi, step))
        rows.append(hi - 1)
    return np.unique(np.asarray(rows, dtype=np.int32))
