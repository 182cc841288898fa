"""The entry point that allocates nothing (bs_attn_prefill_static: packed K / V^T tiles in a static device
array of the library) against bs_attn_prefill, through the C ABI: same kernels, so the outputs must be
identical bit for bit, and within the bf16 tolerance of the oracle.  Two calls in a row, the second on a
smaller prompt (the array keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2507_09071_amd as bs
import workloads as W
from paper_2507_09071_amd import binding
from gpu_util import assert_close, oracle_rows

pytestmark = pytest.mark.gpu
D, S, I, IS = 0, 1, 2, 3
DEV = "cuda:0"


def raw_static(lib, q, k, v, out, tm, p, stream):
    return lib.bs_attn_prefill_static(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), tm.handle,
                                      p.n_q_heads, p.gqa_group, p.head_dim, ctypes.c_float(p.scale),
                                      ctypes.c_void_p(stream))


def test_static_entry_point_matches_the_allocating_one_twice_in_a_row():
    lib = binding.load_library()
    big = W.custom_prompt([("T", 50), ("I", 1900), ("T", 7), ("I", 2300), ("T", 30), ("I", 700), ("T", 64)],
                          [D, S, I, IS, IS, I, S, D], 2, 128, dtype="bf16", sink_len=50, name="static-big")
    small = W.custom_prompt([("T", 9), ("I", 300), ("T", 3), ("I", 140), ("T", 21)],
                            [IS, D, S, I], 2, 128, dtype="bf16", sink_len=9, name="static-small")
    st = torch.cuda.current_stream().cuda_stream
    for i, p in enumerate((big, small)):
        q, k, v = W.make_qkv(p, 20 + i, DEV)
        tm = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len, 128, 64, flags=bs.BS_MAP_PACK_KEYS)
        want = torch.full_like(q, float("nan"))
        bs.bs_attn_prefill(q, k, v, want, tm, bs.BS_BF16, p.n_q_heads, p.gqa_group, p.head_dim, p.scale, st)
        got = torch.full_like(q, float("nan"))
        tm2 = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len, 128, 64, flags=bs.BS_MAP_PACK_KEYS)
        assert raw_static(lib, q, k, v, got, tm2, p, st) == -1          # not prepared: refused, nothing launched
        tm2.prepare(bs.BS_BF16, p.gqa_group, st)
        print("static call", p.name, "L", p.seq_len, flush=True)
        assert raw_static(lib, q, k, v, got, tm2, p, st) == 0
        torch.cuda.synchronize()
        assert torch.equal(got, want), p.name
        ref = oracle_rows(p, q, k, v)
        for h in range(p.n_q_heads):
            assert_close(got[h].float().cpu().numpy(), ref[h], "bf16", f"{p.name} head {h}")
        # a rebind makes the prepared state stale; prepare again and compare again
        hc = np.roll(p.head_class, 1)
        tm2.rebind(hc)
        assert raw_static(lib, q, k, v, got, tm2, p, st) == -1
        tm2.prepare(bs.BS_BF16, p.gqa_group, st)
        assert raw_static(lib, q, k, v, got, tm2, p, st) == 0
        tm.rebind(hc)
        bs.bs_attn_prefill(q, k, v, want, tm, bs.BS_BF16, p.n_q_heads, p.gqa_group, p.head_dim, p.scale, st)
        torch.cuda.synchronize()
        assert torch.equal(got, want), p.name + " rebound"


def test_static_entry_point_rejects_a_prompt_beyond_its_scratch():
    lib = binding.load_library()
    # 8 KV heads x 1024 key tiles x 32 KB = 256 MiB of packed tiles > 96 MiB
    p = W.custom_prompt([("T", 65536)], [D] * 8, 8, 128, dtype="bf16", name="static-too-big")
    tm = bs.bs_build_tilemap(p.spans, p.seq_len, p.head_class, p.sink_len, 128, 64)
    st = torch.cuda.current_stream().cuda_stream
    tm.prepare(bs.BS_BF16, 1, st)
    x = torch.zeros((8, 8, 128), dtype=torch.bfloat16, device=DEV)      # never read: the call is refused first
    rc = lib.bs_attn_prefill_static(x.data_ptr(), x.data_ptr(), x.data_ptr(), x.data_ptr(), tm.handle, 8, 1, 128,
                                    ctypes.c_float(0.1), ctypes.c_void_p(st))
    assert rc == -2 and b"static scratch" in lib.bs_last_error()
    torch.cuda.synchronize()
