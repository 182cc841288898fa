"""The bf16 kernel's matrix phase is inline asm: check in the compiled ISA that the compiler put no
vector access of its own right behind an MFMA (it would read the register before the matrix pipe
has written it).  Needs hipcc (cross-compiles without a GPU); the checker itself is also tested on
hand-written listings."""
import shutil

import pytest

from paper_2507_09071_amd import build as bs_build
import isa_check


def test_checker_flags_a_copy_right_behind_an_mfma():
    ins = ["v_mfma_f32_32x32x16_bf16 v[0:15], v[16:19], v[20:23], v[0:15]",
           "ds_read_b128 v[16:19], v40",
           "v_mov_b64_e32 v[32:33], v[14:15]"]
    found = isa_check.mfma_hazards(ins)
    assert len(found) == 1 and found[0][1] == 1


def test_checker_accepts_waits_accumulation_and_branches():
    acc = "v_mfma_f32_32x32x16_bf16 v[0:15], v[16:19], v[20:23], v[0:15]"
    assert isa_check.mfma_hazards([acc, acc, "s_nop 15", "v_mul_f32_e32 v0, v0, v30"]) == []
    assert isa_check.mfma_hazards([acc, "s_nop 11", "v_mul_f32_e32 v0, v0, v30"]) == []       # 12 wait states
    assert len(isa_check.mfma_hazards([acc, "s_nop 10", "v_mul_f32_e32 v0, v0, v30"])) == 1   # one short of the margin
    assert isa_check.mfma_hazards([acc, "s_barrier", "v_mul_f32_e32 v0, v0, v30"]) == []
    assert isa_check.mfma_hazards([acc, "v_add_f32_e32 v40, v41, v42"]) == []


def test_checker_tracks_lds_reads_in_flight():
    rd = lambda a: f"ds_read_b128 v[{a}:{a + 3}], v60"
    ok = [rd(0), rd(4), rd(8), "s_waitcnt lgkmcnt(2)", "v_mfma_f32_32x32x16_bf16 v[64:79], v[0:3], v[40:43], v[64:79]",
          "s_waitcnt lgkmcnt(0)", "v_mov_b32_e32 v70, v9"]
    assert isa_check.lds_read_hazards(ok) == []
    early = [rd(0), rd(4), "s_waitcnt lgkmcnt(1)", "v_mov_b32_e32 v70, v5"]        # second read still in flight
    assert len(isa_check.lds_read_hazards(early)) == 1
    overwritten = [rd(0), "v_mov_b32_e32 v2, 0", "s_waitcnt lgkmcnt(0)"]           # compiler reuses the register
    assert len(isa_check.lds_read_hazards(overwritten)) == 1


@pytest.mark.skipif(shutil.which(bs_build.hipcc()) is None, reason="hipcc not available")
def test_compiled_bf16_kernels_have_no_mfma_hazard():
    res = isa_check.check()
    assert set(res) == set(isa_check.KERNELS)
    for k, hazards in res.items():
        assert hazards == [], f"{k}: {hazards[:3]}"
