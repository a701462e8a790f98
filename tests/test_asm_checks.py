"""The build's check of registers that a load written as inline assembly still owes their value
(paper_2502_07864_amd/asm_checks.py): what it accepts, what it rejects, and the listing of the
library as built."""
from pathlib import Path

import pytest

from paper_2502_07864_amd import asm_checks

CLEAN = """
_Zkernel_a: ; @kernel
	v_lshl_add_u64 v[62:63], v[4:5], 0, v[6:7]
	global_load_dwordx4 v[2:5], v[62:63], off
	v_lshl_add_u64 v[6:7], v[62:63], 0, 64
	global_load_dwordx4 v[6:9], v[6:7], off
	v_add_u32_e32 v20, v21, v22 ; untouched registers may be used freely
	s_waitcnt vmcnt(0)
	v_mov_b32_e32 v30, v2
	s_endpgm
"""


def body(asm):
    return next(iter(asm_checks.kernels(asm).values()))


def test_a_clean_listing_passes():
    n, bad = asm_checks.pending_register_violations(body(CLEAN))
    assert n == 2 and bad == []
    assert asm_checks.check_listing(CLEAN, "kernel_a") == {"_Zkernel_a": 2}


@pytest.mark.parametrize("line", [
    "\tv_mov_b32_e32 v30, v3",                            # reads a pending register: stale data
    "\tv_mov_b32_e32 v8, 0",                              # writes one: the load overwrites it later
    "\tscratch_store_dwordx4 off, v[2:5], off",           # spills one before its value is there
    "\tglobal_load_dwordx4 v[40:43], v[4:5], off",        # takes an address from one
])
def test_use_of_a_pending_register_is_rejected(line):
    dirty = CLEAN.replace("\tv_add_u32_e32 v20, v21, v22", line)
    n, bad = asm_checks.pending_register_violations(body(dirty))
    assert bad and line.strip() in bad[0]
    with pytest.raises(RuntimeError):
        asm_checks.check_listing(dirty, "kernel_a")


def test_registers_are_free_again_after_the_wait():
    later = CLEAN.replace("\tv_mov_b32_e32 v30, v2", "\tv_mov_b32_e32 v2, 0\n\tv_mov_b32_e32 v9, v2")
    assert asm_checks.pending_register_violations(body(later))[1] == []


def test_the_built_library_s_listing_is_clean():
    listing = Path(asm_checks.__file__).resolve().parent / "_build" / "decode_mfma.s"
    if not listing.exists():
        from paper_2502_07864_amd.build import build_library
        build_library()
    seen = asm_checks.check_listing(listing.read_text(), "decode_mfma_kernel")
    # the d_c = 256 instantiations (ring of 3 and 4, both partitions): 10 query-row loads each
    assert len(seen) == 4 and all(n == 10 for n in seen.values()), seen
