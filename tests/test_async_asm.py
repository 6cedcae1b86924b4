"""The kernels' split asynchronous loads (load in one inline-assembly statement,
wait in a later one) as the compiler has laid them out: no instruction may
touch a destination register between the load and its wait.  CPU only: the
sources are compiled to assembly and scanned."""
import shutil

import pytest

from paper_2402_10876_amd import check_async_asm as chk

BAD = """
_Z1kv:
	;;#ASMSTART
	ds_read_b32 v35, v35
	;;#ASMEND
	v_mov_b32_e32 v76, v35
	;;#ASMSTART
	s_waitcnt lgkmcnt(0)
	;;#ASMEND
	s_endpgm
"""
GOOD = """
_Z1kv:
	;;#ASMSTART
	ds_read_b64_tr_b16 v[2:3], v9 offset:0
	;;#ASMEND
	;;#ASMSTART
	s_load_dwordx4 s[16:19], s[16:17], 0x0
	;;#ASMEND
	v_mfma_f32_32x32x16_f16 a[0:15], v[4:7], v[10:13], a[0:15]
	;;#ASMSTART
	s_waitcnt lgkmcnt(0)
	;;#ASMEND
	v_mov_b32_e32 v76, v2
	v_mov_b32_e32 v77, s17
	ds_read_b32 v1, v76
	v_mov_b32_e32 v5, v1
	s_endpgm
"""


def test_scanner_flags_a_use_before_the_wait_and_nothing_else():
    f = chk.check_assembly(BAD)
    assert len(f) == 1 and f[0][0] == "_Z1kv" and "v76, v35" in f[0][2]
    assert chk.check_assembly(GOOD) == []      # compiler-issued reads outside the markers are its own business


@pytest.mark.skipif(shutil.which(chk.HIPCC) is None, reason="hipcc not available")
def test_kernels_have_no_use_before_wait():
    assert chk.check_sources() == []
