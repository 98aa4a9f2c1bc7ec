"""The build's check of the device assembly: a wide store must not be followed, within two wait
states, by a vector ALU write to the registers it stores."""
import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_1709_04057_amd import build as lr_build
from paper_1709_04057_amd import isa_check

STORE = "\tbuffer_store_dwordx4 v[58:61], v198, s[76:79], s4 offen nt\n"


def test_overwrite_right_behind_the_store_is_found():
    asm = STORE + "\tv_mul_f32_e32 v59, 0x4038aa3b, v180\n\ts_endpgm\n"
    found = isa_check.check_text(asm)
    assert len(found) == 1 and "v[59]" in found[0]


def test_second_wait_state_counts_too():
    asm = STORE + "\ts_mul_i32 s4, s4, s15\n\tv_exp_f32_e32 v61, v3\n\ts_endpgm\n"
    assert len(isa_check.check_text(asm)) == 1
    asm = STORE + "\ts_mul_i32 s4, s4, s15\n\ts_add_i32 s4, s4, 1\n\tv_exp_f32_e32 v61, v3\n\ts_endpgm\n"
    assert isa_check.check_text(asm) == []


def test_pause_or_unrelated_registers_are_fine():
    assert isa_check.check_text(STORE + "\ts_nop 1\n\tv_mul_f32_e32 v59, 2.0, v59\n\ts_endpgm\n") == []
    assert isa_check.check_text(STORE + "\ts_nop 0\n\tv_mul_f32_e32 v59, 2.0, v59\n\ts_endpgm\n") != []
    assert isa_check.check_text(STORE + "\tv_mul_f32_e32 v62, 2.0, v59\n\tv_mov_b32_e32 v57, v58\n\ts_endpgm\n") == []
    # a compare writes a mask, a load's data arrives much later, a narrow store has read its data
    assert isa_check.check_text(STORE + "\tv_cmp_lt_f32_e32 vcc, v59, v60\n\ts_endpgm\n") == []
    assert isa_check.check_text(STORE + "\tbuffer_load_dwordx4 v[58:61], v198, s[76:79], s4 offen\n\ts_endpgm\n") == []
    narrow = "\tbuffer_store_dwordx2 v[58:59], v198, s[76:79], s4 offen nt\n"
    assert isa_check.check_text(narrow + "\tv_mul_f32_e32 v59, 2.0, v59\n\ts_endpgm\n") == []


def test_labels_fall_through_and_branches_are_followed():
    asm = STORE + ".LBB0_1:\n\tv_mov_b64_e32 v[60:61], v[2:3]\n\ts_endpgm\n"
    assert len(isa_check.check_text(asm)) == 1
    asm = (STORE + "\ts_cbranch_vccnz .LBB0_7\n\ts_nop 3\n\ts_endpgm\n"
           ".LBB0_7:\n\tv_add_f32_e32 v58, 1.0, v58\n\ts_endpgm\n")
    assert len(isa_check.check_text(asm)) == 1


def test_global_store_names_its_data_second():
    asm = "\tglobal_store_dwordx4 v[12:13], v[26:29], off nt\n\tv_mov_b32_e32 v12, 0\n\tv_mov_b32_e32 v27, 0\n\ts_endpgm\n"
    found = isa_check.check_text(asm)
    assert len(found) == 1 and "v[27]" in found[0]


def test_packed_fp32_arithmetic_is_reported():
    assert len(isa_check.check_text("\tv_pk_fma_f32 v[0:1], v[2:3], v[4:5], v[6:7]\n\ts_endpgm\n")) == 1
    assert isa_check.check_text("\tv_pk_mov_b32 v[0:1], v[2:3], v[4:5]\n\tv_cvt_pk_bf16_f32 v0, v1, v2\n\ts_endpgm\n") == []


@pytest.mark.skipif(shutil.which(lr_build.HIPCC) is None and not os.path.exists(lr_build.HIPCC), reason="needs hipcc")
def test_the_check_finds_the_hazard_in_real_compiler_output(tmp_path):
    """Tile 3 (four columns, 8 rows per thread) compiled to assembly twice, with every kernel its geometry allows
    (the measured selection builds it for bf16 storage only, where no store is 128 bits wide): as the library
    builds it, and with the pause behind the 128-bit stores of the gated forms taken out.  The first passes the
    check; in the second the compiler schedules the next row's arithmetic into the registers just stored, and
    the check says so."""
    def asm(extra, name):
        out = str(tmp_path / name)
        cmd = [lr_build.HIPCC] + lr_build.FLAGS + ["-DLINREC_TILE_ID=3", "-DLINREC_ALL_SHAPES"] + extra + [
            "-S", "--cuda-device-only", os.path.join(lr_build.CSRC, "linrec_tiles.hip"), "-o", out]
        p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert p.returncode == 0, p.stdout[-2000:]
        with open(out) as f:
            return f.read()

    with ThreadPoolExecutor(max_workers=2) as ex:
        good, bad = ex.map(lambda a: asm(*a), [([], "with_pause.s"), (["-DLINREC_NO_STORE_PAUSE"], "without_pause.s")])
    assert "buffer_store_dwordx4" in good and isa_check.check_text(good, "tile 3") == []
    found = isa_check.check_text(bad, "tile 3 without the pause")
    assert len(found) >= 10 and all("data of the store" in m for m in found)
