"""The streamed GEMM kernels, compiled for gfx950, never touch a register that an LDS read in flight will still
write, and never touch an accumulation register right behind the MFMA that writes it (see asm_check.py: both are
hazards the compiler cannot see, because the reads and the MFMAs are issued from inline assembly).  Compiles
csrc/gemm.hip to device assembly (about a minute and a half) and walks every instantiation of k_gemm_dma,
k_gemm_dma4 and k_gemm_dma64."""
import os
import shutil
import subprocess

import pytest

import asm_check

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_checker_finds_a_planted_hazard_and_accepts_the_waited_form():
    bad = """_Z4demov:
	ds_read_b128 v[10:13], v2 offset:0
	ds_read_b128 v[14:17], v2 offset:1024
	s_waitcnt lgkmcnt(1)
	v_mfma_f32_16x16x32_f16 a[0:3], v[10:13], v[20:23], a[0:3]
	v_lshl_add_u64 v[14:15], v[30:31], 0, s[4:5]
	global_load_lds_dwordx4 v[14:15], off
	s_endpgm
"""
    (name, lines), = list(asm_check.kernels(bad, "demo"))
    msgs = [m for _, m in asm_check.check_kernel(lines)]
    assert len(msgs) == 2 and "writes v[14, 15]" in msgs[0] and "reads v[14, 15]" in msgs[1]
    good = bad.replace("s_waitcnt lgkmcnt(1)", "s_waitcnt lgkmcnt(0)")
    (name, lines), = list(asm_check.kernels(good, "demo"))
    assert asm_check.check_kernel(lines) == []
    # reading a fragment that has not been waited for is reported too
    early = bad.replace("	s_waitcnt lgkmcnt(1)\n", "")
    (name, lines), = list(asm_check.kernels(early, "demo"))
    assert any("reads v[10, 11, 12, 13]" in m for _, m in asm_check.check_kernel(lines))


def test_accumulator_checker_finds_a_copy_right_behind_an_mfma():
    bad = """_Z4demov:
	v_mfma_f32_16x16x32_f16 a[0:3], v[2:5], v[6:9], a[0:3]
	v_mfma_f32_16x16x32_f16 a[4:7], v[2:5], v[6:9], a[4:7]
	s_nop 1
	v_accvgpr_mov_b32 a8, a4
	s_endpgm
"""
    (name, lines), = list(asm_check.kernels(bad, "demo"))
    msgs = [m for _, m in asm_check.check_accumulator_reads(lines)]
    assert len(msgs) == 1 and "a[4]" in msgs[0]
    good = bad.replace("s_nop 1\n", "s_nop 15\n\ts_nop 15\n")
    (name, lines), = list(asm_check.kernels(good, "demo"))
    assert asm_check.check_accumulator_reads(lines) == []
    # the accumulator of the first MFMA is 16 cycles older: a copy of it after one more MFMA and 16 idle cycles is fine
    older = bad.replace("v_accvgpr_mov_b32 a8, a4", "v_accvgpr_mov_b32 a8, a0").replace("s_nop 1\n", "s_nop 15\n")
    (name, lines), = list(asm_check.kernels(older, "demo"))
    assert asm_check.check_accumulator_reads(lines) == []


def test_streamed_gemm_kernels_keep_in_flight_read_registers_untouched(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("no hipcc")
    from paper_1710_03740_amd import build as mpt_build
    out = tmp_path / "gemm.s"
    flags = [f for f in mpt_build.HIP_FLAGS if f != "-fPIC"]
    cmd = [hipcc] + flags + ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_1710_03740_amd", "csrc"),
                             "-x", "hip", "-S", "--cuda-device-only", "-o", str(out),
                             os.path.join(ROOT, "paper_1710_03740_amd", "csrc", "gemm.hip")]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-2000:]
    n = 0
    for name, lines in asm_check.kernels(out.read_text(), r"k_gemm_dma"):
        found = asm_check.check_kernel(lines)
        assert not found, "%s: %s" % (name, found[:5])
        found = asm_check.check_accumulator_reads(lines)
        assert not found, "%s: %s" % (name, found[:5])
        assert sum("v_mfma" in l for l in lines) >= 64          # it is the kernel body that was walked
        n += 1
    assert n >= 15                                               # every instantiation of the three streamed kernels
