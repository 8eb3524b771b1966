"""The streaming kernels load with inline asm and wait explicitly; the compiler must not have put a
spill or a register copy between such a load and its wait.  This compiles the library's device code
to assembly (no GPU needed) and runs the static check that ships next to the kernels."""
import os
import subprocess
import sys

import pytest

from paper_2505_07829_amd import build as bb_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2505_07829_amd", "csrc")
KERNELS = ["_ZN2bb17ffn_stream_kernelILi1EEEvNS_10StreamArgsE", "_ZN2bb17ffn_stream_kernelILi2EEEvNS_10StreamArgsE",
           "_ZN2bb19ffn_stream_t_kernelENS_11StreamTArgsE"]


def test_no_instruction_touches_a_register_whose_load_is_in_flight(tmp_path):
    # the compiler and the flags of the shipped build (paper_2505_07829_amd/build.py), device code to assembly
    assert os.path.exists(bb_build.HIPCC), f"{bb_build.HIPCC} not found: the check cannot run"
    asm = tmp_path / "bb_stream_inst.s"
    cmd = [bb_build.HIPCC, *bb_build.HIPCC_FLAGS, "-S", "--cuda-device-only", "-o", str(asm),
           os.path.join(CSRC, "bb_stream_inst.hip")]
    subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL, timeout=900)
    r = subprocess.run([sys.executable, os.path.join(CSRC, "check_inflight.py"), str(asm)] + KERNELS,
                       capture_output=True, text=True, timeout=300)
    print(r.stdout)
    assert r.returncode == 0, r.stdout + r.stderr
    for k in KERNELS:
        assert f"{k}: 0 suspicious" in r.stdout


def test_checker_follows_loads_into_accumulation_registers(tmp_path):
    # the row-major kernel's queue lives in accumulation registers: a move out of one before the wait is reported
    text = """k:
\t;;#ASMSTART
\tglobal_load_dwordx4 a[4:7], v[0:1], off nt
\t;;#ASMEND
\tv_accvgpr_mov_b32 a20, a5
\tv_accvgpr_read_b32 v9, a6
\t;;#ASMSTART
\ts_waitcnt vmcnt(0)
\t;;#ASMEND
\tv_accvgpr_read_b32 v10, a5
\ts_endpgm
"""
    f = tmp_path / "k.s"
    f.write_text(text)
    r = subprocess.run([sys.executable, os.path.join(CSRC, "check_inflight.py"), str(f), "k"], capture_output=True,
                       text=True)
    assert r.returncode == 1 and "k: 2 suspicious" in r.stdout


def test_checker_flags_a_planted_copy(tmp_path):
    # a copy of a register between its asm load and the wait must be reported; after the wait it must not
    text = """k:
\t;;#ASMSTART
\tglobal_load_dwordx4 v[4:7], v[0:1], off nt
\t;;#ASMEND
\tv_mov_b32_e32 v9, v5
\t;;#ASMSTART
\ts_waitcnt vmcnt(0)
\t;;#ASMEND
\tv_mov_b32_e32 v10, v5
\ts_endpgm
"""
    f = tmp_path / "k.s"
    f.write_text(text)
    r = subprocess.run([sys.executable, os.path.join(CSRC, "check_inflight.py"), str(f), "k"], capture_output=True,
                       text=True)
    assert r.returncode == 1 and "k: 1 suspicious" in r.stdout
