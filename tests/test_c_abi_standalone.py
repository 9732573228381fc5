"""The C-ABI used from plain C, with the system HIP runtime and no Python in the
process: build tests/c/abi_parity.c against include/sparbit.h, libsparbit.so
and the oracle's shared object, and run it."""
import os
import subprocess

import pytest

import oracle
import paper_2109_08751_amd as sb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "tests", "c", "abi_parity.c")
EXE = os.path.join(ROOT, "tests", "c", "abi_parity")


def build_exe():
    lib_dir = os.path.dirname(sb.lib_path())
    ora_dir = os.path.dirname(oracle.build())
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c11", "-Wall", "-O1", SRC, "-o", EXE, "-I", os.path.join(ROOT, "include"),
           "-I", os.path.join(rocm, "include"), "-D__HIP_PLATFORM_AMD__",
           "-L", lib_dir, "-lsparbit", "-L", ora_dir, "-loracle", "-L", os.path.join(rocm, "lib"), "-lamdhip64",
           f"-Wl,-rpath,{lib_dir}", f"-Wl,-rpath,{ora_dir}", f"-Wl,-rpath,{os.path.join(rocm, 'lib')}"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stdout + res.stderr
    return EXE


def test_c_program_builds_against_the_header():
    """Compiles and links on the CPU machine: the header is plain C and every symbol resolves."""
    assert os.path.exists(build_exe())


@pytest.mark.gpu
@pytest.mark.parametrize("p,B,algo", [(6, 1024, 0), (96, 4096, 0), (33, 52, 0), (64, 65536, 0), (16, 4096, 2),
                                      (21, 4096, 1), (21, 4096, 3), (21, 4096, 4), (128, 1028, 0), (257, 1040, 0),
                                      (64, 4100, 2), (256, 128, 0)])
def test_c_program_matches_oracle_on_gpu(p, B, algo):
    exe = EXE if os.path.exists(EXE) else build_exe()
    print("[case] abi_parity", p, B, algo, flush=True)
    out = subprocess.run([exe, str(p), str(B), str(algo)], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "match" in out.stdout
