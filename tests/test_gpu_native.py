"""The C ABI used without Python: tests/native/abi_selftest.cpp is compiled with
hipcc against include/grkan.h, linked with libgrkan.so and with the C oracle as
its checker, and run as a program of its own."""
import shutil
import subprocess
from pathlib import Path

import pytest

pytestmark = pytest.mark.gpu

ROOT = Path(__file__).resolve().parent.parent
SRC = ROOT / "tests" / "native" / "abi_selftest.cpp"


def build_selftest(out_dir: Path) -> Path:
    from paper_2505_13813_amd import binding

    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    gcc = shutil.which("gcc")
    if not Path(hipcc).exists() or gcc is None:
        pytest.skip("no hipcc / gcc on this machine")
    if not binding.LIB_PATH.exists():
        raise RuntimeError("libgrkan.so is not built")
    oracle_obj = out_dir / "grkan_oracle.o"
    subprocess.run([gcc, "-O2", "-std=c99", "-fopenmp", "-c", str(ROOT / "oracle" / "grkan_oracle.c"), "-o",
                    str(oracle_obj)], check=True, capture_output=True, text=True)
    # compile and link in two steps: with a .cpp on the line hipcc would read the objects as HIP source too
    main_obj = out_dir / "abi_selftest.o"
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", "-I", str(ROOT / "include"), "-c",
                          str(SRC), "-o", str(main_obj)], capture_output=True, text=True)
    assert res.returncode == 0, res.stdout + res.stderr
    exe = out_dir / "abi_selftest"
    res = subprocess.run([hipcc, str(main_obj), str(oracle_obj), str(binding.LIB_PATH), "-fopenmp",
                          "-Wl,-rpath," + str(binding.LIB_PATH.parent), "-o", str(exe)],
                         capture_output=True, text=True)
    assert res.returncode == 0, res.stdout + res.stderr
    return exe


def test_c_program_calls_the_abi_and_matches_the_oracle(tmp_path):
    exe = build_selftest(tmp_path)
    res = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300)
    print(res.stdout)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "all cases within tolerance" in res.stdout
