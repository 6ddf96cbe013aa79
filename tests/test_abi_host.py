"""The C ABI without a GPU: the library loads, exports every symbol that
include/grkan.h declares, and rejects bad arguments before touching HIP."""
import ctypes
import re
from pathlib import Path

import pytest

import paper_2505_13813_amd as grkan
from paper_2505_13813_amd import GRKAN_F32, binding

ROOT = Path(__file__).resolve().parent.parent


def declared_functions():
    names = set()
    for header in sorted((ROOT / "include").glob("*.h")):
        text = re.sub(r"/\*.*?\*/", "", header.read_text(), flags=re.S)
        names.update(re.findall(r"\b(grkan_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_expected_entry_points():
    names = declared_functions()
    for n in ("grkan_fwd", "grkan_bwd", "grkan_bwd_workspace_bytes", "grkan_plan",
              "grkan_plan_cover_errors", "grkan_status_string", "grkan_alg1_bwd", "grkan_bwd_noalloc",
              "grkan_tuning_override", "grkan_linear_fwd", "grkan_linear_fwd_packed", "grkan_linear_pack_w",
              "grkan_linear_packed_w_bytes"):
        assert n in names


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(str(binding.LIB_PATH))
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_status_strings():
    seen = set()
    for code in range(0, 10):
        s = grkan.status_string(code)
        assert s and s not in seen
        seen.add(s)
    assert grkan.status_string(0) == "ok"
    assert grkan.status_string(99) == "unknown status"


def test_plan_struct_matches_the_header():
    text = (ROOT / "include" / "grkan.h").read_text()
    body = re.search(r"typedef struct \{(.*?)\} grkan_plan_t;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"(int32_t|int64_t)\s+([a-z_0-9]+)\s*;", body)
    ctype = {"int32_t": ctypes.c_int32, "int64_t": ctypes.c_int64}
    assert [(n, ctype[t]) for t, n in fields] == list(grkan.Plan._fields_)


FWD_BAD = [
    # (x, A, B, y, rows, D, G, m, n, io) -> status
    ((16, 16, 16, 16, 4, 192, 8, 4, 4, 0), 3),   # degree
    ((16, 16, 16, 16, 4, 192, 8, 5, 3, 0), 3),
    ((16, 16, 16, 16, 4, 190, 8, 5, 4, 0), 2),   # D % G
    ((16, 16, 16, 16, -4, 192, 8, 5, 4, 0), 2),
    ((16, 16, 16, 16, 4, 192, 8, 5, 4, 5), 6),   # dtype
    ((0, 16, 16, 16, 4, 192, 8, 5, 4, 0), 1),    # null x
    ((16, 0, 16, 16, 4, 192, 8, 5, 4, 0), 1),    # null A
    ((16, 16, 16, 0, 4, 192, 8, 5, 4, 0), 1),    # null y
    ((18, 16, 16, 16, 4, 192, 8, 5, 4, 0), 4),   # x not 4-byte aligned
    ((17, 16, 16, 16, 4, 192, 8, 5, 4, 1), 4),   # bf16 x not 2-byte aligned
    ((16, 18, 16, 16, 4, 192, 8, 5, 4, 0), 4),   # A not 4-byte aligned
]


@pytest.mark.parametrize("args,status", FWD_BAD)
def test_fwd_rejects_bad_arguments_before_any_launch(args, status):
    x, A, B, y, rows, D, G, m, n, io = args
    st = grkan.grkan_fwd_raw(x, A, B, y, rows, D, G, io, None, m, n)
    assert st == status


def test_bwd_rejects_bad_arguments_before_any_launch():
    ok = dict(x=16, dy=16, A=16, B=16, dx=16, dA=16, dB=16, ws=16, wsb=1 << 20, rows=4, D=192, G=8, io=GRKAN_F32)

    def call(**kw):
        a = dict(ok, **kw)
        return grkan.grkan_bwd_raw(a["x"], a["dy"], a["A"], a["B"], a["dx"], a["dA"], a["dB"], a["ws"], a["wsb"],
                                   a["rows"], a["D"], a["G"], a["io"], None, a.get("m", 5), a.get("n", 4))

    assert call(m=6) == 3
    assert call(D=100) == 2
    assert call(dy=0) == 1
    assert call(dA=0) == 1
    assert call(dB=0) == 1
    assert call(dx=18) == 4
    assert call(dA=18) == 4
    assert call(io=9) == 6


def test_binding_refuses_cpu_tensors():
    import torch

    x = torch.zeros(4, 192)
    A = torch.zeros(8, 6)
    B = torch.zeros(8, 4)
    with pytest.raises(ValueError):
        grkan.grkan_fwd(x, A, B)
    with pytest.raises(ValueError):
        grkan.grkan_bwd(x, x, A, B)


def test_headers_are_plain_c(tmp_path):
    """The boundary is a C ABI: both headers must compile as C99 on their own,
    in either order, with a call site for every entry point."""
    import shutil
    import subprocess

    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_abi.c"
    src.write_text(
        '#include "grkan_alg1.h"\n#include "grkan.h"\n'
        "int use(void *p, float *f, void *s) {\n"
        "  grkan_plan_t pl; int32_t q[4];\n"
        "  grkan_status_t st = grkan_plan(1, 8, 1, GRKAN_F16, 16, 256, 2, 0, &pl);\n"
        "  st = grkan_fwd(p, f, f, p, 1, 8, 1, 5, 4, GRKAN_F32, s);\n"
        "  st = grkan_bwd(p, p, f, f, p, f, f, p, grkan_bwd_workspace_bytes(1, 8, 1, GRKAN_BF16), 1, 8, 1, 5, 4, GRKAN_BF16, s);\n"
        "  st = grkan_alg1_bwd(p, p, f, f, p, f, f, 1, 8, 1, s);\n"
        "  st = grkan_device_query(q);\n"
        "  return (int)st + (int)grkan_plan_cover_errors(1, 8, 1, GRKAN_F32, &pl) + (grkan_status_string(st) != 0);\n"
        "}\n")
    res = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only",
                          "-I", str(ROOT / "include"), str(src)], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr


def test_device_query_rejects_a_null_pointer():
    lib = grkan.load_library()
    assert lib.grkan_device_query(None) == 1


def test_packed_weight_size_is_host_arithmetic():
    """grkan_linear_packed_w_bytes needs no GPU: (D_in / 32) stages x 16-row tiles of whole channel blocks x 1 KB."""
    lib = binding.load_library()
    f = lib.grkan_linear_packed_w_bytes
    assert f(3072, 768) == (3072 // 32) * (768 // 16) * 1024 == 2 * 768 * 3072     # nothing padded
    assert f(768, 3072) == 2 * 768 * 3072
    assert f(1536, 384) == 2 * 1536 * 384
    assert f(256, 200) == (256 // 32) * (384 // 16) * 1024                            # 200 -> two blocks of 192
    assert f(64, 4) == (64 // 32) * (192 // 16) * 1024
    assert f(100, 768) == 0 and f(3072, 770) == 0 and f(0, 768) == 0 and f(3072, -4) == 0
    assert lib.grkan_linear_pack_w(None, None, 3072, 768, None) == 1                  # null pointers
    assert lib.grkan_linear_pack_w(None, None, 100, 768, None) == 8                   # shape not covered
