"""Thin ctypes binding of libgrkan.so: argument marshalling only.

Every step of the forward and backward pass runs in the HIP kernels behind the
C ABI declared in include/grkan.h.  torch supplies device memory and the
current stream; nothing here computes.  There is no CPU fallback: if the
library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
from pathlib import Path
from typing import Optional, Tuple

_PKG = Path(__file__).resolve().parent
LIB_PATH = _PKG / "libgrkan.so"

GRKAN_F32 = 0
GRKAN_BF16 = 1
GRKAN_F16 = 2
M_DEGREE = 5  # the paper's degrees; (3, 2) and (7, 6) are built too
N_DEGREE = 4
DEGREES = ((5, 4), (3, 2), (7, 6))

_lib = None
_ws_bytes_cache = {}


class GrkanError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__("%s: %s (status %d)" % (where, status_string(status), status))


class Plan(ctypes.Structure):
    _fields_ = [
        ("vec", ctypes.c_int32),
        ("vecs_per_segment", ctypes.c_int32),
        ("waves_per_wg", ctypes.c_int32),
        ("groups_per_wg", ctypes.c_int32),
        ("waves_per_group_in_wg", ctypes.c_int32),
        ("wg_per_bundle", ctypes.c_int32),
        ("grid", ctypes.c_int32),
        ("fixed_col", ctypes.c_int32),
        ("chunk_stride", ctypes.c_int64),
        ("partials_per_group", ctypes.c_int32),
        ("lane_coef", ctypes.c_int32),
        ("column_split", ctypes.c_int32),
    ]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


def load_library():
    """Load libgrkan.so (built in-tree by paper_2505_13813_amd/build.py)."""
    global _lib
    if _lib is not None:
        return _lib
    if not LIB_PATH.exists():
        # nothing built yet: build once (hipcc cross-compiles without a GPU).  There is no
        # fallback path: if this fails, loading fails.
        from . import build as _build

        _build.build_library(force=True)
    # torch first: it ships its own copy of the HIP runtime under the same soname as the
    # system's.  Whichever is loaded first serves the whole process, and the tensors this
    # library is handed live in torch's; loaded the other way round, launches on them fail.
    import torch  # noqa: F401

    lib = ctypes.CDLL(str(LIB_PATH))
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
    lib.grkan_status_string.argtypes = [ctypes.c_int]
    lib.grkan_status_string.restype = ctypes.c_char_p
    lib.grkan_plan.argtypes = [i64, i32, i32, ctypes.c_int, i32, i32, i32, i32, ctypes.POINTER(Plan)]
    lib.grkan_plan.restype = ctypes.c_int
    lib.grkan_plan_cover_errors.argtypes = [i64, i32, i32, ctypes.c_int, ctypes.POINTER(Plan)]
    lib.grkan_plan_cover_errors.restype = i64
    lib.grkan_device_query.argtypes = [ctypes.POINTER(ctypes.c_int32)]
    lib.grkan_device_query.restype = ctypes.c_int
    lib.grkan_tuning_override.argtypes = [i32, i32]
    lib.grkan_tuning_override.restype = None
    lib.grkan_bwd_workspace_bytes.argtypes = [i64, i32, i32, ctypes.c_int]
    lib.grkan_bwd_workspace_bytes.restype = sz
    lib.grkan_fwd.argtypes = [vp, vp, vp, vp, i64, i32, i32, i32, i32, ctypes.c_int, vp]
    lib.grkan_fwd.restype = ctypes.c_int
    lib.grkan_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, sz, i64, i32, i32, i32, i32, ctypes.c_int, vp]
    lib.grkan_bwd.restype = ctypes.c_int
    lib.grkan_linear_fwd.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, i32, i32, ctypes.c_int, ctypes.c_int, vp]
    lib.grkan_linear_fwd.restype = ctypes.c_int
    lib.grkan_linear_fwd_packed.argtypes = lib.grkan_linear_fwd.argtypes
    lib.grkan_linear_fwd_packed.restype = ctypes.c_int
    lib.grkan_linear_packed_w_bytes.argtypes = [i32, i32]
    lib.grkan_linear_packed_w_bytes.restype = ctypes.c_size_t
    lib.grkan_linear_pack_w.argtypes = [vp, vp, i32, i32, vp]
    lib.grkan_linear_pack_w.restype = ctypes.c_int
    lib.grkan_bwd_noalloc.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i32, i32, i32, i32, ctypes.c_int, vp]
    lib.grkan_bwd_noalloc.restype = ctypes.c_int
    lib.grkan_alg1_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i32, i32, vp]
    lib.grkan_alg1_bwd.restype = ctypes.c_int
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().grkan_status_string(int(status)).decode()


def plan(rows: int, D: int, G: int, io: int = GRKAN_F32, align_bytes: int = 16,
         num_cu: int = 256, wg_per_cu: int = 4, forward: bool = False) -> Plan:
    """Host-only: the launch geometry of the backward (default) or forward pass
    for a shape (see grkan_plan in grkan.h)."""
    p = Plan()
    st = load_library().grkan_plan(rows, D, G, io, align_bytes, num_cu, wg_per_cu, 1 if forward else 0,
                                   ctypes.byref(p))
    if st:
        raise GrkanError(st, "grkan_plan")
    return p


def plan_cover_errors(rows: int, D: int, G: int, io: int, p: Plan) -> int:
    return int(load_library().grkan_plan_cover_errors(rows, D, G, io, ctypes.byref(p)))


# ---------------------------------------------------------------- raw pointer level
def device_query() -> dict:
    """Compute units, engine clock, memory clock (kHz) and memory bus width (bits) of the current device."""
    out = (ctypes.c_int32 * 4)()
    st = load_library().grkan_device_query(out)
    if st != 0:
        raise GrkanError(st, "grkan_device_query")
    return {"compute_units": out[0], "engine_clock_khz": out[1], "memory_clock_khz": out[2], "memory_bus_bits": out[3]}


def tuning_override(fwd_wg_per_cu: int = 0, bwd_wg_per_cu: int = 0) -> None:
    """Experiments and tests: size the persistent grids for this many workgroups per
    compute unit (0 = the built-in choice).  Cached workspace sizes are dropped."""
    load_library().grkan_tuning_override(int(fwd_wg_per_cu), int(bwd_wg_per_cu))
    _ws_bytes_cache.clear()


def grkan_bwd_workspace_bytes(rows: int, D: int, G: int, io: int) -> int:
    return int(load_library().grkan_bwd_workspace_bytes(rows, D, G, io))


def grkan_fwd_raw(x_ptr, A_ptr, B_ptr, y_ptr, rows, D, G, io, stream_ptr, m=M_DEGREE, n=N_DEGREE) -> int:
    return int(load_library().grkan_fwd(x_ptr, A_ptr, B_ptr, y_ptr, rows, D, G, m, n, io, stream_ptr))


def grkan_bwd_raw(x_ptr, dy_ptr, A_ptr, B_ptr, dx_ptr, dA_ptr, dB_ptr, ws_ptr, ws_bytes,
                  rows, D, G, io, stream_ptr, m=M_DEGREE, n=N_DEGREE) -> int:
    return int(load_library().grkan_bwd(x_ptr, dy_ptr, A_ptr, B_ptr, dx_ptr, dA_ptr, dB_ptr,
                                        ws_ptr, ws_bytes, rows, D, G, m, n, io, stream_ptr))


# ---------------------------------------------------------------- torch tensors
def _io_of(t) -> int:
    import torch

    if t.dtype == torch.float32:
        return GRKAN_F32
    if t.dtype == torch.bfloat16:
        return GRKAN_BF16
    if t.dtype == torch.float16:
        return GRKAN_F16
    raise TypeError("x must be float32, bfloat16 or float16, got %s" % t.dtype)


def _check(x, A, B) -> Tuple[int, int, int]:
    import torch

    if not x.is_cuda or A.device != x.device or B.device != x.device:
        raise ValueError("grkan runs on the GPU only: tensors must be on one HIP device")
    if not x.is_contiguous() or not A.is_contiguous() or not B.is_contiguous():
        raise ValueError("tensors must be contiguous")
    if A.dtype != torch.float32 or B.dtype != torch.float32:
        raise TypeError("A and B must be float32")
    if A.dim() != 2 or B.dim() != 2 or A.shape[0] != B.shape[0]:
        raise ValueError("A must be [G, m+1] and B [G, n]")
    if x.dim() < 1:
        raise ValueError("x needs at least one dimension")
    D = int(x.shape[-1])
    rows = int(x.numel() // D) if D else 0
    return rows, D, int(A.shape[0])


def _stream_ptr(stream=None):
    import torch

    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def grkan_fwd(x, A, B, out=None, stream=None):
    """y = F(x) group-wise (FlashKAT paper, Eq. "pade").  Enqueues on the current stream."""
    import torch

    rows, D, G = _check(x, A, B)
    y = torch.empty_like(x) if out is None else out
    if y.shape != x.shape or y.dtype != x.dtype or not y.is_contiguous() or y.device != x.device:
        raise ValueError("out must match x")
    st = grkan_fwd_raw(x.data_ptr(), A.data_ptr(), B.data_ptr(), y.data_ptr(), rows, D, G, _io_of(x),
                       _stream_ptr(stream), int(A.shape[1]) - 1, int(B.shape[1]))
    if st:
        raise GrkanError(st, "grkan_fwd")
    return y


def _workspace_bytes_cached(rows: int, D: int, G: int, io: int, device_index: int) -> int:
    """grkan_bwd_workspace_bytes plans the launch for every built degree pair and
    alignment; the answer depends on (shape, dtype, device) only, so it is kept."""
    key = (rows, D, G, io, device_index)
    need = _ws_bytes_cache.get(key)
    if need is None:
        need = grkan_bwd_workspace_bytes(rows, D, G, io)
        if need == 0:
            raise GrkanError(7, "grkan_bwd_workspace_bytes")
        _ws_bytes_cache[key] = need
    return need


def _check_bwd_outputs(x, A, B, dx, dA, dB):
    import torch

    if dx.shape != x.shape or dx.dtype != x.dtype or not dx.is_contiguous() or dx.device != x.device:
        raise ValueError("dx must match x in shape, dtype, device and be contiguous")
    for name, t, like in (("dA", dA, A), ("dB", dB, B)):
        if t.shape != like.shape or t.dtype != torch.float32 or not t.is_contiguous() or t.device != x.device:
            raise ValueError("%s must be a contiguous float32 tensor of the shape of %s on the device of x"
                             % (name, name[1:]))


def grkan_bwd(x, dy, A, B, workspace: Optional["torch.Tensor"] = None, out=None, stream=None):
    """(dx, dA, dB) of the group-wise rational function (Eq. "grad_x", "grad_a",
    "grad_b", "accum", "accum2").  dA, dB are float32 and overwritten.

    `workspace`: a contiguous uint8 tensor on the device of x of at least
    grkan_bwd_workspace_bytes(...) bytes (the library checks the size); one is
    allocated when none is passed."""
    import torch

    rows, D, G = _check(x, A, B)
    if dy.shape != x.shape or dy.dtype != x.dtype or not dy.is_contiguous() or dy.device != x.device:
        raise ValueError("dy must match x")
    io = _io_of(x)
    if out is None:
        dx = torch.empty_like(x)
        dA = torch.empty_like(A)
        dB = torch.empty_like(B)
    else:
        dx, dA, dB = out
        _check_bwd_outputs(x, A, B, dx, dA, dB)
    if workspace is None:
        need = _workspace_bytes_cached(rows, D, G, io, x.device.index or 0)
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    elif (workspace.dtype != torch.uint8 or not workspace.is_contiguous() or workspace.device != x.device
          or workspace.dim() != 1):
        raise ValueError("workspace must be a contiguous one-dimensional uint8 tensor on the device of x")
    st = grkan_bwd_raw(x.data_ptr(), dy.data_ptr(), A.data_ptr(), B.data_ptr(), dx.data_ptr(),
                       dA.data_ptr(), dB.data_ptr(), workspace.data_ptr(), workspace.numel(),
                       rows, D, G, io, _stream_ptr(stream), int(A.shape[1]) - 1, int(B.shape[1]))
    if st:
        raise GrkanError(st, "grkan_bwd")
    return dx, dA, dB


class PackedWeight:
    """The packed copy grkan_linear_pack_w makes of a [D_out, D_in] bfloat16 weight matrix (opaque
    bytes on the device) with the shape it was made from."""

    def __init__(self, data, D_out: int, D_in: int):
        self.data, self.D_out, self.D_in = data, int(D_out), int(D_in)


def grkan_linear_pack_w(W, stream=None) -> PackedWeight:
    """Packed copy of the weights for grkan_linear_fwd (weights that stay the same between calls):
    the layer kernel then fetches them in whole cache lines.  One small kernel; allocates the copy."""
    import torch

    if W.dtype != torch.bfloat16 or W.dim() != 2 or not W.is_contiguous() or not W.is_cuda:
        raise ValueError("W must be a contiguous bfloat16 [D_out, D_in] tensor on the GPU")
    D_out, D_in = int(W.shape[0]), int(W.shape[1])
    need = int(load_library().grkan_linear_packed_w_bytes(D_in, D_out))
    if need == 0:
        raise GrkanError(8, "grkan_linear_packed_w_bytes")
    data = torch.empty(need, dtype=torch.uint8, device=W.device)
    st = int(load_library().grkan_linear_pack_w(W.data_ptr(), data.data_ptr(), D_in, D_out, _stream_ptr(stream)))
    if st:
        raise GrkanError(st, "grkan_linear_pack_w")
    return PackedWeight(data, D_out, D_in)


def grkan_linear_fwd(x, A, B, W, bias=None, out=None, out_dtype=None, stream=None):
    """out = F(x) W^T (+ bias): the GR-KAN layer in one kernel (Eq. "GR_KAN").  x bfloat16; W a
    bfloat16 [D_out, D_in] tensor or its PackedWeight; bias float32 or None; out bfloat16 (default)
    or float32."""
    import torch

    rows, D_in, G = _check(x, A, B)
    packed = isinstance(W, PackedWeight)
    if packed:
        if x.dtype != torch.bfloat16:
            raise TypeError("x must be bfloat16")
        if W.D_in != D_in or W.data.device != x.device:
            raise ValueError("the packed weights were made for another D_in or device")
        D_out, w_ptr = W.D_out, W.data.data_ptr()
    else:
        if x.dtype != torch.bfloat16 or W.dtype != torch.bfloat16:
            raise TypeError("x and W must be bfloat16")
        if W.dim() != 2 or W.shape[1] != D_in or not W.is_contiguous() or W.device != x.device:
            raise ValueError("W must be a contiguous [D_out, D_in] tensor on the device of x")
        D_out, w_ptr = int(W.shape[0]), W.data_ptr()
    if bias is not None and (bias.dtype != torch.float32 or bias.shape != (D_out,) or not bias.is_contiguous()
                             or bias.device != x.device):
        raise ValueError("bias must be a contiguous float32 [D_out] tensor on the device of x")
    if out is None:
        out = torch.empty(x.shape[:-1] + (D_out,), dtype=out_dtype or torch.bfloat16, device=x.device)
    if (out.dtype not in (torch.bfloat16, torch.float32) or out.shape != x.shape[:-1] + (D_out,)
            or not out.is_contiguous() or out.device != x.device):
        raise ValueError("out must be a contiguous bfloat16 or float32 [..., D_out] tensor on the device of x")
    lib = load_library()
    entry = lib.grkan_linear_fwd_packed if packed else lib.grkan_linear_fwd
    st = int(entry(
        x.data_ptr(), A.data_ptr(), B.data_ptr(), w_ptr, bias.data_ptr() if bias is not None else None,
        out.data_ptr(), rows, D_in, D_out, G, int(A.shape[1]) - 1, int(B.shape[1]), GRKAN_BF16,
        GRKAN_BF16 if out.dtype == torch.bfloat16 else GRKAN_F32, _stream_ptr(stream)))
    if st:
        raise GrkanError(st, "grkan_linear_fwd_packed" if packed else "grkan_linear_fwd")
    return out


NOALLOC_SCRATCH_BYTES = 4 << 20


def grkan_bwd_noalloc(x, dy, A, B, out, stream=None):
    """grkan_bwd without a workspace argument and without any allocation: the
    caller passes every output (`out` = (dx, dA, dB)); the workspace rows live in
    the library's fixed 4 MiB device array.  Calls that overlap on one GPU race."""
    rows, D, G = _check(x, A, B)
    if dy.shape != x.shape or dy.dtype != x.dtype or not dy.is_contiguous() or dy.device != x.device:
        raise ValueError("dy must match x")
    dx, dA, dB = out
    _check_bwd_outputs(x, A, B, dx, dA, dB)
    st = int(load_library().grkan_bwd_noalloc(x.data_ptr(), dy.data_ptr(), A.data_ptr(), B.data_ptr(), dx.data_ptr(),
                                              dA.data_ptr(), dB.data_ptr(), rows, D, G, int(A.shape[1]) - 1,
                                              int(B.shape[1]), _io_of(x), _stream_ptr(stream)))
    if st:
        raise GrkanError(st, "grkan_bwd_noalloc")
    return dx, dA, dB


def grkan_alg1_bwd(x, dy, A, B, out=None, stream=None):
    """The paper's Algorithm 1 (per-element global atomics), float32 only: a
    measurement baseline, not the product path (see include/grkan_alg1.h)."""
    import torch

    rows, D, G = _check(x, A, B)
    if x.dtype != torch.float32 or dy.dtype != torch.float32 or dy.shape != x.shape or not dy.is_contiguous():
        raise TypeError("the Algorithm 1 baseline takes contiguous float32 x and dy of one shape")
    if int(A.shape[1]) != M_DEGREE + 1 or int(B.shape[1]) != N_DEGREE:
        raise GrkanError(3, "grkan_alg1_bwd")
    if out is None:
        out = (torch.empty_like(x), torch.empty_like(A), torch.empty_like(B))
    dx, dA, dB = out
    st = load_library().grkan_alg1_bwd(x.data_ptr(), dy.data_ptr(), A.data_ptr(), B.data_ptr(), dx.data_ptr(),
                                       dA.data_ptr(), dB.data_ptr(), rows, D, G, _stream_ptr(stream))
    if st:
        raise GrkanError(st, "grkan_alg1_bwd")
    return dx, dA, dB
