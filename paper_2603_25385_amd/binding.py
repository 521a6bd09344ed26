"""ctypes binding of libglowq.so: the same names and arguments as include/glowq.h.

Argument marshalling only -- every step of the forward runs in the HIP kernels
behind the C ABI.  Device buffers are passed as integer addresses (for a torch
tensor: `t.data_ptr()`), the stream as the integer value of a hipStream_t (for
torch: `torch.cuda.current_stream().cuda_stream`).  There is no CPU fallback: if
the shared library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

GLOWQ_F16, GLOWQ_BF16, GLOWQ_F32 = 0, 1, 2
GLOWQ_MAX_MODULES = 8
GLOWQ_MAX_RANK = 128
GLOWQ_STATIC_SCRATCH_BYTES = 16 << 20
GLOWQ_OK = 0
GLOWQ_ERR_NULL, GLOWQ_ERR_SHAPE, GLOWQ_ERR_ALIGN, GLOWQ_ERR_DTYPE = -1, -2, -3, -4
GLOWQ_ERR_UNSUPPORTED, GLOWQ_ERR_WORKSPACE, GLOWQ_ERR_HIP = -5, -6, -7

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libglowq.so")


class glowq_module(ctypes.Structure):
    _fields_ = [("w_prepared", ctypes.c_void_p), ("A", ctypes.c_void_p), ("Y", ctypes.c_void_p),
                ("d_out", ctypes.c_int32), ("ldy", ctypes.c_int32)]


class glowq_unit(ctypes.Structure):
    _fields_ = [("X", ctypes.c_void_p), ("B", ctypes.c_void_p),
                ("modules", ctypes.POINTER(glowq_module)), ("n_modules", ctypes.c_int32),
                ("T", ctypes.c_int32), ("d_in", ctypes.c_int32), ("r", ctypes.c_int32),
                ("group_size", ctypes.c_int32), ("act_dtype", ctypes.c_int32),
                ("out_dtype", ctypes.c_int32)]


def _share_hip_runtime_with_torch() -> None:
    """One process must hold ONE HIP runtime.  A PyTorch-ROCm wheel bundles its own
    libamdhip64; if this library pulled in the system copy first, torch would then be
    bound to a runtime that does not match its bundled HSA layer and no device would
    be found.  So when torch is installed, its copy is loaded first (without importing
    torch) and libglowq.so resolves its HIP symbols against it."""
    import importlib.util

    spec = importlib.util.find_spec("torch")
    if spec is None or not spec.submodule_search_locations:
        return
    path = os.path.join(list(spec.submodule_search_locations)[0], "lib", "libamdhip64.so")
    if os.path.exists(path):
        ctypes.CDLL(path, mode=ctypes.RTLD_GLOBAL)


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python paper_2603_25385_amd/csrc/build.py` "
            "(there is no fallback path)")
    _share_hip_runtime_with_torch()
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    up = ctypes.POINTER(glowq_unit)
    sigs = {
        "glowq_status_string": (ctypes.c_char_p, [ctypes.c_int]),
        "glowq_last_hip_error": (ctypes.c_char_p, []),
        "glowq_validate_unit": (ctypes.c_int, [up, i32]),
        "glowq_prepared_bytes": (ctypes.c_int, [i32, i32, i32, ctypes.POINTER(sz)]),
        "glowq_prepare_weights": (ctypes.c_int, [vp, vp, vp, i32, i32, i32, vp, vp]),
        "glowq_workspace_bytes": (ctypes.c_int, [up, i32, ctypes.POINTER(sz)]),
        "glowq_workspace_init": (ctypes.c_int, [vp, sz, vp]),
        "glowq_workspace_status": (ctypes.c_int, [up, i32, vp, sz, vp, vp]),
        "glowq_shared_proj": (ctypes.c_int, [up, vp, vp, sz, vp]),
        "glowq_group_forward": (ctypes.c_int, [up, i32, vp, sz, vp]),
        "glowq_group_forward_static": (ctypes.c_int, [up, i32, vp]),
        "glowq_block_forward": (ctypes.c_int, [up, i32, vp, vp, sz, vp]),
        "glowq_layerwise_workspace_bytes": (ctypes.c_int, [up, i32, ctypes.POINTER(sz)]),
        "glowq_layerwise_forward": (ctypes.c_int, [up, i32, ctypes.POINTER(vp), vp, sz, vp]),
        "glowq_unit_importance": (ctypes.c_int, [up, ctypes.POINTER(vp), vp, vp, vp]),
        "glowq_select_units": (ctypes.c_int, [ctypes.POINTER(ctypes.c_double), i32, i32,
                                              ctypes.POINTER(ctypes.c_uint8)]),
        "glowq_quantize_rtn": (ctypes.c_int, [vp, i32, i32, i32, vp, vp, vp, vp]),
        "glowq_factorize_workspace_bytes": (ctypes.c_int, [up, i32, i32, ctypes.POINTER(sz)]),
        "glowq_factorize_unit": (ctypes.c_int, [up, ctypes.POINTER(vp), vp, i32, i32, i32, vp, vp, sz,
                                                ctypes.POINTER(vp), vp, vp, vp]),
        "glowq_mx_prepared_bytes": (ctypes.c_int, [i32, i32, ctypes.POINTER(sz)]),
        "glowq_mx_prepare_weights": (ctypes.c_int, [vp, vp, i32, i32, vp, vp]),
        "glowq_mx_quantize_activations": (ctypes.c_int, [vp, i32, i32, i32, vp, vp, vp]),
        "glowq_mx_workspace_bytes": (ctypes.c_int, [up, ctypes.POINTER(sz)]),
        "glowq_mx_group_forward": (ctypes.c_int, [up, i32, vp, sz, vp]),
        "glowq_debug_unpack": (ctypes.c_int, [vp, i32, i32, i32, vp, vp]),
        "glowq_debug_dequant": (ctypes.c_int, [vp, i32, i32, i32, i32, vp, vp]),
        # include/glowq_probe.h
        "glowq_probe_stream_read": (ctypes.c_int32, [vp, sz, vp, vp]),
        "glowq_probe_mfma": (ctypes.c_int32, [i32, i32, i32, vp, ctypes.POINTER(ctypes.c_double), vp]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(lib, name)          # AttributeError if a declared symbol is not exported
        fn.restype, fn.argtypes = res, args
    return lib, tuple(sigs)


_lib, EXPORTED = _load()


class GlowqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = f" [{glowq_last_hip_error()}]" if status == GLOWQ_ERR_HIP else ""
        super().__init__(f"{where}: {glowq_status_string(status)} ({status}){detail}")


def _check(status: int, where: str) -> None:
    if status != GLOWQ_OK:
        raise GlowqError(status, where)


def make_module(w_prepared: int, A: int, Y: int, d_out: int, ldy: int) -> glowq_module:
    return glowq_module(w_prepared or None, A or None, Y or None, d_out, ldy)


def make_unit(X: int, B: int, modules: Sequence[glowq_module], T: int, d_in: int, r: int,
              group_size: int, act_dtype: int, out_dtype: int) -> glowq_unit:
    arr = (glowq_module * len(modules))(*modules) if modules else None
    u = glowq_unit(X or None, B or None, arr, len(modules), T, d_in, r, group_size, act_dtype,
                   out_dtype)
    u._keepalive = arr       # the descriptor array lives as long as the unit object
    return u


def _units_array(units):
    if isinstance(units, ctypes.Array):      # already packed by pack_units()
        return units
    arr = (glowq_unit * len(units))()
    for i, u in enumerate(units):
        ctypes.memmove(ctypes.byref(arr[i]), ctypes.byref(u), ctypes.sizeof(glowq_unit))
    arr._keepalive = list(units)
    return arr


def pack_units(units: Sequence[glowq_unit]):
    """Pack unit descriptors into one C array once, for callers that issue the same
    glowq_block_forward / glowq_workspace_bytes call many times."""
    return _units_array(list(units))


def pack_mask(restore_mask) -> "ctypes.Array":
    return (ctypes.c_uint8 * len(restore_mask))(*[1 if b else 0 for b in restore_mask])


def glowq_status_string(status: int) -> str:
    return _lib.glowq_status_string(status).decode()


def glowq_last_hip_error() -> str:
    return _lib.glowq_last_hip_error().decode()


def glowq_validate_unit(unit: glowq_unit, check_pointers: bool = True) -> int:
    """Returns the status code (does not raise)."""
    return _lib.glowq_validate_unit(ctypes.byref(unit) if unit is not None else None,
                                    1 if check_pointers else 0)


def glowq_prepared_bytes(d_out: int, d_in: int, group_size: int) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.glowq_prepared_bytes(d_out, d_in, group_size, ctypes.byref(n)),
           "glowq_prepared_bytes")
    return n.value


def glowq_prepare_weights(wq: int, scales: int, zeros: int, d_out: int, d_in: int,
                          group_size: int, w_prepared: int, stream: int = 0) -> None:
    _check(_lib.glowq_prepare_weights(wq or None, scales or None, zeros or None, d_out, d_in,
                                      group_size, w_prepared or None, stream or None),
           "glowq_prepare_weights")


def glowq_workspace_bytes(units: Sequence[glowq_unit]) -> int:
    n = ctypes.c_size_t(0)
    arr = _units_array(units)
    _check(_lib.glowq_workspace_bytes(arr, len(units), ctypes.byref(n)), "glowq_workspace_bytes")
    return n.value


def glowq_workspace_init(workspace: int, workspace_bytes: int, stream: int = 0) -> None:
    _check(_lib.glowq_workspace_init(workspace or None, workspace_bytes, stream or None),
           "glowq_workspace_init")


def glowq_workspace_status(units: Sequence[glowq_unit], workspace: int, workspace_bytes: int,
                           failed_units: int, stream: int = 0) -> None:
    """failed_units: address of a 4-byte device word that receives the count."""
    arr = _units_array(units)
    _check(_lib.glowq_workspace_status(arr, len(units), workspace or None, workspace_bytes,
                                       failed_units or None, stream or None),
           "glowq_workspace_status")


def glowq_shared_proj(unit: glowq_unit, R_out: int, workspace: int, workspace_bytes: int,
                      stream: int = 0) -> None:
    _check(_lib.glowq_shared_proj(ctypes.byref(unit), R_out or None, workspace or None,
                                  workspace_bytes, stream or None), "glowq_shared_proj")


def glowq_group_forward(unit: glowq_unit, restore: bool, workspace: int, workspace_bytes: int,
                        stream: int = 0) -> None:
    _check(_lib.glowq_group_forward(ctypes.byref(unit), 1 if restore else 0, workspace or None,
                                    workspace_bytes, stream or None), "glowq_group_forward")


def glowq_group_forward_static(unit: glowq_unit, restore: bool, stream: int = 0) -> None:
    _check(_lib.glowq_group_forward_static(ctypes.byref(unit), 1 if restore else 0,
                                           stream or None), "glowq_group_forward_static")


def glowq_block_forward(units: Sequence[glowq_unit], restore_mask: Optional[bytes],
                        workspace: int, workspace_bytes: int, stream: int = 0) -> None:
    arr = _units_array(units)
    mask = None
    if isinstance(restore_mask, ctypes.Array):
        mask = restore_mask
    elif restore_mask is not None:
        mask = pack_mask(restore_mask)
    _check(_lib.glowq_block_forward(arr, len(units), mask, workspace or None, workspace_bytes,
                                    stream or None), "glowq_block_forward")


def glowq_layerwise_workspace_bytes(units: Sequence[glowq_unit]) -> int:
    n = ctypes.c_size_t(0)
    arr = _units_array(units)
    _check(_lib.glowq_layerwise_workspace_bytes(arr, len(units), ctypes.byref(n)),
           "glowq_layerwise_workspace_bytes")
    return n.value


def pack_pointers(addresses: Sequence[int]):
    """A host array of device addresses (one call's B_modules)."""
    return (ctypes.c_void_p * len(addresses))(*[a or None for a in addresses])


def glowq_layerwise_forward(units: Sequence[glowq_unit], B_modules, workspace: int,
                            workspace_bytes: int, stream: int = 0) -> None:
    """B_modules: one device address per module, unit after unit (a sequence of ints or
    the result of pack_pointers)."""
    arr = _units_array(units)
    ptrs = B_modules if isinstance(B_modules, ctypes.Array) else pack_pointers(B_modules)
    _check(_lib.glowq_layerwise_forward(arr, len(units), ptrs, workspace or None,
                                        workspace_bytes, stream or None), "glowq_layerwise_forward")


GLOWQ_IMPORTANCE_SCRATCH_BYTES = 4096


def glowq_unit_importance(unit: glowq_unit, W_modules, scratch: int, scores: int, stream: int = 0) -> None:
    """W_modules: one device address (fp32 [d_out][d_in]) per module; scores: device double[2]."""
    ptrs = W_modules if isinstance(W_modules, ctypes.Array) else pack_pointers(W_modules)
    _check(_lib.glowq_unit_importance(ctypes.byref(unit), ptrs, scratch or None, scores or None,
                                      stream or None), "glowq_unit_importance")


def glowq_select_units(scores: Sequence[float], k: int) -> list:
    n = len(scores)
    arr = (ctypes.c_double * n)(*scores)
    mask = (ctypes.c_uint8 * n)()
    _check(_lib.glowq_select_units(arr, n, k, mask), "glowq_select_units")
    return list(mask)


def glowq_quantize_rtn(W: int, d_out: int, d_in: int, group_size: int, wq: int, scales: int,
                       zeros: int, stream: int = 0) -> None:
    _check(_lib.glowq_quantize_rtn(W or None, d_out, d_in, group_size, wq or None, scales or None,
                                   zeros or None, stream or None), "glowq_quantize_rtn")


GLOWQ_MAX_SKETCH = 256
GLOWQ_MAX_POWER_STEPS = 8


def glowq_factorize_workspace_bytes(unit: glowq_unit, r: int, p: int) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.glowq_factorize_workspace_bytes(ctypes.byref(unit), r, p, ctypes.byref(n)),
           "glowq_factorize_workspace_bytes")
    return n.value


def glowq_factorize_unit(unit: glowq_unit, W_modules, sigma_x_diag: int, r: int, p: int, q: int,
                         Omega: int, workspace: int, workspace_bytes: int, A_out, B_out: int,
                         sigma_out: int = 0, stream: int = 0) -> None:
    """W_modules / A_out: one device address per module (fp32 weights in, act-dtype [d_out][r]
    out); sigma_x_diag: device double[d_in] or 0; Omega: device double[d_in][r + p]."""
    w = W_modules if isinstance(W_modules, ctypes.Array) else pack_pointers(W_modules)
    a = A_out if isinstance(A_out, ctypes.Array) else pack_pointers(A_out)
    _check(_lib.glowq_factorize_unit(ctypes.byref(unit), w, sigma_x_diag or None, r, p, q,
                                     Omega or None, workspace or None, workspace_bytes, a,
                                     B_out or None, sigma_out or None, stream or None),
           "glowq_factorize_unit")


def glowq_mx_prepared_bytes(d_out: int, d_in: int) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.glowq_mx_prepared_bytes(d_out, d_in, ctypes.byref(n)), "glowq_mx_prepared_bytes")
    return n.value


def glowq_mx_prepare_weights(codes: int, scales: int, d_out: int, d_in: int, w_prepared: int,
                             stream: int = 0) -> None:
    _check(_lib.glowq_mx_prepare_weights(codes or None, scales or None, d_out, d_in, w_prepared or None,
                                         stream or None), "glowq_mx_prepare_weights")


def glowq_mx_quantize_activations(X: int, T: int, d_in: int, act_dtype: int, codes: int, scales: int,
                                  stream: int = 0) -> None:
    _check(_lib.glowq_mx_quantize_activations(X or None, T, d_in, act_dtype, codes or None, scales or None,
                                              stream or None), "glowq_mx_quantize_activations")


def glowq_mx_workspace_bytes(unit: glowq_unit) -> int:
    n = ctypes.c_size_t(0)
    _check(_lib.glowq_mx_workspace_bytes(ctypes.byref(unit), ctypes.byref(n)), "glowq_mx_workspace_bytes")
    return n.value


def glowq_mx_group_forward(unit: glowq_unit, restore: int, workspace: int, workspace_bytes: int,
                           stream: int = 0) -> None:
    _check(_lib.glowq_mx_group_forward(ctypes.byref(unit), restore, workspace or None, workspace_bytes,
                                       stream or None), "glowq_mx_group_forward")


def glowq_debug_unpack(w_prepared: int, d_out: int, d_in: int, group_size: int, q_out: int,
                       stream: int = 0) -> None:
    _check(_lib.glowq_debug_unpack(w_prepared or None, d_out, d_in, group_size, q_out or None,
                                   stream or None), "glowq_debug_unpack")


def glowq_debug_dequant(w_prepared: int, d_out: int, d_in: int, group_size: int, act_dtype: int,
                        w_out: int, stream: int = 0) -> None:
    _check(_lib.glowq_debug_dequant(w_prepared or None, d_out, d_in, group_size, act_dtype,
                                    w_out or None, stream or None), "glowq_debug_dequant")


def glowq_probe_stream_read(src: int, nbytes: int, sink: int, stream: int = 0) -> None:
    rc = _lib.glowq_probe_stream_read(src or None, nbytes, sink or None, stream or None)
    if rc != 0:
        raise GlowqError(rc, "glowq_probe_stream_read")


def glowq_probe_mfma(iters: int, bf16: bool, waves_per_simd: int, sink: int, stream: int = 0) -> float:
    """Returns the floating-point operations of the launch."""
    fl = ctypes.c_double(0.0)
    rc = _lib.glowq_probe_mfma(iters, 1 if bf16 else 0, waves_per_simd, sink or None,
                               ctypes.byref(fl), stream or None)
    if rc != 0:
        raise GlowqError(rc, "glowq_probe_mfma")
    return fl.value
