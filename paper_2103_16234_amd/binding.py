"""ctypes binding of libconvfwd.so: argument marshalling only.

Every step of the convolution runs in the library's HIP kernels; torch is used for device
memory and streams. There is no CPU or eager fallback: if the library is missing, loading
raises and tells how to build it.
"""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "libconvfwd.so")
_lib = None

CONV_KERNEL_GENERIC = 0
CONV_KERNEL_TAP = 1
CONV_KERNEL_POINTWISE = 2
CONV_KERNEL_PANEL = 3
CONV_LOADER_REGISTERS = 1
CONV_LOADER_DIRECT = 2
CONV_LOADER_DIRECT_WAVES = 3
CONV_LOADER_DIRECT_DEEP = 4
CONV_ORDER_CHANNEL_FAST = 1
CONV_ORDER_PIXEL_FAST = 2
CONV_ORDER_CHANNEL_GROUPS = 3

EXPORTS = ("conv_fwd", "conv_fwd_plan", "conv_fwd_planned", "conv_fwd_bias_relu", "conv_fwd_find", "conv_two_stage_workspace_bytes",
           "conv_fwd_two_stage", "conv_fwd_plan_split_c", "conv_fwd_split_c", "conv_fwd_split_c_static", "conv_fwd_plan_request", "conv_probe_mfma", "conv_probe_copy",
           "conv_variant_count", "conv_variant_info", "conv_set_stream", "conv_strerror")


class ConvPlan(ctypes.Structure):
    """Mirror of conv_plan_t in include/convfwd.h."""
    _fields_ = [(n, ctypes.c_int) for n in (
        "kernel", "variant", "tile_k", "tile_pix", "chunk_c", "x_vec", "w_vec", "lds_rows", "lds_pitch",
        "lds_plane", "grid", "block", "lds_bytes", "P", "Q", "c_splits", "loader", "order", "k_group")] + [
        ("workspace_bytes", ctypes.c_longlong), ("flops", ctypes.c_longlong), ("bytes", ctypes.c_longlong)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class ConvError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"convfwd error {code}: {text}")
        self.code = code


def library_path() -> str:
    return _LIB_PATH


def build_library(force: bool = False) -> str:
    from . import build as _build
    return _build.build(force=force)


def load_library():
    """Load libconvfwd.so (built in-tree by `python -m paper_2103_16234_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python -m paper_2103_16234_amd.build` "
                          "(there is no fallback path)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, ci = ctypes.c_void_p, ctypes.c_int
    dims = [ci] * 9
    lib.conv_fwd.argtypes = [vp, vp, vp] + dims
    lib.conv_fwd_plan.argtypes = dims + [ctypes.POINTER(ConvPlan)]
    lib.conv_fwd_planned.argtypes = [vp, vp, vp] + dims + [ctypes.POINTER(ConvPlan), ctypes.POINTER(ConvPlan)]
    lib.conv_fwd_bias_relu.argtypes = [vp, vp, vp, vp] + dims + [ci, ctypes.POINTER(ConvPlan), ctypes.POINTER(ConvPlan)]
    lib.conv_fwd_find.argtypes = [vp, vp, vp] + dims + [vp, ctypes.c_longlong, ctypes.POINTER(ConvPlan),
                                                        ctypes.POINTER(ctypes.c_float)]
    lib.conv_two_stage_workspace_bytes.argtypes = dims
    lib.conv_two_stage_workspace_bytes.restype = ctypes.c_longlong
    lib.conv_fwd_two_stage.argtypes = [vp, vp, vp, vp, ctypes.c_longlong] + dims
    lib.conv_fwd_plan_split_c.argtypes = dims + [ctypes.POINTER(ConvPlan)]
    lib.conv_fwd_plan_request.argtypes = dims + [ctypes.POINTER(ConvPlan), ctypes.POINTER(ConvPlan), ctypes.POINTER(ctypes.c_double)]
    lib.conv_fwd_split_c.argtypes = [vp, vp, vp, vp, vp, ctypes.c_longlong] + dims + [ci, ctypes.POINTER(ConvPlan),
                                                                                   ctypes.POINTER(ConvPlan)]
    lib.conv_fwd_split_c_static.argtypes = [vp, vp, vp, vp] + dims + [ci, ctypes.POINTER(ConvPlan), ctypes.POINTER(ConvPlan)]
    lib.conv_probe_mfma.argtypes = [ci, vp]
    lib.conv_probe_mfma.restype = ctypes.c_longlong
    lib.conv_probe_copy.argtypes = [vp, vp, ctypes.c_longlong]
    lib.conv_variant_count.argtypes = [ci]
    lib.conv_variant_info.argtypes = [ci, ci] + [ctypes.POINTER(ci)] * 3
    lib.conv_set_stream.argtypes = [vp]
    lib.conv_strerror.argtypes = [ci]
    lib.conv_strerror.restype = ctypes.c_char_p
    for name in EXPORTS:
        if name not in ("conv_strerror", "conv_two_stage_workspace_bytes", "conv_probe_mfma"):
            getattr(lib, name).restype = ci
    _lib = lib
    return lib


def conv_strerror(code: int) -> str:
    return load_library().conv_strerror(code).decode()


def _check(code: int):
    if code != 0:
        raise ConvError(code, conv_strerror(code))


def conv_fwd_plan(N, C, H, W, K, R, S, pad_h, pad_w) -> ConvPlan:
    plan = ConvPlan()
    _check(load_library().conv_fwd_plan(N, C, H, W, K, R, S, pad_h, pad_w, ctypes.byref(plan)))
    return plan


def conv_variant_count(kernel: int) -> int:
    return load_library().conv_variant_count(kernel)


def conv_variant_info(kernel: int, variant: int):
    tk, mp, bl = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    _check(load_library().conv_variant_info(kernel, variant, ctypes.byref(tk), ctypes.byref(mp), ctypes.byref(bl)))
    return tk.value, mp.value, bl.value


def conv_set_stream(stream=None):
    """Use a torch.cuda.Stream (or a raw hipStream_t integer, or None for the null stream)."""
    handle = getattr(stream, "cuda_stream", stream)
    _check(load_library().conv_set_stream(ctypes.c_void_p(handle or 0)))


def _device_args(x, w, y, pad_h, pad_w):
    import torch
    for name, t in (("x", x), ("w", w)):
        if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()
                and t.dim() == 4):
            raise TypeError(f"{name} must be a contiguous 4-d float32 tensor on the GPU")
    N, C, H, W = x.shape
    K, Cw, R, S = w.shape
    if Cw != C:
        raise ValueError("x and w disagree on the number of channels")
    P, Q = H + 2 * pad_h - R + 1, W + 2 * pad_w - S + 1
    if y is None:
        if P <= 0 or Q <= 0:
            _check(-3)
        y = torch.empty((N, K, P, Q), device=x.device, dtype=torch.float32)
    elif not (y.is_cuda and y.dtype == torch.float32 and y.is_contiguous() and tuple(y.shape) == (N, K, P, Q)):
        raise TypeError("y must be a contiguous float32 GPU tensor of shape [N,K,P,Q]")
    return y, (N, C, H, W, K, R, S, pad_h, pad_w)


def conv_fwd(x, w, pad_h: int, pad_w: int, y=None, use_current_stream: bool = True):
    """y[N,K,P,Q] = stride-1 forward convolution of x[N,C,H,W] with w[K,C,R,S] (device tensors)."""
    import torch
    y, dims = _device_args(x, w, y, pad_h, pad_w)
    lib = load_library()
    if use_current_stream:
        conv_set_stream(torch.cuda.current_stream(x.device))
    _check(lib.conv_fwd(x.data_ptr(), w.data_ptr(), y.data_ptr(), *dims))
    return y


def conv_fwd_planned(x, w, pad_h: int, pad_w: int, kernel: int, variant: int = 0, tile_pix: int = 0,
                     chunk_c: int = 0, y=None, use_current_stream: bool = True, loader: int = 0, order: int = 0, k_group: int = 0):
    """As conv_fwd with a requested kernel family / tile shape; returns (y, resolved ConvPlan)."""
    import torch
    y, dims = _device_args(x, w, y, pad_h, pad_w)
    lib = load_library()
    if use_current_stream:
        conv_set_stream(torch.cuda.current_stream(x.device))
    req, res = ConvPlan(), ConvPlan()
    req.kernel, req.variant, req.tile_pix, req.chunk_c, req.loader = kernel, variant, tile_pix, chunk_c, loader
    req.order, req.k_group = order, k_group
    _check(lib.conv_fwd_planned(x.data_ptr(), w.data_ptr(), y.data_ptr(), *dims, ctypes.byref(req), ctypes.byref(res)))
    return y, res


def conv_fwd_bias_relu(x, w, bias, pad_h: int, pad_w: int, relu: bool, kernel=None, variant: int = 0, tile_pix: int = 0,
                       y=None, use_current_stream: bool = True, loader: int = 0):
    """y = act(conv(x, w) + bias) in one kernel; bias may be None. kernel=None plans as conv_fwd does. Returns (y, plan)."""
    import torch
    y, dims = _device_args(x, w, y, pad_h, pad_w)
    if bias is not None and (not bias.is_cuda or bias.dtype != torch.float32 or not bias.is_contiguous()
                             or bias.numel() != w.shape[0]):
        raise ValueError("bias must be a contiguous fp32 device tensor of K elements")
    lib = load_library()
    if use_current_stream:
        conv_set_stream(torch.cuda.current_stream(x.device))
    res = ConvPlan()
    req = None
    if kernel is not None:
        req = ConvPlan()
        req.kernel, req.variant, req.tile_pix, req.loader = kernel, variant, tile_pix, loader
    _check(lib.conv_fwd_bias_relu(x.data_ptr(), w.data_ptr(), bias.data_ptr() if bias is not None else None, y.data_ptr(),
                                  *dims, int(bool(relu)), ctypes.byref(req) if req is not None else None,
                                  ctypes.byref(res)))
    return y, res


def conv_fwd_plan_request(N, C, H, W, K, R, S, pad_h, pad_w, kernel: int, variant: int = 0, tile_pix: int = 0,
                          c_splits: int = 0, loader: int = 0, order: int = 0, k_group: int = 0):
    """Host-only: resolve a requested mapping without launching it; returns (plan, modelled cycles - tap family only)."""
    req, res, cycles = ConvPlan(), ConvPlan(), ctypes.c_double(0)
    req.kernel, req.variant, req.tile_pix, req.c_splits, req.loader = kernel, variant, tile_pix, c_splits, loader
    req.order, req.k_group = order, k_group
    _check(load_library().conv_fwd_plan_request(N, C, H, W, K, R, S, pad_h, pad_w, ctypes.byref(req), ctypes.byref(res),
                                                ctypes.byref(cycles)))
    return res, float(cycles.value)


def conv_fwd_plan_split_c(N, C, H, W, K, R, S, pad_h, pad_w) -> ConvPlan:
    plan = ConvPlan()
    _check(load_library().conv_fwd_plan_split_c(N, C, H, W, K, R, S, pad_h, pad_w, ctypes.byref(plan)))
    return plan


def conv_fwd_split_c(x, w, pad_h: int, pad_w: int, bias=None, relu: bool = False, c_splits: int = 0, variant=None,
                     tile_pix: int = 0, workspace=None, y=None, use_current_stream: bool = True, loader: int = 0):
    """Channel-splitting mode: y = act(conv(x, w) + bias) with the channels of an output tile shared by c_splits
    work-groups and a second pass that adds their partial outputs. variant=None lets the library choose the
    mapping (then c_splits is ignored); otherwise the tap variant / tile_pix / c_splits are requested.
    workspace: fp32 device tensor (allocated here when None). Returns (y, plan)."""
    import torch
    y, dims = _device_args(x, w, y, pad_h, pad_w)
    if bias is not None and (not bias.is_cuda or bias.dtype != torch.float32 or not bias.is_contiguous()
                             or bias.numel() != w.shape[0]):
        raise ValueError("bias must be a contiguous fp32 device tensor of K elements")
    lib = load_library()
    if use_current_stream:
        conv_set_stream(torch.cuda.current_stream(x.device))
    res = ConvPlan()
    req = None
    if variant is not None:
        req = ConvPlan()
        req.kernel, req.variant, req.tile_pix, req.c_splits, req.loader = 1, variant, tile_pix, c_splits, loader
    if workspace is None:
        need = max(c_splits, 16) * y.numel() if variant is not None else conv_fwd_plan_split_c(*dims).workspace_bytes // 4
        workspace = torch.empty(max(int(need), 4), dtype=torch.float32, device=x.device)
    _check(lib.conv_fwd_split_c(x.data_ptr(), w.data_ptr(), bias.data_ptr() if bias is not None else None, y.data_ptr(),
                                workspace.data_ptr(), workspace.numel() * 4, *dims, int(bool(relu)),
                                ctypes.byref(req) if req is not None else None, ctypes.byref(res)))
    return y, res


STATIC_SCRATCH_BYTES = 16 << 20


def conv_fwd_split_c_static(x, w, pad_h: int, pad_w: int, y, bias=None, relu: bool = False, c_splits: int = 0, variant=None,
                            tile_pix: int = 0, use_current_stream: bool = True, loader: int = 0):
    """conv_fwd_split_c on the library's static scratch array: no workspace, and nothing is allocated here either
    (y must be given). Returns (y, plan)."""
    import torch
    y, dims = _device_args(x, w, y, pad_h, pad_w)
    lib = load_library()
    if use_current_stream:
        conv_set_stream(torch.cuda.current_stream(x.device))
    res = ConvPlan()
    req = None
    if variant is not None:
        req = ConvPlan()
        req.kernel, req.variant, req.tile_pix, req.c_splits, req.loader = 1, variant, tile_pix, c_splits, loader
    _check(lib.conv_fwd_split_c_static(x.data_ptr(), w.data_ptr(), bias.data_ptr() if bias is not None else None, y.data_ptr(),
                                       *dims, int(bool(relu)), ctypes.byref(req) if req is not None else None, ctypes.byref(res)))
    return y, res


def conv_fwd_find(x, w, pad_h: int, pad_w: int, y=None, flush=None, use_current_stream: bool = True):
    """Time every mapping for this layer, keep the fastest for later conv_fwd calls; returns (y, plan, microseconds).
    flush: optional device tensor (>= 1 MiB, overwritten) streamed through the caches before every timed launch."""
    import torch
    y, dims = _device_args(x, w, y, pad_h, pad_w)
    lib = load_library()
    if use_current_stream:
        conv_set_stream(torch.cuda.current_stream(x.device))
    plan, us = ConvPlan(), ctypes.c_float(0)
    fptr, fbytes = (flush.data_ptr(), flush.numel() * flush.element_size()) if flush is not None else (None, 0)
    _check(lib.conv_fwd_find(x.data_ptr(), w.data_ptr(), y.data_ptr(), *dims, fptr, fbytes, ctypes.byref(plan),
                             ctypes.byref(us)))
    return y, plan, float(us.value)


def conv_two_stage_workspace_bytes(N, C, H, W, K, R, S, pad_h, pad_w) -> int:
    n = load_library().conv_two_stage_workspace_bytes(N, C, H, W, K, R, S, pad_h, pad_w)
    if n < 0:
        _check(int(n))
    return int(n)


def conv_fwd_two_stage(x, w, pad_h: int, pad_w: int, workspace=None, y=None, use_current_stream: bool = True):
    """The paper's two-stage scheme (opt-in): y = conv(x, w) through an explicit workspace tensor."""
    import torch
    y, dims = _device_args(x, w, y, pad_h, pad_w)
    lib = load_library()
    need = conv_two_stage_workspace_bytes(*dims)
    if workspace is None and need:
        workspace = torch.empty(need // 4, device=x.device, dtype=torch.float32)
    if use_current_stream:
        conv_set_stream(torch.cuda.current_stream(x.device))
    ws_ptr = workspace.data_ptr() if workspace is not None else 0
    ws_bytes = workspace.numel() * 4 if workspace is not None else 0
    _check(lib.conv_fwd_two_stage(x.data_ptr(), w.data_ptr(), y.data_ptr(), ws_ptr, ws_bytes, *dims))
    return y
