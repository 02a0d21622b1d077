"""Thin ctypes binding of libhashgrid.so (C ABI in include/hashgrid.h).

Argument marshalling only: every step of the encoding runs in the library's
HIP kernels.  PyTorch supplies device memory and the stream.  There is no CPU
fallback: if the shared library has not been built, importing this module's
entry points raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch  # imported before the library so that both share one HIP runtime

from .build import LIB_PATH, PROBES_LIB_PATH

HG_OK = 0
HG_F32, HG_F16 = 0, 1
HG_INTERP_LINEAR, HG_INTERP_SMOOTHSTEP = 0, 1
HG_MAX_LEVELS = 32
HG_BWD_COUNTED = 1
HG_BWD_OVERWRITE = 2
HG_ERR_UNSUPPORTED = 2
HG_STATIC_SCRATCH_BYTES = 64 << 20
HG_LOSS_L2, HG_LOSS_MAPE = 0, 1
_LOSSES = {"l2": HG_LOSS_L2, "mape": HG_LOSS_MAPE, HG_LOSS_L2: HG_LOSS_L2, HG_LOSS_MAPE: HG_LOSS_MAPE}

_DTYPES = {"f32": HG_F32, "f16": HG_F16, torch.float32: HG_F32, torch.float16: HG_F16}
_TORCH = {HG_F32: torch.float32, HG_F16: torch.float16}

EXPORTS = ("hashgrid_create", "hashgrid_destroy", "hashgrid_n_entries", "hashgrid_level_info",
           "hashgrid_encode_fwd", "hashgrid_encode_bwd", "hashgrid_encode_bwd_input",
           "hashgrid_debug_indices", "hashgrid_debug_count_outside", "hashgrid_strerror", "hashgrid_bwd_workspace_bytes",
           "hashgrid_encode_bwd_ws", "hashgrid_encode_fwd_ws", "hashgrid_bwd_ws_pays", "hashgrid_adam_step",
           "hashgrid_encode_mlp_fwd", "hashgrid_encode_bwd_static", "hashgrid_encode_mlp_fwd_train", "hashgrid_mlp_bwd",
           "hashgrid_adam_step_half_grad", "hashgrid_loss_grad", "hashgrid_mlp_fwd")
PROBE_EXPORTS = ("hashgrid_probe_copy", "hashgrid_probe_gather", "hashgrid_probe_atomic_add",
                 "hashgrid_probe_gather_lines")


class HashGridError(RuntimeError):
    pass


class hashgrid_config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in
                ("d", "L", "F", "T", "N_min", "N_max", "param_dtype", "io_dtype", "interp", "grad_dtype")]


class hashgrid_adam_config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_float) for n in ("lr", "beta1", "beta2", "eps", "l2_reg")]


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads the in-tree shared library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise HashGridError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = ctypes.CDLL(LIB_PATH)
    vp, u32, u64 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64
    lib.hashgrid_create.argtypes = [ctypes.POINTER(hashgrid_config), ctypes.POINTER(vp)]
    lib.hashgrid_create.restype = ctypes.c_int
    lib.hashgrid_destroy.argtypes = [vp]
    lib.hashgrid_destroy.restype = None
    lib.hashgrid_n_entries.argtypes = [vp]
    lib.hashgrid_n_entries.restype = u64
    lib.hashgrid_level_info.argtypes = [vp, u32, ctypes.POINTER(u32), ctypes.POINTER(u64), ctypes.POINTER(u32),
                                        ctypes.POINTER(ctypes.c_int)]
    lib.hashgrid_level_info.restype = ctypes.c_int
    lib.hashgrid_encode_fwd.argtypes = [vp, u32, vp, vp, vp, vp]
    lib.hashgrid_encode_fwd.restype = ctypes.c_int
    lib.hashgrid_encode_bwd.argtypes = [vp, u32, vp, vp, vp, vp]
    lib.hashgrid_encode_bwd.restype = ctypes.c_int
    lib.hashgrid_encode_bwd_input.argtypes = [vp, u32, vp, vp, vp, vp, vp]
    lib.hashgrid_encode_bwd_input.restype = ctypes.c_int
    lib.hashgrid_debug_indices.argtypes = [vp, u32, vp, u32, vp, vp, vp]
    lib.hashgrid_debug_indices.restype = ctypes.c_int
    lib.hashgrid_debug_count_outside.argtypes = [vp, u32, vp, vp, vp]
    lib.hashgrid_debug_count_outside.restype = ctypes.c_int
    lib.hashgrid_bwd_workspace_bytes.argtypes = [vp, u32]
    lib.hashgrid_bwd_workspace_bytes.restype = u64
    lib.hashgrid_encode_bwd_ws.argtypes = [vp, u32, vp, vp, vp, vp, u64, u32, vp]
    lib.hashgrid_encode_bwd_static.argtypes = [vp, u32, vp, vp, vp, u32, vp]
    lib.hashgrid_encode_bwd_static.restype = ctypes.c_int
    lib.hashgrid_encode_fwd_ws.argtypes = [vp, u32, vp, vp, vp, vp, u64, vp]
    lib.hashgrid_encode_fwd_ws.restype = ctypes.c_int
    lib.hashgrid_encode_mlp_fwd.argtypes = [vp, u32, vp, vp, vp, vp, vp, u32, vp, vp]
    lib.hashgrid_encode_mlp_fwd.restype = ctypes.c_int
    lib.hashgrid_encode_mlp_fwd_train.argtypes = [vp, u32, vp, vp, vp, vp, vp, u32, vp, vp, vp]
    lib.hashgrid_encode_mlp_fwd_train.restype = ctypes.c_int
    lib.hashgrid_mlp_bwd.argtypes = [u32, u32, u32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.hashgrid_mlp_bwd.restype = ctypes.c_int
    lib.hashgrid_mlp_fwd.argtypes = [u32, u32, u32, vp, vp, vp, vp, vp, vp]
    lib.hashgrid_mlp_fwd.restype = ctypes.c_int
    lib.hashgrid_bwd_ws_pays.argtypes = [vp, u32]
    lib.hashgrid_bwd_ws_pays.restype = ctypes.c_int
    lib.hashgrid_encode_bwd_ws.restype = ctypes.c_int
    lib.hashgrid_adam_step.argtypes = [u64, vp, vp, vp, vp, vp, ctypes.POINTER(hashgrid_adam_config), u32, ctypes.c_int,
                                       vp]
    lib.hashgrid_adam_step.restype = ctypes.c_int
    lib.hashgrid_adam_step_half_grad.argtypes = [u64, vp, vp, vp, vp, vp, ctypes.POINTER(hashgrid_adam_config), u32,
                                                 ctypes.c_int, ctypes.c_float, vp]
    lib.hashgrid_adam_step_half_grad.restype = ctypes.c_int
    lib.hashgrid_loss_grad.argtypes = [u64, vp, vp, u32, ctypes.c_float, vp, vp, vp]
    lib.hashgrid_loss_grad.restype = ctypes.c_int
    lib.hashgrid_strerror.argtypes = [ctypes.c_int]
    lib.hashgrid_strerror.restype = ctypes.c_char_p
    _lib = lib
    return lib


_probes = None


def load_probes() -> ctypes.CDLL:
    """Loads the in-tree library of machine probes (the benchmark's); raises if it has not been built."""
    global _probes
    if _probes is not None:
        return _probes
    if not os.path.exists(PROBES_LIB_PATH):
        raise HashGridError(
            f"{PROBES_LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    lib = ctypes.CDLL(PROBES_LIB_PATH)
    vp, u32, u64 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64
    lib.hashgrid_probe_copy.argtypes = [vp, vp, u64, vp]
    lib.hashgrid_probe_copy.restype = ctypes.c_int
    lib.hashgrid_probe_gather.argtypes = [vp, u64, u64, u32, vp, vp]
    lib.hashgrid_probe_gather.restype = ctypes.c_int
    lib.hashgrid_probe_atomic_add.argtypes = [vp, u64, u64, u32, vp]
    lib.hashgrid_probe_atomic_add.restype = ctypes.c_int
    lib.hashgrid_probe_gather_lines.argtypes = [vp, u64, u32, u64, u32, u32, vp, vp]
    lib.hashgrid_probe_gather_lines.restype = ctypes.c_int
    _probes = lib
    return lib


def strerror(status: int) -> str:
    return load_library().hashgrid_strerror(status).decode()


def _check(status: int, what: str) -> None:
    if status != HG_OK:
        raise HashGridError(f"{what}: {strerror(status)} (status {status})")


@dataclass(frozen=True)
class LevelInfo:
    N: int
    entry_offset: int
    n_entries: int
    is_dense: bool


def _stream_ptr(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def _dev(t: torch.Tensor, dtype, shape, name: str) -> int:
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()):
        raise HashGridError(f"{name} must be a contiguous device tensor")
    if t.dtype != dtype or tuple(t.shape) != tuple(shape):
        raise HashGridError(f"{name}: expected {dtype} {tuple(shape)}, got {t.dtype} {tuple(t.shape)}")
    return t.data_ptr()


class HashGrid:
    """Handle on one encoding configuration (hashgrid_create / hashgrid_destroy)."""

    def __init__(self, d: int, L: int, F: int, T: int, N_min: int, N_max: int, param_dtype="f16",
                 io_dtype="f16", interp: int = HG_INTERP_LINEAR, grad_dtype="f32"):
        self._lib = load_library()
        self.cfg = hashgrid_config(d, L, F, T, N_min, N_max, _DTYPES[param_dtype], _DTYPES[io_dtype], interp,
                                   _DTYPES[grad_dtype])
        h = ctypes.c_void_p()
        _check(self._lib.hashgrid_create(ctypes.byref(self.cfg), ctypes.byref(h)), "hashgrid_create")
        self._h = h
        self.d, self.L, self.F, self.T = d, L, F, T
        self.param_dtype = _TORCH[self.cfg.param_dtype]
        self.io_dtype = _TORCH[self.cfg.io_dtype]
        self.grad_dtype = _TORCH[self.cfg.grad_dtype]
        self.n_entries = int(self._lib.hashgrid_n_entries(self._h))
        self._ws = {}  # (device, stream) -> scratch buffer kept for calls that pass none
        self._counted = None  # (x pointer, B, workspace pointer, x version, stream) the workspace holds counts for

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h:
            self._lib.hashgrid_destroy(h)

    def level_info(self, l: int) -> LevelInfo:
        N, off, n, dense = ctypes.c_uint32(), ctypes.c_uint64(), ctypes.c_uint32(), ctypes.c_int()
        _check(self._lib.hashgrid_level_info(self._h, l, ctypes.byref(N), ctypes.byref(off), ctypes.byref(n),
                                             ctypes.byref(dense)), "hashgrid_level_info")
        return LevelInfo(N.value, off.value, n.value, bool(dense.value))

    def levels(self):
        return [self.level_info(l) for l in range(self.L)]

    def _workspace(self, need: int, device, stream) -> torch.Tensor:
        """The scratch buffer this object keeps for calls that pass none: one per (device, stream), because
        calls that overlap in time need separate buffers and calls on one stream never overlap."""
        key = (device, _stream_ptr(stream))
        ws = self._ws.get(key)
        if ws is None or ws.numel() < need:
            ws = torch.empty(need, dtype=torch.uint8, device=device)
            self._ws[key] = ws
        if stream is not None:
            ws.record_stream(stream)  # allocated on torch's current stream, used on this one
        return ws

    def bwd_ws_pays(self, B: int) -> bool:
        return bool(self._lib.hashgrid_bwd_ws_pays(self._h, B))

    def encode_fwd(self, x: torch.Tensor, params: torch.Tensor, y: torch.Tensor | None = None, stream=None,
                   count_for_bwd=False, workspace: torch.Tensor | None = None):
        """hashgrid_encode_fwd; with count_for_bwd, hashgrid_encode_fwd_ws where the configuration
        is served by it and the batch is large enough for the sorted backward pass to pay
        (count_for_bwd="always": whatever the batch): the next encode_bwd on the same, unmodified x and
        the same workspace then skips its counting pass."""
        B = x.shape[0]
        if y is None:
            y = torch.empty((B, self.L * self.F), dtype=self.io_dtype, device=x.device)
        self._counted = None
        want = bool(count_for_bwd) and B and (count_for_bwd == "always" or self.bwd_ws_pays(B))
        need = self.bwd_workspace_bytes(B) if want else 0
        if need:
            ws = workspace if workspace is not None else self._workspace(need, x.device, stream)
            st = self._lib.hashgrid_encode_fwd_ws(
                self._h, B, _dev(x, torch.float32, (B, self.d), "x"),
                _dev(params, self.param_dtype, (self.n_entries, self.F), "params"),
                _dev(y, self.io_dtype, (B, self.L * self.F), "y"), ws.data_ptr(), ws.numel() * ws.element_size(),
                _stream_ptr(stream))
            if st != HG_ERR_UNSUPPORTED:
                _check(st, "hashgrid_encode_fwd_ws")
                self._counted = (x.data_ptr(), B, ws.data_ptr(), x._version, _stream_ptr(stream))  # x unchanged since, as far as torch knows
                return y
        _check(self._lib.hashgrid_encode_fwd(
            self._h, B, _dev(x, torch.float32, (B, self.d), "x"),
            _dev(params, self.param_dtype, (self.n_entries, self.F), "params"),
            _dev(y, self.io_dtype, (B, self.L * self.F), "y"), _stream_ptr(stream)), "hashgrid_encode_fwd")
        return y

    def bwd_workspace_bytes(self, B: int) -> int:
        return int(self._lib.hashgrid_bwd_workspace_bytes(self._h, B))

    def encode_bwd(self, x: torch.Tensor, dLdy: torch.Tensor, grad_params: torch.Tensor | None = None,
                   stream=None, workspace: torch.Tensor | None = None, use_workspace: bool | None = None,
                   overwrite: bool = False):
        """hashgrid_encode_bwd_ws (the scratch buffer is `workspace` or one kept on this object) or
        hashgrid_encode_bwd.  use_workspace: True = the former wherever the configuration is served
        by it, False = the latter, None = whichever hashgrid_bwd_ws_pays expects to be faster.
        overwrite: grad_params becomes the gradient of this batch instead of growing by it
        (HG_BWD_OVERWRITE; where the atomic pass runs, the buffer is cleared on the stream first)."""
        B = x.shape[0]
        fresh = grad_params is None
        if fresh:
            grad_params = torch.zeros((self.n_entries, self.F), dtype=self.grad_dtype, device=x.device)
        if use_workspace is None:
            use_workspace = self._counted is not None or self.bwd_ws_pays(B)
        need = self.bwd_workspace_bytes(B) if use_workspace else 0
        counted, self._counted = self._counted, None  # the pass consumes the counts
        if need:
            if workspace is None:
                workspace = self._workspace(need, x.device, stream)
            # the counts are only there for a call ordered after the forward: same stream
            flags = HG_BWD_COUNTED if counted == (x.data_ptr(), B, workspace.data_ptr(), x._version, _stream_ptr(stream)) else 0
            if overwrite and not fresh:
                flags |= HG_BWD_OVERWRITE
            _check(self._lib.hashgrid_encode_bwd_ws(
                self._h, B, _dev(x, torch.float32, (B, self.d), "x"),
                _dev(dLdy, self.io_dtype, (B, self.L * self.F), "dLdy"),
                _dev(grad_params, self.grad_dtype, (self.n_entries, self.F), "grad_params"),
                workspace.data_ptr(), workspace.numel() * workspace.element_size(), flags, _stream_ptr(stream)),
                "hashgrid_encode_bwd_ws")
            return grad_params
        if overwrite and not fresh:  # the atomic pass only adds: clear first, on the same stream
            _dev(grad_params, self.grad_dtype, (self.n_entries, self.F), "grad_params")
            with torch.cuda.stream(torch.cuda.current_stream() if stream is None else stream):
                grad_params.zero_()
        _check(self._lib.hashgrid_encode_bwd(
            self._h, B, _dev(x, torch.float32, (B, self.d), "x"),
            _dev(dLdy, self.io_dtype, (B, self.L * self.F), "dLdy"),
            _dev(grad_params, self.grad_dtype, (self.n_entries, self.F), "grad_params"), _stream_ptr(stream)),
            "hashgrid_encode_bwd")
        return grad_params

    def encode_bwd_static(self, x: torch.Tensor, dLdy: torch.Tensor, grad_params: torch.Tensor, stream=None,
                          overwrite: bool = False):
        """hashgrid_encode_bwd_static: the sorted backward pass on the library's own fixed scratch array
        (no workspace, no allocation inside the call); grad_params must be given."""
        B = x.shape[0]
        _check(self._lib.hashgrid_encode_bwd_static(
            self._h, B, _dev(x, torch.float32, (B, self.d), "x"),
            _dev(dLdy, self.io_dtype, (B, self.L * self.F), "dLdy"),
            _dev(grad_params, self.grad_dtype, (self.n_entries, self.F), "grad_params"),
            HG_BWD_OVERWRITE if overwrite else 0, _stream_ptr(stream)), "hashgrid_encode_bwd_static")
        return grad_params

    def encode_bwd_input(self, x: torch.Tensor, params: torch.Tensor, dLdy: torch.Tensor,
                         dLdx: torch.Tensor | None = None, stream=None):
        B = x.shape[0]
        if dLdx is None:
            dLdx = torch.empty((B, self.d), dtype=torch.float32, device=x.device)
        _check(self._lib.hashgrid_encode_bwd_input(
            self._h, B, _dev(x, torch.float32, (B, self.d), "x"),
            _dev(params, self.param_dtype, (self.n_entries, self.F), "params"),
            _dev(dLdy, self.io_dtype, (B, self.L * self.F), "dLdy"),
            _dev(dLdx, torch.float32, (B, self.d), "dLdx"), _stream_ptr(stream)), "hashgrid_encode_bwd_input")
        return dLdx

    def encode_mlp_fwd(self, x: torch.Tensor, params: torch.Tensor, W1: torch.Tensor, W2: torch.Tensor,
                       W3: torch.Tensor, out: torch.Tensor | None = None, stream=None, y: torch.Tensor | None = None):
        """hashgrid_encode_mlp_fwd: the encoding followed by the 64-64 ReLU network, fp16 weights
        W1 [64, L*F], W2 [64, 64], W3 [n_out, 64]; returns out [B, n_out] fp32.  With y [B, L*F] fp16:
        hashgrid_encode_mlp_fwd_train, which also keeps the encoded features for mlp_bwd."""
        B, n_out = x.shape[0], W3.shape[0]
        if out is None:
            out = torch.empty((B, n_out), dtype=torch.float32, device=x.device)
        args = (self._h, B, _dev(x, torch.float32, (B, self.d), "x"),
                _dev(params, self.param_dtype, (self.n_entries, self.F), "params"),
                _dev(W1, torch.float16, (64, self.L * self.F), "W1"), _dev(W2, torch.float16, (64, 64), "W2"),
                _dev(W3, torch.float16, (n_out, 64), "W3"), n_out, _dev(out, torch.float32, (B, n_out), "out"))
        if y is None:
            _check(self._lib.hashgrid_encode_mlp_fwd(*args, _stream_ptr(stream)), "hashgrid_encode_mlp_fwd")
        else:
            _check(self._lib.hashgrid_encode_mlp_fwd_train(
                *args, _dev(y, torch.float16, (B, self.L * self.F), "y"), _stream_ptr(stream)),
                "hashgrid_encode_mlp_fwd_train")
        return out

    def debug_count_outside(self, x: torch.Tensor, stream=None) -> int:
        """hashgrid_debug_count_outside: coordinates of x that are not in [0,1) (synchronises)."""
        B = x.shape[0]
        count = torch.zeros(1, dtype=torch.int32, device=x.device)
        _check(self._lib.hashgrid_debug_count_outside(
            self._h, B, _dev(x, torch.float32, (B, self.d), "x"), count.data_ptr(), _stream_ptr(stream)),
            "hashgrid_debug_count_outside")
        return int(count.item())

    def debug_indices(self, x: torch.Tensor, level: int, stream=None):
        B = x.shape[0]
        idx = torch.empty((B, 1 << self.d), dtype=torch.int32, device=x.device)
        w = torch.empty((B, self.d), dtype=torch.float32, device=x.device)
        _check(self._lib.hashgrid_debug_indices(
            self._h, B, _dev(x, torch.float32, (B, self.d), "x"), level, idx.data_ptr(), w.data_ptr(),
            _stream_ptr(stream)), "hashgrid_debug_indices")
        return idx, w


def adam_step(params_master: torch.Tensor, grad: torch.Tensor, m: torch.Tensor, v: torch.Tensor, step: int,
              lr: float = 1e-2, beta1: float = 0.9, beta2: float = 0.99, eps: float = 1e-15,
              params_half: torch.Tensor | None = None, zero_grad: bool = True, stream=None,
              grad_scale: float = 1.0, l2_reg: float = 0.0) -> None:
    """hashgrid_adam_step on flat or [n, F] fp32 tensors (in place); with an fp16 gradient (grad_dtype "f16")
    hashgrid_adam_step_half_grad, which multiplies every gradient scalar by grad_scale as it reads it.  l2_reg: the
    factor of the L2 regularisation (the paper: 1e-6 on the network's weights, 0 on the tables)."""
    n = params_master.numel()
    for name, t in (("params_master", params_master), ("m", m), ("v", v)):
        if not (t.is_cuda and t.is_contiguous() and t.dtype == torch.float32 and t.numel() == n):
            raise HashGridError(f"{name} must be a contiguous fp32 device tensor of {n} scalars")
    if not (grad.is_cuda and grad.is_contiguous() and grad.dtype in (torch.float32, torch.float16) and grad.numel() == n):
        raise HashGridError(f"grad must be a contiguous fp32 or fp16 device tensor of {n} scalars")
    if grad.dtype == torch.float32 and grad_scale != 1.0:
        raise HashGridError("grad_scale applies to fp16 gradients only")
    half_ptr = None
    if params_half is not None:
        if not (params_half.is_cuda and params_half.is_contiguous() and params_half.dtype == torch.float16
                and params_half.numel() == n):
            raise HashGridError("params_half must be a contiguous fp16 device tensor of the same size")
        half_ptr = params_half.data_ptr()
    cfg = hashgrid_adam_config(lr, beta1, beta2, eps, l2_reg)
    lib = load_library()
    if grad.dtype == torch.float16:
        _check(lib.hashgrid_adam_step_half_grad(n, params_master.data_ptr(), half_ptr, grad.data_ptr(), m.data_ptr(),
                                                v.data_ptr(), ctypes.byref(cfg), step, int(zero_grad), grad_scale,
                                                _stream_ptr(stream)), "hashgrid_adam_step_half_grad")
    else:
        _check(lib.hashgrid_adam_step(n, params_master.data_ptr(), half_ptr, grad.data_ptr(), m.data_ptr(),
                                      v.data_ptr(), ctypes.byref(cfg), step, int(zero_grad), _stream_ptr(stream)),
               "hashgrid_adam_step")


def loss_grad(prediction: torch.Tensor, target: torch.Tensor, loss, scale: float, dLdout: torch.Tensor,
              loss_sum: torch.Tensor | None = None, stream=None) -> None:
    """hashgrid_loss_grad: dLdout = scale * d loss / d prediction per scalar ("l2" or "mape"); the unscaled loss values
    are added to loss_sum (one fp64 device scalar) when given."""
    n = prediction.numel()
    for name, t in (("prediction", prediction), ("target", target), ("dLdout", dLdout)):
        if not (t.is_cuda and t.is_contiguous() and t.dtype == torch.float32 and t.numel() == n):
            raise HashGridError(f"{name} must be a contiguous fp32 device tensor of {n} scalars")
    if loss not in _LOSSES:
        raise HashGridError(f"unknown loss {loss!r}")
    sum_ptr = None
    if loss_sum is not None:
        if not (loss_sum.is_cuda and loss_sum.dtype == torch.float64 and loss_sum.numel() == 1):
            raise HashGridError("loss_sum must be one fp64 device scalar")
        sum_ptr = loss_sum.data_ptr()
    _check(load_library().hashgrid_loss_grad(n, prediction.data_ptr(), target.data_ptr(), _LOSSES[loss], scale,
                                             dLdout.data_ptr(), sum_ptr, _stream_ptr(stream)), "hashgrid_loss_grad")


def probe_copy(src: torch.Tensor, dst: torch.Tensor, stream=None) -> None:
    """hashgrid_probe_copy: dst = src (contiguous device tensors of equal byte size)."""
    nbytes = src.numel() * src.element_size()
    if not (src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()
            and dst.numel() * dst.element_size() == nbytes):
        raise HashGridError("src and dst must be contiguous device tensors of equal size")
    _check(load_probes().hashgrid_probe_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream_ptr(stream)),
           "hashgrid_probe_copy")


def probe_gather(table: torch.Tensor, n_gathers: int, sink: torch.Tensor, seed: int = 1, stream=None) -> None:
    """hashgrid_probe_gather over an int32 device tensor with a power-of-two number of words."""
    if not (table.is_cuda and table.is_contiguous() and table.element_size() == 4 and sink.is_cuda
            and sink.is_contiguous() and sink.element_size() == 4 and sink.numel() >= n_gathers // 16):
        raise HashGridError("table and sink must be contiguous 4-byte device tensors, sink of n_gathers/16 words")
    _check(load_probes().hashgrid_probe_gather(table.data_ptr(), table.numel(), n_gathers, seed, sink.data_ptr(),
                                                _stream_ptr(stream)), "hashgrid_probe_gather")


def probe_atomic_add(table: torch.Tensor, n_adds: int, seed: int = 1, stream=None) -> None:
    """hashgrid_probe_atomic_add over an fp32 device tensor with a power-of-two number of words."""
    if not (table.is_cuda and table.is_contiguous() and table.dtype == torch.float32):
        raise HashGridError("table must be a contiguous fp32 device tensor")
    _check(load_probes().hashgrid_probe_atomic_add(table.data_ptr(), table.numel(), n_adds, seed,
                                                    _stream_ptr(stream)), "hashgrid_probe_atomic_add")


def probe_gather_lines(table: torch.Tensor, slice_words: int, n_slices: int, n_points: int, n_levels: int,
                       sink: torch.Tensor, seed: int = 1, stream=None) -> None:
    """hashgrid_probe_gather_lines: the forward pass's access shape (4 lines x 2 adjacent words per point
    and level, a barrier per level, slice l mod n_slices of the table for level l)."""
    if not (table.is_cuda and table.is_contiguous() and table.element_size() == 4
            and table.numel() >= slice_words * n_slices and sink.is_cuda and sink.is_contiguous()
            and sink.element_size() == 4 and sink.numel() >= n_points):
        raise HashGridError("table must hold n_slices * slice_words 4-byte words, sink n_points words")
    _check(load_probes().hashgrid_probe_gather_lines(table.data_ptr(), slice_words, n_slices, n_points, n_levels,
                                                     seed, sink.data_ptr(), _stream_ptr(stream)),
           "hashgrid_probe_gather_lines")


def mlp_fwd(y: torch.Tensor, W1: torch.Tensor, W2: torch.Tensor, W3: torch.Tensor, out: torch.Tensor | None = None,
            stream=None) -> torch.Tensor:
    """hashgrid_mlp_fwd: the 64-64 ReLU network on features y [B, n_in] fp16 that are in memory; out [B, n_out] fp32."""
    B, n_in = y.shape
    n_out = W3.shape[0]
    if out is None:
        out = torch.empty((B, n_out), dtype=torch.float32, device=y.device)
    _check(load_library().hashgrid_mlp_fwd(
        B, n_in, n_out, _dev(y, torch.float16, (B, n_in), "y"), _dev(W1, torch.float16, (64, n_in), "W1"),
        _dev(W2, torch.float16, (64, 64), "W2"), _dev(W3, torch.float16, (n_out, 64), "W3"),
        _dev(out, torch.float32, (B, n_out), "out"), _stream_ptr(stream)), "hashgrid_mlp_fwd")
    return out


def mlp_bwd(y: torch.Tensor, W1: torch.Tensor, W2: torch.Tensor, W3: torch.Tensor, dLdout: torch.Tensor,
            dLdy: torch.Tensor, dW1: torch.Tensor, dW2: torch.Tensor, dW3: torch.Tensor, stream=None) -> None:
    """hashgrid_mlp_bwd: y [B, n_in] fp16, fp16 weights, dLdout [B, n_out] fp32 -> dLdy [B, n_in] fp16 (written),
    dW1, dW2, dW3 fp32 (accumulated into)."""
    B, n_in = y.shape
    n_out = W3.shape[0]
    _check(load_library().hashgrid_mlp_bwd(
        B, n_in, n_out, _dev(y, torch.float16, (B, n_in), "y"), _dev(W1, torch.float16, (64, n_in), "W1"),
        _dev(W2, torch.float16, (64, 64), "W2"), _dev(W3, torch.float16, (n_out, 64), "W3"),
        _dev(dLdout, torch.float32, (B, n_out), "dLdout"), _dev(dLdy, torch.float16, (B, n_in), "dLdy"),
        _dev(dW1, torch.float32, (64, n_in), "dW1"), _dev(dW2, torch.float32, (64, 64), "dW2"),
        _dev(dW3, torch.float32, (n_out, 64), "dW3"), _stream_ptr(stream)), "hashgrid_mlp_bwd")
