"""ctypes loader for the CPU oracle of the multiresolution hash encoding.

TEST INFRASTRUCTURE ONLY: the test-suite, the smoke check and the benchmark's
CPU-baseline leg use this module; the GPU library never does.  All arithmetic
lives in ``hashgrid_oracle.c`` (paper Section 3, Eq. 2-4; Appendix A); this file
only compiles that C file with gcc, widens arrays to fp64 (exact for fp16 and
fp32 inputs) and marshals pointers.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hashgrid_oracle.c")
_LIB = os.path.join(_HERE, "libhashgrid_oracle.so")
_MAX_LEVELS = 64

INTERP_LINEAR = 0
INTERP_SMOOTHSTEP = 1


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (fp contraction off so that the fp32
    scale step stays one rounded multiply)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
               "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


class _Config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in ("d", "L", "F", "T", "N_min", "N_max", "interp")]


class _Levels(ctypes.Structure):
    _fields_ = [
        ("N", ctypes.c_uint32 * _MAX_LEVELS),
        ("verts", ctypes.c_uint32 * _MAX_LEVELS),
        ("offset", ctypes.c_uint64 * _MAX_LEVELS),
        ("size", ctypes.c_uint32 * _MAX_LEVELS),
        ("dense", ctypes.c_int32 * _MAX_LEVELS),
        ("total", ctypes.c_uint64),
    ]


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        vp, u64, u32 = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32
        cfgp = ctypes.POINTER(_Config)
        lib.hgo_num_threads.restype = ctypes.c_int
        lib.hgo_set_num_threads.argtypes = [ctypes.c_int]
        lib.hgo_set_num_threads.restype = None
        lib.hgo_levels.argtypes = [cfgp, ctypes.POINTER(_Levels)]
        lib.hgo_index.argtypes = [u32, u32, u32, ctypes.c_int, vp]
        lib.hgo_index.restype = u32
        lib.hgo_check_x.argtypes = [u64, vp]
        lib.hgo_check_x.restype = u64
        lib.hgo_fwd.argtypes = [cfgp, u64, vp, vp, vp]
        lib.hgo_bwd.argtypes = [cfgp, u64, vp, vp, vp]
        lib.hgo_bwd_input.argtypes = [cfgp, u64, vp, vp, vp, vp]
        lib.hgo_indices.argtypes = [cfgp, u64, vp, u32, vp, vp]
        dbl = ctypes.c_double
        lib.hgo_adam_step.argtypes = [u64, vp, vp, vp, vp, dbl, dbl, dbl, dbl, dbl, u32]
        _lib = lib
    return _lib


@dataclass(frozen=True)
class LevelTable:
    N: np.ndarray       # [L] uint32   resolution N_l
    verts: np.ndarray   # [L] uint32   grid vertices per axis
    offset: np.ndarray  # [L] uint64   first entry of the level
    size: np.ndarray    # [L] uint32   entries in the level
    dense: np.ndarray   # [L] bool     1:1 indexed level
    total: int          # entries over all levels


@dataclass(frozen=True)
class OracleConfig:
    d: int
    L: int
    F: int
    T: int
    N_min: int
    N_max: int
    interp: int = INTERP_LINEAR

    def _c(self) -> _Config:
        return _Config(self.d, self.L, self.F, self.T, self.N_min, self.N_max, self.interp)


def num_threads() -> int:
    return int(_load().hgo_num_threads())


def set_num_threads(n: int) -> None:
    """Threads the following calls may use (for timing on one core); results do not depend on it."""
    _load().hgo_set_num_threads(int(n))


def levels(cfg: OracleConfig) -> LevelTable:
    lv = _Levels()
    if _load().hgo_levels(ctypes.byref(cfg._c()), ctypes.byref(lv)) != 0:
        raise ValueError(f"invalid configuration {cfg}")
    L = cfg.L
    return LevelTable(
        N=np.array(lv.N[:L], dtype=np.uint32), verts=np.array(lv.verts[:L], dtype=np.uint32),
        offset=np.array(lv.offset[:L], dtype=np.uint64), size=np.array(lv.size[:L], dtype=np.uint32),
        dense=np.array(lv.dense[:L], dtype=bool), total=int(lv.total))


def index(d: int, verts: int, T: int, dense: bool, v) -> int:
    vv = np.ascontiguousarray(v, dtype=np.uint32)
    assert vv.shape == (d,)
    return int(_load().hgo_index(d, verts, T, int(dense), vv.ctypes.data))


def _x32(cfg: OracleConfig, x) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    if x.ndim != 2 or x.shape[1] != cfg.d:
        raise ValueError(f"x must be [B,{cfg.d}], got {x.shape}")
    return x


def _f64(a, shape) -> np.ndarray:
    a = np.ascontiguousarray(np.asarray(a).astype(np.float64, copy=False))
    if a.shape != shape:
        raise ValueError(f"expected shape {shape}, got {a.shape}")
    return a


def _check(rc: int) -> None:
    if rc == -1:
        raise ValueError("invalid configuration")
    if rc == -2:
        raise ValueError("x has a coordinate outside [0,1) or not finite")
    if rc != 0:
        raise RuntimeError(f"oracle returned {rc}")


def encode_fwd(cfg: OracleConfig, x, theta) -> np.ndarray:
    """y [B, L*F] in fp64 from x [B,d] fp32 and theta [total, F] (any float dtype)."""
    x = _x32(cfg, x)
    total = levels(cfg).total
    theta = _f64(theta, (total, cfg.F))
    y = np.zeros((x.shape[0], cfg.L * cfg.F), dtype=np.float64)
    _check(_load().hgo_fwd(ctypes.byref(cfg._c()), x.shape[0], x.ctypes.data, theta.ctypes.data, y.ctypes.data))
    return y


def encode_bwd(cfg: OracleConfig, x, dy, dtheta=None) -> np.ndarray:
    """dtheta [total, F] fp64 (accumulated into ``dtheta`` when given) from dy [B, L*F]."""
    x = _x32(cfg, x)
    total = levels(cfg).total
    dy = _f64(dy, (x.shape[0], cfg.L * cfg.F))
    if dtheta is None:
        dtheta = np.zeros((total, cfg.F), dtype=np.float64)
    assert dtheta.dtype == np.float64 and dtheta.flags.c_contiguous and dtheta.shape == (total, cfg.F)
    _check(_load().hgo_bwd(ctypes.byref(cfg._c()), x.shape[0], x.ctypes.data, dy.ctypes.data, dtheta.ctypes.data))
    return dtheta


def encode_bwd_input(cfg: OracleConfig, x, theta, dy) -> np.ndarray:
    """dx [B, d] fp64."""
    x = _x32(cfg, x)
    total = levels(cfg).total
    theta = _f64(theta, (total, cfg.F))
    dy = _f64(dy, (x.shape[0], cfg.L * cfg.F))
    dx = np.zeros((x.shape[0], cfg.d), dtype=np.float64)
    _check(_load().hgo_bwd_input(ctypes.byref(cfg._c()), x.shape[0], x.ctypes.data, theta.ctypes.data,
                                 dy.ctypes.data, dx.ctypes.data))
    return dx


def indices(cfg: OracleConfig, x, level: int):
    """(idx [B, 2^d] uint32 level-local, w [B, d] fp32) as decided in fp32."""
    x = _x32(cfg, x)
    idx = np.zeros((x.shape[0], 1 << cfg.d), dtype=np.uint32)
    w = np.zeros((x.shape[0], cfg.d), dtype=np.float32)
    _check(_load().hgo_indices(ctypes.byref(cfg._c()), x.shape[0], x.ctypes.data, level, idx.ctypes.data,
                               w.ctypes.data))
    return idx, w


def adam_step(theta, grad, m, v, lr, beta1=0.9, beta2=0.99, eps=1e-15, step=1, l2=0.0):
    """One optimiser step on fp64 arrays, in place (theta, m, v); entries with grad == 0 are skipped; l2: the
    factor of the L2 regularisation (Section 4, "Training": 1e-6 on the network's weights, none on the tables)."""
    for a in (theta, m, v):
        assert a.dtype == np.float64 and a.flags.c_contiguous
    g = np.ascontiguousarray(grad, dtype=np.float64)
    assert theta.shape == g.shape == m.shape == v.shape
    rc = _load().hgo_adam_step(theta.size, theta.ctypes.data, g.ctypes.data, m.ctypes.data, v.ctypes.data,
                               float(lr), float(beta1), float(beta2), float(eps), float(l2), int(step))
    if rc != 0:
        raise ValueError("invalid arguments")
