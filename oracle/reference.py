"""ctypes access to the CPU oracle -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Only tests/, the smoke check and the benchmark's cpu-baseline leg may import this module.
It loads oracle/liboracle_cser.so (built from cser_oracle.cpp by oracle/build.py) and adds
the iteration loop of Algorithm 3 around the oracle's per-statement routines: count t from 1,
run the local step, and run the error reset when t mod H = 0.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


class _Problem(ctypes.Structure):
    _fields_ = [("d", ctypes.c_uint64), ("seed", ctypes.c_uint64), ("col0", ctypes.c_uint64),
                ("ncols", ctypes.c_uint64), ("ld", ctypes.c_uint64), ("W", ctypes.c_uint32),
                ("block", ctypes.c_uint32)]


def load(path):
    """Open an oracle library and declare its signatures."""
    L = ctypes.CDLL(path)
    u64, u32, dbl, vp = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_double, ctypes.c_void_p
    L.oracle_philox4x32_10.argtypes = [vp, vp, vp]
    L.oracle_philox4x32_10.restype = None
    L.oracle_blocks_kept.argtypes = [u64, u64]
    L.oracle_blocks_kept.restype = u64
    L.oracle_block_perm.argtypes = [u64, u32, u64, u64, u64]
    L.oracle_block_perm.restype = u64
    L.oracle_block_perm_inverse.argtypes = [u64, u32, u64, u64, u64]
    L.oracle_block_perm_inverse.restype = u64
    L.oracle_select_blocks.argtypes = [u64, u32, u64, u64, u64, vp, vp]
    L.oracle_select_blocks.restype = ctypes.c_int
    pp = ctypes.POINTER(_Problem)
    for sfx in ("f32", "f64"):
        getattr(L, "oracle_mcser_local_step_" + sfx).argtypes = [pp, u64, u64, dbl, dbl, vp, vp, vp, vp]
        getattr(L, "oracle_mcser_error_reset_" + sfx).argtypes = [pp, u64, u64, vp, vp]
        getattr(L, "oracle_cser2_local_step_" + sfx).argtypes = [pp, u64, u64, dbl, dbl, vp, vp, vp]
        getattr(L, "oracle_cser2_model_sync_" + sfx).argtypes = [pp, u64, u64, vp]
    return L


def lib():
    global _LIB
    if _LIB is None:
        _LIB = load(_build.build(force=False))
    return _LIB


def philox4x32_10(counter, key):
    c = np.asarray(counter, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(c.ctypes.data, k.ctypes.data, out.ctypes.data)
    return out


def blocks_kept(B, R):
    return int(lib().oracle_blocks_kept(int(B), int(R)))


def block_perm(seed, stream, t, B, v):
    return int(lib().oracle_block_perm(int(seed), int(stream), int(t), int(B), int(v)))


def block_perm_inverse(seed, stream, t, B, v):
    return int(lib().oracle_block_perm_inverse(int(seed), int(stream), int(t), int(B), int(v)))


def select_blocks(seed, stream, t, B, k):
    """Return (idx[k] uint32 in draw order, mask[B] uint8) for the given stream (0 step, 1 reset)."""
    idx = np.zeros(int(k), dtype=np.uint32)
    mask = np.zeros(int(B), dtype=np.uint8)
    rc = lib().oracle_select_blocks(int(seed), int(stream), int(t), int(B), int(k),
                                    idx.ctypes.data if k else None, mask.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_select_blocks: bad argument")
    return idx, mask


class OracleCSER:
    """M-CSER (Algorithm 3), or implementation II when with_error=False, for W workers.

    State arrays are numpy [W][ncols] and hold the global columns of blocks [b0, b1); the
    block choice is always made over all B blocks, so a slice evolves exactly as it does in
    the full run.
    """

    def __init__(self, d, W, block, R_step, R_reset, H, lr, momentum, seed, x0_row, dtype=np.float32,
                 b0=0, b1=None, with_error=True):
        self.d, self.W, self.block = int(d), int(W), int(block)
        self.R_step, self.R_reset, self.H = int(R_step), int(R_reset), int(H)
        self.dtype = np.dtype(dtype)
        self.sfx = {"float32": "f32", "float64": "f64"}[self.dtype.name]
        # the step size and momentum the float path uses are the float-rounded ones
        self.lr = float(np.float32(lr)) if self.sfx == "f32" else float(lr)
        self.momentum = float(np.float32(momentum)) if self.sfx == "f32" else float(momentum)
        self.seed = int(seed)
        self.B = -(-self.d // self.block)
        self.b0 = int(b0)
        self.b1 = self.B if b1 is None else int(b1)
        self.col0 = self.b0 * self.block
        self.col1 = min(self.d, self.b1 * self.block)
        n = self.col1 - self.col0
        x0_row = np.asarray(x0_row)
        assert x0_row.shape == (n,), (x0_row.shape, n)
        self.x = np.ascontiguousarray(np.broadcast_to(x0_row.astype(self.dtype), (self.W, n)))
        self.m = np.zeros((self.W, n), dtype=self.dtype)
        self.e = np.zeros((self.W, n), dtype=self.dtype) if with_error else None
        self.t = 0
        self._pb = _Problem(self.d, self.seed, self.col0, n, n, self.W, self.block)

    @property
    def k_step(self):
        return blocks_kept(self.B, self.R_step)

    @property
    def k_reset(self):
        return blocks_kept(self.B, self.R_reset)

    def set_lr(self, lr):
        self.lr = float(np.float32(lr)) if self.sfx == "f32" else float(lr)

    def step(self, g):
        g = np.ascontiguousarray(g, dtype=self.dtype)
        assert g.shape == self.x.shape
        self.t += 1
        L = lib()
        if self.e is not None:
            rc = getattr(L, "oracle_mcser_local_step_" + self.sfx)(
                ctypes.byref(self._pb), self.t, self.R_step, self.lr, self.momentum,
                self.x.ctypes.data, self.e.ctypes.data, self.m.ctypes.data, g.ctypes.data)
        else:
            rc = getattr(L, "oracle_cser2_local_step_" + self.sfx)(
                ctypes.byref(self._pb), self.t, self.R_step, self.lr, self.momentum,
                self.x.ctypes.data, self.m.ctypes.data, g.ctypes.data)
        assert rc == 0
        if self.H > 0 and self.t % self.H == 0:
            self.error_reset()

    def error_reset(self):
        L = lib()
        if self.e is not None:
            rc = getattr(L, "oracle_mcser_error_reset_" + self.sfx)(
                ctypes.byref(self._pb), self.t, self.R_reset, self.x.ctypes.data, self.e.ctypes.data)
        else:
            rc = getattr(L, "oracle_cser2_model_sync_" + self.sfx)(
                ctypes.byref(self._pb), self.t, self.R_reset, self.x.ctypes.data)
        assert rc == 0
