"""Thin ctypes binding of the C ABI in include/cser.h (and of the measurement entry points in
include/cser_measure.h): same names, argument marshalling only.

Every step of the update runs in the HIP kernels of libcser_hip.so; this module never computes
anything and has no fallback: if the library is missing or does not load, the first call raises.
PyTorch appears only as the owner of device memory (tensors) and of the current stream.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIBRARY = os.path.join(_HERE, "libcser_hip.so")

CSER_OK, CSER_EINVAL, CSER_EALIGN, CSER_ENOMEM, CSER_EHIP, CSER_ERANGE = 0, -1, -2, -3, -4, -5
CSER_STATIC_MAX_BLOCKS = 524288

EXPORTS = ("cser_create", "cser_step", "cser_step_many", "cser_step_static", "cser_error_reset", "cser_destroy", "cser_select_blocks",
           "cser_preset_csea", "cser_preset_cser_pl", "cser_overall_ratio",
           "cser_block_counts", "cser_set_lr", "cser_get_step", "cser_set_step", "cser_strerror", "cser_last_hip_error")
MEASURE_EXPORTS = ("cser_profile_enable", "cser_profile_read", "cser_profile_clear", "cser_set_tuning",
                   "cser_measure_counters", "cser_measure_residency", "cser_measure_kernel_choice", "cser_copy_probe")

# cser_tuning_key
CSER_TUNE_KERNEL, CSER_TUNE_NONTEMPORAL, CSER_TUNE_FUSE_RESET = 0, 1, 2
CSER_TUNE_TILE_WAVES_PER_CU, CSER_TUNE_SHARED_GROUPS_PER_CU = 3, 4
KERNEL_AUTO, KERNEL_TILE, KERNEL_SHARED, KERNEL_GENERAL, KERNEL_SPLIT = 0, 1, 2, 3, 4


class cser_config(ctypes.Structure):
    _fields_ = [("d", ctypes.c_uint64), ("ld", ctypes.c_uint64), ("W", ctypes.c_uint32),
                ("block", ctypes.c_uint32), ("R_step", ctypes.c_uint32), ("R_reset", ctypes.c_uint32),
                ("H", ctypes.c_uint32), ("lr", ctypes.c_float), ("momentum", ctypes.c_float),
                ("seed", ctypes.c_uint64)]


class cser_counters(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint64) for n in ("steps", "window_draws", "resets_fused", "resets_separate",
                                               "launches_tile", "launches_shared", "launches_general",
                                               "launches_split")]


class cser_residency(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in ("tile_lds", "tile_groups_per_cu", "shared_lds", "shared_groups_per_cu",
                                               "shared_reset_lds", "shared_reset_groups_per_cu", "reset_lds",
                                               "reset_groups_per_cu")]


class CSERError(RuntimeError):
    def __init__(self, status, where):
        text = _lib().cser_strerror(status).decode()
        detail = _lib().cser_last_hip_error().decode() if status == CSER_EHIP else ""
        super().__init__(f"{where}: {text} ({status})" + (f": {detail}" if detail else ""))
        self.status = status


_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIBRARY):
            raise RuntimeError(f"{LIBRARY} is missing: build it with `python -m paper_2007_13221_amd.build` "
                               "(there is no CPU fallback)")
        # torch first: the library must bind to the HIP runtime instance torch has loaded, because the
        # device pointers and streams it is handed belong to that instance
        import torch  # noqa: F401
        L = ctypes.CDLL(LIBRARY)
        vp, u64, u32, i64 = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int64
        L.cser_create.argtypes = [ctypes.POINTER(cser_config), vp, vp, vp, vp, ctypes.POINTER(vp)]
        L.cser_step.argtypes = [vp, vp, vp]
        L.cser_step_many.argtypes = [vp, vp, u32, vp, ctypes.POINTER(u32)]
        L.cser_step_static.argtypes = [ctypes.POINTER(cser_config), u64, vp, vp, vp, vp, vp]
        L.cser_error_reset.argtypes = [vp, vp]
        L.cser_destroy.argtypes = [vp]
        L.cser_select_blocks.argtypes = [vp, ctypes.c_int, u64, vp, vp, ctypes.POINTER(u32)]
        L.cser_block_counts.argtypes = [vp, ctypes.POINTER(u64), ctypes.POINTER(u32), ctypes.POINTER(u32)]
        L.cser_preset_csea.argtypes = [ctypes.POINTER(cser_config)]
        L.cser_preset_cser_pl.argtypes = [ctypes.POINTER(cser_config)]
        L.cser_overall_ratio.argtypes = [ctypes.POINTER(cser_config), ctypes.POINTER(ctypes.c_double)]
        L.cser_set_lr.argtypes = [vp, ctypes.c_float]
        L.cser_get_step.argtypes = [vp, ctypes.POINTER(u64)]
        L.cser_set_step.argtypes = [vp, u64]
        L.cser_profile_enable.argtypes = [vp, ctypes.c_int]
        L.cser_profile_read.argtypes = [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(u64)]
        L.cser_profile_clear.argtypes = [vp]
        L.cser_set_tuning.argtypes = [vp, ctypes.c_int, i64]
        L.cser_copy_probe.argtypes = [vp, vp, u64, vp]
        L.cser_measure_counters.argtypes = [vp, ctypes.POINTER(cser_counters)]
        L.cser_measure_residency.argtypes = [vp, ctypes.POINTER(cser_residency)]
        L.cser_measure_kernel_choice.argtypes = [ctypes.POINTER(cser_config), ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
        L.cser_strerror.argtypes = [ctypes.c_int]
        L.cser_strerror.restype = ctypes.c_char_p
        L.cser_last_hip_error.argtypes = []
        L.cser_last_hip_error.restype = ctypes.c_char_p
        for name in EXPORTS + MEASURE_EXPORTS:
            if name not in ("cser_strerror", "cser_last_hip_error"):
                getattr(L, name).restype = ctypes.c_int
        _LIB = L
    return _LIB


def _check(status, where):
    if status != CSER_OK:
        raise CSERError(status, where)


def _ptr(t):
    """Device address of a torch tensor (or None, or a raw integer address)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    """Raw hipStream_t: None means torch's current stream."""
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def cser_create(cfg: cser_config, x, e, m, stream=None):
    """x, e, m: device tensors [W][ld] fp32 (e and/or m may be None, see cser.h). Returns a handle."""
    handle = ctypes.c_void_p()
    _check(_lib().cser_create(ctypes.byref(cfg), _ptr(x), _ptr(e), _ptr(m), _stream(stream), ctypes.byref(handle)),
           "cser_create")
    return handle


def cser_step(ctx, g, stream=None):
    _check(_lib().cser_step(ctx, _ptr(g), _stream(stream)), "cser_step")


def cser_step_many(ctx, grads, stream=None):
    """grads: a sequence of device tensors (or raw addresses), one per iteration; or a prepared
    (ctypes pointer array, n) pair from gradient_list()."""
    if not (isinstance(grads, tuple) and len(grads) == 2 and isinstance(grads[1], int)):
        grads = gradient_list(grads)
    arr, n = grads
    done = ctypes.c_uint32()
    _check(_lib().cser_step_many(ctx, arr, n, _stream(stream), ctypes.byref(done)), "cser_step_many")
    return done.value


def cser_step_static(cfg: cser_config, t, x, e, m, g, stream=None):
    """Iteration t of configuration cfg on the caller's buffers, without a context and without any allocation."""
    _check(_lib().cser_step_static(ctypes.byref(cfg), int(t), _ptr(x), _ptr(e), _ptr(m), _ptr(g), _stream(stream)),
           "cser_step_static")


def gradient_list(grads):
    """The host array of device pointers cser_step_many takes, built once for repeated use."""
    arr = (ctypes.c_void_p * len(grads))(*[_ptr(g) for g in grads])
    return arr, len(grads)


def cser_error_reset(ctx, stream=None):
    _check(_lib().cser_error_reset(ctx, _stream(stream)), "cser_error_reset")


def cser_destroy(ctx):
    _check(_lib().cser_destroy(ctx), "cser_destroy")


def cser_block_counts(ctx):
    B, ks, kr = ctypes.c_uint64(), ctypes.c_uint32(), ctypes.c_uint32()
    _check(_lib().cser_block_counts(ctx, ctypes.byref(B), ctypes.byref(ks), ctypes.byref(kr)), "cser_block_counts")
    return B.value, ks.value, kr.value


def cser_select_blocks(ctx, which, t):
    """Returns (idx[k] uint32 in draw order, mask[B] uint8) as numpy arrays."""
    B, ks, kr = cser_block_counts(ctx)
    k = ks if which == 0 else kr
    idx = np.zeros(max(k, 1), dtype=np.uint32)
    mask = np.zeros(B, dtype=np.uint8)
    kout = ctypes.c_uint32()
    _check(_lib().cser_select_blocks(ctx, int(which), int(t), idx.ctypes.data, mask.ctypes.data, ctypes.byref(kout)),
           "cser_select_blocks")
    assert kout.value == k
    return idx[:k], mask


def cser_preset_csea(cfg: cser_config) -> cser_config:
    _check(_lib().cser_preset_csea(ctypes.byref(cfg)), "cser_preset_csea")
    return cfg


def cser_preset_cser_pl(cfg: cser_config) -> cser_config:
    _check(_lib().cser_preset_cser_pl(ctypes.byref(cfg)), "cser_preset_cser_pl")
    return cfg


def cser_overall_ratio(cfg: cser_config) -> float:
    r = ctypes.c_double()
    _check(_lib().cser_overall_ratio(ctypes.byref(cfg), ctypes.byref(r)), "cser_overall_ratio")
    return r.value


def cser_set_lr(ctx, lr):
    _check(_lib().cser_set_lr(ctx, float(lr)), "cser_set_lr")


def cser_get_step(ctx):
    t = ctypes.c_uint64()
    _check(_lib().cser_get_step(ctx, ctypes.byref(t)), "cser_get_step")
    return t.value


def cser_set_step(ctx, t):
    _check(_lib().cser_set_step(ctx, int(t)), "cser_set_step")


def cser_profile_enable(ctx, on=True):
    _check(_lib().cser_profile_enable(ctx, 1 if on else 0), "cser_profile_enable")


def cser_profile_read(ctx, which):
    """Returns (total_ms, launches) of the fused-step kernel (which=0) or the reset kernel (which=1)."""
    ms, n = ctypes.c_double(), ctypes.c_uint64()
    _check(_lib().cser_profile_read(ctx, int(which), ctypes.byref(ms), ctypes.byref(n)), "cser_profile_read")
    return ms.value, n.value


def cser_profile_clear(ctx):
    _check(_lib().cser_profile_clear(ctx), "cser_profile_clear")


def cser_set_tuning(ctx, key, value):
    _check(_lib().cser_set_tuning(ctx, int(key), int(value)), "cser_set_tuning")


def cser_measure_counters(ctx):
    c = cser_counters()
    _check(_lib().cser_measure_counters(ctx, ctypes.byref(c)), "cser_measure_counters")
    return {n: getattr(c, n) for n, _ in cser_counters._fields_}


def cser_measure_residency(ctx):
    r = cser_residency()
    _check(_lib().cser_measure_residency(ctx, ctypes.byref(r)), "cser_measure_residency")
    return {n: getattr(r, n) for n, _ in cser_residency._fields_}


def cser_measure_kernel_choice(cfg: cser_config, reset_iteration=False) -> int:
    """The fused-step kernel (KERNEL_TILE, KERNEL_SHARED, KERNEL_GENERAL or KERNEL_SPLIT) an iteration of cfg takes."""
    k = ctypes.c_int()
    _check(_lib().cser_measure_kernel_choice(ctypes.byref(cfg), int(bool(reset_iteration)), ctypes.byref(k)),
           "cser_measure_kernel_choice")
    return k.value


def cser_copy_probe(dst, src, n_bytes, stream=None):
    _check(_lib().cser_copy_probe(_ptr(dst), _ptr(src), int(n_bytes), _stream(stream)), "cser_copy_probe")


def cser_strerror(status):
    return _lib().cser_strerror(int(status)).decode()


def make_config(d, W, block, R_step, R_reset, H, lr, momentum, seed, ld=None) -> cser_config:
    return cser_config(int(d), int(d if ld is None else ld), int(W), int(block), int(R_step), int(R_reset),
                       int(H), float(lr), float(momentum), int(seed))


class CSER:
    """Convenience owner of a context and its state tensors (allocation and lifetime only)."""

    def __init__(self, cfg: cser_config, x, with_error=True, with_momentum=True, stream=None, e=None, m=None):
        """e, m: tensors to use for the residual and the momentum (cser_create zero-fills them); allocated here if None."""
        import torch
        assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and tuple(x.shape) == (cfg.W, cfg.ld)
        for t in (e, m):
            assert t is None or (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.shape == x.shape)
        self.cfg = cfg
        self.x = x
        self.e = (torch.zeros_like(x) if e is None else e) if with_error else None
        self.m = (torch.zeros_like(x) if m is None else m) if with_momentum else None
        self.ctx = cser_create(cfg, self.x, self.e, self.m, stream)

    def step(self, g, stream=None):
        cser_step(self.ctx, g, stream)

    def step_many(self, grads, stream=None):
        return cser_step_many(self.ctx, grads, stream)

    def error_reset(self, stream=None):
        cser_error_reset(self.ctx, stream)

    def close(self):
        if self.ctx is not None:
            cser_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
