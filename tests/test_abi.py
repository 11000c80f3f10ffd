"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2007_13221_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cser_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared("cser.h")
    assert "cser_create" in names and "cser_step" in names and "cser_error_reset" in names and "cser_destroy" in names
    measure = _declared("cser_measure.h")
    assert "cser_set_tuning" in measure and not set(measure) & set(names)
    lib = ctypes.CDLL(B.LIBRARY)
    for name in names + measure:
        assert hasattr(lib, name), name
    assert sorted(B.EXPORTS) == names          # the binding covers both headers, nothing more
    assert sorted(B.MEASURE_EXPORTS) == measure


def test_config_struct_layout_matches_the_header():
    assert ctypes.sizeof(B.cser_config) == 56
    assert B.cser_config.seed.offset == 48 and B.cser_config.lr.offset == 36


def test_strerror_and_null_destroy():
    assert B.cser_strerror(0) == "ok"
    assert "invalid" in B.cser_strerror(B.CSER_EINVAL)
    assert B._lib().cser_destroy(None) == B.CSER_OK


@pytest.mark.parametrize("change,status", [
    (dict(d=0), B.CSER_EINVAL), (dict(W=0), B.CSER_EINVAL), (dict(block=0), B.CSER_EINVAL),
    (dict(ld=10), B.CSER_EINVAL), (dict(R_reset=0), B.CSER_EINVAL), (dict(momentum=1.0), B.CSER_EINVAL),
    (dict(momentum=-0.1), B.CSER_EINVAL), (dict(lr=float("nan")), B.CSER_EINVAL),
    (dict(d=2**40, ld=2**40, block=1), B.CSER_ERANGE),
])
def test_create_rejects_bad_configs_without_a_device(change, status):
    kw = dict(d=64, W=2, block=8, R_step=2, R_reset=2, H=2, lr=0.1, momentum=0.9, seed=1, ld=64)
    kw.update(change)
    cfg = B.make_config(**kw)
    out = ctypes.c_void_p(123)
    fake = 0x1000   # never dereferenced: validation fails first
    rc = B._lib().cser_create(ctypes.byref(cfg), fake, fake, fake, None, ctypes.byref(out))
    assert rc == status and out.value is None


def test_create_rejects_null_and_misaligned_pointers():
    cfg = B.make_config(64, 2, 8, 2, 2, 2, 0.1, 0.9, 1)
    out = ctypes.c_void_p()
    assert B._lib().cser_create(ctypes.byref(cfg), None, 0x1000, 0x1000, None, ctypes.byref(out)) == B.CSER_EINVAL
    assert B._lib().cser_create(ctypes.byref(cfg), 0x1002, 0x1000, 0x1000, None, ctypes.byref(out)) == B.CSER_EALIGN
    assert B._lib().cser_create(ctypes.byref(cfg), 0x1000, 0x1000, None, None, ctypes.byref(out)) == B.CSER_EINVAL  # no m with beta > 0
    assert B._lib().cser_create(None, 0x1000, 0x1000, 0x1000, None, ctypes.byref(out)) == B.CSER_EINVAL
    assert B._lib().cser_step(None, 0x1000, None) == B.CSER_EINVAL
    assert B._lib().cser_error_reset(None, None) == B.CSER_EINVAL


def test_overall_ratio_matches_the_printed_table4_rows():
    """Section 5.1's formula through the C ABI on the ten CSER rows of Table 4 (tests/golden)."""
    rows = [tuple(int(v) for v in l.split()) for l in open(os.path.join(ROOT, "tests", "golden", "table4_cser_rows.txt"))
            if l.strip() and l[0] != "#"]
    assert len(rows) == 10
    for overall, r_step, r_reset, H in rows:
        cfg = B.make_config(1000, 8, 10, r_step, r_reset, H, 0.1, 0.9, 0)
        assert B.cser_overall_ratio(cfg) == pytest.approx(overall, rel=1e-12)
    # the large workload mirrors the 256x row's pattern with R_step halved: 1 / (1/256 + 1/512) = 170.67
    assert B.cser_overall_ratio(B.make_config(1000, 8, 10, 256, 16, 32, 0.1, 0.9, 0)) == pytest.approx(512 / 3)


def test_table4_workloads_carry_the_printed_rows():
    from paper_2007_13221_amd import inputs as I
    rows = [tuple(int(v) for v in l.split()) for l in open(os.path.join(ROOT, "tests", "golden", "table4_cser_rows.txt"))
            if l.strip() and l[0] != "#"]
    assert tuple(rows) == I.TABLE4_CSER
    for wl, (overall, r_step, r_reset, H) in zip(I.table4_workloads(), rows):
        assert (wl.R_step, wl.R_reset, wl.H) == (r_step, r_reset, H) and wl.steps >= 2 * H and wl.d == 25_557_032
        cfg = B.make_config(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, wl.lr, wl.momentum, wl.seed)
        assert B.cser_overall_ratio(cfg) == pytest.approx(overall, rel=1e-12)


def test_presets_of_the_special_cases():
    cfg = B.cser_preset_csea(B.make_config(1000, 8, 10, 64, 4, 16, 0.1, 0.0, 0))
    assert (cfg.R_step, cfg.H, cfg.R_reset) == (0, 1, 4) and B.cser_overall_ratio(cfg) == 4.0   # CSEA: R = R_C1
    cfg = B.cser_preset_cser_pl(B.make_config(1000, 8, 10, 64, 4, 16, 0.1, 0.0, 0))
    assert (cfg.R_step, cfg.H, cfg.R_reset) == (0, 16, 4) and B.cser_overall_ratio(cfg) == 64.0  # CSER-PL: R_C1 * H
    cfg = B.make_config(1000, 8, 10, 0, 4, 0, 0.1, 0.0, 0)
    assert B.cser_overall_ratio(cfg) == float("inf")
    assert B._lib().cser_preset_csea(None) == B.CSER_EINVAL


def test_default_kernel_by_worker_count_block_size_and_synchronised_share():
    """Host logic of the launch: which fused-step kernel an iteration takes by default (measured break-even points;
    every choice computes the same bits, which the GPU parity tests check)."""
    T, S, G, P = B.KERNEL_TILE, B.KERNEL_SHARED, B.KERNEL_GENERAL, B.KERNEL_SPLIT

    def choice(reset=False, **kw):
        base = dict(d=25_557_032, W=8, block=1024, R_step=256, R_reset=16, H=32, lr=0.1, momentum=0.9, seed=2)
        base.update(kw)
        return B.cser_measure_kernel_choice(B.make_config(**base), reset)

    assert choice() == T and choice(reset=True) == T                   # the large workload: few blocks synchronised
    assert choice(R_step=8) == T and choice(R_step=4) == T
    assert choice(R_step=2) == P                                       # half of the blocks: pair of launches
    assert choice(R_step=2, block=4096) == P and choice(R_step=2, block=256) == P
    assert choice(R_step=2, block=64) == S                             # tiles hold both kinds of blocks: one kernel
    assert choice(R_step=1) == S                                       # everything synchronised
    assert choice(R_step=4, R_reset=2, reset=True) == P and choice(R_step=4, R_reset=2) == T   # Table 4's first row
    assert choice(R_step=0, R_reset=1, reset=True) == S and choice(R_step=0, R_reset=1) == T   # local SGD with period H
    for W in (3, 6, 12, 16):
        assert choice(W=W, R_step=256) == T and choice(W=W, R_step=8) == P and choice(W=W, R_step=1) == S
    for W in (17, 32, 64, 96, 1000):
        assert choice(W=W, R_step=256) == P and choice(W=W, R_step=2) == P and choice(W=W, R_step=1) == G
    assert choice(W=32, R_step=0) == T and choice(W=96, R_step=0) == P  # nothing synchronised; beyond 64 workers only the pair's first half fits
    assert choice(W=32, R_step=32, block=64) == P and choice(W=32, R_step=4, block=64) == G   # short blocks: few / many tiles hold both kinds
    assert choice(block=6) == G and choice(block=1022) == G            # not a multiple of 4 columns: element-wise kernels
    assert choice(W=70_000) == G                                       # more workers than a grid dimension takes
    assert B._lib().cser_measure_kernel_choice(None, 0, None) == B.CSER_EINVAL
