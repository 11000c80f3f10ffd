"""The entry point that allocates nothing, cser_step_static, against cser_step: same bits on the same inputs.

Collected last (file name): it keeps calling into one per-GPU array that earlier calls have written, first
with a larger configuration, then with smaller ones.
"""
import ctypes

import pytest
import torch

from paper_2007_13221_amd import binding as B
from paper_2007_13221_amd import inputs as I

pytestmark = pytest.mark.gpu


def _pair(wl, steps, with_error=True, with_momentum=True, ld=None):
    """`steps` iterations through a context (cser_step) and through cser_step_static; returns both sets of states."""
    dev = torch.device("cuda:0")
    ld = wl.ld if ld is None else ld
    momentum = wl.momentum if with_momentum else 0.0
    cfg = B.make_config(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, wl.lr, momentum, wl.seed, ld=ld)
    opt = B.CSER(cfg, I.initial_model(wl, dev, ld=ld), with_error=with_error, with_momentum=with_momentum)
    x = I.initial_model(wl, dev, ld=ld)
    e = torch.zeros_like(x) if with_error else None
    m = torch.zeros_like(x) if with_momentum else None
    for t in range(1, steps + 1):
        g = I.gradient(wl, t, dev, ld=ld)
        opt.step(g)
        B.cser_step_static(cfg, t, x, e, m, g)
    torch.cuda.synchronize()
    out = (opt.x.clone(), None if e is None else opt.e.clone(), None if m is None else opt.m.clone()), (x, e, m)
    opt.close()
    return out


def _same(a, b):
    for u, v in zip(a, b):
        assert (u is None) == (v is None)
        if u is not None:
            assert torch.equal(u, v)
    assert a[0].abs().max() > 0


def _wl(**kw):
    base = dict(name="case", d=5000, W=4, block=64, R_step=4, R_reset=2, H=3, lr=0.1, momentum=0.9,
                x_var=1e-2, g_var=1e-2, seed=11, steps=12)
    base.update(kw)
    return I.Workload(**base)


def test_two_calls_in_a_row_the_second_with_a_smaller_input():
    # larger first: 7,813 blocks of 64 columns, 8 workers, resets every other iteration (fused into the same kernel pass)
    _same(*_pair(_wl(d=500_000, W=8, R_step=4, R_reset=2, H=2, seed=3), 6))
    # then smaller: 79 blocks; the array still holds the larger call's masks beyond them
    _same(*_pair(_wl(d=5000, W=4, R_step=3, R_reset=2, H=3, seed=4), 7))
    # and larger again, with most blocks chosen (the selector then fills with ones and clears the exceptions)
    _same(*_pair(_wl(d=200_000, W=8, block=8, R_step=1, R_reset=1, H=2, seed=5), 4))


@pytest.mark.parametrize("kw,with_error,with_momentum", [
    (dict(), False, True), (dict(momentum=0.0), True, False), (dict(momentum=0.0), False, False),
    (dict(W=3), True, True), (dict(W=20, d=3000), True, True), (dict(W=70, d=2000), True, True),
    (dict(block=6, d=4099), True, True), (dict(d=4099, block=4), True, True), (dict(R_step=0, H=1), True, True), (dict(H=0), True, True),
    (dict(block=256, d=40_000, W=8, R_step=2), True, True),    # half of the tiles synchronised: the pair of launches
    (dict(block=512, d=40_000, W=6, R_step=4, R_reset=1, H=2), True, True),
])
def test_state_variants_worker_counts_and_layouts(kw, with_error, with_momentum):
    wl = _wl(**kw)
    _same(*_pair(wl, 7, with_error=with_error, with_momentum=with_momentum))


def test_unpadded_rows():
    _same(*_pair(_wl(d=4099), 6, ld=4099))


def test_sizes_beyond_the_fixed_array_and_bad_arguments_are_rejected():
    dev = torch.device("cuda:0")
    x = torch.zeros(1, 64, device=dev)
    too_many = B.make_config((B.CSER_STATIC_MAX_BLOCKS + 1) * 4, 1, 4, 2, 2, 2, 0.1, 0.0, 1)
    assert B._lib().cser_step_static(ctypes.byref(too_many), 1, x.data_ptr(), None, None, x.data_ptr(), None) == B.CSER_ERANGE
    just_fits = B.make_config(B.CSER_STATIC_MAX_BLOCKS * 4, 1, 4, 2, 2, 2, 0.1, 0.0, 1)
    assert B._lib().cser_step_static(ctypes.byref(just_fits), 1, x.data_ptr(), None, None, None, None) == B.CSER_EINVAL   # no g
    ok = B.make_config(64, 1, 4, 2, 2, 2, 0.1, 0.9, 1)
    assert B._lib().cser_step_static(ctypes.byref(ok), 1, x.data_ptr(), None, None, x.data_ptr(), None) == B.CSER_EINVAL  # beta > 0 without m
    assert B._lib().cser_step_static(None, 1, x.data_ptr(), None, None, x.data_ptr(), None) == B.CSER_EINVAL
    assert B._lib().cser_step_static(ctypes.byref(ok), 1, x.data_ptr() + 2, None, x.data_ptr(), x.data_ptr(), None) == B.CSER_EALIGN
    torch.cuda.synchronize()
    assert not x.any()      # nothing was launched


def test_largest_size_the_array_takes():
    """B = CSER_STATIC_MAX_BLOCKS exactly: both masks fill their halves of the array to the last byte."""
    wl = _wl(d=B.CSER_STATIC_MAX_BLOCKS * 4 - 1, W=2, block=4, R_step=3, R_reset=2, H=1, seed=6)
    assert wl.B == B.CSER_STATIC_MAX_BLOCKS
    _same(*_pair(wl, 2))


# ---------------------------------------------------------------------------- under HIP graph capture
# The call allocates nothing, so once its per-device set-up has run it can be recorded into a HIP graph; every replay,
# with eager work in between, must give what the same eager call gives.
@pytest.mark.parametrize("kw", [dict(d=50_000, W=4, block=64, R_step=4, R_reset=2, H=2),
                                dict(d=40_000, W=8, block=256, R_step=2, R_reset=2, H=3)])
def test_recorded_call_replays_like_the_eager_call(kw):
    dev = torch.device("cuda:0")
    wl = I.Workload(name="graph", lr=0.1, momentum=0.9, x_var=1e-2, g_var=1e-2, seed=21, steps=8, **kw)
    cfg = B.make_config(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, wl.lr, wl.momentum, wl.seed, ld=wl.ld)
    t_rec = 2 * wl.H if wl.H else 2          # an iteration that carries an error reset as well
    state = [I.initial_model(wl, dev), torch.zeros(wl.W, wl.ld, device=dev), torch.zeros(wl.W, wl.ld, device=dev)]
    ref = [s.clone() for s in state]
    g = I.gradient(wl, 1, dev)
    B.cser_step_static(cfg, 1, *state, g)    # first call on the device: looks up the array and the launch shapes
    B.cser_step_static(cfg, 1, *ref, g)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        with torch.cuda.graph(graph, stream=s):
            B.cser_step_static(cfg, t_rec, *state, g, stream=s)
    torch.cuda.synchronize()
    for replay in range(4):
        g.copy_(I.gradient(wl, 10 + replay, dev))           # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        B.cser_step_static(cfg, t_rec, *ref, g)
        torch.cuda.synchronize()
        for a, b in zip(state, ref):
            assert torch.equal(a, b), replay
    assert state[0].abs().max() > 0
