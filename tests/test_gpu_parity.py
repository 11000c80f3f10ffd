"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Block indices and masks must be bit-exact; fp32 states must satisfy
|gpu - oracle| <= 1e-7 + 1e-6 |oracle| (the stated bar); with the shared arithmetic contract
(written-out fused multiply-adds, in-order worker sum, true division) the two are in fact expected
to agree bit for bit, which the tests also record.
"""
import ctypes

import numpy as np
import pytest
import torch

from oracle import reference as R
from paper_2007_13221_amd import binding as B
from paper_2007_13221_amd import inputs as I

pytestmark = pytest.mark.gpu

ABS_TOL, REL_TOL = 1e-7, 1e-6

# launch shapes (measurement interface): every one must give the same bits
K, NT, FUSE, TILE_CAP, SHARED_CAP = (B.CSER_TUNE_KERNEL, B.CSER_TUNE_NONTEMPORAL, B.CSER_TUNE_FUSE_RESET,
                                     B.CSER_TUNE_TILE_WAVES_PER_CU, B.CSER_TUNE_SHARED_GROUPS_PER_CU)
TILE, SHARED, GENERAL, SPLIT = B.KERNEL_TILE, B.KERNEL_SHARED, B.KERNEL_GENERAL, B.KERNEL_SPLIT


def assert_states_close(name, got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (name, got.shape, want.shape)
    err = np.abs(got - want)
    bound = ABS_TOL + REL_TOL * np.abs(want)
    bad = err > bound
    assert not bad.any(), f"{name}: {int(bad.sum())} of {bad.size} beyond tolerance, worst {err.max():.3e}"
    return int((got != want).sum())


def run_pair(wl, steps, ld=None, with_error=True, with_momentum=True, tuning=None, lr_schedule=None,
             x_offset=0, check_every=None):
    """Run `steps` iterations on the GPU and in the fp32 oracle on identical inputs; compare at the end
    (and every `check_every` steps).  Returns (gpu object, oracle, number of elements not bit-identical)."""
    dev = torch.device("cuda:0")
    ld = wl.ld if ld is None else ld
    x = I.initial_model(wl, dev, ld=ld)
    if x_offset:   # deliberately misaligned rows: a view into a larger buffer
        big = torch.zeros(wl.W * ld + 8, device=dev, dtype=torch.float32)
        view = big[x_offset:x_offset + wl.W * ld].view(wl.W, ld)
        view.copy_(x)
        x = view
    cfg = B.make_config(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, wl.lr, wl.momentum, wl.seed, ld=ld)
    e = torch.zeros_like(x) if with_error else None
    m = torch.zeros_like(x) if with_momentum else None
    if x_offset:
        ebig = torch.zeros(wl.W * ld + 8, device=dev, dtype=torch.float32)
        mbig = torch.zeros(wl.W * ld + 8, device=dev, dtype=torch.float32)
        e = ebig[x_offset:x_offset + wl.W * ld].view(wl.W, ld) if with_error else None
        m = mbig[x_offset:x_offset + wl.W * ld].view(wl.W, ld) if with_momentum else None
    ctx = B.cser_create(cfg, x, e, m)
    for key, value in (tuning or {}).items():
        B.cser_set_tuning(ctx, key, value)
    x0 = I.initial_model_row(wl, dev).cpu().numpy()
    o = R.OracleCSER(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, wl.lr, wl.momentum if with_momentum else 0.0,
                     wl.seed, x0, dtype=np.float32, with_error=with_error)
    g = torch.zeros(wl.W, ld, device=dev, dtype=torch.float32)
    if x_offset:
        gbig = torch.zeros(wl.W * ld + 8, device=dev, dtype=torch.float32)
        g = gbig[x_offset:x_offset + wl.W * ld].view(wl.W, ld)
    diff = 0

    def compare():
        torch.cuda.synchronize()
        n = assert_states_close("x", x[:, :wl.d].cpu().numpy(), o.x)
        if with_error:
            n += assert_states_close("e", e[:, :wl.d].cpu().numpy(), o.e)
        if with_momentum:
            n += assert_states_close("m", m[:, :wl.d].cpu().numpy(), o.m)
        return n

    for t in range(1, steps + 1):
        if lr_schedule is not None:
            B.cser_set_lr(ctx, lr_schedule(t))
            o.set_lr(lr_schedule(t))
        I.gradient(wl, t, dev, ld=ld, out=g)
        B.cser_step(ctx, g)
        o.step(g[:, :wl.d].cpu().numpy())
        if check_every and t % check_every == 0:
            diff += compare()
    diff += compare()
    assert B.cser_get_step(ctx) == steps == o.t
    B.cser_destroy(ctx)
    return diff


# ---------------------------------------------------------------------------- selector
@pytest.mark.parametrize("d,block,R_step,R_reset", [
    (65536, 256, 8, 4), (855770, 512, 32, 8), (25557032, 1024, 256, 16), (25557032, 64, 2, 16),
    (25557032, 4096, 1024, 16), (335000000, 4096, 512, 32), (100, 7, 3, 1), (5, 8, 1, 1), (64, 1, 0, 2), (3, 1, 2, 3),
])
def test_selector_indices_and_masks_are_bit_exact(d, block, R_step, R_reset):
    dev = torch.device("cuda:0")
    x = torch.zeros(1, 64, device=dev)   # never touched: only the selector runs
    cfg = B.make_config(d, 1, block, R_step, R_reset, 1, 0.1, 0.0, 0xDEADBEEF12345, ld=d)
    ctx = B.cser_create(cfg, x, None, None)   # no e, no m: nothing is filled, x is a dummy
    Bn, ks, kr = B.cser_block_counts(ctx)
    assert Bn == -(-d // block) and ks == R.blocks_kept(Bn, R_step) and kr == R.blocks_kept(Bn, R_reset)
    for which, k in ((0, ks), (1, kr)):
        for t in (0, 1, 2, 31, 2**32 + 5, 2**63 + 11):
            idx, mask = B.cser_select_blocks(ctx, which, t)
            ridx, rmask = R.select_blocks(cfg.seed, which, t, Bn, k)
            assert np.array_equal(mask, rmask), (which, t)
            assert np.array_equal(idx, ridx), (which, t)
    B.cser_destroy(ctx)


# ---------------------------------------------------------------------------- named workloads
@pytest.mark.parametrize("tuning", [None, {FUSE: 0}, {K: TILE}, {K: SHARED}, {K: SHARED, FUSE: 0}, {K: GENERAL},
                                    {K: GENERAL, FUSE: 0}, {K: SPLIT}, {K: SPLIT, FUSE: 0}],
                         ids=["auto-fused-reset", "auto-separate-reset", "one-wavefront", "lds-shared",
                              "lds-shared-separate-reset", "lane-walks-workers", "lane-walks-separate",
                              "launch-pair", "launch-pair-separate-reset"])
def test_tiny_workload_100_steps(tuning):
    wl = I.WORKLOADS["tiny"]
    diff = run_pair(wl, 100, check_every=20, tuning=tuning)
    assert diff == 0, f"{diff} elements not bit-identical"


def test_small_cnn_workload_200_steps_ragged_tail():
    wl = I.WORKLOADS["small_cnn"]          # d = 855,770: last block has 218 columns, d % 4 == 2
    assert wl.d % 4 == 2 and wl.d % wl.block == 218
    diff = run_pair(wl, 200, check_every=100)
    assert diff == 0, f"{diff} elements not bit-identical"


# ---------------------------------------------------------------------------- layouts and degenerate cases
def _wl(**kw):
    base = dict(name="case", d=5000, W=4, block=64, R_step=4, R_reset=2, H=3, lr=0.1, momentum=0.9,
                x_var=1e-2, g_var=1e-2, seed=11, steps=12)
    base.update(kw)
    return I.Workload(**base)


@pytest.mark.parametrize("kw", [
    dict(),                                   # plain
    dict(W=1),                                # one worker: plain SGD
    dict(W=3), dict(W=5), dict(W=9),          # division by a non power of two; batch remainder
    dict(W=16),
    dict(R_step=0),                           # C_step keeps nothing (CSER-PL)
    dict(R_step=0, H=1),                      # CSEA
    dict(R_step=1),                           # identity: fully synchronous
    dict(R_reset=1),                          # full reset
    dict(H=0),                                # never reset
    dict(H=1),
    dict(d=40, block=64),                     # d smaller than one block
    dict(d=1, block=1, W=2),
    dict(d=4099, block=4),                    # smallest vector block, ragged d
    dict(d=4099, block=1),                    # element-wise blocks
    dict(d=4099, block=6),                    # block not a multiple of 4: the only case for element-wise kernels
    dict(d=70000, block=4096, R_step=2),      # block larger than a workgroup's columns
    dict(momentum=0.0),
    dict(lr=0.0),
    dict(W=33, d=3000, R_step=2),             # more workers than the in-register chosen-block path holds
    dict(W=64, d=2000, R_step=2, R_reset=2, H=2),
    dict(d=50000, block=65536, R_step=1, R_reset=1, H=2),   # a single block, always chosen by both compressors
    dict(d=50000, block=65536, R_step=0, R_reset=1, H=2),
])
def test_edge_cases_match_bit_for_bit(kw):
    wl = _wl(**kw)
    assert run_pair(wl, wl.steps) == 0


def test_row_stride_equal_to_an_odd_d_keeps_rows_only_4_byte_aligned():
    wl = _wl(d=4099)
    assert run_pair(wl, 12, ld=4099) == 0


def test_misaligned_base_pointers():
    wl = _wl(d=4096)
    assert run_pair(wl, 12, ld=4096, x_offset=1) == 0
    assert run_pair(wl, 12, ld=4096, x_offset=4) == 0


def test_implementation_two_without_residual_buffer():
    wl = _wl(d=20000, W=8, steps=16)
    for tuning in (None, {FUSE: 0}, {K: SHARED}, {K: SHARED, FUSE: 0}, {K: GENERAL}, {K: SPLIT}):
        assert run_pair(wl, 16, with_error=False, tuning=tuning) == 0
    for tuning in (None, {K: SHARED}, {K: GENERAL}, {K: SPLIT}):
        assert run_pair(_wl(d=20000, W=5, R_step=2, R_reset=2, H=1), 8, with_error=False, tuning=tuning) == 0


def test_blocks_chosen_by_both_compressors_at_once():
    # R_step = R_reset = 2 with H = 1: a quarter of the blocks is in both choices at every iteration
    for kw in (dict(), dict(W=3), dict(block=6), dict(momentum=0.0)):
        wl = _wl(d=30000, R_step=2, R_reset=2, H=1, **kw)
        assert run_pair(wl, 10) == 0
        for kernel in (TILE, SHARED, GENERAL, SPLIT):
            assert run_pair(wl, 10, tuning={K: kernel}) == 0


def test_no_momentum_buffer_is_algorithm_2():
    wl = _wl(d=20000, W=8, momentum=0.0)
    for tuning in (None, {K: SHARED}, {K: GENERAL}, {K: SPLIT}):
        assert run_pair(wl, 12, with_momentum=False, tuning=tuning) == 0
        assert run_pair(wl, 12, with_momentum=False, with_error=False, tuning=tuning) == 0


@pytest.mark.parametrize("tuning", [{K: TILE}, {K: TILE, NT: 0}, {K: TILE, NT: 1}, {K: TILE, TILE_CAP: 0}, {K: TILE, TILE_CAP: 7},
                                    {K: TILE, FUSE: 0}, {K: SHARED}, {K: SHARED, NT: 0}, {K: SHARED, NT: 1},
                                    {K: SHARED, SHARED_CAP: 0}, {K: SHARED, SHARED_CAP: 1}, {K: SHARED, FUSE: 0},
                                    {K: GENERAL}, {K: GENERAL, NT: 1}, {K: GENERAL, FUSE: 0}, {NT: 1}, {FUSE: 0},
                                    {K: SPLIT}, {K: SPLIT, NT: 0}, {K: SPLIT, NT: 1}, {K: SPLIT, FUSE: 0},
                                    {K: SPLIT, TILE_CAP: 5, SHARED_CAP: 1}],
                         ids=lambda t: "-".join(f"{k}={v}" for k, v in t.items()))
def test_results_do_not_depend_on_launch_shape(tuning):
    wl = _wl(d=30000, W=8, steps=8)
    assert run_pair(wl, 8, tuning=tuning) == 0


@pytest.mark.parametrize("W", [1, 2, 3, 5, 6, 7, 12, 13, 16, 17, 31, 33, 48, 64, 65])
@pytest.mark.parametrize("R_step", [1, 2, 5])
def test_every_worker_count_in_every_kernel_that_takes_it(W, R_step):
    """The one-wavefront kernel shares a tile's synchronised column groups among its W workgroups in slices of
    floor(64 / W) groups (two rounds when W does not divide 64); the LDS-shared kernel has W wavefronts per
    workgroup; the pair of launches gives the synchronised blocks to the LDS-shared kernel up to 16 workers and to
    the general kernel beyond; beyond 64 workers a lane walks the worker axis."""
    wl = _wl(d=2500, W=W, block=8, R_step=R_step, R_reset=2, H=2, steps=4)
    kernels = [None] + ([TILE] if W <= 64 else []) + ([SHARED] if W <= 16 else []) + [SPLIT, GENERAL]
    for kernel in kernels:
        assert run_pair(wl, 4, tuning=None if kernel is None else {K: kernel}) == 0
        assert run_pair(wl, 4, with_error=False, tuning=None if kernel is None else {K: kernel}) == 0


def test_learning_rate_schedule():
    wl = _wl()
    assert run_pair(wl, 12, lr_schedule=lambda t: 0.1 / t) == 0


def test_forced_reset_and_resume_from_checkpoint():
    dev = torch.device("cuda:0")
    wl = _wl(d=9000, W=4, H=4)
    cfg = B.make_config(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, wl.lr, wl.momentum, wl.seed, ld=wl.ld)

    def run(n0, n1):
        x = I.initial_model(wl, dev)
        opt = B.CSER(cfg, x)
        for t in range(1, n0 + 1):
            opt.step(I.gradient(wl, t, dev))
        if n1:
            # "checkpoint": copy the state, build a fresh context on the copies, restore t
            x2, e2, m2 = opt.x.clone(), opt.e.clone(), opt.m.clone()
            torch.cuda.synchronize()
            opt.close()
            ctx = B.cser_create(cfg, x2, torch.empty_like(e2), torch.empty_like(m2))
            B.cser_destroy(ctx)                      # create zero-fills e and m: restore them afterwards
            e3, m3 = torch.zeros_like(e2), torch.zeros_like(m2)
            ctx = B.cser_create(cfg, x2, e3, m3)
            e3.copy_(e2)
            m3.copy_(m2)
            B.cser_set_step(ctx, n0)
            for t in range(n0 + 1, n0 + n1 + 1):
                B.cser_step(ctx, I.gradient(wl, t, dev))
            torch.cuda.synchronize()
            B.cser_destroy(ctx)
            return x2.cpu(), e3.cpu(), m3.cpu()
        torch.cuda.synchronize()
        out = opt.x.cpu(), opt.e.cpu(), opt.m.cpu()
        opt.close()
        return out

    straight = run(10, 0)
    resumed = run(6, 4)
    for a, b in zip(straight, resumed):
        assert torch.equal(a, b)

    # a forced reset at an arbitrary t matches the oracle's
    x = I.initial_model(wl, dev)
    opt = B.CSER(cfg, x)
    o = R.OracleCSER(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, wl.lr, wl.momentum, wl.seed,
                     I.initial_model_row(wl, dev).cpu().numpy())
    for t in range(1, 4):
        g = I.gradient(wl, t, dev)
        opt.step(g)
        o.step(g[:, :wl.d].cpu().numpy())
    opt.error_reset()
    o.error_reset()
    torch.cuda.synchronize()
    assert assert_states_close("x", opt.x[:, :wl.d].cpu().numpy(), o.x) == 0
    assert assert_states_close("e", opt.e[:, :wl.d].cpu().numpy(), o.e) == 0
    opt.close()


def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        d = int(rng.choice([1, 2, 3, 5, 63, 64, 65, 257, 1000, 1023, 4096, 5003, 20011]))
        block = int(rng.choice([1, 2, 3, 4, 6, 8, 16, 64, 100, 256, 1000, 4096]))
        momentum = float(rng.choice([0.0, 0.5, 0.9]))
        cases.append(dict(
            d=d, W=int(rng.integers(1, 13)), block=block, R_step=int(rng.choice([0, 1, 2, 3, 5, 16, 1000])),
            R_reset=int(rng.choice([1, 2, 3, 7, 64])), H=int(rng.choice([0, 1, 2, 3, 5])), momentum=momentum,
            lr=float(rng.choice([0.1, 0.01, 1.0])), seed=int(rng.integers(0, 2**62)),
            ld=int(rng.choice([d, -(-d // 4) * 4, -(-d // 64) * 64, -(-d // 1024) * 1024])),
            with_error=bool(rng.integers(0, 2)), with_momentum=bool(momentum != 0.0 or rng.integers(0, 2)),
            tuning=[None, {K: GENERAL}, {K: SHARED}, {FUSE: 0}, {K: TILE, NT: 1}, {K: SHARED, NT: 0}, {K: TILE}, {K: SPLIT}][int(rng.integers(0, 8))]))
    return cases


@pytest.mark.parametrize("case", _random_cases(48, 20200725), ids=lambda c: f"d{c['d']}-W{c['W']}-b{c['block']}")
def test_randomly_drawn_configurations(case):
    wl = _wl(d=case["d"], W=case["W"], block=case["block"], R_step=case["R_step"], R_reset=case["R_reset"], H=case["H"],
             momentum=case["momentum"], lr=case["lr"], seed=case["seed"])
    assert run_pair(wl, 7, ld=case["ld"], with_error=case["with_error"], with_momentum=case["with_momentum"],
                    tuning=case["tuning"]) == 0


def test_step_counter_jumps_across_the_mask_window():
    """C_step's masks are drawn 32 iterations per selector launch; moving t backwards, forwards and
    across window edges must still use the mask of the iteration actually being run."""
    dev = torch.device("cuda:0")
    wl = _wl(d=9000, W=4, H=5)
    cfg = B.make_config(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, wl.lr, wl.momentum, wl.seed, ld=wl.ld)
    opt = B.CSER(cfg, I.initial_model(wl, dev))
    o = R.OracleCSER(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, wl.lr, wl.momentum, wl.seed,
                     I.initial_model_row(wl, dev).cpu().numpy())
    schedule = [(0, 35), (3, 4), (31, 4), (2**32 - 2, 4), (2**64 - 40, 36), (64, 2), (63, 3)]
    n = 0
    for start, count in schedule:
        B.cser_set_step(opt.ctx, start)
        o.t = start
        for _ in range(count):
            n += 1
            g = I.gradient(wl, n, dev)
            opt.step(g)
            o.step(g[:, :wl.d].cpu().numpy())
        assert B.cser_get_step(opt.ctx) == o.t == start + count
    torch.cuda.synchronize()
    for name in ("x", "e", "m"):
        assert assert_states_close(name, getattr(opt, name)[:, :wl.d].cpu().numpy(), getattr(o, name)) == 0
    opt.close()


def test_steps_issued_on_alternating_streams():
    """The caller orders its own work between streams; the library orders the mask window it drew on
    one stream before the step kernels it launches on another."""
    dev = torch.device("cuda:0")
    wl = _wl(d=200000, W=8, H=3)
    cfg = B.make_config(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, wl.lr, wl.momentum, wl.seed, ld=wl.ld)
    opt = B.CSER(cfg, I.initial_model(wl, dev))
    torch.cuda.synchronize()
    o = R.OracleCSER(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, wl.lr, wl.momentum, wl.seed,
                     I.initial_model_row(wl, dev).cpu().numpy())
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    grads = [I.gradient(wl, t, dev) for t in range(1, 11)]
    torch.cuda.synchronize()
    prev = None
    for t, g in enumerate(grads, start=1):
        s = streams[t & 1]
        if prev is not None:
            s.wait_stream(prev)
        opt.step(g, stream=s)
        prev = s
        o.step(g[:, :wl.d].cpu().numpy())
    torch.cuda.synchronize()
    for name in ("x", "e", "m"):
        assert assert_states_close(name, getattr(opt, name)[:, :wl.d].cpu().numpy(), getattr(o, name)) == 0
    opt.close()


def test_csea_and_cser_pl_presets_against_their_algorithm_boxes():
    """Independent of the oracle's Algorithm 3: the presets of Appendix A.1 run on the GPU and are compared with
    numpy float64 re-codings of the CSEA and CSER-PL boxes (tests/_np_models.py), to fp32 rounding."""
    from tests import _np_models as M
    dev = torch.device("cuda:0")
    d, W, block, R_reset, T, lr, seed = 3000, 4, 8, 4, 12, 0.1, 99
    Bn = -(-d // block)
    rng = np.random.default_rng(3)
    x0 = (rng.standard_normal(d) * 0.1).astype(np.float32)
    grads = [(rng.standard_normal((W, d)) * 0.1).astype(np.float32) for _ in range(T)]
    masks = {t: R.select_blocks(seed, 1, t, Bn, R.blocks_kept(Bn, R_reset))[1] for t in range(1, T + 1)}
    lr32 = float(np.float32(lr))
    for preset, H, expect in (
            (B.cser_preset_csea, 7, lambda: M.csea_impl1(x0, [g.astype(np.float64) for g in grads], masks, lr32, block)),
            (B.cser_preset_cser_pl, 3, lambda: M.cser_pl_impl1(x0, [g.astype(np.float64) for g in grads], masks, 3, lr32, block))):
        cfg = preset(B.make_config(d, W, block, 64, R_reset, H, lr, 0.0, seed, ld=3072))
        x = torch.zeros(W, 3072, device=dev)
        x[:, :d] = torch.from_numpy(x0).to(dev)
        opt = B.CSER(cfg, x, with_momentum=False)
        g = torch.zeros(W, 3072, device=dev)
        for t in range(T):
            g[:, :d] = torch.from_numpy(grads[t]).to(dev)
            opt.step(g)
        torch.cuda.synchronize()
        want_x, want_e = expect()
        np.testing.assert_allclose(opt.x[:, :d].cpu().numpy(), want_x, rtol=0, atol=2e-6)
        np.testing.assert_allclose(opt.e[:, :d].cpu().numpy(), want_e, rtol=0, atol=2e-6)
        assert np.abs(want_e).max() > 1e-3
        opt.close()


def test_gpu_run_stays_within_rounding_of_the_float64_oracle():
    """Independent of the shared fp32 contract: against the oracle in double precision the fp32 states
    differ by accumulated rounding only (about one rounding of 2^-24 |value| per statement and step)."""
    dev = torch.device("cuda:0")
    wl = I.WORKLOADS["tiny"]
    x = I.initial_model(wl, dev)
    cfg = B.make_config(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, wl.lr, wl.momentum, wl.seed, ld=wl.ld)
    opt = B.CSER(cfg, x)
    o = R.OracleCSER(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, float(np.float32(wl.lr)),
                     float(np.float32(wl.momentum)), wl.seed, I.initial_model_row(wl, dev).cpu().numpy(),
                     dtype=np.float64)
    for t in range(1, 101):
        g = I.gradient(wl, t, dev)
        opt.step(g)
        o.step(g[:, :wl.d].cpu().numpy())
    torch.cuda.synchronize()
    for name, got, want in (("x", opt.x, o.x), ("e", opt.e, o.e), ("m", opt.m, o.m)):
        err = np.abs(got[:, :wl.d].cpu().numpy().astype(np.float64) - want)
        assert err.max() < 100 * 2.0 ** -24 * max(1.0, np.abs(want).max()), (name, err.max())
    opt.close()


def test_profile_timers_counters_and_copy_probe():
    dev = torch.device("cuda:0")
    wl = _wl(d=100000, W=8, H=2, block=256)
    cfg = B.make_config(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, wl.lr, wl.momentum, wl.seed, ld=wl.ld)
    opt = B.CSER(cfg, I.initial_model(wl, dev))
    B.cser_profile_enable(opt.ctx, True)
    g = I.gradient(wl, 1, dev)
    for _ in range(6):
        opt.step(g)
    assert B.cser_profile_read(opt.ctx, 0)[1] == 6
    assert B.cser_profile_read(opt.ctx, 1)[1] == 0      # resets ran inside the fused-step kernel
    c = B.cser_measure_counters(opt.ctx)
    # R_step = 4, R_reset = 2, blocks of one tile: a quarter of the blocks is synchronised on ordinary iterations
    # (one-wavefront kernel), five eighths on reset iterations (the one-wavefront kernel takes the local blocks, then
    # the LDS-shared kernel the rest)
    assert (c["steps"], c["window_draws"], c["resets_fused"], c["resets_separate"]) == (6, 1, 3, 0)
    assert (c["launches_tile"], c["launches_shared"], c["launches_general"], c["launches_split"]) == (3, 0, 0, 3)
    B.cser_profile_clear(opt.ctx)
    B.cser_set_tuning(opt.ctx, FUSE, 0)                  # separate reset kernel
    for _ in range(6):
        opt.step(g)
    ms0, n0 = B.cser_profile_read(opt.ctx, 0)
    ms1, n1 = B.cser_profile_read(opt.ctx, 1)
    assert n0 == 6 and n1 == 3 and ms0 > 0 and ms1 > 0
    c = B.cser_measure_counters(opt.ctx)
    assert (c["steps"], c["window_draws"], c["resets_fused"], c["resets_separate"]) == (12, 2, 3, 3)
    assert (c["launches_tile"], c["launches_shared"], c["launches_split"]) == (9, 0, 3)
    B.cser_profile_clear(opt.ctx)
    assert B.cser_profile_read(opt.ctx, 0) == (0.0, 0)
    opt.close()
    src = torch.arange(1 << 20, device=dev, dtype=torch.float32)
    dst = torch.zeros_like(src)
    B.cser_copy_probe(dst, src, src.numel() * 4)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)


def test_residency_caps_are_what_the_launches_get():
    """The kernels bound the wavefronts resident on a CU by the size of their dynamic LDS request; the request is
    chosen with the runtime's occupancy calculator, and what it reports for the chosen request is the cap asked for."""
    dev = torch.device("cuda:0")
    for with_error, with_momentum, want_tile in ((True, True, 12), (False, True, 18), (True, False, 18), (False, False, None)):
        wl = _wl(d=100000, W=8, momentum=0.9 if with_momentum else 0.0)
        cfg = B.make_config(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, wl.lr, wl.momentum, wl.seed, ld=wl.ld)
        opt = B.CSER(cfg, I.initial_model(wl, dev), with_error=with_error, with_momentum=with_momentum)
        r = B.cser_measure_residency(opt.ctx)
        if want_tile is None:
            assert r["tile_lds"] == 0 and r["tile_groups_per_cu"] >= 24     # two load streams: no cap
        else:
            assert r["tile_groups_per_cu"] == want_tile, r
        assert r["shared_groups_per_cu"] == 3 and r["shared_lds"] >= 8 * 1024, r          # 24 wavefronts per CU at W = 8
        assert r["shared_reset_groups_per_cu"] == 3 and r["shared_reset_lds"] >= 16 * 1024, r
        assert r["reset_groups_per_cu"] == 3, r
        B.cser_set_tuning(opt.ctx, TILE_CAP, 9)
        B.cser_set_tuning(opt.ctx, SHARED_CAP, 2)
        r = B.cser_measure_residency(opt.ctx)
        assert r["tile_groups_per_cu"] == 9 and r["shared_groups_per_cu"] == 2 and r["reset_groups_per_cu"] == 2, r
        opt.close()
    wl = _wl(d=100000, W=3)
    cfg = B.make_config(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, wl.lr, wl.momentum, wl.seed, ld=wl.ld)
    opt = B.CSER(cfg, I.initial_model(wl, dev))
    assert B.cser_measure_residency(opt.ctx)["shared_groups_per_cu"] == 8       # 24 / 3
    opt.close()


def test_many_steps_in_one_call_equal_the_same_steps_one_by_one():
    dev = torch.device("cuda:0")
    wl = _wl(d=9000, W=4, H=3)
    cfg = B.make_config(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, wl.lr, wl.momentum, wl.seed, ld=wl.ld)
    grads = [I.gradient(wl, t, dev) for t in range(1, 41)]
    one = B.CSER(cfg, I.initial_model(wl, dev))
    for g in grads:
        one.step(g)
    many = B.CSER(cfg, I.initial_model(wl, dev))
    assert many.step_many(grads[:7]) == 7
    prepared = B.gradient_list(grads[7:])
    assert many.step_many(prepared) == 33
    assert many.step_many([]) == 0
    torch.cuda.synchronize()
    assert B.cser_get_step(many.ctx) == B.cser_get_step(one.ctx) == 40
    for name in ("x", "e", "m"):
        assert torch.equal(getattr(one, name), getattr(many, name))
    o = R.OracleCSER(wl.d, wl.W, wl.block, wl.R_step, wl.R_reset, wl.H, wl.lr, wl.momentum, wl.seed,
                     I.initial_model_row(wl, dev).cpu().numpy())
    for g in grads:
        o.step(g[:, :wl.d].cpu().numpy())
    for name in ("x", "e", "m"):
        assert assert_states_close(name, getattr(many, name)[:, :wl.d].cpu().numpy(), getattr(o, name)) == 0
    # a bad pointer in the list stops the call there and reports how far it got
    bad = (ctypes.c_void_p * 3)(grads[0].data_ptr(), grads[1].data_ptr() + 2, grads[2].data_ptr())
    done = ctypes.c_uint32()
    assert B._lib().cser_step_many(many.ctx, bad, 3, None, ctypes.byref(done)) == B.CSER_EALIGN and done.value == 1
    one.close()
    many.close()
