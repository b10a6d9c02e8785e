"""The drain entry point that allocates nothing (ps_drain_rows_mitigated, scratch in a fixed device
array) against the context-based entry point it is a variant of (ps_drain_buffered_mitigated), through
the C ABI, on two calls in a row, the second with a smaller input."""
import sys

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2406_05546_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu

DROP_SEED = 7


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def ps():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2406_05546_amd import binding
    binding.load_library()
    return binding


def _rows(seed, n, P):
    rows = synth.gradient_rows(seed, 0, n, P)
    rows *= np.array([0.5, 1.0, 2.0], np.float32)[np.arange(n) % 3][:, None]      # three different norms
    return rows


def _by_context(ps, theta0, rows, mode, lr, ref, clip):
    ctx = ps.ps_init(ps.make_config(1, 1, 1, len(rows), DROP_SEED, 0.25))
    try:
        ps.ps_set_weights(ctx, theta0)
        for i, r in enumerate(rows):
            ps.ps_queue_push_host(ctx, r, 0, 0, i)
        k, used = ps.ps_drain_buffered_mitigated(ctx, mode, lr, ref, clip)
        assert k == len(rows)
        return ps.ps_get_weights(ctx), used
    finally:
        ps.ps_destroy(ctx)


def _padded(a, row_floats):
    import torch
    a = np.atleast_2d(a)
    out = np.zeros((a.shape[0], row_floats), np.float32)
    out[:, :a.shape[1]] = a
    return torch.from_numpy(out).cuda()


def test_two_calls_in_a_row_match_the_context_based_drain(ps):
    import torch
    lr, ref = 0.02, 16.0
    theta0 = synth.he_uniform_theta(21)
    calls = [(37, 0, 4.0), (37, 1, 4.0), (5, 1, 3.0), (5, 0, 0.0), (64, 1, 5.0), (3, 0, 9.0)]   # (rows, mode, clip norm)
    for n, mode, clip in calls:
        rows = _rows(50 + n, n, ps.P)
        want, used_want = _by_context(ps, theta0, rows, mode, lr, ref, clip)
        theta_dev = _padded(theta0, ps.ROW_FLOATS)[0].contiguous()
        grads_dev = _padded(rows, ps.ROW_FLOATS)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        say(f"no_alloc: {n} rows, mode {mode}, clip {clip}")
        used = ps.ps_drain_rows_mitigated(theta_dev, grads_dev, mode, lr, ref, clip)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        got = theta_dev.cpu().numpy()
        assert used == used_want and (got[ps.P:] == 0).all()
        assert np.array_equal(got[:ps.P], want), f"{n} rows, mode {mode}: differs from the context-based drain"
        scales = orc.clip_scales(list(rows), clip)
        assert clip == 0.0 or 0 < sum(s < 1.0 for s in scales) < n           # some rows clipped, some not
        oracle, _ = orc.drain_mitigated(theta0.astype(np.float64), list(rows), lr, mode, ref, clip)
        parity.assert_close(got[:ps.P], oracle, parity.WEIGHT_TOL, f"{n} rows, mode {mode} against the oracle")
        assert np.abs(got[:ps.P] - oracle).max() <= 1e-3 * np.abs(oracle - theta0).max()


def test_limits_and_errors(ps):
    import torch
    theta0 = synth.he_uniform_theta(22)
    theta_dev = _padded(theta0, ps.ROW_FLOATS)[0].contiguous()
    grads_dev = _padded(_rows(9, 2, ps.P), ps.ROW_FLOATS)
    ps.ps_drain_rows_mitigated(theta_dev, grads_dev, 0, 0.1, 0.0, 0.0, n_rows=0)              # no rows: nothing changes
    torch.cuda.synchronize()
    assert np.array_equal(theta_dev.cpu().numpy()[:ps.P], theta0)
    with pytest.raises(ps.PsError) as e:
        ps.ps_drain_rows_mitigated(theta_dev, grads_dev, 0, 0.1, 0.0, 0.0, n_rows=ps.STATIC_DRAIN_MAX_ROWS + 1)
    assert e.value.status == ps.PS_EINVAL and "4096" in str(e.value)
    for bad in (lambda: ps.ps_drain_rows_mitigated(theta_dev, grads_dev, 2, 0.1), lambda: ps.ps_drain_rows_mitigated(theta_dev, grads_dev, 0, 0.1, -1.0),
                lambda: ps.ps_drain_rows_mitigated(theta_dev, grads_dev, 0, 0.1, 0.0, -1.0)):
        with pytest.raises(ps.PsError) as e:
            bad()
        assert e.value.status == ps.PS_EINVAL
    torch.cuda.synchronize()
    assert np.array_equal(theta_dev.cpu().numpy()[:ps.P], theta0)                             # failed calls changed nothing
