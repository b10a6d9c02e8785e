"""Pins for the CPU oracle: everything here checks oracle/ against something other than itself
(the generator's published known answers, hand-enumerated values, closed forms, finite
differences, an independent library's autograd, and the invariants the update rules imply)."""
import math
import os

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2406_05546_amd import synth

TINY = orc.Dims(H=8, W=8, C1=2, C2=3, F=8, NC=3)


def _rand_theta(dims, seed, scale=0.5):
    rng = np.random.default_rng(seed)
    return rng.uniform(-scale, scale, dims.P)


def _rand_batch(dims, B, seed):
    rng = np.random.default_rng(seed)
    return rng.uniform(0, 1, (B, dims.H * dims.W)), rng.integers(0, dims.NC, B).astype(np.int32)


# ---------------------------------------------------------------- generator

def test_philox_known_answers(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) if l[0] != "#"]
    assert len(rows) == 3
    for r in rows:
        v = [int(t, 16) for t in r]
        assert orc.philox4x32_10(v[0:4], v[4:6]) == v[6:10]


def test_dropout_keep_rate_and_edges():
    keep = orc.dropout_keep(seed=7, minibatch_id=(3 << 32) | 11, B=2048, F=512, p=0.25)
    assert keep.size >= 10 ** 6
    assert abs(keep.mean() - 0.75) < 0.002
    # neighbouring units / samples are not copies of each other
    assert abs(np.corrcoef(keep[:, :-1].ravel(), keep[:, 1:].ravel())[0, 1]) < 0.01
    assert abs(np.corrcoef(keep[:-1].ravel(), keep[1:].ravel())[0, 1]) < 0.01
    assert orc.dropout_keep(7, 5, 16, 64, 0.0).all()            # p = 0: identity
    assert orc.dropout_threshold(0.25) == 0x40000000
    # the mask depends on logical ids only: sample rows of a larger batch are the same rows
    small = orc.dropout_keep(7, (3 << 32) | 11, 5, 512, 0.25)
    assert (small == keep[:5]).all()
    assert (orc.dropout_keep(8, (3 << 32) | 11, 5, 512, 0.25) != small).any()
    assert (orc.dropout_keep(7, (3 << 32) | 12, 5, 512, 0.25) != small).any()


def test_dropout_word_assignment():
    """Unit u of sample s takes word u%4 of Philox({mb_lo, mb_hi, s, u/4}, {seed_lo, seed_hi})."""
    seed, mb = (5 << 32) | 9, (2 << 32) | 77
    keep = orc.dropout_keep(seed, mb, 3, 16, 0.25)
    for s in range(3):
        for u in range(16):
            w = orc.philox4x32_10([mb & 0xFFFFFFFF, mb >> 32, s, u // 4], [seed & 0xFFFFFFFF, seed >> 32])
            assert keep[s, u] == (1 if w[u % 4] >= 0x40000000 else 0)


# ---------------------------------------------------------------- sizes and layout

def test_param_count_and_layout():
    d = orc.Dims()
    assert d.P == 813258 == synth.NetDims().P
    offs = {n: o for n, o, _, _ in synth.NetDims().segments()}
    assert offs == {"conv1.W": 0, "conv1.b": 144, "conv2.W": 160, "conv2.b": 4768, "fc1.W": 4800,
                    "fc1.b": 807616, "fc2.W": 808128, "fc2.b": 813248}
    assert 400 * d.P * 4 == 1301212800 and 1024 * d.P * 4 == 3331104768
    assert TINY.P == synth.NetDims(8, 8, 2, 3, 8, 3).P


# ---------------------------------------------------------------- conv / pool against hand values

def _conv1_only(kernel, bias, img4):
    d = orc.Dims(H=4, W=4, C1=1, C2=1, F=2, NC=2)
    theta = np.zeros(d.P)
    theta[0:9] = np.asarray(kernel, float).ravel()
    theta[9] = bias
    x = np.asarray(img4, float).reshape(1, 16)
    _, _, rec = orc.worker_grad(d, theta, x, np.zeros(1, np.int32), np.ones((1, 2), np.uint8), 0.0, records=True)
    return rec


def test_conv_pool_hand_enumerated(golden_dir):
    img = np.arange(1, 17).reshape(4, 4)
    kernels = {"ones": (np.ones((3, 3)), 0.0),
               "up": (np.array([[0, 1, 0], [0, 0, 0], [0, 0, 0]]), 0.0),
               "left": (np.array([[0, 0, 0], [0, 0, 1], [0, 0, 0]]), 0.5)}
    seen = 0
    for line in open(os.path.join(golden_dir, "conv_pool_4x4.txt")):
        t = line.split()
        if not t or t[0] not in kernels:
            continue
        vals = np.array([float(v) for v in t[1:]]).reshape(4, 3)
        rec = _conv1_only(*kernels[t[0]], img)
        assert np.array_equal(rec.top1[0], vals[:, 0]), t[0]
        assert np.array_equal(rec.code1[0], vals[:, 1].astype(np.uint8)), t[0]
        assert np.array_equal(rec.margin1[0], vals[:, 2]), t[0]
        seen += 1
    assert seen == 3


def test_centre_tap_is_identity_and_first_max_wins():
    d = orc.Dims(H=8, W=8, C1=1, C2=1, F=2, NC=2)
    theta = np.zeros(d.P)
    theta[4] = 1.0                                   # centre tap only
    x, _ = _rand_batch(d, 2, 3)
    _, _, rec = orc.worker_grad(d, theta, x, np.zeros(2, np.int32), np.ones((2, 2), np.uint8), 0.0, records=True)
    win = x.reshape(2, 4, 2, 4, 2).transpose(0, 1, 3, 2, 4).reshape(2, 16, 4)
    assert np.array_equal(rec.top1, win.max(-1))
    assert np.array_equal(rec.code1, win.argmax(-1).astype(np.uint8))
    # all-equal window: the first element wins, margin 0
    _, _, rec = orc.worker_grad(d, theta, np.full((1, 64), 0.25), np.zeros(1, np.int32),
                                np.ones((1, 2), np.uint8), 0.0, records=True)
    assert (rec.code1 == 0).all() and (rec.margin1 == 0).all() and (rec.top1 == 0.25).all()


# ---------------------------------------------------------------- whole gradient

def _fd_grad(dims, theta, x, y, keep, p, idx, h=1e-6):
    out = np.empty(len(idx))
    for n, i in enumerate(idx):
        tp, tm = theta.copy(), theta.copy()
        tp[i] += h
        tm[i] -= h
        out[n] = (orc.worker_grad(dims, tp, x, y, keep, p)[1] - orc.worker_grad(dims, tm, x, y, keep, p)[1]) / (2 * h)
    return out


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_gradient_matches_central_differences(seed):
    """Mask held fixed; evaluation points are kept away from ReLU / pool kinks by a margin check."""
    d, B, p = TINY, 2, 0.25
    x, y = _rand_batch(d, B, 100 + seed)
    keep = orc.dropout_keep(11, seed, B, d.F, p)
    keep[:, 0] = 1
    for attempt in range(50):
        theta = _rand_theta(d, 1000 * seed + attempt)
        g, loss, rec = orc.worker_grad(d, theta, x, y, keep, p, records=True)
        if min(rec.margin1.min(), rec.margin2.min(), np.abs(rec.top1).min(), np.abs(rec.top2).min(),
               np.abs(rec.hpre).min()) > 1e-3:
            break
    else:
        pytest.fail("no kink-free point found")
    fd = _fd_grad(d, theta, x, y, keep, p, range(d.P))
    assert np.abs(g).max() > 1e-3
    for name, off, shape, _ in synth.NetDims(d.H, d.W, d.C1, d.C2, d.F, d.NC).segments():
        n = int(np.prod(shape))
        a, b = g[off:off + n], fd[off:off + n]
        assert np.linalg.norm(a - b) <= 1e-6 * max(np.linalg.norm(b), 1e-3), name


def _torch_grad(dims, theta, x, y, keep, p):
    import torch
    import torch.nn.functional as Fn
    t = torch.tensor(theta, dtype=torch.float64, requires_grad=True)
    nd = synth.NetDims(dims.H, dims.W, dims.C1, dims.C2, dims.F, dims.NC)
    seg = {n: t[o:o + int(np.prod(s))].reshape(s) for n, o, s, _ in nd.segments()}
    a = torch.tensor(x, dtype=torch.float64).reshape(-1, 1, dims.H, dims.W)
    a = Fn.max_pool2d(Fn.relu(Fn.conv2d(a, seg["conv1.W"], seg["conv1.b"], padding=1)), 2)
    a = Fn.max_pool2d(Fn.relu(Fn.conv2d(a, seg["conv2.W"], seg["conv2.b"], padding=1)), 2)
    a = Fn.relu(Fn.linear(a.flatten(1), seg["fc1.W"], seg["fc1.b"]))
    a = a * torch.tensor(keep, dtype=torch.float64) / (1.0 - p)
    z = Fn.linear(a, seg["fc2.W"], seg["fc2.b"])
    loss = Fn.cross_entropy(z, torch.tensor(y, dtype=torch.long))
    loss.backward()
    return t.grad.numpy(), float(loss), z.detach().numpy()


@pytest.mark.parametrize("dims,B", [(TINY, 3), (orc.Dims(H=12, W=8, C1=3, C2=4, F=16, NC=5), 4), (orc.Dims(), 3)])
def test_gradient_matches_independent_autograd(dims, B):
    """Same network written with a library's conv / pool / linear / cross-entropy and its autograd."""
    x, y = _rand_batch(dims, B, 5)
    theta = synth.he_uniform_theta(3, synth.NetDims(dims.H, dims.W, dims.C1, dims.C2, dims.F, dims.NC)).astype(float)
    theta += np.random.default_rng(1).uniform(-0.05, 0.05, dims.P)      # non-zero biases too
    keep = orc.dropout_keep(21, 9, B, dims.F, 0.25)
    g, loss, rec = orc.worker_grad(dims, theta, x, y, keep, 0.25, records=True)
    tg, tloss, tz = _torch_grad(dims, theta, x, y, keep, 0.25)
    assert abs(loss - tloss) <= 1e-12 * abs(tloss)
    assert np.allclose(rec.z, tz, rtol=1e-11, atol=1e-12)
    for name, off, shape, _ in synth.NetDims(dims.H, dims.W, dims.C1, dims.C2, dims.F, dims.NC).segments():
        n = int(np.prod(shape))
        assert np.linalg.norm(g[off:off + n] - tg[off:off + n]) <= 1e-11 * np.linalg.norm(tg[off:off + n]), name


def test_zero_weights_closed_form():
    d, B = orc.Dims(), 8
    x, y = synth.minibatch(1, 2, B)
    g, loss = orc.worker_grad(d, np.zeros(d.P), x, y, orc.dropout_keep(1, 2, B, d.F, 0.25), 0.25)
    assert abs(loss - math.log(10.0)) < 1e-15
    expect = np.zeros(d.P)
    expect[813248:] = 0.1 - np.bincount(y, minlength=10) / B
    assert np.allclose(g, expect, rtol=0, atol=1e-16)


def test_softmax_gradient_sums_to_zero_and_batch_mean():
    d, B = TINY, 5
    x, y = _rand_batch(d, B, 8)
    theta = _rand_theta(d, 4)
    keep = orc.dropout_keep(2, 3, B, d.F, 0.25)
    g, loss = orc.worker_grad(d, theta, x, y, keep, 0.25)
    assert abs(g[-d.NC:].sum()) < 1e-15
    # gradient of the mean loss over B samples = mean of the B single-sample gradients (same mask rows)
    singles = [orc.worker_grad(d, theta, x[i:i + 1], y[i:i + 1], keep[i:i + 1], 0.25) for i in range(B)]
    assert np.allclose(g, np.mean([s[0] for s in singles], axis=0), rtol=1e-12, atol=1e-15)
    assert abs(loss - np.mean([s[1] for s in singles])) < 1e-14


def test_dropout_p0_is_identity_and_mask_zeroes_units():
    d, B = TINY, 2
    x, y = _rand_batch(d, B, 9)
    theta = _rand_theta(d, 5)
    g0, l0 = orc.worker_grad(d, theta, x, y, np.ones((B, d.F), np.uint8), 0.0)
    tg, tl, _ = _torch_grad(d, theta, x, y, np.ones((B, d.F)), 0.0)
    assert abs(l0 - tl) < 1e-13 and np.allclose(g0, tg, rtol=1e-10, atol=1e-14)
    # a fully dropped layer: only the output bias sees a gradient
    g, _ = orc.worker_grad(d, theta, x, y, np.zeros((B, d.F), np.uint8), 0.25)
    assert np.all(g[:-d.NC] == 0) and np.any(g[-d.NC:] != 0)


def test_batched_workers_match_single_calls_and_use_their_snapshot():
    d, B, n = TINY, 3, 4
    rng = np.random.default_rng(0)
    x = rng.uniform(0, 1, (n, B, 64))
    y = rng.integers(0, 3, (n, B)).astype(np.int32)
    thetas = np.stack([_rand_theta(d, s) for s in (1, 2)])
    keep = np.stack([orc.dropout_keep(4, i, B, d.F, 0.25) for i in range(n)])
    slot = [0, 1, 1, 0]
    grads, losses, used = orc.worker_grads(d, thetas, slot, x, y, keep, 0.25, n_threads=2)
    assert used == 2
    for i in range(n):
        g, l = orc.worker_grad(d, thetas[slot[i]], x[i], y[i], keep[i], 0.25)
        assert np.array_equal(g, grads[i]) and l == losses[i]


# ---------------------------------------------------------------- update rules

def _server(dims, n_slots, seed=3):
    nd = synth.NetDims(dims.H, dims.W, dims.C1, dims.C2, dims.F, dims.NC)
    return orc.OracleServer(dims, seed=seed, dropout_p=0.25, n_slots=n_slots, theta=synth.he_uniform_theta(seed, nd))


def _mb(dims, seed, ids, B):
    return synth.minibatches(seed, ids, B, h=dims.H, w=dims.W, n_classes=dims.NC)


def test_sync_with_one_worker_equals_async_bit_exact():
    """Section 2.1: with a single worker "wait for all, apply at once" is "apply on arrival"."""
    a, b = _server(TINY, 1), _server(TINY, 1)
    for step in range(5):
        ids = [synth.minibatch_id(0, step)]
        x, y = _mb(TINY, 3, ids, 4)
        ea = a.worker_grads_batched([0], [0], ids, x, y)
        a.apply_sync([e.seq for e in ea], 0.05)
        a.snapshot_weights(0)
        eb = b.worker_grads_batched([0], [0], ids, x, y)
        b.apply_async(eb[0].seq, 0.05)
        b.snapshot_weights(0)
    assert np.array_equal(a.theta, b.theta) and a.version == b.version == 5
    assert not np.array_equal(a.theta, _server(TINY, 1).theta)


def test_zero_outage_drain_equals_async_bit_exact():
    """Section 3.3: a stateless server step that finds one pending gradient is an async update."""
    arrivals = synth.async_cyclic_arrivals(5, 3, 12)
    for mode in (orc.DRAIN_SUM, orc.DRAIN_SEQ):
        a, b = _server(TINY, 3), _server(TINY, 3)
        for arr in arrivals:
            x, y = _mb(TINY, 3, [arr.mb_id], 4)
            e = a.worker_grads_batched([arr.worker], [arr.slot], [arr.mb_id], x, y)[0]
            a.apply_async(e.seq, 0.05)
            a.snapshot_weights(arr.slot)
            b.worker_grads_batched([arr.worker], [arr.slot], [arr.mb_id], x, y)
            assert b.drain_buffered(mode, 0.05) == 1
            b.snapshot_weights(arr.slot)
        assert np.array_equal(a.theta, b.theta) and a.version == b.version == 12


def test_async_uses_stale_snapshots():
    """A gradient is computed on the slot's snapshot, not on the server's current weights."""
    s = _server(TINY, 2)
    ids = [synth.minibatch_id(0, 0), synth.minibatch_id(1, 0)]
    x, y = _mb(TINY, 3, ids, 4)
    theta0 = s.theta.copy()
    e0 = s.worker_grads_batched([0], [0], ids[:1], x[:1], y[:1])[0]
    s.apply_async(e0.seq, 0.5)
    e1 = s.worker_grads_batched([1], [1], ids[1:], x[1:], y[1:])[0]        # slot 1 still holds theta0
    keep = orc.dropout_keep(3, ids[1], 4, TINY.F, 0.25)
    g_stale, _ = orc.worker_grad(TINY, theta0, x[1], y[1], keep, 0.25)
    g_fresh, _ = orc.worker_grad(TINY, s.theta, x[1], y[1], keep, 0.25)
    assert np.array_equal(e1.grad, g_stale) and not np.array_equal(e1.grad, g_fresh)
    assert e1.version == 0 and s.version == 1
    s.snapshot_weights(1)
    e2 = s.worker_grads_batched([1], [1], ids[1:], x[1:], y[1:])[0]
    assert np.array_equal(e2.grad, g_fresh) and e2.version == 1


def test_sum_and_seq_drain_agree_and_queue_semantics():
    plan = synth.OutagePlan(n_workers=3, up_steps=2, down_steps=4)
    out = {}
    for mode in (orc.DRAIN_SUM, orc.DRAIN_SEQ):
        s = _server(TINY, 1)
        for r, up, ids in plan.rounds():
            x, y = _mb(TINY, 3, ids, 4)
            s.worker_grads_batched(range(3), [0] * 3, ids, x, y)
            if up:
                assert s.drain_buffered(orc.DRAIN_SEQ, 0.05) == 3
                s.snapshot_weights(0)
        assert len(s.pending) == plan.n_buffered == 12
        # every outage gradient was computed on the same (last published) snapshot, on new data
        assert {e.version for e in s.pending} == {6}
        assert [e.seq for e in s.pending] == list(range(6, 18))
        assert [e.worker for e in s.pending] == [0, 1, 2] * 4
        assert len({e.mb_id for e in s.pending}) == 12
        before = s.theta.copy()
        manual = before - 0.05 * np.sum([e.grad for e in s.pending], axis=0)
        assert s.drain_buffered(mode, 0.05) == 12
        assert len(s.pending) == 0 and s.drain_buffered(mode, 0.05) == 0      # read once, then gone
        assert np.allclose(s.theta, manual, rtol=1e-12, atol=1e-15)
        assert not np.array_equal(s.theta, before)
        out[mode] = s.theta
    assert np.linalg.norm(out[0] - out[1]) <= 1e-12 * np.linalg.norm(out[0])


def test_apply_rules_on_plain_vectors():
    theta = np.array([1.0, -2.0, 0.5])
    g = [np.array([0.5, 0.25, -1.0]), np.array([-1.5, 0.75, 2.0])]
    assert np.array_equal(orc.apply_async(theta, g[0], 0.5), [0.75, -2.125, 1.0])
    assert np.array_equal(orc.apply_sync(theta, g, 0.5), [1.5, -2.5, 0.0])
    assert np.array_equal(orc.drain(theta, g, 0.5, orc.DRAIN_SEQ), [1.5, -2.5, 0.0])
    assert np.array_equal(orc.drain(theta, g, 0.5, orc.DRAIN_SUM), [1.5, -2.5, 0.0])
    assert orc.drain(theta, [], 0.5, orc.DRAIN_SUM) is theta


def test_update_direction_first_order():
    """theta - lr*g descends: loss(theta) - loss(theta - lr*g) = lr*|g|^2 to first order."""
    d, B = TINY, 4
    x, y = _rand_batch(d, B, 12)
    theta = _rand_theta(d, 6)
    keep = orc.dropout_keep(2, 3, B, d.F, 0.25)
    g, l0 = orc.worker_grad(d, theta, x, y, keep, 0.25)
    lr = 1e-7
    for new in (orc.apply_async(theta, g, lr), orc.apply_sync(theta, [g], lr), orc.drain(theta, [g], lr, orc.DRAIN_SEQ)):
        l1 = orc.worker_grad(d, new, x, y, keep, 0.25)[1]
        assert abs((l0 - l1) / (lr * g.dot(g)) - 1.0) < 1e-3


# ---------------------------------------------------------------- forced tie decisions

def test_forcing_the_oracles_own_decisions_changes_nothing():
    d, B = TINY, 3
    x, y = _rand_batch(d, B, 31)
    theta = _rand_theta(d, 32)
    keep = orc.dropout_keep(1, 1, B, d.F, 0.25)
    g, loss, rec = orc.worker_grad(d, theta, x, y, keep, 0.25, records=True)
    forced = []
    for s in range(B):
        forced += [[s, 1, i, int(rec.code1[s, i]) | (4 if rec.top1[s, i] > 0 else 0)] for i in range(d.n1)]
        forced += [[s, 2, i, int(rec.code2[s, i]) | (4 if rec.top2[s, i] > 0 else 0)] for i in range(d.n2)]
        forced += [[s, 3, u, int(rec.hpre[s, u] > 0)] for u in range(d.F)]
    g2, loss2 = orc.worker_grad(d, theta, x, y, keep, 0.25, forced=np.array(forced, np.int32))
    assert np.array_equal(g, g2) and loss == loss2


def test_forced_decision_equals_the_natural_one_across_a_tie():
    """Nudging an input across a tie by 1e-12 flips the natural decision; forcing that decision on the
    un-nudged side must give the same gradient up to the size of the nudge."""
    d, B = orc.Dims(H=8, W=8, C1=2, C2=3, F=8, NC=3), 2
    theta = _rand_theta(d, 40)
    theta[0:18] = 0.0
    theta[4] = 1.0          # conv1 channel 0 = identity on the image
    theta[9 + 4] = 0.7      # conv1 channel 1 = 0.7 * image
    theta[18:20] = 0.0
    x, y = _rand_batch(d, B, 41)
    keep = np.ones((B, d.F), np.uint8)
    # pool1 winner tie: window (0,0) of sample 1, elements 1 and 2 are the two largest and nearly equal
    xa = x.copy().reshape(B, 8, 8)
    xa[1, 0, 0], xa[1, 1, 1] = 0.1, 0.2
    xa[1, 0, 1], xa[1, 1, 0] = 0.9 + 1e-12, 0.9
    xb = xa.copy()
    xb[1, 0, 1], xb[1, 1, 0] = 0.9, 0.9 + 1e-12
    ga, _, ra = orc.worker_grad(d, theta, xa.reshape(B, 64), y, keep, 0.0, records=True)
    gb, _, rb = orc.worker_grad(d, theta, xb.reshape(B, 64), y, keep, 0.0, records=True)
    assert ra.code1[1, 0] == 1 and rb.code1[1, 0] == 2 and ra.margin1[1, 0] < 1e-11
    assert np.linalg.norm(ga - gb) > 1e-6 * np.linalg.norm(ga)          # the choice matters
    forced = np.array([[1, 1, 0, 2 | 4], [1, 1, 16, 2 | 4]], np.int32)   # both channels see the same window
    gf, _ = orc.worker_grad(d, theta, xa.reshape(B, 64), y, keep, 0.0, forced=forced)
    assert np.linalg.norm(gf - gb) <= 1e-9 * np.linalg.norm(gb)
    # fc1 ReLU gate: put unit 3 of sample 0 a hair above / below zero through its bias
    off_b = d.C1 * 10 + d.C2 * d.C1 * 9 + d.C2 + d.F * d.n2
    _, _, r0 = orc.worker_grad(d, theta, x, y, keep, 0.0, records=True)
    tp, tm = theta.copy(), theta.copy()
    tp[off_b + 3] += -r0.hpre[0, 3] + 1e-12
    tm[off_b + 3] += -r0.hpre[0, 3] - 1e-12
    gp, _, rp = orc.worker_grad(d, tp, x, y, keep, 0.0, records=True)
    gm, _, rm = orc.worker_grad(d, tm, x, y, keep, 0.0, records=True)
    assert 0 < rp.hpre[0, 3] < 1e-11 and -1e-11 < rm.hpre[0, 3] < 0
    assert np.linalg.norm(gp - gm) > 1e-6 * np.linalg.norm(gp)
    gf, _ = orc.worker_grad(d, tp, x, y, keep, 0.0, forced=np.array([[0, 3, 3, 0]], np.int32))
    assert np.linalg.norm(gf - gm) <= 1e-9 * np.linalg.norm(gm)
    # pool gate: a window whose winner sits a hair above zero, forced shut
    xz = x.copy().reshape(B, 8, 8)
    xz[0, 2:4, 2:4] = [[-0.3, -0.2], [1e-12, -0.5]]
    xn = xz.copy()
    xn[0, 3, 2] = -1e-12
    gz, _, rz = orc.worker_grad(d, theta, xz.reshape(B, 64), y, keep, 0.0, records=True)
    gn, _, _ = orc.worker_grad(d, theta, xn.reshape(B, 64), y, keep, 0.0, records=True)
    assert rz.code1[0, 5] == 2 and 0 < rz.top1[0, 5] < 1e-11
    gf, _ = orc.worker_grad(d, theta, xz.reshape(B, 64), y, keep, 0.0,
                            forced=np.array([[0, 1, 5, 2], [0, 1, 21, 2]], np.int32))
    assert np.linalg.norm(gf - gn) <= 1e-9 * max(np.linalg.norm(gn), 1e-3)


# ---------------------------------------------------------------- stale-gradient mitigation in the drain

def test_mitigated_drain_closed_forms():
    rng = np.random.default_rng(3)
    theta = rng.normal(size=50)
    pending = [rng.normal(size=50) * s for s in (0.1, 1.0, 5.0, 0.0)]
    norms = [np.linalg.norm(g) for g in pending]
    clip = 2.0
    scales = orc.clip_scales(pending, clip)
    for g, s, n in zip(pending, scales, norms):
        assert abs(np.linalg.norm(g * s) - min(n, clip)) < 1e-12          # clipped norm = min(norm, c)
        assert s == 1.0 if n <= clip else s < 1.0
    assert orc.clip_scales(pending, 0.0) == [1.0] * 4                      # clipping off
    # learning rate turned down only beyond the reference backlog
    assert orc.backlog_lr(0.01, 3, 0.0) == 0.01 and orc.backlog_lr(0.01, 3, 4.0) == 0.01
    assert orc.backlog_lr(0.01, 8, 4.0) == 0.005
    for mode in (orc.DRAIN_SUM, orc.DRAIN_SEQ):
        # both mitigations off: exactly the plain drain
        t0, used = orc.drain_mitigated(theta, pending, 0.01, mode, 0.0, 0.0)
        assert used == 0.01 and np.array_equal(t0, orc.drain(theta, pending, 0.01, mode))
        # backlog scaling alone = plain drain at the reduced rate
        t1, used = orc.drain_mitigated(theta, pending, 0.01, mode, 2.0, 0.0)
        assert used == 0.005 and np.array_equal(t1, orc.drain(theta, pending, 0.005, mode))
        # clipping alone = plain drain of the hand-clipped gradients
        t2, _ = orc.drain_mitigated(theta, pending, 0.01, mode, 0.0, clip)
        by_hand = [g if n <= clip else g * (clip / n) for g, n in zip(pending, norms)]
        assert np.allclose(t2, orc.drain(theta, by_hand, 0.01, mode), rtol=1e-14, atol=1e-16)
        # the update can never be longer than lr * K * clip
        assert np.linalg.norm(t2 - theta) <= 0.01 * 4 * clip + 1e-12


# ---------------------------------------------------------------- evaluation and checkpoint recovery

def test_evaluate_matches_independent_forward():
    d, n = orc.Dims(), 6
    x, y = synth.minibatch(4, 9, n)
    theta = synth.he_uniform_theta(4).astype(float) + np.random.default_rng(2).uniform(-0.02, 0.02, d.P)
    loss, acc, pred, z = orc.evaluate(d, theta, x, y)
    _, tloss, tz = _torch_grad(d, theta, x, y, np.ones((n, d.F)), 0.0)          # no dropout, scale 1
    assert abs(loss - tloss) <= 1e-12 * abs(tloss) and np.allclose(z, tz, rtol=1e-11, atol=1e-12)
    assert np.array_equal(pred, tz.argmax(1)) and acc == float(np.mean(tz.argmax(1) == y))
    # lowest index wins a tie: zero weights give all-equal logits
    _, acc0, pred0, _ = orc.evaluate(d, np.zeros(d.P), x, np.zeros(n, np.int32))
    assert (pred0 == 0).all() and acc0 == 1.0


def test_restore_continues_from_the_checkpointed_state():
    sc = synth.scenario_checkpoint(2, 4, 5, 0.05, period=2, kills=[2], kills_inflight=[4])
    nd = synth.NetDims(8, 8, 2, 3, 8, 3)
    theta0 = synth.he_uniform_theta(3, nd)
    mb = lambda seed, ids, B: synth.minibatches(seed, ids, B, h=8, w=8, n_classes=3)
    from oracle.sim import OracleReplay
    o = OracleReplay(sc, 3, 7, theta0, mb, 0.25, dims=TINY)
    seen = []
    for ev, _ in o.steps():
        if ev[0] == "snapshot" and ev[1] == 1:
            ckpt = (o.server.theta.copy(), o.server.version)
        if ev[0] == "restore":
            assert np.array_equal(o.server.theta, ckpt[0]) and o.server.version == ckpt[1] and not o.server.pending
            seen.append(o.dropped[-1])
    assert seen == [0, 2]                                   # the in-flight kill loses that step's two gradients
    # updates 1,2 -> checkpoint; update 3, kill -> back to 2; update -> 3, checkpoint; in-flight kill -> 3
    assert o.server.version == 3


def test_store_consume_is_a_prefix_in_arrival_order_read_once_then_deleted():
    """Section 3.3, last paragraph: write once, read once, delete.  Closed forms on hand-made
    gradients g_i = (i + 1) * e_i: a SUM step over the first k moves exactly coordinates 0..k-1 by
    lr * (i + 1) in one version; SEQ steps split anywhere give what one step gives; nothing is
    applied twice and the rest stays pending in order."""
    n, lr = 6, 0.5
    def server():
        s = orc.OracleServer(TINY, 7, 0.25, 1, np.zeros(n))
        for i in range(n):
            g = np.zeros(n)
            g[i] = i + 1.0
            s.pending.append(orc.QueueEntry(s.next_seq, i, 0, 100 + i, g, 0.0))
            s.next_seq += 1
        return s
    s = server()
    assert s.consume(orc.DRAIN_SUM, lr, 4) == 4
    assert np.array_equal(s.theta, [-0.5, -1.0, -1.5, -2.0, 0, 0]) and s.version == 1
    assert [e.seq for e in s.pending] == [4, 5]
    assert s.consume(orc.DRAIN_SEQ, lr, 10) == 2 and s.version == 3 and not s.pending
    assert np.array_equal(s.theta, -lr * np.arange(1.0, n + 1))
    assert s.consume(orc.DRAIN_SEQ, lr, 3) == 0 and s.version == 3          # empty store: nothing happens
    a, b = server(), server()
    a.consume(orc.DRAIN_SEQ, lr, 2), a.consume(orc.DRAIN_SEQ, lr, 1), a.consume(orc.DRAIN_SEQ, lr, 3)
    b.consume(orc.DRAIN_SEQ, lr, n)
    assert np.array_equal(a.theta, b.theta) and a.version == b.version == n


def test_adadelta_drain_against_an_independent_library_and_closed_forms():
    """Section 2.3 names an adaptive learning rate (Adadelta) for the stale gradients.  The oracle's
    recursion is pinned against torch.optim.Adadelta run on the same gradient sequence in fp64, and
    against the first step's closed form dx = -sqrt(eps) / sqrt((1 - rho) g^2 + eps) * g."""
    import torch
    rng = np.random.default_rng(5)
    n, K, lr, rho, eps = 37, 9, 0.7, 0.9, 1e-6
    theta0 = rng.standard_normal(n)
    grads = [rng.standard_normal(n) * 10.0 ** rng.integers(-3, 2) for _ in range(K)]
    got, g2, dx2 = orc.drain_adadelta(theta0, grads, lr, rho, eps, np.zeros(n), np.zeros(n))
    p = torch.nn.Parameter(torch.tensor(theta0, dtype=torch.float64))
    opt = torch.optim.Adadelta([p], lr=lr, rho=rho, eps=eps)
    for g in grads:
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
    assert np.allclose(got, p.detach().numpy(), rtol=1e-12, atol=1e-14)
    st = opt.state[p]
    assert np.allclose(g2, st["square_avg"].numpy(), rtol=1e-12) and np.allclose(dx2, st["acc_delta"].numpy(), rtol=1e-12)
    one, g2_1, dx2_1 = orc.drain_adadelta(theta0, grads[:1], lr, rho, eps, np.zeros(n), np.zeros(n))
    dx = -np.sqrt(eps) / np.sqrt((1 - rho) * grads[0] ** 2 + eps) * grads[0]
    assert np.allclose(one, theta0 + lr * dx, rtol=1e-15) and np.allclose(g2_1, (1 - rho) * grads[0] ** 2)
    assert np.allclose(dx2_1, (1 - rho) * dx ** 2)
    # the state carries over: two drains equal one drain of the concatenation; zero gradients move nothing
    a, ag, ad = orc.drain_adadelta(theta0, grads[:4], lr, rho, eps, np.zeros(n), np.zeros(n))
    b, _, _ = orc.drain_adadelta(a, grads[4:], lr, rho, eps, ag, ad)
    assert np.array_equal(b, got)
    z, zg, zd = orc.drain_adadelta(theta0, [np.zeros(n)] * 3, lr, rho, eps, np.zeros(n), np.zeros(n))
    assert np.array_equal(z, theta0) and not zg.any() and not zd.any()
    # and on the server model: version += K, queue emptied
    s = orc.OracleServer(TINY, 7, 0.25, 1, theta0)
    for i, g in enumerate(grads):
        s.pending.append(orc.QueueEntry(i, 0, 0, i, g, 0.0))
    assert s.drain_adadelta(lr, rho, eps) == K and s.version == K and not s.pending
    assert np.array_equal(s.theta, got)


def test_elastic_averaging_step_invariants_and_closed_forms():
    """Elastic averaging SGD (Section 2.3 names it): the forces between centre and workers cancel, so
    centre + sum_i x_i is conserved; equal weights are a fixed point; one worker with alpha = 1/2
    meets the centre half way; differences follow (x_i - c)' = (1 - alpha)(x_i - c) - alpha sum_j (x_j - c)."""
    rng = np.random.default_rng(2)
    n, W, alpha = 11, 5, 0.07
    c = rng.standard_normal(n)
    xs = [rng.standard_normal(n) for _ in range(W)]
    c1, xs1 = orc.elastic_average(c, xs, alpha)
    assert np.allclose(c1 + sum(xs1), c + sum(xs), rtol=0, atol=1e-13)
    tot = sum(x - c for x in xs)
    for x, x1 in zip(xs, xs1):
        assert np.allclose(x1 - c1, (1 - alpha) * (x - c) - alpha * tot, rtol=0, atol=1e-13)
    same_c, same = orc.elastic_average(c, [c.copy()] * 3, 0.3)
    assert np.array_equal(same_c, c) and all(np.array_equal(x, c) for x in same)
    mid_c, (mid_x,) = orc.elastic_average(c, [xs[0]], 0.5)
    assert np.allclose(mid_c, (c + xs[0]) / 2) and np.allclose(mid_x, (c + xs[0]) / 2)
    zero_c, zero = orc.elastic_average(c, xs, 0.0)
    assert np.array_equal(zero_c, c) and all(np.array_equal(a, b) for a, b in zip(zero, xs))
    # on the server model: a local step touches only its slot; the elastic step counts as one update
    s = orc.OracleServer(TINY, 7, 0.25, 2, c)
    g = rng.standard_normal(n)
    s.pending.append(orc.QueueEntry(0, 1, 0, 0, g, 0.0))
    s.next_seq = 1
    s.apply_local(1, 0, 0.1)
    assert np.array_equal(s.theta, c) and np.array_equal(s.ring[0], c) and np.allclose(s.ring[1], c - 0.1 * g)
    assert not s.pending and s.version == 0
    s.elastic_average([0, 1], 0.25)
    assert s.version == 1 and np.allclose(s.theta + s.ring[0] + s.ring[1], 3 * c - 0.1 * g)
