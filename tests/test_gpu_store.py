"""The lock-free gradient store (workers and server on two streams) vs the CPU oracle and vs the
ordered path, through the C ABI."""
import sys

import numpy as np
import pytest

from oracle import oracle as orc
from paper_2406_05546_amd import synth
from tests import parity

pytestmark = pytest.mark.gpu

DATA_SEED = 23
DROP_SEED = (0x5EED << 32) | 0x2406
P_DROP = 0.25


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


def _dev(x, y):
    import torch
    return torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()


def _valid_steps(steps, consumed, version0=0):
    """A server-step log is valid iff the steps tile [0, consumed) in order and the version grows by
    1 per SUM step and by the count per SEQ step."""
    at, v = 0, version0
    for first, count, mode, version_after in steps:
        assert first == at and count >= 1 and mode in (0, 1)
        at += count
        v += 1 if mode == 0 else count
        assert version_after == v
    assert at == consumed
    return v


def test_store_in_lockstep_with_the_oracle_over_a_wrapping_queue(ps):
    """5 rounds of 4 workers over 12 rows (positions wrap), two ring slots published in turn from the
    server stream, SUM and SEQ steps alternating; every gradient, the weights after every step,
    versions and counters against the oracle."""
    W, B, V, CAP, ROUNDS, lr = 4, 16, 2, 12, 5, 0.05
    theta0 = synth.he_uniform_theta(DATA_SEED)
    o = orc.OracleServer(orc.Dims(), DROP_SEED, P_DROP, V, theta0)
    ctx = ps.ps_init(ps.make_config(W, B, V, CAP, DROP_SEED, P_DROP))
    try:
        ps.ps_set_weights(ctx, theta0)
        expected_steps = []
        for r in range(ROUNDS):
            slot, mode = r % 2, r % 2
            workers = [(3 * r + i) % 7 for i in range(W)]
            mbs = [synth.minibatch_id(w, r) for w in workers]
            x, y = synth.minibatches(DATA_SEED, mbs, B)
            xd, yd = _dev(x, y)
            say(f"store lockstep: round {r} append on slot {slot}")
            import torch
            loss = torch.zeros(W, device="cuda")
            ps.worker_grads_append(ctx, workers, [slot] * W, mbs, xd, yd, loss)
            st = ps.ps_store_state(ctx)
            assert (st["claimed"], st["published"], st["consumed"]) == (W * (r + 1), W * (r + 1), W * r)
            ref = o.worker_grads_batched(workers, [slot] * W, mbs, x, y)
            losses = loss.cpu().numpy()
            for i in range(W):
                g, wk, ver, mb = ps.ps_store_entry(ctx, W * r + i)
                assert (wk, ver, mb) == (workers[i], ref[i].version, mbs[i])
                assert abs(losses[i] - ref[i].loss) <= 2e-5 * abs(ref[i].loss)
                if not parity.is_close(g, ref[i].grad, parity.TIE_LOOK):
                    res = parity.check_worker(ps, ctx, i, -1, o.ring[slot], x[i], y[i], mbs[i], DROP_SEED, P_DROP,
                                              f"round {r} worker {i}", grad=g)
                    ref[i].grad[:] = res["grad"]            # the oracle goes on from the branch taken
            ps.ps_store_consume(ctx, mode, lr, 0, True)
            assert o.consume(mode, lr, W) == W
            expected_steps.append((W * r, W, mode, o.version))
            ps.ps_store_publish(ctx, 1 - slot)
            o.snapshot_weights(1 - slot)
            if r == 2:
                # evaluation in the middle of a store session waits for both streams and sees the step just enqueued
                ex, ey = synth.eval_batch(DATA_SEED, r, 2 * B)
                exd, eyd = _dev(ex, ey)
                gl, ga, gp = ps.ps_evaluate(ctx, -1, exd, eyd)
                ol, oa, op, oz = orc.evaluate(orc.Dims(), o.theta, ex, ey)
                zs = np.sort(oz, axis=1)
                clear = (zs[:, -1] - zs[:, -2]) > 2.0 * parity.REACH[4] * np.abs(oz).max()
                assert abs(gl - ol) <= 2e-5 * abs(ol) and np.array_equal(gp[clear], op[clear])
            parity.assert_close(ps.ps_get_weights(ctx), o.theta, parity.WEIGHT_TOL, f"weights after round {r}")
            parity.assert_close(ps.ps_get_weights(ctx, 1 - slot), o.ring[1 - slot], parity.WEIGHT_TOL, "published slot")
            st = ps.ps_store_state(ctx)
            assert st == {"claimed": W * (r + 1), "published": W * (r + 1), "consumed": W * (r + 1),
                          "version": o.version, "steps": r + 1}
            with pytest.raises(ps.PsError) as e:                # read once, then deleted
                ps.ps_store_entry(ctx, W * r, want_grad=False)
            assert e.value.status == ps.PS_ESTATE
        assert ps.ps_store_steps(ctx) == expected_steps
        assert ps.ps_version(ctx) == o.version
    finally:
        ps.ps_destroy(ctx)


def test_store_limits_capacity_and_hand_over_to_the_ordered_calls(ps):
    W, B, CAP, lr = 4, 8, 6, 0.1
    theta0 = synth.he_uniform_theta(4)
    o = orc.OracleServer(orc.Dims(), DROP_SEED, P_DROP, 1, theta0)
    mbs = [synth.minibatch_id(w, 0) for w in range(W)]
    x, y = synth.minibatches(DATA_SEED, mbs, B)
    xd, yd = _dev(x, y)
    ctx = ps.ps_init(ps.make_config(W, B, 1, CAP, DROP_SEED, P_DROP))
    try:
        ps.ps_set_weights(ctx, theta0)
        # an ordered update first: the store must carry on from version 1
        q = ps.worker_grads_batched(ctx, [0], [0], mbs[:1], xd, yd)
        ps.ps_apply_sync(ctx, q, lr)
        ps.ps_snapshot_weights(ctx, 0)
        o.worker_grads_batched([0], [0], mbs[:1], x[:1], y[:1])
        o.consume(orc.DRAIN_SUM, lr, 1)
        o.snapshot_weights(0)
        ps.worker_grads_append(ctx, range(W), [0] * W, mbs, xd, yd)
        ref = o.worker_grads_batched(range(W), [0] * W, mbs, x, y)
        with pytest.raises(ps.PsError) as e:                    # 4 + 4 > 6: refused, nothing claimed
            ps.worker_grads_append(ctx, range(W), [0] * W, mbs, xd, yd)
        assert e.value.status == ps.PS_EFULL
        for call in (lambda: ps.worker_grads_batched(ctx, [0], [0], mbs[:1], xd, yd),
                     lambda: ps.ps_snapshot_weights(ctx, 0), lambda: ps.ps_drain_buffered(ctx, 0, lr),
                     lambda: ps.ps_restore_weights(ctx, 0), lambda: ps.ps_set_weights(ctx, theta0),
                     lambda: ps.ps_queue_push_host(ctx, theta0, 0, 0, 0)):
            with pytest.raises(ps.PsError) as e:                # the store holds gradients
                call()
            assert e.value.status == ps.PS_ESTATE
        st = ps.ps_store_state(ctx)
        assert (st["claimed"], st["published"], st["consumed"], st["version"]) == (4, 4, 0, 1)
        assert ps.ps_store_entry(ctx, 2, want_grad=False)[1:] == (2, 1, mbs[2])      # snapshot version 1
        for i in range(W):
            g = ps.ps_store_entry(ctx, i)[0]
            if not parity.is_close(g, ref[i].grad, parity.TIE_LOOK):
                ref[i].grad[:] = parity.check_worker(ps, ctx, i, -1, o.ring[0], x[i], y[i], mbs[i], DROP_SEED, P_DROP,
                                                     f"worker {i}", grad=g)["grad"]
        with pytest.raises(ps.PsError) as e:
            ps.ps_store_entry(ctx, 4, want_grad=False)          # never appended
        assert e.value.status == ps.PS_ESTATE
        ps.ps_store_consume(ctx, ps.DRAIN_SEQ, lr, 3, True)     # a limit: exactly three are taken
        o.consume(orc.DRAIN_SEQ, lr, 3)
        st = ps.ps_store_state(ctx)
        assert (st["consumed"], st["version"], st["steps"]) == (3, 4, 1)
        parity.assert_close(ps.ps_get_weights(ctx), o.theta, parity.WEIGHT_TOL, "weights after three")
        ps.worker_grads_append(ctx, range(W), [0] * W, mbs, xd, yd)      # 1 + 4 <= 6 now; rows 4, 5, 0, 1
        o.worker_grads_batched(range(W), [0] * W, mbs, x, y)
        for i in range(W):
            o.pending[1 + i].grad[:] = ref[i].grad                        # same inputs, same snapshot
        ps.ps_store_consume(ctx, ps.DRAIN_SUM, lr, 0, True)
        o.consume(orc.DRAIN_SUM, lr, 5)
        ps.ps_store_consume(ctx, ps.DRAIN_SUM, lr, 0, True)               # nothing left: no step, no version
        st = ps.ps_store_state(ctx)
        assert st == {"claimed": 8, "published": 8, "consumed": 8, "version": 5, "steps": 2}
        assert ps.ps_store_steps(ctx) == [(0, 3, 1, 4), (3, 5, 0, 5)]
        parity.assert_close(ps.ps_get_weights(ctx), o.theta, parity.WEIGHT_TOL, "weights after all")
        # back to the ordered calls, which continue from the store's version
        assert ps.ps_version(ctx) == 5 and ps.ps_snapshot_weights(ctx, 0) == 5
        q = ps.worker_grads_batched(ctx, [1], [0], mbs[1:2], xd[1:2].contiguous(), yd[1:2].contiguous())
        with pytest.raises(ps.PsError) as e:                    # ordered queue not empty
            ps.worker_grads_append(ctx, range(W), [0] * W, mbs, xd, yd)
        assert e.value.status == ps.PS_ESTATE
        assert ps.ps_drain_buffered(ctx, ps.DRAIN_SEQ, lr) == 1 and ps.ps_version(ctx) == 6
        ps.worker_grads_append(ctx, [0], [0], mbs[:1], xd, yd)
        ps.ps_store_consume(ctx, ps.DRAIN_SEQ, lr, 0, True)
        st = ps.ps_store_state(ctx)
        assert (st["claimed"], st["consumed"], st["version"]) == (9, 9, 7)
        for bad in (lambda: ps.ps_store_consume(ctx, 2, lr), lambda: ps.ps_store_consume(ctx, 0, lr, -1),
                    lambda: ps.ps_store_publish(ctx, 1), lambda: ps.worker_grads_append(ctx, [0], [1], mbs[:1], xd, yd),
                    lambda: ps.worker_grads_append(ctx, range(W + 1), [0] * (W + 1), mbs + mbs[:1], xd, yd)):
            with pytest.raises((ps.PsError, AssertionError)) as e:
                bad()
            assert not isinstance(e.value, ps.PsError) or e.value.status == ps.PS_EINVAL
    finally:
        ps.ps_destroy(ctx)


def test_versions_come_back_from_the_store_without_reading_its_state(ps):
    """Store calls, then ordered calls with nothing but ps_sync in between (no ps_store_state): the
    update count and the snapshot versions the device kept must be what the ordered calls continue from,
    and a second store session must start from the ordered calls' count."""
    W, B, lr = 3, 8, 0.05
    theta0 = synth.he_uniform_theta(6)
    mbs = [synth.minibatch_id(w, 0) for w in range(W)]
    x, y = synth.minibatches(DATA_SEED, mbs, B)
    xd, yd = _dev(x, y)
    ctx = ps.ps_init(ps.make_config(W, B, 2, W, DROP_SEED, P_DROP))
    try:
        ps.ps_set_weights(ctx, theta0)
        ps.worker_grads_append(ctx, range(W), [0] * W, mbs, xd, yd)
        ps.ps_store_consume(ctx, ps.DRAIN_SEQ, lr, 0, True)            # version 3 on the device
        ps.ps_store_publish(ctx, 1)                                    # slot 1 holds version 3
        ps.ps_sync(ctx)
        assert ps.ps_snapshot_weights(ctx, 0) == W                     # first ordered call: no ps_store_state before it
        assert ps.ps_version(ctx) == W
        q = ps.worker_grads_batched(ctx, [0, 1], [0, 1], mbs[:2], xd, yd)
        assert [(m[1], m[2]) for m in ps.ps_queue_meta(ctx)] == [(0, W), (1, W)]   # both snapshots carry version 3
        ps.ps_apply_sync(ctx, q, lr)
        assert ps.ps_version(ctx) == W + 1
        # and the other way round without a read in between
        ps.worker_grads_append(ctx, [2], [1], mbs[2:], xd[2:].contiguous(), yd[2:].contiguous())
        ps.ps_store_consume(ctx, ps.DRAIN_SUM, lr, 0, True)
        assert ps.ps_version(ctx) == W + 2                              # waits for both streams, reads the device count
        ps.ps_sync(ctx)
        assert ps.ps_restore_weights(ctx, 1) == 0 and ps.ps_version(ctx) == W
        st = ps.ps_store_state(ctx)
        assert (st["claimed"], st["consumed"]) == (W + 1, W + 1)
    finally:
        ps.ps_destroy(ctx)


@pytest.mark.parametrize("mode", [1, 0])
def test_store_server_racing_the_workers(ps, mode):
    """Server steps enqueued without waiting for the workers take whatever is complete when they run.
    Whatever the timing: the log tiles the positions in order; in SEQ mode the final weights equal,
    bit for bit, those of the ordered path on the same inputs (same updates in the same order); in SUM
    mode they match the oracle applying the logged groups."""
    W, B, ROUNDS, lr = 8, 32, 6, 0.02
    theta0 = synth.he_uniform_theta(9)
    rounds = []
    for r in range(ROUNDS):
        mbs = [synth.minibatch_id(w, r) for w in range(W)]
        x, y = synth.minibatches(DATA_SEED, mbs, B)
        rounds.append((mbs, x, y) + _dev(x, y))
    ctx = ps.ps_init(ps.make_config(W, B, 1, W * ROUNDS, DROP_SEED, P_DROP))
    try:
        ps.ps_set_weights(ctx, theta0)
        for mbs, x, y, xd, yd in rounds:
            ps.worker_grads_batched(ctx, range(W), [0] * W, mbs, xd, yd)
        assert ps.ps_drain_buffered(ctx, ps.DRAIN_SEQ, lr) == W * ROUNDS
        ordered = ps.ps_get_weights(ctx)
        ps.ps_set_weights(ctx, theta0)
        say(f"store race: mode {mode}")
        for mbs, x, y, xd, yd in rounds:
            ps.worker_grads_append(ctx, range(W), [0] * W, mbs, xd, yd)
            ps.ps_store_consume(ctx, mode, lr, 0, False)
            ps.ps_store_consume(ctx, mode, lr, 5, False)
        ps.ps_store_consume(ctx, mode, lr, 0, True)
        st = ps.ps_store_state(ctx)
        assert st["claimed"] == st["published"] == st["consumed"] == W * ROUNDS
        steps = ps.ps_store_steps(ctx)
        assert _valid_steps(steps, W * ROUNDS) == st["version"] and len(steps) == st["steps"]
        say(f"store race: groups {[s[1] for s in steps]}")
        got = ps.ps_get_weights(ctx)
        if mode == 1:
            assert np.array_equal(got, ordered)
        else:
            o = orc.OracleServer(orc.Dims(), DROP_SEED, P_DROP, 1, theta0)
            for mbs, x, y, xd, yd in rounds:
                o.worker_grads_batched(range(W), [0] * W, mbs, x, y)
            for _, count, _, _ in steps:
                o.consume(orc.DRAIN_SUM, lr, count)
            parity.assert_close(got, o.theta, parity.WEIGHT_TOL, "weights after racing SUM steps")
    finally:
        ps.ps_destroy(ctx)


def test_store_full_size_overlapped_rounds(ps):
    """W=256, B=256, 1024 rows: four appended rounds, each consumed on the server stream while the next
    one computes (the bench's overlapped schedule).  Sampled gradients against the oracle; final
    weights bit for bit those of the ordered path (4 rounds, then a SEQ drain)."""
    W, B, ROUNDS, lr = 256, 256, 4, 0.005
    theta0 = synth.he_uniform_theta(DATA_SEED)
    ctx = ps.ps_init(ps.make_config(W, B, 2, W * ROUNDS, DROP_SEED, P_DROP))
    try:
        ps.ps_set_weights(ctx, theta0)
        rounds = []
        for r in range(ROUNDS):
            mbs = [synth.minibatch_id(w, r) for w in range(W)]
            x, y = synth.minibatches(DATA_SEED, mbs, B)
            rounds.append((mbs, x, y) + _dev(x, y))
        for mbs, x, y, xd, yd in rounds:
            ps.worker_grads_batched(ctx, range(W), [0] * W, mbs, xd, yd)
        assert ps.ps_drain_buffered(ctx, ps.DRAIN_SEQ, lr) == W * ROUNDS
        ordered = ps.ps_get_weights(ctx)
        ps.ps_set_weights(ctx, theta0)
        say("store full size: first round, sampled against the oracle")
        mbs, x, y, xd, yd = rounds[0]
        ps.worker_grads_append(ctx, range(W), [0] * W, mbs, xd, yd)
        for w in (3, 200):
            g, wk, ver, mb = ps.ps_store_entry(ctx, w)
            assert (wk, ver, mb) == (w, 0, mbs[w])
            r = parity.check_worker(ps, ctx, w, -1, theta0.astype(np.float64), x[w], y[w], mbs[w], DROP_SEED, P_DROP,
                                    f"worker {w}", grad=g)
            say(f"store full size: worker {w} rel err {r['worst']:.2e}")
        ps.ps_store_consume(ctx, ps.DRAIN_SEQ, lr, 0, True)
        for mbs, x, y, xd, yd in rounds[1:]:
            ps.worker_grads_append(ctx, range(W), [0] * W, mbs, xd, yd)
            ps.ps_store_consume(ctx, ps.DRAIN_SEQ, lr, 0, True)
        ps.ps_store_publish(ctx, 1)
        st = ps.ps_store_state(ctx)
        assert st == {"claimed": 1024, "published": 1024, "consumed": 1024, "version": 1024, "steps": 4}
        assert ps.ps_store_steps(ctx) == [(256 * r, 256, 1, 256 * (r + 1)) for r in range(4)]
        assert np.array_equal(ps.ps_get_weights(ctx), ordered)
        assert np.array_equal(ps.ps_get_weights(ctx, 1), ordered)
    finally:
        ps.ps_destroy(ctx)


def test_store_many_small_steps_wrap_the_step_log_and_the_readback_ring(ps):
    """1100 one-gradient appends, each consumed by its own server step, over a 3-row queue: the
    device keeps the last 1024 steps, positions wrap the queue 366 times, and the host's view of the
    consumed count has to keep up without ever reporting a full store.  The weights must equal, bit
    for bit, those of the ordered path applying the same 1100 gradients one by one."""
    B, STEPS, lr = 2, 1100, 0.01
    theta0 = synth.he_uniform_theta(12)
    mbs = [synth.minibatch_id(0, k) for k in range(8)]
    x, y = synth.minibatches(DATA_SEED, mbs, B)
    xd, yd = _dev(x, y)
    ctx = ps.ps_init(ps.make_config(1, B, 1, 3, DROP_SEED, P_DROP))
    try:
        ps.ps_set_weights(ctx, theta0)
        for k in range(STEPS):
            i = k % 8
            (q,) = ps.worker_grads_batched(ctx, [0], [0], [mbs[i]], xd[i:i + 1], yd[i:i + 1])
            ps.ps_apply_async(ctx, q, lr)
        ordered = ps.ps_get_weights(ctx)
        assert ps.ps_version(ctx) == STEPS
        ps.ps_set_weights(ctx, theta0)
        say("store small steps: 1100 appends")
        for k in range(STEPS):
            i = k % 8
            ps.worker_grads_append(ctx, [0], [0], [mbs[i]], xd[i:i + 1], yd[i:i + 1])
            ps.ps_store_consume(ctx, ps.DRAIN_SEQ, lr, 0, True)
        st = ps.ps_store_state(ctx)
        assert st == {"claimed": STEPS, "published": STEPS, "consumed": STEPS, "version": STEPS, "steps": STEPS}
        steps = ps.ps_store_steps(ctx, 2000)
        assert steps == [(k, 1, 1, k + 1) for k in range(STEPS - 1024, STEPS)]
        assert ps.ps_store_steps(ctx, 5) == [(k, 1, 1, k + 1) for k in range(STEPS - 5, STEPS)]
        assert np.array_equal(ps.ps_get_weights(ctx), ordered)
    finally:
        ps.ps_destroy(ctx)
