"""Seeded synthetic inputs and replay schedules.

This module serves both the HIP path's harness and the CPU oracle's harness and
therefore holds none of the method's arithmetic: it only produces inputs
(pixels, labels, initial weights, stand-in gradient rows) and the order of
events (which worker's gradient arrives when, when the server is down).

Inputs stand in for FashionMNIST (Section 4 of the paper), which is not
shipped: one-channel 28x28 images with pixels uniform in [0, 1) and labels
uniform over the 10 classes, drawn from numpy's Philox bit generator keyed by
(seed, stream, minibatch id) so that a minibatch's content depends only on its
logical id and never on how workers are batched into a call.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Iterator, List, Sequence, Tuple

import numpy as np

IMG_H = 28
IMG_W = 28
N_CLASSES = 10

_STREAM_PIXELS = 1
_STREAM_LABELS = 2
_STREAM_THETA = 3
_STREAM_PERM = 4
_STREAM_GRAD = 5


def _raw(seed: int, stream: int, ident: int, n: int) -> np.ndarray:
    """n raw 64-bit words of the (seed, stream, ident) Philox stream."""
    key = np.array([seed & 0xFFFFFFFFFFFFFFFF, ((stream & 0xFF) << 56) ^ (ident & 0x00FFFFFFFFFFFFFF)],
                   dtype=np.uint64)
    return np.random.Philox(key=key).random_raw(n)


def _unit_f32(raw: np.ndarray) -> np.ndarray:
    """Top 24 bits of each word as a float32 in [0, 1) (exactly representable)."""
    return ((raw >> np.uint64(40)).astype(np.float32)) * np.float32(2.0 ** -24)


def minibatch_id(worker: int, local_step: int) -> int:
    """64-bit logical id of a worker's minibatch: strictly increasing per worker, also while
    the server is down (Section 2.3: workers keep computing on new data)."""
    return ((worker & 0xFFFFFFFF) << 32) | (local_step & 0xFFFFFFFF)


def minibatch(seed: int, mb_id: int, batch: int, h: int = IMG_H, w: int = IMG_W,
              n_classes: int = N_CLASSES) -> Tuple[np.ndarray, np.ndarray]:
    """(x float32 [batch, h*w] in [0,1), y int32 [batch] in [0, n_classes))."""
    x = _unit_f32(_raw(seed, _STREAM_PIXELS, mb_id, batch * h * w)).reshape(batch, h * w)
    r = _raw(seed, _STREAM_LABELS, mb_id, batch) >> np.uint64(32)
    y = ((r * np.uint64(n_classes)) >> np.uint64(32)).astype(np.int32)
    return x, y


def minibatches(seed: int, mb_ids: Sequence[int], batch: int, **kw) -> Tuple[np.ndarray, np.ndarray]:
    """Stacked minibatches: x [n, batch, h*w], y [n, batch]."""
    xs, ys = zip(*(minibatch(seed, m, batch, **kw) for m in mb_ids))
    return np.stack(xs), np.stack(ys)


@dataclass(frozen=True)
class NetDims:
    """Sizes of the paper's CNN (model endnote); smaller values give the tiny nets used by tests."""
    H: int = IMG_H
    W: int = IMG_W
    C1: int = 16
    C2: int = 32
    F: int = 512
    NC: int = N_CLASSES

    @property
    def feat(self) -> int:
        return self.C2 * (self.H // 4) * (self.W // 4)

    def segments(self) -> List[Tuple[str, int, Tuple[int, ...], int]]:
        """(name, offset, shape, fan_in) of the 8 tensors in the flat parameter vector."""
        out, off = [], 0
        for name, shape, fan in (
            ("conv1.W", (self.C1, 1, 3, 3), 9), ("conv1.b", (self.C1,), 0),
            ("conv2.W", (self.C2, self.C1, 3, 3), 9 * self.C1), ("conv2.b", (self.C2,), 0),
            ("fc1.W", (self.F, self.feat), self.feat), ("fc1.b", (self.F,), 0),
            ("fc2.W", (self.NC, self.F), self.F), ("fc2.b", (self.NC,), 0),
        ):
            out.append((name, off, shape, fan))
            off += int(np.prod(shape))
        return out

    @property
    def P(self) -> int:
        name, off, shape, _ = self.segments()[-1]
        return off + int(np.prod(shape))


def he_uniform_theta(seed: int, dims: NetDims = NetDims()) -> np.ndarray:
    """Initial flat parameter vector, float32: weights U(-sqrt(6/fan_in), +sqrt(6/fan_in)), biases 0."""
    theta = np.zeros(dims.P, dtype=np.float32)
    for i, (name, off, shape, fan) in enumerate(dims.segments()):
        if fan == 0:
            continue
        n = int(np.prod(shape))
        u = _unit_f32(_raw(seed, _STREAM_THETA, i, n))
        bound = np.float32(np.sqrt(6.0 / fan))
        theta[off:off + n] = (u * np.float32(2.0) - np.float32(1.0)) * bound
    return theta


def gradient_rows(seed: int, first: int, count: int, P: int, scale: float = 1e-2) -> np.ndarray:
    """Stand-in gradient rows (float32 [count, P], uniform in [-scale, scale)) for exercising the
    server's apply rules at sizes where real gradients would take the oracle too long."""
    out = np.empty((count, P), dtype=np.float32)
    for i in range(count):
        u = _unit_f32(_raw(seed, _STREAM_GRAD, first + i, P))
        out[i] = (u * np.float32(2.0) - np.float32(1.0)) * np.float32(scale)
    return out


# --------------------------------------------------------------------------- schedules

@dataclass(frozen=True)
class Arrival:
    """One gradient arriving at the server."""
    seq: int          # arrival number, 0-based
    worker: int
    slot: int         # ring slot holding the snapshot the gradient was computed on
    mb_id: int        # logical minibatch id


def worker_permutation(seed: int, n_workers: int) -> List[int]:
    """Seeded permutation of the workers (Fisher-Yates on the raw stream)."""
    perm = list(range(n_workers))
    r = _raw(seed, _STREAM_PERM, n_workers, n_workers)
    for i in range(n_workers - 1, 0, -1):
        j = int(r[i] % np.uint64(i + 1))
        perm[i], perm[j] = perm[j], perm[i]
    return perm


def async_cyclic_arrivals(seed: int, n_workers: int, n_arrivals: int) -> List[Arrival]:
    """Asynchronous arrival order: one seeded permutation of the workers repeated cyclically.
    Worker w owns ring slot w.  On arrival the server applies the gradient, then that worker
    pulls the new weights into its slot and starts its next minibatch, so a gradient is at most
    n_workers-1 server versions stale."""
    perm = worker_permutation(seed, n_workers)
    step = [0] * n_workers
    out = []
    for t in range(n_arrivals):
        w = perm[t % n_workers]
        out.append(Arrival(seq=t, worker=w, slot=w, mb_id=minibatch_id(w, step[w])))
        step[w] += 1
    return out


@dataclass(frozen=True)
class OutagePlan:
    """Stateless-server run: `up_steps` rounds with the server up, then `down_steps` rounds with it
    down (workers keep appending gradients computed on the last published snapshot), then recovery."""
    n_workers: int
    up_steps: int
    down_steps: int

    def rounds(self) -> Iterator[Tuple[int, bool, List[int]]]:
        """Yields (round index, server_up, minibatch ids in worker order)."""
        for r in range(self.up_steps + self.down_steps):
            yield r, r < self.up_steps, [minibatch_id(w, r) for w in range(self.n_workers)]

    @property
    def n_buffered(self) -> int:
        return self.n_workers * self.down_steps


# --------------------------------------------------------------------------- scenarios
# A scenario is a list of events that both the HIP harness and the oracle harness replay:
#   ("grads", workers, slots, mb_ids)   each listed worker computes one gradient on its slot's
#                                       snapshot; gradients get consecutive arrival numbers (seq)
#   ("sync", seqs, lr)                  one update with all listed gradients
#   ("async", seq, lr)                  one update with one gradient
#   ("drain", mode, lr[, ref, clip])    stateless server step over everything pending; with ref / clip
#                                       the learning rate is scaled by min(1, ref / K) and every
#                                       gradient clipped to 2-norm clip (0 = off)
#   ("snapshot", slot)                  a worker pulls the current weights into a ring slot (or the
#                                       server checkpoints / replicates them into it)
#   ("restore", slot)                   the server is killed and comes back with the weights of that slot;
#                                       pending gradients are lost
#   ("eval", n_images, eval_id)         periodic evaluation of the current weights on a held-out batch

DRAIN_SUM = 0
DRAIN_SEQ = 1


@dataclass(frozen=True)
class Scenario:
    name: str
    n_workers: int
    batch: int
    n_slots: int
    queue_capacity: int
    events: Tuple[tuple, ...]

    @property
    def max_call(self) -> int:
        return max((len(e[1]) for e in self.events if e[0] == "grads"), default=1)

    @property
    def n_gradients(self) -> int:
        return sum(len(e[1]) for e in self.events if e[0] == "grads")


def scenario_sync(n_workers: int, batch: int, steps: int, lr: float) -> Scenario:
    """Synchronous SGD: every step all workers compute on the same snapshot, the server waits for
    all of them and updates once."""
    ev, seq = [], 0
    for step in range(steps):
        ws = list(range(n_workers))
        ev.append(("grads", ws, [0] * n_workers, [minibatch_id(w, step) for w in ws]))
        ev.append(("sync", list(range(seq, seq + n_workers)), lr))
        ev.append(("snapshot", 0))
        seq += n_workers
    return Scenario("sync", n_workers, batch, 1, n_workers, tuple(ev))


def scenario_async(seed: int, n_workers: int, batch: int, n_arrivals: int, lr: float) -> Scenario:
    """Asynchronous SGD with the cyclic seeded arrival order of async_cyclic_arrivals.  The W
    gradients in flight at the start of a cycle are computed in one batched call, each on its own
    worker's slot; they then arrive one by one, and after each arrival that worker pulls."""
    arr = async_cyclic_arrivals(seed, n_workers, n_arrivals)
    ev = []
    for r0 in range(0, n_arrivals, n_workers):
        cyc = arr[r0:r0 + n_workers]
        ev.append(("grads", [a.worker for a in cyc], [a.slot for a in cyc], [a.mb_id for a in cyc]))
        for a in cyc:
            ev.append(("async", a.seq, lr))
            ev.append(("snapshot", a.slot))
    return Scenario("async", n_workers, batch, n_workers, n_workers, tuple(ev))


def scenario_outage(n_workers: int, batch: int, up_steps: int, down_steps: int, lr: float,
                    recovery_mode: int = DRAIN_SEQ, recovery_lr: float = None, lr_backlog_ref: float = 0.0,
                    clip_norm: float = 0.0) -> Scenario:
    """Stateless server: while it is up every round ends with a server step over the W new
    gradients and a publish; while it is down rounds only append; recovery is one server step over
    the whole backlog."""
    plan = OutagePlan(n_workers, up_steps, down_steps)
    ev = []
    for r, up, ids in plan.rounds():
        ev.append(("grads", list(range(n_workers)), [0] * n_workers, ids))
        if up:
            ev.append(("drain", DRAIN_SEQ, lr))
            ev.append(("snapshot", 0))
    ev.append(("drain", recovery_mode, lr if recovery_lr is None else recovery_lr, lr_backlog_ref, clip_norm))
    ev.append(("snapshot", 0))
    return Scenario("outage", n_workers, batch, 1, max(n_workers, plan.n_buffered), tuple(ev))


def scenario_versions(n_workers: int, batch: int, n_slots: int, steps: int, lr: float) -> Scenario:
    """Batched asynchronous steps with `n_slots` weight versions resident: worker w reads slot
    w % n_slots; after a step's gradients have been applied one by one in worker order the new
    weights are published into slot step % n_slots, so snapshots are 0..n_slots-1 steps stale."""
    ev, seq = [], 0
    for step in range(steps):
        ws = list(range(n_workers))
        ev.append(("grads", ws, [w % n_slots for w in ws], [minibatch_id(w, step) for w in ws]))
        for i in range(n_workers):
            ev.append(("async", seq + i, lr))
        ev.append(("snapshot", step % n_slots))
        seq += n_workers
    return Scenario("versions", n_workers, batch, n_slots, n_workers, tuple(ev))


def scenario_checkpoint(n_workers: int, batch: int, steps: int, lr: float, period: int, kills: Sequence[int],
                        asynchronous: bool = False, eval_images: int = 0, kills_inflight: Sequence[int] = ()) -> Scenario:
    """Checkpointing / chain-replication arm: sync (or async in worker order) training in which the
    weights are copied to a checkpoint slot (a file in the checkpointing arms, the backup server's
    memory in the chain arms) after every `period` weight updates; after each step listed in `kills`
    the server dies and comes back with the checkpointed weights, and the workers pull them; in a
    step listed in `kills_inflight` it dies while that step's gradients are still pending, which are
    lost.  With eval_images > 0 the weights are evaluated after every step."""
    ckpt = 1
    ev, seq, updates = [("snapshot", ckpt)], 0, 0
    for step in range(steps):
        ws = list(range(n_workers))
        ev.append(("grads", ws, [0] * n_workers, [minibatch_id(w, step) for w in ws]))
        if step in kills_inflight:
            ev.append(("restore", ckpt))
        elif asynchronous:
            for i in range(n_workers):
                ev.append(("async", seq + i, lr))
                updates += 1
                if updates % period == 0:
                    ev.append(("snapshot", ckpt))
        else:
            ev.append(("sync", list(range(seq, seq + n_workers)), lr))
            updates += 1
            if updates % period == 0:
                ev.append(("snapshot", ckpt))
        seq += n_workers
        if step in kills:
            ev.append(("restore", ckpt))
        ev.append(("snapshot", 0))
        if eval_images:
            ev.append(("eval", eval_images, step))
    return Scenario("checkpoint", n_workers, batch, 2, n_workers, tuple(ev))


def eval_batch(seed: int, eval_id: int, n_images: int) -> Tuple[np.ndarray, np.ndarray]:
    """Held-out evaluation images: a minibatch id space no worker uses."""
    return minibatch(seed, minibatch_id(0xFFFFFFFF, eval_id), n_images)


def paper_configs() -> dict:
    """The five evaluation configurations (sizes fixed by this build; the paper states none)."""
    return {
        "sync_w2_b32": scenario_sync(2, 32, 10, 0.01),
        "async_w4_b64": scenario_async(1, 4, 64, 100, 0.01),
        "outage_w8_b64": scenario_outage(8, 64, 20, 50, 0.01),
        # 64 summed updates per step from snapshots up to 7 steps old: at 0.01 the run diverges (the loss
        # triples within three steps and rounding is amplified without bound); 0.01 / 8 gives the same
        # summed rate per step, W * lr = 0.08, as the 8-worker outage configuration
        "versions_w64_b128": scenario_versions(64, 128, 8, 50, 0.00125),
        "outage_w256_b256": scenario_outage(256, 256, 0, 4, 0.005, DRAIN_SUM),
    }
