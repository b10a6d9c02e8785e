"""CPU oracle: Python face of ps_oracle.c plus the server's three update rules.

TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64; shares no code with the HIP path
and never imports it.  Only tests, the smoke check and the bench's CPU-baseline
leg may use it.

Update rules (stated in the paper in prose; restated here):
  sync      (Section 2.1, Section 3.1): wait for every worker's gradient, then
            update once with all of them:  theta <- theta - lr * sum_w g_w
  async     (Section 2.1, Section 3.1): update as soon as any gradient arrives:
            theta <- theta - lr * g, g computed on whatever (possibly stale)
            snapshot that worker held
  stateless (Section 2.3, Section 3.3 and its pseudo-code figure): one server
            step gathers ALL pending gradients, applies them to the stored
            weights, publishes the result and removes the applied gradients;
            while the server is down the list only grows.
Readings where the paper is silent: the aggregate is a SUM (not a mean) of the
per-worker mean-loss gradients, so that applying pending gradients "all at once"
and "one by one" agree up to rounding; plain SGD without momentum.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ps_oracle.c")
_LIB = os.path.join(_HERE, "libps_oracle.so")


def build(force: bool = False) -> str:
    """Compile ps_oracle.c with gcc (IEEE semantics: no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Dims(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("H", "W", "C1", "C2", "F", "NC")]


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.oracle_param_count.restype = ctypes.c_int64
        lib.oracle_param_count.argtypes = [ctypes.POINTER(_Dims)]
        lib.oracle_philox4x32_10.restype = None
        lib.oracle_dropout_keep.restype = None
        lib.oracle_dropout_keep.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int32, ctypes.c_int32,
                                            ctypes.c_uint32, ctypes.c_void_p]
        lib.oracle_worker_grad.restype = None
        lib.oracle_worker_grad.argtypes = [ctypes.POINTER(_Dims)] + [ctypes.c_void_p] * 3 + [ctypes.c_int32] + \
            [ctypes.c_void_p, ctypes.c_double] + [ctypes.c_void_p] * 10 + [ctypes.c_void_p, ctypes.c_int32]
        lib.oracle_worker_grads.restype = ctypes.c_int32
        lib.oracle_worker_grads.argtypes = [ctypes.POINTER(_Dims), ctypes.c_int32] + [ctypes.c_void_p] * 4 + \
            [ctypes.c_int32, ctypes.c_void_p, ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32]
        _lib = lib
    return _lib


@dataclass(frozen=True)
class Dims:
    """Layer sizes; defaults are the paper's CNN (model endnote)."""
    H: int = 28
    W: int = 28
    C1: int = 16
    C2: int = 32
    F: int = 512
    NC: int = 10

    def _c(self) -> _Dims:
        return _Dims(self.H, self.W, self.C1, self.C2, self.F, self.NC)

    @property
    def P(self) -> int:
        return int(_load().oracle_param_count(ctypes.byref(self._c())))

    @property
    def n1(self) -> int:
        return self.C1 * (self.H // 2) * (self.W // 2)

    @property
    def n2(self) -> int:
        return self.C2 * (self.H // 4) * (self.W // 4)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def philox4x32_10(ctr: Sequence[int], key: Sequence[int]) -> List[int]:
    c = (ctypes.c_uint32 * 4)(*ctr)
    k = (ctypes.c_uint32 * 2)(*key)
    o = (ctypes.c_uint32 * 4)()
    _load().oracle_philox4x32_10(c, k, o)
    return [int(v) for v in o]


def dropout_threshold(p: float) -> int:
    """A unit is dropped iff its 32-bit word is below floor(p * 2^32)."""
    return int(np.floor(float(p) * 4294967296.0))


def dropout_keep(seed: int, minibatch_id: int, B: int, F: int, p: float) -> np.ndarray:
    """Keep mask uint8 [B, F] (1 = kept) for one minibatch."""
    keep = np.empty((B, F), dtype=np.uint8)
    _load().oracle_dropout_keep(ctypes.c_uint64(seed), ctypes.c_uint64(minibatch_id), B, F,
                                ctypes.c_uint32(dropout_threshold(p)), _ptr(keep))
    return keep


@dataclass
class Records:
    """Per-sample decisions of one worker's forward pass."""
    code1: np.ndarray
    top1: np.ndarray
    margin1: np.ndarray
    code2: np.ndarray
    top2: np.ndarray
    margin2: np.ndarray
    hpre: np.ndarray
    z: np.ndarray


def worker_grad(dims: Dims, theta: np.ndarray, x: np.ndarray, y: np.ndarray, keep: np.ndarray, p: float,
                records: bool = False, forced: Optional[np.ndarray] = None):
    """Gradient (fp64 [P]) of one worker's mean minibatch loss at `theta`; returns (grad, loss[, Records]).
    `forced` (int32 [k, 4] rows {sample, layer, index, value}) makes tied max / ReLU decisions take a
    stated outcome; see ps_oracle.c."""
    B = int(x.shape[0])
    theta = np.ascontiguousarray(theta, dtype=np.float64)
    x = np.ascontiguousarray(x, dtype=np.float64).reshape(B, dims.H * dims.W)
    y = np.ascontiguousarray(y, dtype=np.int32)
    keep = np.ascontiguousarray(keep, dtype=np.uint8).reshape(B, dims.F)
    assert theta.shape == (dims.P,) and y.shape == (B,)
    assert int(y.min()) >= 0 and int(y.max()) < dims.NC
    grad = np.empty(dims.P, dtype=np.float64)
    loss = ctypes.c_double(0.0)
    rec = None
    if records:
        rec = Records(np.empty((B, dims.n1), np.uint8), np.empty((B, dims.n1)), np.empty((B, dims.n1)),
                      np.empty((B, dims.n2), np.uint8), np.empty((B, dims.n2)), np.empty((B, dims.n2)),
                      np.empty((B, dims.F)), np.empty((B, dims.NC)))
    r = rec
    if forced is not None:
        forced = np.ascontiguousarray(forced, dtype=np.int32).reshape(-1, 4)
    _load().oracle_worker_grad(ctypes.byref(dims._c()), _ptr(theta), _ptr(x), _ptr(y), B, _ptr(keep),
                               ctypes.c_double(1.0 / (1.0 - p)), _ptr(grad), ctypes.byref(loss),
                               _ptr(r.code1) if r else None, _ptr(r.top1) if r else None,
                               _ptr(r.margin1) if r else None, _ptr(r.code2) if r else None,
                               _ptr(r.top2) if r else None, _ptr(r.margin2) if r else None,
                               _ptr(r.hpre) if r else None, _ptr(r.z) if r else None,
                               _ptr(forced), 0 if forced is None else len(forced))
    return (grad, loss.value, rec) if records else (grad, loss.value)


def worker_grads(dims: Dims, thetas: np.ndarray, theta_of: Sequence[int], x: np.ndarray, y: np.ndarray,
                 keep: np.ndarray, p: float, n_threads: int = 0):
    """n independent workers (x [n,B,H*W], y [n,B], keep [n,B,F]); worker i reads thetas[theta_of[i]].
    Returns (grads fp64 [n,P], losses [n], host threads used)."""
    n, B = int(x.shape[0]), int(x.shape[1])
    thetas = np.ascontiguousarray(thetas, dtype=np.float64).reshape(-1, dims.P)
    theta_of = np.ascontiguousarray(theta_of, dtype=np.int32)
    assert theta_of.shape == (n,) and int(theta_of.max()) < thetas.shape[0] and int(theta_of.min()) >= 0
    x = np.ascontiguousarray(x, dtype=np.float64).reshape(n, B, dims.H * dims.W)
    y = np.ascontiguousarray(y, dtype=np.int32).reshape(n, B)
    assert int(y.min()) >= 0 and int(y.max()) < dims.NC
    keep = np.ascontiguousarray(keep, dtype=np.uint8).reshape(n, B, dims.F)
    grads = np.empty((n, dims.P), dtype=np.float64)
    losses = np.empty(n, dtype=np.float64)
    if n_threads <= 0:
        n_threads = min(16, len(os.sched_getaffinity(0)))
    used = _load().oracle_worker_grads(ctypes.byref(dims._c()), n, _ptr(thetas), _ptr(theta_of), _ptr(x),
                                       _ptr(y), B, _ptr(keep), ctypes.c_double(1.0 / (1.0 - p)), _ptr(grads),
                                       _ptr(losses), n_threads)
    return grads, losses, int(used)


def evaluate(dims: Dims, theta: np.ndarray, x: np.ndarray, y: np.ndarray):
    """Inference forward pass without dropout (Section 3.1: accuracy and loss are evaluated
    periodically).  Returns (mean loss, accuracy, predicted classes, logits); the predicted class is
    the lowest index among the largest logits."""
    n = int(x.shape[0])
    _, loss, rec = worker_grad(dims, theta, x, y, np.ones((n, dims.F), np.uint8), 0.0, records=True)
    pred = rec.z.argmax(axis=1).astype(np.int32)
    return loss, float(np.mean(pred == np.asarray(y))), pred, rec.z


# --------------------------------------------------------------------------- update rules

def apply_sync(theta: np.ndarray, grads: Sequence[np.ndarray], lr: float) -> np.ndarray:
    """One update with all gathered gradients: theta - lr * (g_0 + g_1 + ...), summed in arrival order."""
    total = np.array(grads[0], dtype=np.float64, copy=True)
    for g in grads[1:]:
        total += np.asarray(g, dtype=np.float64)
    return theta - lr * total


def apply_async(theta: np.ndarray, grad: np.ndarray, lr: float) -> np.ndarray:
    """One update per arriving gradient."""
    return theta - lr * np.asarray(grad, dtype=np.float64)


DRAIN_SUM = 0
DRAIN_SEQ = 1


def drain(theta: np.ndarray, pending: Sequence[np.ndarray], lr: float, mode: int) -> np.ndarray:
    """Stateless server step over all pending gradients in arrival order: either one update with
    their sum (DRAIN_SUM) or one update per gradient (DRAIN_SEQ)."""
    if len(pending) == 0:
        return theta
    if mode == DRAIN_SUM:
        return apply_sync(theta, pending, lr)
    for g in pending:
        theta = apply_async(theta, g, lr)
    return theta


def clip_scales(pending: Sequence[np.ndarray], clip_norm: float) -> List[float]:
    """Per-gradient factor min(1, clip_norm / ||g||_2); 1 where clipping is off or the gradient is zero."""
    out = []
    for g in pending:
        norm = float(np.sqrt(np.sum(np.asarray(g, dtype=np.float64) ** 2)))
        out.append(clip_norm / norm if (clip_norm > 0 and norm > clip_norm) else 1.0)
    return out


def backlog_lr(lr: float, n_pending: int, lr_backlog_ref: float) -> float:
    """Learning rate turned down for a large backlog: lr * min(1, ref / K); ref = 0 leaves lr alone."""
    if lr_backlog_ref > 0 and n_pending > lr_backlog_ref:
        return lr * (lr_backlog_ref / n_pending)
    return lr


def drain_mitigated(theta: np.ndarray, pending: Sequence[np.ndarray], lr: float, mode: int, lr_backlog_ref: float,
                    clip_norm: float):
    """Recovery drain with the stale-gradient mitigations of Section 2.3's last paragraph (the paper names
    them without formulas; these are this build's readings): each pending gradient is clipped to
    2-norm clip_norm and the learning rate is scaled by min(1, lr_backlog_ref / K).
    Returns (new theta, learning rate used)."""
    used = backlog_lr(lr, len(pending), lr_backlog_ref)
    scaled = [np.asarray(g, dtype=np.float64) * s for g, s in zip(pending, clip_scales(pending, clip_norm))]
    return drain(theta, scaled, used, mode), used


def drain_adadelta(theta: np.ndarray, pending: Sequence[np.ndarray], lr: float, rho: float, eps: float,
                   acc_g2: np.ndarray, acc_dx2: np.ndarray):
    """Recovery drain with an adaptive learning rate, which Section 2.3's last paragraph names as a
    candidate for applying the stale gradients (Adadelta; the paper gives no details, so this is the
    method as published: Zeiler 2012, Algorithm 1).  The pending gradients are applied one by one in
    arrival order; per parameter
        E[g^2]  <- rho E[g^2] + (1 - rho) g^2
        dx      <- - sqrt(E[dx^2] + eps) / sqrt(E[g^2] + eps) * g
        E[dx^2] <- rho E[dx^2] + (1 - rho) dx^2
        theta   <- theta + lr * dx
    Returns (theta, E[g^2], E[dx^2]) after the last gradient."""
    theta = np.array(theta, dtype=np.float64, copy=True)
    g2 = np.array(acc_g2, dtype=np.float64, copy=True)
    dx2 = np.array(acc_dx2, dtype=np.float64, copy=True)
    for g in pending:
        g = np.asarray(g, dtype=np.float64)
        g2 = rho * g2 + (1.0 - rho) * g * g
        dx = -np.sqrt(dx2 + eps) / np.sqrt(g2 + eps) * g
        dx2 = rho * dx2 + (1.0 - rho) * dx * dx
        theta = theta + lr * dx
    return theta, g2, dx2


def elastic_average(centre: np.ndarray, locals_: Sequence[np.ndarray], alpha: float):
    """One synchronous elastic-averaging step (Zhang, Choromanska, LeCun 2015, "Deep learning with
    elastic averaging SGD", the update of its Section 2 with alpha = eta * rho), which Section 2.3's
    last paragraph names among the methods to try for the work done while the server was away:
    worker-local weights x_i and the centre are pulled towards each other,
        x_i     <- x_i - alpha (x_i - centre)
        centre  <- centre + alpha sum_i (x_i - centre)
    with every difference taken before the update.  Returns (new centre, list of new x_i)."""
    c = np.asarray(centre, dtype=np.float64)
    xs = [np.asarray(x, dtype=np.float64) for x in locals_]
    total = np.zeros_like(c)
    out = []
    for x in xs:
        d = x - c
        out.append(x - alpha * d)
        total = total + d
    return c + alpha * total, out


# --------------------------------------------------------------------------- server model

@dataclass
class QueueEntry:
    seq: int
    worker: int
    version: int
    mb_id: int
    grad: np.ndarray
    loss: float


@dataclass
class OracleServer:
    """The weights cell, the ring of worker snapshots and the pending-gradient list, in fp64."""
    dims: Dims
    seed: int
    dropout_p: float
    n_slots: int
    theta: np.ndarray
    ring: List[np.ndarray] = field(default_factory=list)
    ring_version: List[int] = field(default_factory=list)
    pending: List[QueueEntry] = field(default_factory=list)
    version: int = 0           # number of weight updates so far
    next_seq: int = 0
    n_threads: int = 0
    threads_used: int = 1

    def __post_init__(self):
        self.theta = np.array(self.theta, dtype=np.float64, copy=True)
        self.ring = [self.theta.copy() for _ in range(self.n_slots)]
        self.ring_version = [0] * self.n_slots

    def snapshot_weights(self, slot: int) -> int:
        self.ring[slot] = self.theta.copy()
        self.ring_version[slot] = self.version
        return self.version

    def worker_grads_batched(self, workers: Sequence[int], slots: Sequence[int], mb_ids: Sequence[int],
                             x: np.ndarray, y: np.ndarray) -> List[QueueEntry]:
        """Each listed worker computes one gradient on its slot's snapshot; gradients are appended
        to the pending list in array order (= arrival order)."""
        n, B = x.shape[0], x.shape[1]
        keep = np.stack([dropout_keep(self.seed, m, B, self.dims.F, self.dropout_p) for m in mb_ids])
        thetas = np.stack(self.ring)
        grads, losses, used = worker_grads(self.dims, thetas, list(slots), x, y, keep, self.dropout_p,
                                           self.n_threads)
        self.threads_used = used
        out = []
        for i in range(n):
            e = QueueEntry(self.next_seq, int(workers[i]), self.ring_version[slots[i]], int(mb_ids[i]),
                           grads[i], float(losses[i]))
            self.next_seq += 1
            self.pending.append(e)
            out.append(e)
        return out

    def _take(self, seqs: Sequence[int]) -> List[QueueEntry]:
        by_seq = {e.seq: e for e in self.pending}
        taken = [by_seq[s] for s in seqs]
        drop = set(seqs)
        self.pending = [e for e in self.pending if e.seq not in drop]
        return taken

    def apply_sync(self, seqs: Sequence[int], lr: float) -> None:
        taken = self._take(seqs)
        self.theta = apply_sync(self.theta, [e.grad for e in taken], lr)
        self.version += 1

    def apply_async(self, seq: int, lr: float) -> None:
        (e,) = self._take([seq])
        self.theta = apply_async(self.theta, e.grad, lr)
        self.version += 1

    def consume(self, mode: int, lr: float, k: int) -> int:
        """Server step of the lock-free gradient store (Section 3.3, last paragraph: a gradient is
        written once, read once by the server and then deleted): the first k pending gradients, in
        arrival order, are applied as one summed update or as k successive updates, and removed."""
        k = min(k, len(self.pending))
        if k == 0:
            return 0
        seqs = [e.seq for e in self.pending[:k]]
        if mode == DRAIN_SUM:
            self.apply_sync(seqs, lr)
        else:
            for s in seqs:
                self.apply_async(s, lr)
        return k

    def apply_local(self, slot: int, seq: int, lr: float) -> None:
        """A worker that trains on its own copy of the weights (elastic averaging SGD): plain SGD
        step on ring slot `slot` with one pending gradient; the server's weights do not change."""
        (e,) = self._take([seq])
        self.ring[slot] = apply_async(self.ring[slot], e.grad, lr)

    def elastic_average(self, slots: Sequence[int], alpha: float) -> None:
        self.theta, new = elastic_average(self.theta, [self.ring[s] for s in slots], alpha)
        for s, x in zip(slots, new):
            self.ring[s] = x
        self.version += 1

    def drain_adadelta(self, lr: float, rho: float, eps: float) -> int:
        """Recovery with Adadelta steps over the pending gradients (see drain_adadelta); the two
        accumulators are server state, zero until first used."""
        if not hasattr(self, "acc_g2"):
            self.acc_g2 = np.zeros_like(self.theta)
            self.acc_dx2 = np.zeros_like(self.theta)
        k = len(self.pending)
        self.theta, self.acc_g2, self.acc_dx2 = drain_adadelta(self.theta, [e.grad for e in self.pending], lr, rho, eps,
                                                               self.acc_g2, self.acc_dx2)
        self.version += k
        self.pending = []
        return k

    def restore_weights(self, slot: int) -> int:
        """Checkpoint / replica takeover: continue from the older state in `slot`; gradients still
        pending are lost."""
        dropped = len(self.pending)
        self.theta = self.ring[slot].copy()
        self.version = self.ring_version[slot]
        self.pending = []
        return dropped

    def drain_buffered(self, mode: int, lr: float, lr_backlog_ref: float = 0.0, clip_norm: float = 0.0) -> int:
        k = len(self.pending)
        self.theta, _ = drain_mitigated(self.theta, [e.grad for e in self.pending], lr, mode, lr_backlog_ref, clip_norm)
        self.version += 0 if k == 0 else (1 if mode == DRAIN_SUM else k)
        self.pending = []
        return k
