"""ctypes binding of libps_hotpath.so: same names as include/ps_hotpath.h, argument marshalling
only.  torch supplies device memory (the workspace, inputs) and the stream; every step of the
path runs in the library's HIP kernels.  There is no fallback: if the library is missing or a
call fails, an exception is raised."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

P = 813258
IMAGE_PIXELS = 784
N_CLASSES = 10
FC1_UNITS = 512
POOL1_SIZE = 3136
POOL2_SIZE = 1568
DRAIN_SUM = 0
DRAIN_SEQ = 1

PS_OK, PS_EINVAL, PS_ENOMEM, PS_ESTATE, PS_EFULL, PS_EDEVICE = range(6)
_STATUS = {0: "PS_OK", 1: "PS_EINVAL", 2: "PS_ENOMEM", 3: "PS_ESTATE", 4: "PS_EFULL", 5: "PS_EDEVICE"}

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libps_hotpath.so")

EXPORTS = ["ps_workspace_bytes", "ps_init", "ps_destroy", "ps_sync", "ps_set_weights", "ps_get_weights",
           "ps_snapshot_weights", "worker_grads_batched", "ps_queue_push_host", "ps_apply_sync", "ps_apply_async",
           "ps_drain_buffered", "ps_drain_buffered_mitigated", "ps_drain_rows_mitigated", "ps_drain_buffered_adadelta", "ps_apply_local", "ps_elastic_average", "ps_restore_weights", "ps_load_snapshot", "ps_evaluate",
           "worker_grads_append", "ps_store_consume", "ps_store_publish", "ps_store_state", "ps_store_steps",
           "ps_store_entry", "ps_get_grad", "ps_queue_meta", "ps_version", "ps_debug_last_batch", "ps_debug_last_activations", "ps_profile_enable",
           "ps_profile_read", "ps_profile_kernel_count", "ps_profile_kernel_name", "ps_measure_ceilings", "ps_last_error"]


class PsError(RuntimeError):
    def __init__(self, call: str, status: int, message: str = ""):
        super().__init__(f"{call}: {_STATUS.get(status, status)} {message}".strip())
        self.status = status


class ps_drain_policy(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("lr_backlog_ref", ctypes.c_float), ("clip_norm", ctypes.c_float)]


class ps_store_counters(ctypes.Structure):
    _fields_ = [("claimed", ctypes.c_uint64), ("published", ctypes.c_uint64), ("consumed", ctypes.c_uint64),
                ("version", ctypes.c_uint64), ("steps", ctypes.c_uint64)]


class ps_store_step(ctypes.Structure):
    _fields_ = [("first", ctypes.c_uint64), ("count", ctypes.c_uint32), ("mode", ctypes.c_uint32),
                ("version_after", ctypes.c_uint64)]


class ps_ceilings(ctypes.Structure):
    _fields_ = [("compute_units", ctypes.c_int32), ("mfma_32x32x2_tflops", ctypes.c_double),
                ("mfma_32x32x2_first_launch_tflops", ctypes.c_double), ("mfma_16x16x4_tflops", ctypes.c_double),
                ("ns_per_mfma_16x16x4", ctypes.c_double), ("ns_per_mfma_with_valu", ctypes.c_double * 4),
                ("shared_simd_ms", ctypes.c_double * 3), ("ns_per_mfma_with_lds_reads", ctypes.c_double * 3), ("hbm_read_GBps", ctypes.c_double), ("hbm_copy_GBps", ctypes.c_double),
                ("hbm_read_bytes", ctypes.c_uint64)]


class ps_config(ctypes.Structure):
    _fields_ = [("max_workers", ctypes.c_int32), ("batch", ctypes.c_int32), ("n_versions", ctypes.c_int32),
                ("queue_capacity", ctypes.c_int32), ("seed", ctypes.c_uint64), ("dropout_p", ctypes.c_float)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads the in-tree HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        # torch first: it brings its own copy of the HIP runtime, and the workspace and the stream come
        # from it, so this library must bind to that same runtime instance (loading the library before
        # torch would pull in a second runtime that does not see torch's device context)
        import torch  # noqa: F401
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32, u64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_uint64, ctypes.c_float
        sig = {
            "ps_workspace_bytes": [ctypes.POINTER(ps_config), ctypes.POINTER(u64)],
            "ps_init": [ctypes.POINTER(vp), ctypes.POINTER(ps_config), vp, u64, vp],
            "ps_destroy": [vp], "ps_sync": [vp],
            "ps_set_weights": [vp, vp], "ps_get_weights": [vp, i32, vp],
            "ps_snapshot_weights": [vp, i32, ctypes.POINTER(u64)],
            "worker_grads_batched": [vp, i32, vp, vp, vp, vp, vp, vp, vp],
            "ps_queue_push_host": [vp, vp, i32, u64, u64, ctypes.POINTER(i32)],
            "ps_apply_sync": [vp, vp, i32, f32], "ps_apply_async": [vp, i32, f32],
            "ps_drain_buffered": [vp, i32, f32, ctypes.POINTER(i32)],
            "ps_drain_buffered_mitigated": [vp, i32, ctypes.POINTER(ps_drain_policy), ctypes.POINTER(i32),
                                            ctypes.POINTER(f32)],
            "ps_drain_rows_mitigated": [vp, vp, i32, i32, ctypes.POINTER(ps_drain_policy), ctypes.POINTER(f32), vp],
            "ps_drain_buffered_adadelta": [vp, f32, f32, f32, ctypes.POINTER(i32)],
            "ps_apply_local": [vp, i32, vp, vp, f32],
            "ps_elastic_average": [vp, vp, i32, f32],
            "ps_restore_weights": [vp, i32, ctypes.POINTER(i32)],
            "ps_load_snapshot": [vp, i32, vp, u64],
            "ps_evaluate": [vp, i32, i32, vp, vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double), vp],
            "worker_grads_append": [vp, i32, vp, vp, vp, vp, vp, vp],
            "ps_store_consume": [vp, i32, f32, i32, i32],
            "ps_store_publish": [vp, i32],
            "ps_store_state": [vp, ctypes.POINTER(ps_store_counters)],
            "ps_store_steps": [vp, i32, ctypes.POINTER(i32), ctypes.POINTER(ps_store_step)],
            "ps_store_entry": [vp, u64, vp, ctypes.POINTER(i32), ctypes.POINTER(u64), ctypes.POINTER(u64)],
            "ps_get_grad": [vp, i32, vp],
            "ps_queue_meta": [vp, i32, ctypes.POINTER(i32), vp, vp, vp, vp, vp],
            "ps_version": [vp, ctypes.POINTER(u64)],
            "ps_debug_last_batch": [vp, i32, vp, vp, vp, vp, vp, vp],
            "ps_debug_last_activations": [vp, i32, vp, vp, vp, vp],
            "ps_profile_enable": [vp, i32],
            "ps_profile_read": [vp, i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)],
            "ps_measure_ceilings": [vp, u64, vp, ctypes.POINTER(ps_ceilings)],
        }
        for name, args in sig.items():
            fn = getattr(lib, name)
            fn.argtypes = args
            fn.restype = ctypes.c_int
        lib.ps_profile_kernel_count.argtypes = []
        lib.ps_profile_kernel_count.restype = ctypes.c_int32
        lib.ps_profile_kernel_name.argtypes = [i32]
        lib.ps_profile_kernel_name.restype = ctypes.c_char_p
        lib.ps_last_error.argtypes = [vp]
        lib.ps_last_error.restype = ctypes.c_char_p
        _lib = lib
    return _lib


@dataclass
class Context:
    """Handle of one ps_ctx plus the torch tensor that owns its device workspace."""
    handle: ctypes.c_void_p
    workspace: object
    cfg: ps_config
    closed: bool = False


def _check(ctx: Optional[Context], call: str, status: int) -> None:
    if status != PS_OK:
        msg = ""
        if ctx is not None and ctx.handle:
            msg = (load_library().ps_last_error(ctx.handle) or b"").decode()
        raise PsError(call, status, msg)


def _np(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def _vp(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def make_config(max_workers: int, batch: int, n_versions: int, queue_capacity: int, seed: int,
                dropout_p: float = 0.25) -> ps_config:
    return ps_config(max_workers, batch, n_versions, queue_capacity, seed, dropout_p)


def ps_workspace_bytes(cfg: ps_config) -> int:
    out = ctypes.c_uint64(0)
    _check(None, "ps_workspace_bytes", load_library().ps_workspace_bytes(ctypes.byref(cfg), ctypes.byref(out)))
    return int(out.value)


def ps_init(cfg: ps_config, device: str = "cuda:0") -> Context:
    """Allocates the workspace with torch on `device` and creates the context on torch's current stream."""
    import torch
    lib = load_library()
    nbytes = ps_workspace_bytes(cfg)
    dev = torch.device(device)
    torch.cuda.set_device(dev)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    handle = ctypes.c_void_p()
    stream = torch.cuda.current_stream(dev).cuda_stream
    st = lib.ps_init(ctypes.byref(handle), ctypes.byref(cfg), ctypes.c_void_p(ws.data_ptr()), nbytes,
                     ctypes.c_void_p(stream))
    _check(None, "ps_init", st)
    return Context(handle, ws, cfg)


def ps_destroy(ctx: Context) -> None:
    if not ctx.closed:
        _check(ctx, "ps_destroy", load_library().ps_destroy(ctx.handle))
        ctx.closed = True
        ctx.workspace = None


def ps_sync(ctx: Context) -> None:
    _check(ctx, "ps_sync", load_library().ps_sync(ctx.handle))


def ps_set_weights(ctx: Context, theta: np.ndarray) -> None:
    theta = _np(theta, np.float32)
    assert theta.shape == (P,)
    _check(ctx, "ps_set_weights", load_library().ps_set_weights(ctx.handle, _vp(theta)))


def ps_get_weights(ctx: Context, slot: int = -1) -> np.ndarray:
    out = np.empty(P, dtype=np.float32)
    _check(ctx, "ps_get_weights", load_library().ps_get_weights(ctx.handle, slot, _vp(out)))
    return out


def ps_snapshot_weights(ctx: Context, slot: int) -> int:
    v = ctypes.c_uint64(0)
    _check(ctx, "ps_snapshot_weights", load_library().ps_snapshot_weights(ctx.handle, slot, ctypes.byref(v)))
    return int(v.value)


def worker_grads_batched(ctx: Context, worker_id: Sequence[int], version_slot: Sequence[int],
                         minibatch_id: Sequence[int], x_dev, y_dev, loss_dev=None) -> List[int]:
    """x_dev: torch float32 cuda tensor [n, B, 784]; y_dev: torch int32 cuda tensor [n, B];
    loss_dev: optional torch float32 cuda tensor [n].  Returns the queue entry of each gradient."""
    n = len(worker_id)
    w = _np(worker_id, np.int32)
    s = _np(version_slot, np.int32)
    m = _np(minibatch_id, np.uint64)
    assert w.shape == s.shape == m.shape == (n,)
    if n:
        import torch
        B = ctx.cfg.batch
        assert x_dev.is_cuda and x_dev.dtype == torch.float32 and x_dev.is_contiguous()
        assert y_dev.is_cuda and y_dev.dtype == torch.int32 and y_dev.is_contiguous()
        assert x_dev.numel() >= n * B * IMAGE_PIXELS and y_dev.numel() >= n * B
        assert loss_dev is None or (loss_dev.is_cuda and loss_dev.dtype == torch.float32 and loss_dev.numel() >= n)
    q = np.full(n, -1, dtype=np.int32)
    st = load_library().worker_grads_batched(
        ctx.handle, n, _vp(w), _vp(s), _vp(m),
        ctypes.c_void_p(x_dev.data_ptr()) if n else None, ctypes.c_void_p(y_dev.data_ptr()) if n else None, _vp(q),
        ctypes.c_void_p(loss_dev.data_ptr()) if loss_dev is not None else None)
    _check(ctx, "worker_grads_batched", st)
    return [int(v) for v in q]


def ps_queue_push_host(ctx: Context, grad: np.ndarray, worker_id: int, version: int, minibatch_id: int) -> int:
    grad = _np(grad, np.float32)
    assert grad.shape == (P,)
    q = ctypes.c_int32(-1)
    st = load_library().ps_queue_push_host(ctx.handle, _vp(grad), worker_id, version, minibatch_id, ctypes.byref(q))
    _check(ctx, "ps_queue_push_host", st)
    return int(q.value)


def ps_apply_sync(ctx: Context, queue_index: Sequence[int], lr: float) -> None:
    q = _np(queue_index, np.int32)
    _check(ctx, "ps_apply_sync", load_library().ps_apply_sync(ctx.handle, _vp(q), len(q), lr))


def ps_apply_async(ctx: Context, queue_index: int, lr: float) -> None:
    _check(ctx, "ps_apply_async", load_library().ps_apply_async(ctx.handle, queue_index, lr))


def ps_drain_buffered(ctx: Context, mode: int, lr: float) -> int:
    k = ctypes.c_int32(0)
    _check(ctx, "ps_drain_buffered", load_library().ps_drain_buffered(ctx.handle, mode, lr, ctypes.byref(k)))
    return int(k.value)


def ps_drain_buffered_mitigated(ctx: Context, mode: int, lr: float, lr_backlog_ref: float = 0.0,
                                clip_norm: float = 0.0) -> Tuple[int, float]:
    """Returns (number of gradients applied, learning rate used)."""
    pol = ps_drain_policy(lr, lr_backlog_ref, clip_norm)
    k, used = ctypes.c_int32(0), ctypes.c_float(0.0)
    st = load_library().ps_drain_buffered_mitigated(ctx.handle, mode, ctypes.byref(pol), ctypes.byref(k), ctypes.byref(used))
    _check(ctx, "ps_drain_buffered_mitigated", st)
    return int(k.value), float(used.value)


ROW_FLOATS = 813312
STATIC_DRAIN_MAX_ROWS = 4096


def ps_drain_rows_mitigated(theta_dev, grads_dev, mode: int, lr: float, lr_backlog_ref: float = 0.0,
                            clip_norm: float = 0.0, n_rows: Optional[int] = None) -> float:
    """theta_dev: torch float32 cuda tensor of ROW_FLOATS elements, updated in place; grads_dev: torch float32
    cuda tensor [n_rows, ROW_FLOATS].  Runs on torch's current stream; returns the learning rate used."""
    import torch
    n = int(grads_dev.shape[0]) if n_rows is None else n_rows
    assert theta_dev.is_cuda and theta_dev.dtype == torch.float32 and theta_dev.is_contiguous() and theta_dev.numel() == ROW_FLOATS
    assert grads_dev.is_cuda and grads_dev.dtype == torch.float32 and grads_dev.is_contiguous()
    assert n > STATIC_DRAIN_MAX_ROWS or grads_dev.numel() >= n * ROW_FLOATS       # too many rows: the library refuses
    pol = ps_drain_policy(lr, lr_backlog_ref, clip_norm)
    used = ctypes.c_float(0.0)
    stream = torch.cuda.current_stream(theta_dev.device).cuda_stream
    st = load_library().ps_drain_rows_mitigated(ctypes.c_void_p(theta_dev.data_ptr()), ctypes.c_void_p(grads_dev.data_ptr()), n, mode,
                                                ctypes.byref(pol), ctypes.byref(used), ctypes.c_void_p(stream))
    if st != PS_OK:
        raise PsError("ps_drain_rows_mitigated", st, (load_library().ps_last_error(None) or b"").decode())
    return float(used.value)


def ps_drain_buffered_adadelta(ctx: Context, lr: float, rho: float, eps: float) -> int:
    k = ctypes.c_int32(0)
    _check(ctx, "ps_drain_buffered_adadelta", load_library().ps_drain_buffered_adadelta(ctx.handle, lr, rho, eps, ctypes.byref(k)))
    return int(k.value)


def ps_apply_local(ctx: Context, slot: Sequence[int], queue_index: Sequence[int], lr: float) -> None:
    s, q = _np(slot, np.int32), _np(queue_index, np.int32)
    assert s.shape == q.shape
    _check(ctx, "ps_apply_local", load_library().ps_apply_local(ctx.handle, len(s), _vp(s), _vp(q), lr))


def ps_elastic_average(ctx: Context, slot: Sequence[int], alpha: float) -> None:
    s = _np(slot, np.int32)
    _check(ctx, "ps_elastic_average", load_library().ps_elastic_average(ctx.handle, _vp(s), len(s), alpha))


def ps_restore_weights(ctx: Context, slot: int) -> int:
    """theta := ring[slot]; returns the number of pending gradients that were dropped."""
    n = ctypes.c_int32(0)
    _check(ctx, "ps_restore_weights", load_library().ps_restore_weights(ctx.handle, slot, ctypes.byref(n)))
    return int(n.value)


def ps_load_snapshot(ctx: Context, slot: int, theta: np.ndarray, version: int) -> None:
    theta = _np(theta, np.float32)
    assert theta.shape == (P,)
    _check(ctx, "ps_load_snapshot", load_library().ps_load_snapshot(ctx.handle, slot, _vp(theta), version))


def ps_evaluate(ctx: Context, slot: int, x_dev, y_dev) -> Tuple[float, float, np.ndarray]:
    """x_dev: torch float32 cuda [n_images, 784]; y_dev: torch int32 cuda [n_images].
    Returns (mean loss, accuracy, predicted classes)."""
    n = int(y_dev.numel())
    assert x_dev.is_cuda and x_dev.is_contiguous() and x_dev.numel() == n * IMAGE_PIXELS
    assert y_dev.is_cuda and y_dev.is_contiguous()
    loss, acc = ctypes.c_double(0.0), ctypes.c_double(0.0)
    pred = np.empty(n, dtype=np.int32)
    st = load_library().ps_evaluate(ctx.handle, slot, n, ctypes.c_void_p(x_dev.data_ptr()), ctypes.c_void_p(y_dev.data_ptr()),
                                    ctypes.byref(loss), ctypes.byref(acc), _vp(pred))
    _check(ctx, "ps_evaluate", st)
    return float(loss.value), float(acc.value), pred


def worker_grads_append(ctx: Context, worker_id: Sequence[int], version_slot: Sequence[int],
                        minibatch_id: Sequence[int], x_dev, y_dev, loss_dev=None) -> None:
    """As worker_grads_batched, into the lock-free store: positions are claimed on the device."""
    n = len(worker_id)
    w = _np(worker_id, np.int32)
    s = _np(version_slot, np.int32)
    m = _np(minibatch_id, np.uint64)
    assert w.shape == s.shape == m.shape == (n,)
    if n:
        import torch
        B = ctx.cfg.batch
        assert x_dev.is_cuda and x_dev.dtype == torch.float32 and x_dev.is_contiguous()
        assert y_dev.is_cuda and y_dev.dtype == torch.int32 and y_dev.is_contiguous()
        assert x_dev.numel() >= n * B * IMAGE_PIXELS and y_dev.numel() >= n * B
        assert loss_dev is None or (loss_dev.is_cuda and loss_dev.dtype == torch.float32 and loss_dev.numel() >= n)
    st = load_library().worker_grads_append(
        ctx.handle, n, _vp(w), _vp(s), _vp(m),
        ctypes.c_void_p(x_dev.data_ptr()) if n else None, ctypes.c_void_p(y_dev.data_ptr()) if n else None,
        ctypes.c_void_p(loss_dev.data_ptr()) if loss_dev is not None else None)
    _check(ctx, "worker_grads_append", st)


def ps_store_consume(ctx: Context, mode: int, lr: float, max_entries: int = 0, wait_for_workers: bool = True) -> None:
    st = load_library().ps_store_consume(ctx.handle, mode, lr, max_entries, 1 if wait_for_workers else 0)
    _check(ctx, "ps_store_consume", st)


def ps_store_publish(ctx: Context, slot: int) -> None:
    _check(ctx, "ps_store_publish", load_library().ps_store_publish(ctx.handle, slot))


def ps_store_state(ctx: Context) -> dict:
    c = ps_store_counters()
    _check(ctx, "ps_store_state", load_library().ps_store_state(ctx.handle, ctypes.byref(c)))
    return {k: int(getattr(c, k)) for k, _ in ps_store_counters._fields_}


def ps_store_steps(ctx: Context, capacity: int = 1024) -> List[Tuple[int, int, int, int]]:
    """Server steps that applied something, oldest first, as (first position, count, mode, version after)."""
    n = ctypes.c_int32(0)
    buf = (ps_store_step * max(capacity, 1))()
    _check(ctx, "ps_store_steps", load_library().ps_store_steps(ctx.handle, capacity, ctypes.byref(n), buf))
    return [(int(buf[i].first), int(buf[i].count), int(buf[i].mode), int(buf[i].version_after)) for i in range(n.value)]


def ps_store_entry(ctx: Context, position: int, want_grad: bool = True) -> Tuple[Optional[np.ndarray], int, int, int]:
    """(gradient or None, worker id, version of the snapshot used, minibatch id) of an unconsumed position."""
    g = np.empty(P, dtype=np.float32) if want_grad else None
    w, v, m = ctypes.c_int32(0), ctypes.c_uint64(0), ctypes.c_uint64(0)
    st = load_library().ps_store_entry(ctx.handle, position, _vp(g), ctypes.byref(w), ctypes.byref(v), ctypes.byref(m))
    _check(ctx, "ps_store_entry", st)
    return g, int(w.value), int(v.value), int(m.value)


def ps_get_grad(ctx: Context, queue_index: int) -> np.ndarray:
    out = np.empty(P, dtype=np.float32)
    _check(ctx, "ps_get_grad", load_library().ps_get_grad(ctx.handle, queue_index, _vp(out)))
    return out


def ps_queue_meta(ctx: Context) -> List[Tuple[int, int, int, int, int]]:
    """Pending entries in arrival order as (seq, worker, version, minibatch_id, queue_index)."""
    cap = ctx.cfg.queue_capacity
    n = ctypes.c_int32(0)
    seq, ver, mb = (np.zeros(cap, np.uint64) for _ in range(3))
    wk, qi = (np.zeros(cap, np.int32) for _ in range(2))
    st = load_library().ps_queue_meta(ctx.handle, cap, ctypes.byref(n), _vp(seq), _vp(wk), _vp(ver), _vp(mb), _vp(qi))
    _check(ctx, "ps_queue_meta", st)
    return [(int(seq[i]), int(wk[i]), int(ver[i]), int(mb[i]), int(qi[i])) for i in range(n.value)]


def ps_version(ctx: Context) -> int:
    v = ctypes.c_uint64(0)
    _check(ctx, "ps_version", load_library().ps_version(ctx.handle, ctypes.byref(v)))
    return int(v.value)


def ps_debug_last_batch(ctx: Context, i: int) -> dict:
    B = ctx.cfg.batch
    out = {"pool1": np.empty((B, POOL1_SIZE), np.uint8), "pool2": np.empty((B, POOL2_SIZE), np.uint8),
           "keep": np.empty((B, FC1_UNITS), np.uint8), "hdrop": np.empty((B, FC1_UNITS), np.float32),
           "z": np.empty((B, N_CLASSES), np.float32), "pred": np.empty(B, np.int32)}
    st = load_library().ps_debug_last_batch(ctx.handle, i, _vp(out["pool1"]), _vp(out["pool2"]), _vp(out["keep"]),
                                            _vp(out["hdrop"]), _vp(out["z"]), _vp(out["pred"]))
    _check(ctx, "ps_debug_last_batch", st)
    return out


def ps_debug_last_activations(ctx: Context, i: int) -> dict:
    B = ctx.cfg.batch
    out = {"pool1_val": np.empty((B, POOL1_SIZE), np.float32), "pool2_val": np.empty((B, POOL2_SIZE), np.float32),
           "d3": np.empty((B, FC1_UNITS), np.float32), "dpool2": np.empty((B, POOL2_SIZE), np.float32)}
    st = load_library().ps_debug_last_activations(ctx.handle, i, _vp(out["pool1_val"]), _vp(out["pool2_val"]), _vp(out["d3"]),
                                                  _vp(out["dpool2"]))
    _check(ctx, "ps_debug_last_activations", st)
    return out


def ps_measure_ceilings(device: str = "cuda:0", gib: float = 2.0) -> dict:
    """Chip ceilings measured with short timing kernels on torch's current stream over a torch buffer."""
    import torch
    dev = torch.device(device)
    torch.cuda.set_device(dev)
    buf = torch.empty(int(gib * (1 << 30)), dtype=torch.uint8, device=dev)
    c = ps_ceilings()
    st = load_library().ps_measure_ceilings(ctypes.c_void_p(buf.data_ptr()), buf.numel(),
                                            ctypes.c_void_p(torch.cuda.current_stream(dev).cuda_stream), ctypes.byref(c))
    if st != PS_OK:
        raise PsError("ps_measure_ceilings", st)
    out = {}
    for name, _ in ps_ceilings._fields_:
        v = getattr(c, name)
        out[name] = list(v) if hasattr(v, "__len__") else v
    return out


def ps_profile_enable(ctx: Context, enable: bool) -> None:
    _check(ctx, "ps_profile_enable", load_library().ps_profile_enable(ctx.handle, 1 if enable else 0))


def ps_profile_read(ctx: Context) -> dict:
    """{kernel name: (total milliseconds, launches)} since timing was last enabled."""
    lib = load_library()
    out = {}
    for k in range(lib.ps_profile_kernel_count()):
        ms, n = ctypes.c_double(0.0), ctypes.c_int64(0)
        _check(ctx, "ps_profile_read", lib.ps_profile_read(ctx.handle, k, ctypes.byref(ms), ctypes.byref(n)))
        out[lib.ps_profile_kernel_name(k).decode()] = (float(ms.value), int(n.value))
    return out
