"""CPU-only checks of the harness's schedules and of the C-ABI library's host side."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2406_05546_amd import binding as ps
from paper_2406_05546_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "ps_hotpath.h")).read()
    declared = re.findall(r"^PS_API\s+[\w\s\*]+?\b(\w+)\(", header, flags=re.M)
    assert sorted(declared) == sorted(ps.EXPORTS) and len(declared) == 37
    lib = ps.load_library()
    for name in declared:
        assert getattr(lib, name) is not None


def test_workspace_bytes_and_argument_checks_without_a_gpu():
    cfg = ps.make_config(max_workers=2, batch=32, n_versions=1, queue_capacity=2, seed=1)
    small = ps.ps_workspace_bytes(cfg)
    row = 813312 * 4
    assert small >= 4 * row and small % 256 == 0
    big = ps.ps_workspace_bytes(ps.make_config(256, 256, 1, 1024, 1))
    assert 1024 * row < big < 12 * 2 ** 30          # 3.3 GB queue + activations, far below 288 GB
    for bad in (ps.make_config(0, 32, 1, 2, 1), ps.make_config(2, 0, 1, 2, 1), ps.make_config(2, 32, 0, 2, 1),
                ps.make_config(2, 32, 1, 0, 1), ps.make_config(2, 32, 1, 2, 1, dropout_p=1.0)):
        with pytest.raises(ps.PsError) as e:
            ps.ps_workspace_bytes(bad)
        assert e.value.status == ps.PS_EINVAL
    lib = ps.load_library()
    h = ctypes.c_void_p()
    assert lib.ps_init(ctypes.byref(h), ctypes.byref(cfg), None, 0, None) == ps.PS_EINVAL and not h.value
    assert lib.ps_init(ctypes.byref(h), ctypes.byref(cfg), ctypes.c_void_p(4096), 16, None) == ps.PS_ENOMEM
    assert lib.ps_init(ctypes.byref(h), ctypes.byref(cfg), ctypes.c_void_p(4097), small, None) == ps.PS_EINVAL
    assert lib.ps_sync(None) == ps.PS_EINVAL and lib.ps_destroy(None) == ps.PS_EINVAL
    assert lib.ps_last_error(None) == b""
    names = [lib.ps_profile_kernel_name(k).decode() for k in range(lib.ps_profile_kernel_count())]
    assert len(names) == 17 and len(set(names)) == 17 and lib.ps_profile_kernel_name(99) == b""


def test_minibatches_depend_only_on_logical_ids():
    x, y = synth.minibatch(3, synth.minibatch_id(2, 5), 8)
    assert x.dtype == np.float32 and y.dtype == np.int32 and x.shape == (8, 784)
    assert 0 <= x.min() and x.max() < 1 and 0 <= y.min() and y.max() <= 9
    xs, ys = synth.minibatches(3, [synth.minibatch_id(0, 0), synth.minibatch_id(2, 5)], 8)
    assert np.array_equal(xs[1], x) and np.array_equal(ys[1], y) and not np.array_equal(xs[0], x)
    x16, _ = synth.minibatch(3, synth.minibatch_id(2, 5), 16)
    assert np.array_equal(x16[:8], x)
    big_x, big_y = synth.minibatch(9, 1, 4096)
    assert abs(big_x.mean() - 0.5) < 0.002 and np.bincount(big_y, minlength=10).min() > 300


def test_he_uniform_bounds():
    theta = synth.he_uniform_theta(4)
    for name, off, shape, fan in synth.NetDims().segments():
        seg = theta[off:off + int(np.prod(shape))]
        if fan == 0:
            assert (seg == 0).all()
        else:
            b = np.sqrt(6.0 / fan)
            assert np.abs(seg).max() <= b and np.abs(seg).max() > 0.9 * b and abs(seg.mean()) < 0.1 * b


def test_async_schedule_staleness():
    arr = synth.async_cyclic_arrivals(1, 4, 100)
    assert sorted(a.worker for a in arr[:4]) == [0, 1, 2, 3]
    assert [a.worker for a in arr[:4]] == [a.worker for a in arr[4:8]]
    assert len({a.mb_id for a in arr}) == 100
    # replay versions: a gradient's snapshot version lags the server's by at most W-1 = 3
    pulled = {w: 0 for w in range(4)}
    worst = 0
    for t, a in enumerate(arr):
        worst = max(worst, t - pulled[a.worker])
        pulled[a.worker] = t + 1
    assert worst == 3
    sc = synth.scenario_async(1, 4, 64, 100, 0.01)
    assert sc.n_gradients == 100 and sc.max_call == 4 and sc.queue_capacity == 4
    seqs = [e[1] for e in sc.events if e[0] == "async"]
    assert seqs == list(range(100))


def test_outage_scenario_shape():
    sc = synth.paper_configs()["outage_w8_b64"]
    assert sc.n_gradients == 560 and sc.queue_capacity == 400
    drains = [e for e in sc.events if e[0] == "drain"]
    assert len(drains) == 21 and drains[-1][1] == synth.DRAIN_SEQ
    ids = [m for e in sc.events if e[0] == "grads" for m in e[3]]
    assert len(set(ids)) == 560
    big = synth.paper_configs()["outage_w256_b256"]
    assert big.n_gradients == 1024 and big.queue_capacity == 1024 and big.max_call == 256
    v = synth.paper_configs()["versions_w64_b128"]
    assert v.n_slots == 8 and v.n_gradients == 3200
    assert [e[2] for e in v.events if e[0] == "grads"][0][:10] == [0, 1, 2, 3, 4, 5, 6, 7, 0, 1]


def test_checkpoint_scenario_shape():
    sc = synth.scenario_checkpoint(2, 8, 6, 0.01, period=2, kills=[3], eval_images=16, kills_inflight=[4])
    kinds = [e[0] for e in sc.events]
    assert kinds.count("restore") == 2 and kinds.count("eval") == 6 and kinds.count("grads") == 6
    assert kinds.count("sync") == 5                       # the in-flight step is never applied
    assert sc.n_slots == 2 and sc.max_call == 2
    # checkpoints after updates 2 and 4 (and the initial one)
    assert [e for e in sc.events if e == ("snapshot", 1)].__len__() == 3
    x, y = synth.eval_batch(5, 0, 16)
    xw, _ = synth.minibatch(5, synth.minibatch_id(0, 0), 16)
    assert x.shape == (16, 784) and not np.array_equal(x, xw)


def test_loading_the_library_brings_in_torch_first():
    """The library must bind to the HIP runtime that torch ships (torch owns the device memory and the
    stream), whatever the caller imports first."""
    import subprocess
    import sys
    code = ("import sys; from paper_2406_05546_amd import binding; assert 'torch' not in sys.modules; "
            "binding.load_library(); assert 'torch' in sys.modules; print('ok')")
    out = subprocess.run([sys.executable, "-c", code], cwd=ROOT, capture_output=True, text=True, timeout=300)
    assert out.returncode == 0 and out.stdout.strip().endswith("ok"), out.stderr[-2000:]


def test_bench_reads_its_traffic_figures_from_the_tracked_counter_summary():
    """bench.py reports HBM traffic per launch; the figures must be the rocprofv3 counter summary kept under
    profiles/ (FETCH_SIZE and WRITE_SIZE, scaled by the plain-copy reference), read from that file at run time."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    got = bench.measured_hbm_bytes()
    assert set(got) == set(bench.COUNTER_ROWS) - set(bench.STALE_COUNTERS)
    text = open(bench.COUNTER_SUMMARY).read()
    for name, value in got.items():
        mib = value / bench.MIB
        assert mib > 100, name
        # the two numbers that make up the figure stand in the summary as printed
        row = [l for l in text.splitlines() if bench.COUNTER_ROWS[name] in l][0].split()
        f_mib, w_mib, max_f, max_w = float(row[-5]), float(row[-3]), float(row[-2]), float(row[-1])
        assert abs(mib - ((max_f + max_w) if name.startswith("apply_kernel") else (f_mib + w_mib))) < 1e-6
    # the drain reads its algorithmic bytes and nothing more: 1024 rows of P floats plus the weights
    algorithmic = (1024 * 813258 * 4 + 2 * 813258 * 4) / bench.MIB
    assert abs(got["apply_kernel<0>"] / bench.MIB - algorithmic) < 0.01 * algorithmic
    assert bench.measured_hbm_bytes("/nonexistent") == {}
