"""How far do two runs of the W=64, B=128, 8-version asynchronous scenario separate when they differ
only in the precision the weights are STORED in?

TEST INFRASTRUCTURE ONLY (CPU, oracle arithmetic only; never imported by the product path).

Two oracle servers replay the same scenario (Section 2.1 / 3.1 asynchronous rule: every arriving
gradient is applied at once; workers read snapshots up to 7 steps old).  Server A keeps the weights in
fp64.  Server B rounds the weights to fp32 after every update and every gradient to fp32 before it is
applied, with all gradient arithmetic still exact fp64: the least any fp32 implementation of the rule
must do.  Printed per step: mean loss, gradient norm, weight norm, the relative distance of the two
weight vectors and the largest per-tensor relative difference between the two servers' gradients.

If the gradients of A and B part by more than the 1e-4 parity bound, no fp32 implementation can be
compared with the fp64 oracle gradient by gradient along that trajectory, whatever its kernels do: the
scenario amplifies rounding (it diverges), and a lower learning rate has to be used for parity.

    python -m oracle.drift_study --steps 12 --lr 0.01
"""
from __future__ import annotations

import argparse
import time

import numpy as np

from oracle import oracle as orc
from paper_2406_05546_amd import synth


def per_tensor_rel(a: np.ndarray, b: np.ndarray) -> dict:
    out = {}
    for name, off, shape, _ in synth.NetDims().segments():
        n = int(np.prod(shape))
        out[name] = float(np.linalg.norm(a[off:off + n] - b[off:off + n]) / max(np.linalg.norm(b[off:off + n]), 1e-300))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=12)
    ap.add_argument("--lr", type=float, default=0.01)
    ap.add_argument("--workers", type=int, default=64)
    ap.add_argument("--batch", type=int, default=128)
    ap.add_argument("--slots", type=int, default=8)
    ap.add_argument("--data-seed", type=int, default=11)
    args = ap.parse_args()
    drop_seed = (0x5EED << 32) | 0x2406
    sc = synth.scenario_versions(args.workers, args.batch, args.slots, args.steps, args.lr)
    theta0 = synth.he_uniform_theta(args.data_seed)
    a = orc.OracleServer(orc.Dims(), drop_seed, 0.25, args.slots, theta0)
    b = orc.OracleServer(orc.Dims(), drop_seed, 0.25, args.slots, theta0)
    print(f"# W={args.workers} B={args.batch} V={args.slots} lr={args.lr}: A = fp64 weights, B = weights and gradients "
          f"rounded to fp32 for storage")
    print("# step  loss  |g|  |theta|  |theta_B-theta_A|/|theta_A|  max over workers of |g_B-g_A|/|g_A| per tensor: "
          "conv1.W conv2.W fc1.W fc2.W  seconds")
    step, t0 = 0, time.time()
    for ev in sc.events:
        if ev[0] == "grads":
            _, workers, slots, mbs = ev
            x, y = synth.minibatches(args.data_seed, mbs, sc.batch)
            ea = a.worker_grads_batched(workers, slots, mbs, x, y)
            eb = b.worker_grads_batched(workers, slots, mbs, x, y)
            worst = {}
            for p, q in zip(ea, eb):
                q.grad[:] = q.grad.astype(np.float32).astype(np.float64)
                for k, v in per_tensor_rel(q.grad, p.grad).items():
                    worst[k] = max(worst.get(k, 0.0), v)
            print(f"{step:3d}  {np.mean([e.loss for e in ea]):8.4f}  {np.mean([np.linalg.norm(e.grad) for e in ea]):9.3e}  "
                  f"{np.linalg.norm(a.theta):8.3f}  {np.linalg.norm(a.theta - b.theta) / np.linalg.norm(a.theta):9.2e}  "
                  f"{worst['conv1.W']:9.2e} {worst['conv2.W']:9.2e} {worst['fc1.W']:9.2e} {worst['fc2.W']:9.2e}  "
                  f"{time.time() - t0:5.0f}", flush=True)
            step += 1
        elif ev[0] == "async":
            a.apply_async(ev[1], ev[2])
            b.apply_async(ev[1], ev[2])
            b.theta = b.theta.astype(np.float32).astype(np.float64)
        elif ev[0] == "snapshot":
            a.snapshot_weights(ev[1])
            b.snapshot_weights(ev[1])


if __name__ == "__main__":
    main()
