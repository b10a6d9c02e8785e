"""Replays a synth.Scenario through the C ABI (host-side sequencing only)."""
from __future__ import annotations

from typing import Dict, Iterator, List, Tuple

import numpy as np

from . import binding as ps
from . import synth


class Replay:
    """Keeps the map arrival number -> queue entry; all arithmetic happens inside the library."""

    def __init__(self, sc: synth.Scenario, data_seed: int, dropout_seed: int, theta0: np.ndarray,
                 dropout_p: float = 0.25, device: str = "cuda:0"):
        import torch
        self.torch = torch
        self.sc = sc
        self.data_seed = data_seed
        self.device = device
        self.ctx = ps.ps_init(ps.make_config(sc.max_call, sc.batch, sc.n_slots, sc.queue_capacity, dropout_seed,
                                             dropout_p), device)
        ps.ps_set_weights(self.ctx, theta0)
        self.entry_of: Dict[int, int] = {}
        self.next_seq = 0
        self.meta_log: List[tuple] = []      # (seq, worker, version, mb_id) in arrival order
        self.losses: Dict[int, float] = {}
        self.evals: List[tuple] = []         # (eval_id, loss, accuracy, predictions)
        self.dropped: List[int] = []         # pending gradients lost at each restore
        self.last_inputs = None              # (x, y host arrays, x, y device tensors) of the latest worker step

    def close(self):
        ps.ps_destroy(self.ctx)

    def steps(self) -> Iterator[Tuple[tuple, List[int]]]:
        """Executes the events one by one; yields (event, arrival numbers it appended) after each."""
        torch = self.torch
        for ev in self.sc.events:
            kind, seqs = ev[0], []
            if kind == "grads":
                _, workers, slots, mbs = ev
                x, y = synth.minibatches(self.data_seed, mbs, self.sc.batch)
                xd = torch.from_numpy(x).to(self.device)
                yd = torch.from_numpy(y).to(self.device)
                loss = torch.empty(len(workers), dtype=torch.float32, device=self.device)
                self.last_inputs = (x, y, xd, yd)
                entries = ps.worker_grads_batched(self.ctx, workers, slots, mbs, xd, yd, loss)
                seqs = list(range(self.next_seq, self.next_seq + len(workers)))
                self.next_seq += len(workers)
                by_entry = {m[4]: m for m in ps.ps_queue_meta(self.ctx)}
                for s, q in zip(seqs, entries):
                    self.entry_of[s] = q
                    m = by_entry[q]
                    self.meta_log.append((m[0], m[1], m[2], m[3]))
                ps.ps_sync(self.ctx)                      # x, y, loss are borrowed until the work is done
                for s, l in zip(seqs, loss.cpu().numpy()):
                    self.losses[s] = float(l)
            elif kind == "sync":
                ps.ps_apply_sync(self.ctx, [self.entry_of.pop(s) for s in ev[1]], ev[2])
            elif kind == "async":
                ps.ps_apply_async(self.ctx, self.entry_of.pop(ev[1]), ev[2])
            elif kind == "drain":
                if len(ev) > 3 and (ev[3] or ev[4]):
                    k, _ = ps.ps_drain_buffered_mitigated(self.ctx, ev[1], ev[2], ev[3], ev[4])
                else:
                    k = ps.ps_drain_buffered(self.ctx, ev[1], ev[2])
                assert k == len(self.entry_of)
                self.entry_of.clear()
            elif kind == "snapshot":
                ps.ps_snapshot_weights(self.ctx, ev[1])
            elif kind == "restore":
                self.dropped.append(ps.ps_restore_weights(self.ctx, ev[1]))
                self.entry_of.clear()
            elif kind == "eval":
                x, y = synth.eval_batch(self.data_seed, ev[2], ev[1])
                xd, yd = torch.from_numpy(x).to(self.device), torch.from_numpy(y).to(self.device)
                self.evals.append((ev[2],) + ps.ps_evaluate(self.ctx, -1, xd, yd))
            else:
                raise ValueError(kind)
            yield ev, seqs

    def run(self) -> np.ndarray:
        for _ in self.steps():
            pass
        return self.weights()

    def weights(self) -> np.ndarray:
        return ps.ps_get_weights(self.ctx)

    def grad(self, seq: int) -> np.ndarray:
        return ps.ps_get_grad(self.ctx, self.entry_of[seq])
