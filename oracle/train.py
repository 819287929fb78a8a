"""Training drivers of the oracle.

train_model / train_all: the plain definition.  Each of the K models is
trained on its own, unsharded, one after another: per step one forward pass,
one backward pass, one update; the loss reported for a step is the loss before
that step's update.  All models consume the same batch sequence (they are
configurations of one task; paper, Introduction, "Model Selection
Integration").

train_sharded_interleaved: a second driver that cuts every model at given
layer boundaries, runs forward (F), backward (B) and update (U) tasks of
(model, shard) pairs in a caller-given or round-robin interleaved order, and
hands boundary features / gradients between the shards of a model.  It calls
the same unit functions; the paper's third desideratum (sharding must not
change the training output) says its result must be bit-identical to
train_all, which the tests check.  It also refuses an order that violates a
dependency, which pins the dependency rules.  Test infrastructure only.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import model as M
from . import optim as O

PH_F, PH_B, PH_U = 0, 1, 2


def batch_at(data: Dict, t: int) -> Dict:
    """Batch of step t (1-based): index (t-1) mod n_batches."""
    i = (t - 1) % data["inputs"].shape[0]
    return {k: (v[i] if v is not None else None) for k, v in data.items()}


def train_model(arch, hp, data, steps: int, seed: int, model: int, params=None):
    """Returns (losses fp64 [steps], params list of fp32 arrays, optimizer state)."""
    params = M.init_params(arch, seed, model) if params is None else [p.copy() for p in params]
    st = O.new_state(params)
    losses = np.zeros(steps, dtype=np.float64)
    for t in range(1, steps + 1):
        loss, grads = M.loss_and_grads(arch, params, batch_at(data, t))
        losses[t - 1] = loss
        for j, g in enumerate(grads):
            O.update_tensor(hp, t, params[j], g, st["m"][j], st["v"][j])
    return losses, params, st


def train_all(archs, hps, data, steps: int, seed: int, models: Optional[Sequence[int]] = None):
    """Trains models (default all) one after another.  Returns {model: (losses, params)}."""
    out = {}
    for k in (range(len(archs)) if models is None else models):
        losses, params, _ = train_model(archs[k], hps[k], data, steps, seed, k)
        out[k] = (losses, params)
    return out


def shard_ranges(arch, cuts: Sequence[int]) -> List[Tuple[int, int]]:
    b = [0] + list(cuts) + [M.n_units(arch)]
    assert all(b[i] < b[i + 1] for i in range(len(b) - 1)), "cut points must be strictly increasing and interior"
    return [(b[i], b[i + 1]) for i in range(len(b) - 1)]


def round_robin_order(n_shards: Sequence[int]) -> List[Tuple[int, int, int]]:
    """One step's tasks, interleaved over models: at every turn each model that
    still has work runs its next task (F shards ascending, then B and U shards descending)."""
    per_model = []
    for k, S in enumerate(n_shards):
        seq = [(k, s, PH_F) for s in range(S)]
        for s in reversed(range(S)):
            seq += [(k, s, PH_B), (k, s, PH_U)]
        per_model.append(seq)
    order, i = [], 0
    while any(i < len(q) for q in per_model):
        order += [q[i] for q in per_model if i < len(q)]
        i += 1
    return order


def train_sharded_interleaved(archs, hps, data, steps: int, seed: int, cuts: Sequence[Sequence[int]],
                              order: Optional[List[Tuple[int, int, int]]] = None):
    """order: (model, shard, phase) triples for ONE step, replayed every step."""
    K = len(archs)
    ranges = [shard_ranges(archs[k], cuts[k]) for k in range(K)]
    order = round_robin_order([len(r) for r in ranges]) if order is None else order
    params = [M.init_params(archs[k], seed, k) for k in range(K)]
    state = [O.new_state(params[k]) for k in range(K)]
    losses = np.zeros((K, steps), dtype=np.float64)
    for t in range(1, steps + 1):
        batch = batch_at(data, t)
        done = set()
        act = {}      # (k, s) -> output of shard s forward
        gin = {}      # (k, s) -> gradient w.r.t. shard s input
        caches, grads = {}, {}
        for (k, s, ph) in order:
            S = len(ranges[k])
            u0, u1 = ranges[k][s]
            if ph == PH_F:
                if s > 0 and (k, s - 1, PH_F) not in done:
                    raise ValueError(f"F({k},{s}) before F({k},{s - 1})")
                x = act.get((k, s - 1))
                for u in range(u0, u1):
                    x, caches[(k, u)] = M.unit_fwd(archs[k], params[k], u, x, batch)
                act[(k, s)] = x
                if s == S - 1:
                    losses[k, t - 1] = x
            elif ph == PH_B:
                need = (k, s, PH_F) if s == S - 1 else (k, s + 1, PH_B)
                if need not in done or (k, s, PH_F) not in done:
                    raise ValueError(f"B({k},{s}) before {need}")
                dx = gin.get((k, s + 1))
                for u in reversed(range(u0, u1)):
                    dx, g = M.unit_bwd(archs[k], params[k], u, caches.pop((k, u)), dx)
                    grads.update({(k, j): gj for j, gj in g.items()})
                gin[(k, s)] = dx
            else:
                if (k, s, PH_B) not in done:
                    raise ValueError(f"U({k},{s}) before B({k},{s})")
                for u in range(u0, u1):
                    for j in M.unit_tensors(archs[k], u):
                        O.update_tensor(hps[k], t, params[k][j], grads.pop((k, j)).reshape(params[k][j].shape),
                                        state[k]["m"][j], state[k]["v"][j])
            if (k, s, ph) in done:
                raise ValueError(f"task {(k, s, ph)} listed twice")
            done.add((k, s, ph))
        want = {(k, s, ph) for k in range(K) for s in range(len(ranges[k])) for ph in (PH_F, PH_B, PH_U)}
        if done != want:
            raise ValueError("order does not cover every (model, shard, phase) exactly once")
    return {k: (losses[k], params[k]) for k in range(K)}
