"""Model selection on top of the trainer (paper, Introduction, "Model Selection Integration": many configurations
of one task are trained together and compared): successive halving.  After every rung (a number of epochs) the
worse half of the models still running, by the mean loss of their latest epoch, is marked inactive with
hydra_set_active and drops out of the schedule; the shard queues of the remaining models are rebuilt by the next
hydra_train_epoch.  Bookkeeping only: every training step runs in libhydra.so.
"""
from __future__ import annotations

from typing import Dict, List

import numpy as np

from . import hydra as H


def successive_halving(ctx: "H.Context", n_models: int, epochs_per_rung: int = 1, keep_fraction: float = 0.5,
                       min_models: int = 1, policy: int = H.SCHED_SHARD_PARALLEL, max_rungs: int = 32) -> Dict:
    """ctx: a context with models defined, sharded and data set.  Returns the surviving models, the order in which
    models were stopped (with the rung and the score that stopped them) and per-rung statistics."""
    alive = list(range(n_models))
    stopped: List[Dict] = []
    rungs: List[Dict] = []
    for rung in range(max_rungs):
        stats = [H.hydra_train_epoch(ctx, policy) for _ in range(epochs_per_rung)]
        steps = stats[-1]["steps"]
        score = {k: float(np.mean(H.hydra_read_loss(ctx, k)[-steps:])) for k in alive}
        rungs.append(dict(rung=rung, models=list(alive), scores=score, wall_ms=sum(s["wall_ms"] for s in stats),
                          launches=sum(s["launches"] for s in stats)))
        if len(alive) <= min_models:
            break
        n_keep = max(min_models, int(np.ceil(len(alive) * keep_fraction)))
        ranked = sorted(alive, key=lambda k: (score[k], k))       # lower loss is better; ties by model index
        for k in ranked[n_keep:]:
            H.hydra_set_active(ctx, k, False)
            stopped.append(dict(model=k, rung=rung, score=score[k]))
        alive = sorted(ranked[:n_keep])
    return dict(survivors=alive, stopped=stopped, rungs=rungs)
