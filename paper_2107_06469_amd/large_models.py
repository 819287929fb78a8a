"""Decoders of the largest workload's shape (d=4096, 32 heads, gated FFN 11008, S=2048, batch 8) on one GPU.

    python -m paper_2107_06469_amd.large_models K steps layers device_budget_GiB activation_budget_GiB

K such models are trained for `steps` steps under the shard-parallel and the sequential model-parallel schedule,
then model 0 alone with resident state; losses and four probed tensors must agree bit for bit (the paper's exact
replication, Approach, "Desiderata").  device_budget_GiB > 0 smaller than the models' state spills master weights
and Adam moments to pinned host memory; activation_budget_GiB > 0 smaller than the activations makes every
backward task recompute its shard's forward.  Prints per-step times, spill traffic and per-kernel times as JSON.
A machine that can pin less host memory than 12 bytes per parameter of all K models cannot spill them: reduce K or
the depth (the full workload, K=8 x 32 layers, needs 648 GB of pinned memory).

Argument marshalling and reporting only: every step of training runs in libhydra.so.
"""
from __future__ import annotations

import json
import os
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

import numpy as np


def decoder_workload(K: int, steps: int, layers: int, n_shards: int = 4):
    """Workload 4 cut down to K models of `layers` blocks, n_shards equal shards each."""
    from hydra_workloads import workload
    w = workload(4)
    for a in w.archs:
        a["n_layers"] = layers
    cuts = [layers * i // n_shards for i in range(1, n_shards)]
    w.archs, w.hparams, w.boundaries = w.archs[:K], w.hparams[:K], [cuts] * K
    w.steps = w.n_batches = steps
    return w


def run(w, data, n_models: int, policy: int, device_budget: int, activation_budget: int, tag: str = ""):
    """Trains the first n_models models of w; returns (losses per model, four probed tensors of model 0, report)."""
    import torch
    from paper_2107_06469_amd import hydra as H
    t0 = time.time()
    ctx = H.hydra_create(n_streams=4, device_budget_bytes=device_budget, activation_budget_bytes=activation_budget)
    try:
        H.hydra_define_models(ctx, w.archs[:n_models], w.hparams[:n_models], w.init_seed)
        for k in range(n_models):
            H.hydra_shard(ctx, k, w.boundaries[k])
        H.hydra_set_data(ctx, data["inputs"], data["target_pos"], data["targets"])
        setup_s = time.time() - t0
        H.hydra_profile_enable(ctx, True)
        st = H.hydra_train_epoch(ctx, policy)
        prof = H.hydra_profile_read(ctx)
        busy, ovl = H.hydra_profile_busy(ctx), H.hydra_profile_copy_overlap(ctx)
        losses = [H.hydra_read_loss(ctx, k) for k in range(n_models)]
        n_t = len(H.hydra_tensor_shapes(ctx, 0))
        probe = [2, 4, n_t - 6, n_t - 3]  # Wqkv and Wo of block 0, W2 of the last block, the final LayerNorm's bias
        tensors = [H.hydra_read_params(ctx, 0, j) for j in probe]
    finally:
        H.hydra_destroy(ctx)
        torch.cuda.empty_cache()
    sec = st["wall_ms"] / 1e3
    report = {"run": tag, "models": n_models, "setup_s": round(setup_s, 1), "ms_per_step": st["wall_ms"] / w.steps,
              "samples_per_s": n_models * w.batch * w.steps / sec,
              "h2d_GB": st["h2d_bytes"] / 1e9, "d2h_GB": st["d2h_bytes"] / 1e9,
              "host_link_GBps_each_way": st["h2d_bytes"] / 1e9 / sec,
              "peak_dev_GiB": st["peak_dev_bytes"] / 2 ** 30, "peak_host_GiB": st["peak_host_bytes"] / 2 ** 30,
              "launches_per_step": st["launches"] / w.steps, "losses": [l.tolist() for l in losses],
              "gpu_busy_fraction": busy["busy_ms"] / st["wall_ms"],
              "copy_busy_fraction": ovl["copy_ms"] / st["wall_ms"],
              "copy_time_under_kernels": ovl["overlapped_ms"] / ovl["copy_ms"] if ovl["copy_ms"] > 0 else None,
              "kernel_ms_per_step": {k: round(v["total_ms"] / w.steps, 1) for k, v in prof.items()}}
    return losses, tensors, report


def compare(K: int, steps: int, layers: int, device_budget: int, activation_budget: int, n_shards: int = 4, out=print):
    """The three runs and the bitwise comparisons; returns True when everything agrees."""
    from hydra_workloads import make_data
    from paper_2107_06469_amd import hydra as H
    w = decoder_workload(K, steps, layers, n_shards)
    data = make_data(w)
    ls, ts, r = run(w, data, K, H.SCHED_SHARD_PARALLEL, device_budget, activation_budget, "shard-parallel")
    out(json.dumps(r))
    lq, tq, r = run(w, data, K, H.SCHED_SEQUENTIAL, device_budget, activation_budget, "sequential model-parallel")
    out(json.dumps(r))
    l1, t1, r = run(w, data, 1, H.SCHED_SHARD_PARALLEL, 0, activation_budget, "model 0 alone, resident state")
    out(json.dumps(r))
    alone = np.array_equal(ls[0], l1[0]) and all(np.array_equal(a, b) for a, b in zip(ts, t1))
    sched = all(np.array_equal(a, b) for a, b in zip(ls, lq)) and all(np.array_equal(a, b) for a, b in zip(ts, tq))
    finite = all(np.all(np.isfinite(l)) for l in ls)
    out(f"model 0 inside the K={K} run == model 0 alone, bitwise (losses, 4 probed tensors): {alone}")
    out(f"shard-parallel == sequential model-parallel, bitwise: {sched}")
    out(f"first losses (ln 32000 = {np.log(32000):.4f}): {[float(l[0]) for l in ls]}")
    return alone and sched and finite


def main(argv):
    K = int(argv[1]) if len(argv) > 1 else 2
    steps = int(argv[2]) if len(argv) > 2 else 2
    layers = int(argv[3]) if len(argv) > 3 else 8
    db = int(float(argv[4]) * 2 ** 30) if len(argv) > 4 else 40 << 30
    ab = int(float(argv[5]) * 2 ** 30) if len(argv) > 5 else 30 << 30
    return 0 if compare(K, steps, layers, db, ab, out=lambda s: print(s, flush=True)) else 1


if __name__ == "__main__":
    sys.exit(main(sys.argv))
