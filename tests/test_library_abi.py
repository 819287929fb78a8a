"""The C boundary without a GPU: the library loads, exports every declared symbol, and its host
logic (argument checks, call order, shard cutting, schedule validation, planning) behaves."""
import os
import re

import numpy as np
import pytest

from hydra_workloads import make_data, scaled_workload, workload
from paper_2107_06469_amd import hydra as H

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    for f in os.listdir(os.path.join(ROOT, "include")):
        if f.endswith(".h"):
            src = open(os.path.join(ROOT, "include", f)).read()
            src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
            names |= set(re.findall(r"\b(hydra_\w+)\s*\(", src))
    return names


def test_library_exports_every_declared_symbol():
    L = H.lib()
    names = _declared()
    assert {"hydra_define_models", "hydra_shard", "hydra_train_epoch", "hydra_read_params", "hydra_read_loss"} <= names
    for n in sorted(names):
        assert hasattr(L, n), f"libhydra.so does not export {n}"


def _dry(w, data=None):
    ctx = H.hydra_create(n_streams=4, dry_run=True)
    H.hydra_define_models(ctx, w.archs, w.hparams, w.init_seed)
    for k in range(w.K):
        H.hydra_shard(ctx, k, w.boundaries[k])
    if data is not None:
        H.hydra_set_data(ctx, data["inputs"], data["target_pos"], data["targets"])
    return ctx


def test_call_order_is_enforced():
    w = workload(0)
    d = make_data(w)
    ctx = H.hydra_create(dry_run=True)
    with pytest.raises(H.HydraError) as e:
        H.hydra_shard(ctx, 0, [2])
    assert e.value.status == 2
    with pytest.raises(H.HydraError) as e:
        H.hydra_train_epoch(ctx)
    assert e.value.status == 2
    H.hydra_define_models(ctx, w.archs, w.hparams, 1)
    with pytest.raises(H.HydraError) as e:
        H.hydra_define_models(ctx, w.archs, w.hparams, 1)
    assert e.value.status == 2
    with pytest.raises(H.HydraError) as e:
        H.hydra_set_data(ctx, d["inputs"], None, d["targets"])
    assert e.value.status == 2
    H.hydra_shard(ctx, -1, [2])
    with pytest.raises(H.HydraError) as e:
        H.hydra_train_epoch(ctx)
    assert e.value.status == 2
    H.hydra_set_data(ctx, d["inputs"], None, d["targets"])
    assert H.hydra_train_epoch(ctx)["steps"] == 10
    H.hydra_destroy(ctx)


def test_argument_checks():
    w = workload(0)
    ctx = H.hydra_create(dry_run=True)
    bad = dict(w.archs[0], d_model=250)
    with pytest.raises(H.HydraError) as e:
        H.hydra_define_models(ctx, [bad] * 4, w.hparams, 1)
    assert e.value.status == 7
    with pytest.raises(H.HydraError) as e:
        H.hydra_define_models(ctx, w.archs, [dict(h, lr=-1.0) for h in w.hparams], 1)
    assert e.value.status == 1
    H.hydra_define_models(ctx, w.archs, w.hparams, 1)
    for cuts in ([0], [5], [3, 3], [3, 2], [1, 2, 3, 4, 5]):
        with pytest.raises(H.HydraError) as e:
            H.hydra_shard(ctx, 0, cuts)
        assert e.value.status == 1
    H.hydra_shard(ctx, 0, [1, 2, 3, 4])
    assert H.hydra_shard_count(ctx, 0) == 5 and H.hydra_shard_count(ctx, 1) == 1
    with pytest.raises(H.HydraError):
        H.hydra_shard(ctx, 9, [1])
    d = make_data(w)
    y = d["targets"].copy()
    y[0, 0] = 10
    with pytest.raises(H.HydraError) as e:
        H.hydra_set_data(ctx, d["inputs"], None, y)
    assert e.value.status == 1
    H.hydra_destroy(ctx)


def test_tensor_shapes_follow_the_canonical_order():
    w = workload(0)
    ctx = _dry(w)
    assert H.hydra_tensor_shapes(ctx, 3) == [(256, 256), (1, 256)] * 4 + [(10, 256), (1, 10)]
    H.hydra_destroy(ctx)


def test_explicit_schedules_are_validated_before_anything_runs():
    w = workload(0)
    ctx = _dry(w, make_data(w))
    F, B, U = H.PHASE_F, H.PHASE_B, H.PHASE_U
    one = [(0, 0, F), (0, 1, F), (0, 1, B), (0, 0, B), (0, 0, U), (0, 1, U)]
    full = [(k, s, p) for k in range(4) for (_, s, p) in one]
    assert H.hydra_train_epoch(ctx, H.SCHED_EXPLICIT, full)["steps"] == 10
    bad = [
        [(0, 1, F)] + full,                                             # F before its predecessor
        [t for t in full if t != (2, 0, U)],                            # a task is missing
        full + [(1, 1, U)],                                             # listed twice
        [(0, 0, F), (0, 1, F), (0, 0, B)] + full[3:],                   # B(0,0) before B(0,1)
        [(0, 0, F), (0, 1, F), (0, 1, U)] + full[2:],                   # U before B
        [(7, 0, F)] + full,                                             # no such model
    ]
    for tasks in bad:
        with pytest.raises(H.HydraError) as e:
            H.hydra_train_epoch(ctx, H.SCHED_EXPLICIT, tasks)
        assert e.value.status == 3, tasks[:3]
    H.hydra_destroy(ctx)


def test_shard_parallel_plan_groups_models_and_sequential_does_not():
    w = workload(1)
    d = make_data(scaled_workload(1, d=4096, n_out=1000, batch=8, steps=2))     # shapes only matter in a dry run
    ctx = H.hydra_create(n_streams=4, dry_run=True)
    H.hydra_define_models(ctx, w.archs, w.hparams, w.init_seed)
    H.hydra_shard(ctx, -1, w.boundaries[0])
    H.hydra_set_data(ctx, d["inputs"], None, d["targets"])
    seq = H.hydra_train_epoch(ctx, H.SCHED_SEQUENTIAL)
    par = H.hydra_train_epoch(ctx, H.SCHED_SHARD_PARALLEL)
    assert seq["grouped_tasks"] == 0
    assert par["grouped_tasks"] == 2 * 8 * 4 * 3                                 # every task of both steps
    assert seq["launches"] == 8 * par["launches"]
    # 8 models x (4 fp32 state blocks + 1 bf16 copy) of 272.6 M parameters
    assert par["peak_dev_bytes"] > 8 * 272_000_000 * 18
    H.hydra_destroy(ctx)


def test_read_buffers_report_required_size():
    import ctypes as C
    w = workload(0)
    ctx = _dry(w)
    n = C.c_size_t(0)
    st = H.lib().hydra_read_params(ctx.handle, 0, -1, None, 0, C.byref(n))
    assert st == 8 and n.value == 4 * (256 * 256 + 256) + 2560 + 10
    st = H.lib().hydra_read_params(ctx.handle, 0, 8, None, 0, C.byref(n))
    assert st == 8 and n.value == 2560
    H.hydra_destroy(ctx)


def _brute_force_partition(cost, S):
    """Smallest possible largest part over all contiguous partitions into S parts (exhaustive)."""
    from itertools import combinations
    U, best = len(cost), None
    for cuts in combinations(range(1, U), S - 1):
        b = (0,) + cuts + (U,)
        worst = max(sum(cost[b[i]:b[i + 1]]) for i in range(S))
        best = worst if best is None else min(best, worst)
    return best


def test_automatic_sharder_balances_and_respects_the_byte_bound():
    # transformer with a heavy first unit (embeddings) and last unit (output matrix): 6 blocks
    w = scaled_workload(2, K=2, depths=[6, 6])
    ctx = H.hydra_create(dry_run=True)
    try:
        H.hydra_define_models(ctx, w.archs, w.hparams, w.init_seed)
        shapes = H.hydra_tensor_shapes(ctx, 0)
        per = 18                                     # master, gradient, two Adam moments, bf16 copy
        pad = [(r * c + 63) // 64 * 64 * per for r, c in shapes]
        cost = [sum(pad[:2 + 12])] + [sum(pad[2 + 12 * l:14 + 12 * l]) for l in range(1, 5)] + [sum(pad[2 + 60:])]
        for S in (1, 2, 3, 4, 6):
            cuts = H.hydra_auto_shard(ctx, 0, n_shards=S)
            assert len(cuts) == S - 1 and H.hydra_shard_count(ctx, 0) == S
            b = [0] + cuts + [6]
            worst = max(sum(cost[b[i]:b[i + 1]]) for i in range(S))
            assert worst == _brute_force_partition(cost, S), (S, cuts)
        # byte bound: fewest shards that respect it
        bound = _brute_force_partition(cost, 3)
        cuts = H.hydra_auto_shard(ctx, 0, max_shard_bytes=bound)
        assert len(cuts) == 2
        cuts = H.hydra_auto_shard(ctx, 0, max_shard_bytes=bound - 1)
        assert len(cuts) >= 3
        assert H.hydra_auto_shard(ctx, 1, max_shard_bytes=bound, n_shards=5) is not None and H.hydra_shard_count(ctx, 1) == 5
        with pytest.raises(H.HydraError) as e:
            H.hydra_auto_shard(ctx, 0, max_shard_bytes=max(cost) - 1)
        assert e.value.status == 1 and "one layer unit" in str(e.value)
        with pytest.raises(H.HydraError):
            H.hydra_auto_shard(ctx, 0, n_shards=7)
        H.hydra_auto_shard(ctx, -1, n_shards=2)
        assert H.hydra_shard_count(ctx, 0) == H.hydra_shard_count(ctx, 1) == 2
    finally:
        H.hydra_destroy(ctx)


def test_task_parallel_plan_and_inactive_models():
    w = workload(0)
    d = make_data(w)
    ctx = _dry(w, d)
    try:
        par = H.hydra_train_epoch(ctx, H.SCHED_SHARD_PARALLEL)
        task = H.hydra_train_epoch(ctx, H.SCHED_TASK_PARALLEL)
        seq = H.hydra_train_epoch(ctx, H.SCHED_SEQUENTIAL)
        assert task["grouped_tasks"] == 0 and task["launches"] == seq["launches"] > par["launches"]
        H.hydra_set_active(ctx, 1, False)
        H.hydra_set_active(ctx, 3, False)
        half = H.hydra_train_epoch(ctx, H.SCHED_SEQUENTIAL)
        assert half["launches"] * 2 == seq["launches"]
        assert len(H.hydra_read_loss(ctx, 1)) == 3 * w.steps and len(H.hydra_read_loss(ctx, 0)) == 4 * w.steps
        with pytest.raises(H.HydraError) as e:   # an explicit order may not name an inactive model
            H.hydra_train_epoch(ctx, H.SCHED_EXPLICIT, [(1, 0, H.PHASE_F)])
        assert e.value.status == 3
        for k in (0, 2):
            H.hydra_set_active(ctx, k, False)
        with pytest.raises(H.HydraError) as e:
            H.hydra_train_epoch(ctx, H.SCHED_SHARD_PARALLEL)
        assert e.value.status == 2
    finally:
        H.hydra_destroy(ctx)


def test_benchmark_refuses_more_than_one_gpu():
    """One GPU is all the library drives: asking the benchmark for more ends with a message, before any device call."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def _padded_blocks(w):
    ctx = H.hydra_create(dry_run=True)
    H.hydra_define_models(ctx, w.archs, w.hparams, w.init_seed)
    nb = [sum((r * c + 63) // 64 * 64 for r, c in H.hydra_tensor_shapes(ctx, k)) for k in range(w.K)]
    H.hydra_destroy(ctx)
    return nb


@pytest.mark.parametrize("slots", [1, 2, 3, 5])
def test_every_policy_plans_with_fewer_state_slots_than_models(slots):
    """Spilled state, K = 4 models of equal depth, fewer state slots than models: a slot is held from a shard's
    backward to its update, so no policy may keep more shards between those two tasks than there are slots."""
    w = scaled_workload(1, K=4, steps=2)
    d = make_data(w)
    nb = _padded_blocks(w)
    slot = max(nb) // 2 * 16 + 64 * 1024
    budget = sum(nb) * 2 + 256 * 1024 + int((slots + 0.5) * slot)
    for n_streams in (1, 4):
        ctx = H.hydra_create(n_streams=n_streams, dry_run=True, device_budget_bytes=budget)
        try:
            H.hydra_define_models(ctx, w.archs, w.hparams, w.init_seed)
            H.hydra_shard(ctx, -1, w.boundaries[0])
            H.hydra_set_data(ctx, d["inputs"], None, d["targets"])
            per_epoch = sum(3 * 4 * n for n in nb) * w.steps
            for policy in (H.SCHED_SEQUENTIAL, H.SCHED_SHARD_PARALLEL, H.SCHED_TASK_PARALLEL):
                st = H.hydra_train_epoch(ctx, policy)
                assert st["h2d_bytes"] == st["d2h_bytes"] >= 0.99 * per_epoch, (policy, slots)
            F, B, U = H.PHASE_F, H.PHASE_B, H.PHASE_U
            # an explicit order that keeps two shards between backward and update needs two slots
            one = lambda k: [(k, 0, F), (k, 1, F), (k, 1, B), (k, 0, B), (k, 0, U), (k, 1, U)]
            tasks = [t for k in range(4) for t in one(k)]
            if slots >= 2:
                H.hydra_train_epoch(ctx, H.SCHED_EXPLICIT, tasks)
            else:
                with pytest.raises(H.HydraError) as e:
                    H.hydra_train_epoch(ctx, H.SCHED_EXPLICIT, tasks)
                assert e.value.status == 3 and "slots" in str(e.value)
        finally:
            H.hydra_destroy(ctx)


def test_models_with_different_optimizers_never_share_a_launch_group():
    """A grid may vary the optimizer: a launch group applies one optimizer to all its members, so SGD and Adam models
    form separate groups (and the epoch plans without error)."""
    w = scaled_workload(1, K=4, steps=2, dtype=1)
    for k in (1, 3):
        w.hparams[k]["opt"] = 0
    d = make_data(w)
    ctx = H.hydra_create(n_streams=4, dry_run=True)
    try:
        H.hydra_define_models(ctx, w.archs, w.hparams, w.init_seed)
        H.hydra_shard(ctx, -1, w.boundaries[0])
        H.hydra_set_data(ctx, d["inputs"], None, d["targets"])
        mixed = H.hydra_train_epoch(ctx, H.SCHED_SHARD_PARALLEL)
        seq = H.hydra_train_epoch(ctx, H.SCHED_SEQUENTIAL)
        assert mixed["grouped_tasks"] == 2 * 4 * 2 * 3            # every task still runs in a group (of two)
        assert mixed["launches"] * 2 == seq["launches"]            # ... and never in a group of four
    finally:
        H.hydra_destroy(ctx)
    w2 = scaled_workload(1, K=4, steps=2, dtype=1)
    ctx = H.hydra_create(n_streams=4, dry_run=True)
    try:
        H.hydra_define_models(ctx, w2.archs, w2.hparams, w2.init_seed)
        H.hydra_shard(ctx, -1, w2.boundaries[0])
        H.hydra_set_data(ctx, d["inputs"], None, d["targets"])
        same = H.hydra_train_epoch(ctx, H.SCHED_SHARD_PARALLEL)
        assert same["launches"] * 4 == seq["launches"] or same["launches"] < mixed["launches"]
    finally:
        H.hydra_destroy(ctx)


def _plan_stats(w, d, **opts):
    ctx = H.hydra_create(dry_run=True, **opts)
    try:
        H.hydra_define_models(ctx, w.archs, w.hparams, w.init_seed)
        for k in range(w.K):
            H.hydra_shard(ctx, k, w.boundaries[k])
        H.hydra_set_data(ctx, d["inputs"], d["target_pos"], d["targets"])
        return H.hydra_train_epoch(ctx, H.SCHED_SHARD_PARALLEL)
    finally:
        H.hydra_destroy(ctx)


def test_automatic_launch_groups_follow_the_tile_count_of_the_products():
    """Automatic group size: ready same-shaped tasks are split over the compute streams only while every group
    still brings 384 output tiles to its smallest product.  Workload 2 (16384 tokens x 768: 192 tiles per model)
    with two compute streams runs forward and backward in two groups of two; with one stream, and workload 1
    (512 tokens x 4096: 32 tiles per model) always, in one group of all models.  Update tasks stay in one group."""
    w = workload(2)
    w.steps = w.n_batches = 1
    d = make_data(w)
    auto4, full4, two4 = (_plan_stats(w, d, n_streams=4, max_group=g) for g in (0, 4, 2))
    assert auto4["grouped_tasks"] == full4["grouped_tasks"] == 4 * 3 * 3
    assert full4["launches"] < auto4["launches"] < two4["launches"]            # F and B in halves, U whole
    assert _plan_stats(w, d, n_streams=1, max_group=0)["launches"] == _plan_stats(w, d, n_streams=1, max_group=4)["launches"]
    w1 = workload(1)
    w1.steps = w1.n_batches = 1
    d1 = make_data(w1)
    assert _plan_stats(w1, d1, n_streams=8, max_group=0)["launches"] == _plan_stats(w1, d1, n_streams=8, max_group=16)["launches"]


def test_small_fp32_mlps_merge_the_launch_groups_of_consecutive_shards():
    """Workload 0 (fp32 MLPs of width 256, 32 rows: the kernels that run a whole shard phase per launch): the
    shard-parallel plan merges the forward groups of consecutive shards, the backward groups likewise, and then the
    two into one group of two launches (forward + input-gradient chain, weight gradients with the update) for the
    4 x 2 shards; with gradients kept the update groups between the backward groups launch the optimizer and nothing
    is merged across them; the sequential plan keeps one launch group per task."""
    w = workload(0)
    w.steps = w.n_batches = 2
    d = make_data(w)
    merged = _plan_stats(w, d, n_streams=4)
    assert merged["launches"] == w.steps * 2 and merged["grouped_tasks"] == w.steps * w.K * 2 * 3
    kept = _plan_stats(w, d, n_streams=4, keep_grads=True)
    assert kept["launches"] > merged["launches"]
    ctx = H.hydra_create(dry_run=True, n_streams=4)
    try:
        H.hydra_define_models(ctx, w.archs, w.hparams, w.init_seed)
        for k in range(w.K):
            H.hydra_shard(ctx, k, w.boundaries[k])
        H.hydra_set_data(ctx, d["inputs"], d["target_pos"], d["targets"])
        seq = H.hydra_train_epoch(ctx, H.SCHED_SEQUENTIAL)
    finally:
        H.hydra_destroy(ctx)
    # per model: forward 1 + 1, backward of the last shard chain + gradients, of the first shard chain + gradients
    assert seq["launches"] == w.steps * w.K * (2 + 2 + 2) and seq["grouped_tasks"] == 0


def test_automatic_budgets_spill_and_recompute_only_when_the_device_is_too_small():
    """auto_budget: with room for everything nothing is spilled or recomputed; with a capacity below the models' state
    the state is spilled to the host; with a capacity between state and state + activations the backward tasks
    recompute their shard's forward (more launches).  A dry run must be told the capacity."""
    w = scaled_workload(4, K=3, depths=[4, 4, 4], steps=2, batch=8, seq=128)   # activations 1.6 x the state
    d = make_data(w)
    nb = _padded_blocks(w)
    state = sum(nb) * 18                                      # fp32 master, gradient, two moments, bf16 copy
    roomy = _plan_stats(w, d, n_streams=4, auto_budget=True, device_capacity_bytes=1 << 40)
    plain = _plan_stats(w, d, n_streams=4)
    assert roomy["h2d_bytes"] == 0 and roomy["launches"] == plain["launches"] and roomy["peak_dev_bytes"] == plain["peak_dev_bytes"]
    acts = plain["peak_dev_bytes"] - state                    # activations, data and scratch of the resident plan
    assert acts > 0
    tight = _plan_stats(w, d, n_streams=4, auto_budget=True, device_capacity_bytes=state + acts // 2)
    assert tight["h2d_bytes"] == 0 and tight["launches"] > plain["launches"]          # state resident, forward recomputed
    assert tight["peak_dev_bytes"] < plain["peak_dev_bytes"]
    small = _plan_stats(w, d, n_streams=4, auto_budget=True, device_capacity_bytes=int(state * 0.9))
    assert small["h2d_bytes"] > 0 and small["peak_host_bytes"] >= sum(nb) * 12       # master and moments live on the host
    assert small["peak_dev_bytes"] <= int(state * 0.9)
    with pytest.raises(H.HydraError) as e:
        _plan_stats(w, d, auto_budget=True)
    assert e.value.status == 1


def test_optimizer_state_calls_check_their_arguments():
    import ctypes as C
    w = scaled_workload(1, K=2)                         # Adam
    ctx = _dry(w)
    try:
        n, steps = C.c_size_t(0), C.c_int64(-1)
        st = H.lib().hydra_read_optimizer_state(ctx.handle, 0, None, None, 0, C.byref(n), C.byref(steps))
        assert st == 8 and n.value == sum(r * c for r, c in H.hydra_tensor_shapes(ctx, 0))
        buf = np.zeros(n.value, dtype=np.float32)
        with pytest.raises(H.HydraError) as e:
            H.hydra_write_optimizer_state(ctx, 0, buf[:-1], buf[:-1], 3)
        assert e.value.status == 1
        with pytest.raises(H.HydraError) as e:
            H.hydra_write_optimizer_state(ctx, 0, buf, buf, -1)
        assert e.value.status == 1
        with pytest.raises(H.HydraError):
            H.hydra_write_optimizer_state(ctx, 5, buf, buf, 0)
        H.hydra_write_optimizer_state(ctx, 0, buf, buf, 7)      # a dry run records the step count only
    finally:
        H.hydra_destroy(ctx)
    w0 = workload(0)                                     # SGD: no moments
    ctx = _dry(w0)
    try:
        n, steps = C.c_size_t(9), C.c_int64(-1)
        st = H.lib().hydra_read_optimizer_state(ctx.handle, 0, None, None, 0, C.byref(n), C.byref(steps))
        assert st == 2 and "dry-run" in H.lib().hydra_last_error(ctx.handle).decode()   # nothing to size, no values to give
    finally:
        H.hydra_destroy(ctx)
