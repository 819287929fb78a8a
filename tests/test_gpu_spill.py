"""Spilling optimizer state to pinned host memory (GPU only): a device budget smaller than the models'
state forces master weights and Adam moments of inactive shards out to the host.  Because the same
kernels see the same numbers, the result must be bit-identical to the resident run (the paper's third
desideratum read strictly), under the overlapped and the synchronous (sequential) schedule."""
import numpy as np
import pytest

from hydra_workloads import make_data, scaled_workload

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a HIP device"
    from paper_2107_06469_amd import hydra
    return hydra


def _blocks(H, w):
    """Padded element count of every model's parameter block (tensor starts are 64-element aligned)."""
    ctx = H.hydra_create(dry_run=True)
    H.hydra_define_models(ctx, w.archs, w.hparams, w.init_seed)
    nb = [sum((r * c + 63) // 64 * 64 for r, c in H.hydra_tensor_shapes(ctx, k)) for k in range(w.K)]
    H.hydra_destroy(ctx)
    return nb


@pytest.mark.parametrize("i", [1, 4])
@pytest.mark.parametrize("slots", [1, 2, 5])
def test_spilled_training_is_bit_identical_to_resident_training(H, i, slots):
    w = scaled_workload(i, steps=3)
    data = make_data(w)
    ref, ref_stats = H.train_workload(w, data, H.SCHED_SHARD_PARALLEL)
    assert ref_stats[0]["h2d_bytes"] == 0
    nb = _blocks(H, w)
    # budget: bf16 working weights + resident vectors (<= 4 B/param) of all models, plus `slots` state slots sized for
    # the largest shard (16 B per element; a shard is at most a whole model here)
    n_shards = len(w.boundaries[0]) + 1
    slot = max(nb) // n_shards * 16 + 64 * 1024
    budget = sum(nb) * 2 + 256 * 1024 + int((slots + 0.5) * slot)
    assert budget < sum(nb) * 18
    for policy in (H.SCHED_SHARD_PARALLEL, H.SCHED_SEQUENTIAL):
        got, stats = H.train_workload(w, data, policy, device_budget_bytes=budget)
        per_step = sum(3 * 4 * n for n in nb)            # master, m, v of every shard once in, once out
        assert stats[0]["h2d_bytes"] >= 0.99 * per_step * w.steps and stats[0]["d2h_bytes"] == stats[0]["h2d_bytes"]
        assert stats[0]["peak_host_bytes"] >= sum(nb) * 12
        for k in range(w.K):
            assert np.array_equal(got[k][0], ref[k][0]), f"loss differs (policy {policy}, {slots} slots)"
            for a, b in zip(got[k][1], ref[k][1]):
                assert np.array_equal(a, b), f"parameters differ (policy {policy}, {slots} slots)"


def test_budget_too_small_for_one_shard_is_reported(H):
    w = scaled_workload(1, steps=1)
    data = make_data(w)
    nb = _blocks(H, w)
    with pytest.raises(H.HydraError) as e:
        H.train_workload(w, data, H.SCHED_SHARD_PARALLEL, device_budget_bytes=sum(nb) * 2 + 300 * 1024)
    assert e.value.status == 4
