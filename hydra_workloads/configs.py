"""Workload descriptions: K models of one architecture family, a per-model
hyper-parameter grid and the shard cut points of every model.

Integer codes below are the ones the C boundary uses; they are plain labels.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List

import numpy as np

KIND_MLP, KIND_ENCODER, KIND_DECODER = 0, 1, 2
ACT_RELU, ACT_GELU = 0, 1
DTYPE_F32, DTYPE_BF16 = 0, 1          # BF16 = bf16 working weights, fp32 master + optimizer state
OPT_SGD, OPT_ADAM = 0, 1

INIT_SEED = 42                         # weight-initialisation seed of every workload
_DATA_SEED0 = 1234                     # data seed of workload i is _DATA_SEED0 + i


def _arch(kind, n_layers, d_in, d_model, n_heads, d_ffn, n_out, max_seq, act, ffn_gated, causal, dtype):
    return dict(kind=kind, n_layers=n_layers, d_in=d_in, d_model=d_model, n_heads=n_heads, d_ffn=d_ffn,
                n_out=n_out, max_seq=max_seq, act=act, ffn_gated=ffn_gated, causal=causal, dtype=dtype)


def mlp_arch(n_layers, d_in, d_model, n_out, act, dtype):
    """n_layers hidden Linear(d->d_model)+act layers followed by Linear(d_model->n_out)."""
    return _arch(KIND_MLP, n_layers, d_in, d_model, 0, 0, n_out, 0, act, 0, 0, dtype)


def transformer_arch(kind, n_layers, d_model, n_heads, d_ffn, vocab, max_seq, ffn_gated, dtype):
    return _arch(kind, n_layers, 0, d_model, n_heads, d_ffn, vocab, max_seq, ACT_GELU, ffn_gated,
                 1 if kind == KIND_DECODER else 0, dtype)


def hparams(opt, lr, warmup_steps=0, beta1=0.9, beta2=0.999, eps=1e-8):
    return dict(opt=opt, lr=float(lr), beta1=float(beta1), beta2=float(beta2), eps=float(eps),
                warmup_steps=int(warmup_steps))


def equal_cuts(n_units: int, n_shards: int) -> List[int]:
    """Interior cut points that split n_units layer units into n_shards nearly equal runs."""
    return [round(i * n_units / n_shards) for i in range(1, n_shards)]


@dataclass
class Workload:
    name: str
    index: int
    archs: List[Dict]                  # one per model
    hparams: List[Dict]                # one per model
    boundaries: List[List[int]]        # interior cut points per model, in layer units
    batch: int                         # B: rows (MLP) or sequences (Transformer) per step
    seq: int                           # S (0 for MLP)
    n_targets: int                     # P: target positions per sequence (0 for MLP)
    steps: int
    n_batches: int
    data_seed: int
    init_seed: int = INIT_SEED
    notes: str = ""
    extra: Dict = field(default_factory=dict)

    @property
    def K(self) -> int:
        return len(self.archs)

    def samples_per_step(self) -> int:
        return self.K * self.batch


def n_workloads() -> int:
    return 5


def workload(i: int) -> Workload:
    """The five measured configurations (index 0..4)."""
    seed = _DATA_SEED0 + i
    if i == 0:
        K = 4
        a = mlp_arch(4, 256, 256, 10, ACT_RELU, DTYPE_F32)
        lrs = [0.1, 0.05, 0.01, 0.005]
        return Workload("mlp256_f32_sgd", i, [dict(a) for _ in range(K)], [hparams(OPT_SGD, lr) for lr in lrs],
                        [[2]] * K, 32, 0, 0, 10, 10, seed)
    if i == 1:
        K = 8
        a = mlp_arch(16, 4096, 4096, 1000, ACT_GELU, DTYPE_BF16)
        lrs = [1e-4 * 10 ** (k / 7.0) for k in range(K)]
        return Workload("mlp4096_bf16_adam", i, [dict(a) for _ in range(K)], [hparams(OPT_ADAM, lr) for lr in lrs],
                        [[4, 8, 12]] * K, 512, 0, 0, 50, 50, seed)
    if i == 2:
        K, S = 4, 512
        a = transformer_arch(KIND_ENCODER, 12, 768, 12, 3072, 30522, S, 0, DTYPE_BF16)
        lrs = [1e-4, 2e-4, 5e-5, 3e-4]
        return Workload("encoder768_bf16_adam", i, [dict(a) for _ in range(K)],
                        [hparams(OPT_ADAM, lr) for lr in lrs], [[4, 8]] * K, 32, S, int(0.15 * S), 20, 20, seed)
    if i == 3:
        K, S = 16, 512
        rng = np.random.default_rng(seed)
        # depth per model drawn from {12,18,24}; redraw until every depth occurs at least once
        while True:
            depths = [int((12, 18, 24)[int(3 * u)]) for u in rng.random(K)]
            if set(depths) == {12, 18, 24}:
                break
        archs = [transformer_arch(KIND_ENCODER, L, 1024, 16, 4096, 32000, S, 0, DTYPE_BF16) for L in depths]
        lr_axis, wu_axis = [1e-4, 2e-4, 3e-4, 5e-4], [0, 2, 5, 10]
        hps = [hparams(OPT_ADAM, lr_axis[k // 4], wu_axis[k % 4]) for k in range(K)]
        cuts = [list(range(6, L, 6)) for L in depths]
        return Workload("encoder1024_hetero_bf16_adam", i, archs, hps, cuts, 16, S, int(0.15 * S), 20, 20, seed,
                        extra=dict(depths=depths))
    if i == 4:
        K, S = 8, 2048
        a = transformer_arch(KIND_DECODER, 32, 4096, 32, 11008, 32000, S, 1, DTYPE_BF16)
        hps = [hparams(OPT_ADAM, 1e-5 * (k + 1)) for k in range(K)]
        return Workload("decoder4096_spill_bf16_adam", i, [dict(a) for _ in range(K)], hps, [[8, 16, 24]] * K,
                        8, S, S, 5, 5, seed)
    raise IndexError(i)


def paper_shaped_workload(name: str, K: int = 4) -> Workload:
    """Workloads with the shapes the paper's own evaluation names (Evaluation, "Workloads"), on synthetic data:
    "ffn_1p2m": a feed-forward network of about 1.2 M parameters (the model the paper compares sharded against
    single-device training with); "bert_large_384": a BERT-Large-shaped encoder (24 blocks, d=1024, 16 heads,
    FFN 4096, sequences of 384 tokens as in span-extraction fine-tuning).  K configurations differ in learning rate."""
    if name == "ffn_1p2m":
        # 784 -> 768 -> 768 -> 10: 784*768 + 768 + 768*768 + 768 + 768*10 + 10 = 1,201,162 parameters.  The paper
        # names no activation; GeLU (smooth) lets single and double precision agree to rounding.
        a = mlp_arch(2, 784, 768, 10, ACT_GELU, DTYPE_F32)
        lrs = [0.1 * 0.5 ** k for k in range(K)]
        return Workload("ffn_1p2m_f32_sgd", 5, [dict(a) for _ in range(K)], [hparams(OPT_SGD, lr) for lr in lrs],
                        [[1, 2]] * K, 64, 0, 0, 12, 4, _DATA_SEED0 + 5, notes="3 epochs over 4 batches")
    if name == "bert_large_384":
        S = 384
        a = transformer_arch(KIND_ENCODER, 24, 1024, 16, 4096, 30522, S, 0, DTYPE_BF16)
        lrs = [5e-5, 3e-5, 2e-5, 1e-4][:K] + [1e-5 * (k + 1) for k in range(max(0, K - 4))]
        return Workload("bert_large_384_bf16_adam", 6, [dict(a) for _ in range(K)], [hparams(OPT_ADAM, lr) for lr in lrs],
                        [[6, 12, 18]] * K, 8, S, int(0.15 * S), 3, 3, _DATA_SEED0 + 6)
    raise KeyError(name)


def scaled_workload(i: int, **kw) -> Workload:
    """Reduced-size replicas of workload i that exercise the same code path
    (same kinds of layers, optimizer, number of shards, ragged sizes) at a cost
    a CPU reference finishes in seconds."""
    w = workload(i)
    if i == 1:
        K = kw.get("K", 3)
        d = kw.get("d", 320)
        a = mlp_arch(kw.get("n_layers", 5), d, d, kw.get("n_out", 72), ACT_GELU, kw.get("dtype", DTYPE_BF16))
        lrs = [1e-4 * 10 ** (k / 7.0) for k in range(K)]
        L = a["n_layers"] + 1
        return Workload("mlp_small_bf16_adam", i, [dict(a) for _ in range(K)],
                        [hparams(OPT_ADAM, lr) for lr in lrs],
                        [equal_cuts(L - 1, kw.get("n_shards", 2))] * K, kw.get("batch", 96), 0, 0,
                        kw.get("steps", 6), kw.get("n_batches", kw.get("steps", 6)), w.data_seed)
    if i in (2, 3, 4):
        K = kw.get("K", 3)
        S = kw.get("seq", 48)
        d, H = kw.get("d", 128), kw.get("heads", 2)      # head width 64, as in the full-size workloads
        kind = KIND_DECODER if i == 4 else KIND_ENCODER
        depths = kw.get("depths", [4] * K if i != 3 else [2, 4, 6][:K])
        archs = [transformer_arch(kind, L, d, H, kw.get("d_ffn", 4 * d if i != 4 else 344), kw.get("vocab", 301), S,
                                  1 if i == 4 else 0, kw.get("dtype", DTYPE_BF16)) for L in depths]
        hps = [hparams(OPT_ADAM, 1e-3 * (k + 1), kw.get("warmup", 0) * (k % 2)) for k in range(K)]
        per = kw.get("layers_per_shard", 2)
        cuts = [list(range(per, L, per)) for L in depths]
        P = S if i == 4 else int(0.15 * S)
        return Workload("transformer_small", i, archs, hps, cuts, kw.get("batch", 3), S, P,
                        kw.get("steps", 4), kw.get("n_batches", kw.get("steps", 4)), w.data_seed,
                        extra=dict(depths=depths))
    return w


def param_count(arch: Dict) -> int:
    """Number of trainable scalars of one model (bookkeeping for reports)."""
    if arch["kind"] == KIND_MLP:
        d0, d, L, V = arch["d_in"], arch["d_model"], arch["n_layers"], arch["n_out"]
        n = 0
        for l in range(L):
            n += (d0 if l == 0 else d) * d + d
        return n + (d if L > 0 else d0) * V + V
    d, F, V, S, L = arch["d_model"], arch["d_ffn"], arch["n_out"], arch["max_seq"], arch["n_layers"]
    blk = 2 * d + 3 * d * d + 3 * d + d * d + d + 2 * d + d * F + F + F * d + d
    if arch["ffn_gated"]:
        blk += d * F + F
    return V * d + S * d + L * blk + 2 * d + d * V + V


assert math.isclose(0.15 * 512, 76.8)
