"""Seeded draws of the inputs a workload consumes.

MLP workloads: feature rows x ~ N(0,1) (fp32) and labels uniform over the
classes.  Encoder workloads: token ids uniform over the vocabulary, with
P = floor(0.15*S) distinct positions per sequence chosen as prediction
targets; the input id at a target position is replaced by MASK_ID and the
target is the original id.  Decoder workloads: S+1 uniform tokens per
sequence, inputs are the first S, the target at position i is token i+1.

All K models of a workload consume the same batches (they are configurations
of one task; paper, Introduction, "Model Selection Integration").
"""
from __future__ import annotations

from typing import Dict

import numpy as np

from .configs import KIND_MLP, KIND_DECODER, Workload

MASK_ID = 0


def mask_positions(rng: np.random.Generator, n_seq: int, S: int, P: int) -> np.ndarray:
    """P distinct positions per sequence, ascending, int32 [n_seq, P]."""
    out = np.empty((n_seq, P), dtype=np.int32)
    for i in range(n_seq):
        out[i] = np.sort(rng.permutation(S)[:P])
    return out


def make_data(w: Workload) -> Dict[str, np.ndarray]:
    """Returns host arrays in the layout the training boundary takes:
    MLP:         inputs fp32 [n_batches, B, d_in], targets int32 [n_batches, B]
    Transformer: inputs int32 [n_batches, B, S], target_pos int32 [n_batches, B, P],
                 targets int32 [n_batches, B, P]
    """
    rng = np.random.default_rng(w.data_seed)
    a = w.archs[0]
    nb, B = w.n_batches, w.batch
    if a["kind"] == KIND_MLP:
        x = rng.standard_normal((nb, B, a["d_in"])).astype(np.float32)
        y = rng.integers(0, a["n_out"], size=(nb, B), dtype=np.int32)
        return dict(inputs=x, target_pos=None, targets=y)
    S, V, P = w.seq, a["n_out"], w.n_targets
    if a["kind"] == KIND_DECODER:
        tok = rng.integers(0, V, size=(nb, B, S + 1), dtype=np.int32)
        ids = np.ascontiguousarray(tok[:, :, :S])
        tgt = np.ascontiguousarray(tok[:, :, 1:])
        pos = np.broadcast_to(np.arange(S, dtype=np.int32), (nb, B, S)).copy()
        return dict(inputs=ids, target_pos=pos, targets=tgt)
    ids = rng.integers(0, V, size=(nb, B, S), dtype=np.int32)
    pos = mask_positions(rng, nb * B, S, P).reshape(nb, B, P)
    tgt = np.take_along_axis(ids, pos, axis=2).astype(np.int32)
    np.put_along_axis(ids, pos, np.int32(MASK_ID), axis=2)
    return dict(inputs=ids, target_pos=pos, targets=tgt)
