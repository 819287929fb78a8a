"""Seeded synthetic workloads for multi-model shard-parallel training.

This module only *describes* workloads (architectures, hyper-parameter grids,
shard cut points) and draws the random inputs they consume (feature rows,
labels, token ids, masked positions).  It holds none of the training method's
arithmetic: no layer, loss, gradient, optimizer or weight-initialisation code
lives here.  Both the CPU oracle and the GPU library are fed from it, and it
imports neither.

The workloads stand in for the model-selection setting of the paper
(Introduction, "Model Selection Integration": many hyper-parameter
configurations of one model trained on the same task) and for its evaluation
models (Evaluation, "Workloads": a small feed-forward net and a BERT-shaped
encoder).  No item of any public dataset is reproduced; every input is drawn
from a seeded generator.
"""
from .configs import (  # noqa: F401
    KIND_MLP, KIND_ENCODER, KIND_DECODER, ACT_RELU, ACT_GELU,
    DTYPE_F32, DTYPE_BF16, OPT_SGD, OPT_ADAM,
    Workload, workload, scaled_workload, paper_shaped_workload, n_workloads, INIT_SEED,
)
from .data import make_data, mask_positions  # noqa: F401
