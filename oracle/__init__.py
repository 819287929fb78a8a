"""CPU oracle: plain, slow, unsharded training of K independent models.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this
package; it exists so that tests, the smoke check and the benchmark's CPU
baseline leg have an independent statement of what training must compute.
It shares no code with the GPU library and never imports it.

What it computes follows the paper's problem statement: several
hyper-parameter configurations of one task are each trained by ordinary
mini-batch gradient descent, forward pass then backpropagation layer by layer
(Introduction, "Motivation"; "Model Selection Integration"), and sharding a
model must not change the result in any way (Approach, "Desiderata", third
item).  The oracle is therefore the plain definition: every model trained on
its own, unsharded, one after another.  The paper prints no formula; layer,
loss and optimizer definitions are the textbook ones and each function says
which.

Numerics: parameters and optimizer state are stored in fp32 (the meaning the
GPU library gives them); every product, reduction and transcendental is
evaluated in fp64.  No bf16 rounding happens anywhere.

Pins (tests marked "not gpu"): closed-form gradients, finite differences on
tiny models, ln(C) loss at zero weights, LayerNorm/attention/GeLU/Adam closed
forms, published splitmix64 vectors, shard-replay bit-identity.  The paper
prints no worked numeric example, so beyond those pins the end-to-end loss
values are "parity unpinned" against the paper itself.
"""
