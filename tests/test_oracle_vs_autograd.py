"""Pins of the oracle against an independent implementation: the same models written with PyTorch's own CPU
primitives (layer_norm, gelu, softmax, cross_entropy, embedding) in fp64 and differentiated by autograd, and
torch.optim's SGD / Adam.  The oracle is numpy with hand-written adjoints; nothing is shared between the two.

What the models are (paper, Introduction "Motivation": features flow layer to layer, gradients back; the paper
names the layer types only): MLP of Linear+activation layers, pre-LN Transformer blocks with a fused QKV projection,
optional gated FFN, final LayerNorm, untied head on the target rows, mean cross-entropy."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from hydra_workloads import configs as C
from oracle import model as M
from oracle import optim as O

F64 = torch.float64


def _batch(arch, seed):
    r = np.random.default_rng(seed)
    if arch["kind"] == C.KIND_MLP:
        return dict(inputs=r.normal(size=(6, arch["d_in"])).astype(np.float32), target_pos=None,
                    targets=r.integers(0, arch["n_out"], size=6).astype(np.int32))
    B, S, V = 3, arch["max_seq"], arch["n_out"]
    ids = r.integers(0, V, size=(B, S)).astype(np.int32)
    ids[1, 2] = ids[1, 0]                                    # a repeated token: its embedding row gets two contributions
    if arch["kind"] == C.KIND_DECODER:
        pos = np.broadcast_to(np.arange(S, dtype=np.int32), (B, S)).copy()
    else:
        pos = np.sort(np.stack([r.permutation(S)[:3] for _ in range(B)]), axis=1).astype(np.int32)
    return dict(inputs=ids, target_pos=pos, targets=r.integers(0, V, size=pos.shape).astype(np.int32))


def _random_params(arch, seed):
    r = np.random.default_rng(seed)
    return [r.normal(size=s) * (0.4 if len(s) > 1 else 0.3) + (1.0 if nm.endswith(".g") else 0.0)
            for nm, s, _ in M.tensor_specs(arch)]


def _torch_loss(arch, p, batch):
    """Loss of one model from its tensors in the canonical order, PyTorch primitives only."""
    act = (lambda z: F.gelu(z, approximate="none")) if arch["act"] == C.ACT_GELU else F.relu
    if arch["kind"] == C.KIND_MLP:
        h = torch.from_numpy(batch["inputs"]).double()
        for l in range(arch["n_layers"]):
            h = act(F.linear(h, p[2 * l], p[2 * l + 1]))
        logits = F.linear(h, p[-2], p[-1])
        return F.cross_entropy(logits, torch.from_numpy(batch["targets"]).long(), reduction="mean")
    d, H, L, gated = arch["d_model"], arch["n_heads"], arch["n_layers"], arch["ffn_gated"]
    dh = d // H
    ids = torch.from_numpy(batch["inputs"]).long()
    B, S = ids.shape
    x = F.embedding(ids, p[0]) + p[1][:S].unsqueeze(0)
    per = 14 if gated else 12
    mask = torch.triu(torch.full((S, S), -math.inf, dtype=F64), diagonal=1) if arch["causal"] else torch.zeros(S, S, dtype=F64)
    for l in range(L):
        t = p[2 + per * l: 2 + per * (l + 1)]
        ln1g, ln1b, Wqkv, bqkv, Wo, bo, ln2g, ln2b, W1, b1 = t[:10]
        a = F.layer_norm(x, (d,), ln1g, ln1b, eps=1e-5)
        q, k, v = F.linear(a, Wqkv, bqkv).split(d, dim=-1)
        heads = lambda z: z.reshape(B, S, H, dh).transpose(1, 2)           # [B, H, S, dh]
        sc = heads(q) @ heads(k).transpose(-1, -2) / math.sqrt(dh) + mask
        o = (torch.softmax(sc, dim=-1) @ heads(v)).transpose(1, 2).reshape(B, S, d)
        x = x + F.linear(o, Wo, bo)
        f = F.layer_norm(x, (d,), ln2g, ln2b, eps=1e-5)
        if gated:
            Wg, bg, W2, b2 = t[10:14]
            hdn = act(F.linear(f, Wg, bg)) * F.linear(f, W1, b1)
        else:
            W2, b2 = t[10:12]
            hdn = act(F.linear(f, W1, b1))
        x = x + F.linear(hdn, W2, b2)
    x = F.layer_norm(x, (d,), p[-4], p[-3], eps=1e-5)
    pos = torch.from_numpy(batch["target_pos"]).long()
    rows = torch.gather(x, 1, pos.unsqueeze(-1).expand(-1, -1, d)).reshape(-1, d)
    logits = F.linear(rows, p[-2], p[-1])
    return F.cross_entropy(logits, torch.from_numpy(batch["targets"]).long().reshape(-1), reduction="mean")


ARCHS = {
    "mlp_relu": C.mlp_arch(3, 5, 7, 4, C.ACT_RELU, C.DTYPE_F32),
    "mlp_gelu": C.mlp_arch(3, 5, 7, 4, C.ACT_GELU, C.DTYPE_F32),
    "encoder": C.transformer_arch(C.KIND_ENCODER, 2, 12, 3, 20, 13, 5, 0, C.DTYPE_F32),
    "encoder_gated": C.transformer_arch(C.KIND_ENCODER, 2, 12, 3, 20, 13, 5, 1, C.DTYPE_F32),
    "decoder": C.transformer_arch(C.KIND_DECODER, 2, 12, 2, 20, 13, 6, 0, C.DTYPE_F32),
    "decoder_gated": C.transformer_arch(C.KIND_DECODER, 3, 8, 2, 12, 9, 4, 1, C.DTYPE_F32),
}


@pytest.mark.parametrize("name", sorted(ARCHS))
def test_loss_and_every_gradient_match_autograd(name):
    arch = ARCHS[name]
    params = _random_params(arch, 5)
    batch = _batch(arch, 6)
    loss, grads = M.loss_and_grads(arch, params, batch)
    tp = [torch.tensor(p, dtype=F64, requires_grad=True) for p in params]
    tl = _torch_loss(arch, tp, batch)
    tl.backward()
    assert loss == pytest.approx(tl.item(), rel=1e-12)
    for (nm, _, _), g, t in zip(M.tensor_specs(arch), grads, tp):
        ref = t.grad.numpy() if t.grad is not None else np.zeros_like(g)
        scale = max(np.abs(ref).max(), 1e-3)
        assert np.abs(g - ref).max() <= 1e-10 * scale, nm


def test_canonical_tensor_order_matches_the_layout_used_above():
    specs = M.tensor_specs(ARCHS["encoder_gated"])
    names = [n for n, _, _ in specs]
    assert len(names) == 2 + 14 * 2 + 4
    shapes = [s for _, s, _ in specs]
    d, Fw, V, S = 12, 20, 13, 5
    assert shapes[0] == (V, d) and shapes[1] == (S, d)
    assert shapes[4] == (3 * d, d) and shapes[6] == (d, d) and shapes[10] == (Fw, d) and shapes[12] == (Fw, d)
    assert shapes[14] == (d, Fw) and shapes[-2] == (V, d) and shapes[-1] == (V,)


@pytest.mark.parametrize("warmup", [0, 3])
def test_adam_matches_torch_optim(warmup):
    r = np.random.default_rng(3)
    hp = C.hparams(C.OPT_ADAM, 3e-3, warmup_steps=warmup, beta1=0.9, beta2=0.999, eps=1e-8)
    p = r.normal(size=(4, 5)).astype(np.float32)
    m, v = np.zeros_like(p), np.zeros_like(p)
    tp = torch.tensor(p.astype(np.float64), dtype=F64, requires_grad=True)
    opt = torch.optim.Adam([tp], lr=hp["lr"], betas=(0.9, 0.999), eps=1e-8, weight_decay=0.0, amsgrad=False)
    for t in range(1, 8):
        g = r.normal(size=p.shape) * (1.0 + t)
        for grp in opt.param_groups:                          # the per-step rate is the oracle's schedule's input, not its output
            grp["lr"] = hp["lr"] * (min(1.0, t / warmup) if warmup > 0 else 1.0)
        tp.grad = torch.tensor(g, dtype=F64)
        opt.step()
        O.update_tensor(hp, t, p, g, m, v)
        # the oracle stores p, m, v in fp32 after every step: agreement to fp32 rounding accumulated over the steps
        np.testing.assert_allclose(p, tp.detach().numpy(), rtol=0, atol=4e-7 * t)
        st = opt.state[tp]
        np.testing.assert_allclose(m, st["exp_avg"].numpy(), rtol=2e-6, atol=1e-7)
        np.testing.assert_allclose(v, st["exp_avg_sq"].numpy(), rtol=2e-6, atol=1e-7)


def test_sgd_matches_torch_optim():
    r = np.random.default_rng(4)
    hp = C.hparams(C.OPT_SGD, 0.05)
    p = r.normal(size=(3, 6)).astype(np.float32)
    tp = torch.tensor(p.astype(np.float64), dtype=F64, requires_grad=True)
    opt = torch.optim.SGD([tp], lr=0.05, momentum=0.0, weight_decay=0.0)
    for t in range(1, 6):
        g = r.normal(size=p.shape)
        tp.grad = torch.tensor(g, dtype=F64)
        opt.step()
        O.update_tensor(hp, t, p, g, None, None)
        np.testing.assert_allclose(p, tp.detach().numpy(), rtol=0, atol=3e-7 * t)
