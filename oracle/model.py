"""Models of the oracle as a chain of layer units.

A model is a list of fp32 tensors in a canonical order plus a chain of units
(MLP: one Linear(+activation) per unit, the last unit is the output Linear
with the loss; Transformer: one pre-LN block per unit, the first also embeds
the tokens, the last also applies the final LayerNorm, the output Linear on
the target rows and the loss).  A unit has a forward and an adjoint; training
one step is: all forwards in order, all adjoints in reverse, then the update.
Features flow unit to unit forward and gradients flow back (paper,
Introduction, "Motivation").  Test infrastructure only.

Canonical tensor order
  MLP:          W_0,b_0, ..., W_{L-1},b_{L-1}, W_out,b_out            (W stored [out,in])
  Transformer:  tok_emb[V,d], pos_emb[S,d],
                per block: ln1.g, ln1.b, Wqkv[3d,d], bqkv, Wo[d,d], bo, ln2.g, ln2.b,
                           W1[F,d], b1, (Wg[F,d], bg,) W2[d,F], b2,
                lnf.g, lnf.b, Whead[V,d], bhead
  Wqkv rows [0,d) produce q, [d,2d) k, [2d,3d) v; head h owns columns [h*dh,(h+1)*dh) of each.

Initialisation (seed, model k, tensor j -> stream (k<<20)|j of the counter RNG):
  MLP weights    U(-a,a), a = fp32(sqrt(6/fan_in))      (He/Kaiming uniform, gain sqrt 2); biases 0
  Transformer    matrices and embeddings U(-a,a), a = fp32(0.02*sqrt(3)) (std 0.02); biases 0; LN gamma 1, beta 0
"""
from __future__ import annotations

from typing import Dict, List, Tuple

import numpy as np

from . import layers as L
from .rng import tensor_stream, uniform_sym

F64 = np.float64
KIND_MLP, KIND_ENCODER, KIND_DECODER = 0, 1, 2
ACT_RELU, ACT_GELU = 0, 1


def tensor_specs(arch: Dict) -> List[Tuple[str, Tuple[int, ...], str]]:
    """(name, shape, init) per tensor; init in {"he", "n02", "zero", "one"}."""
    out = []
    if arch["kind"] == KIND_MLP:
        d_prev = arch["d_in"]
        for l in range(arch["n_layers"]):
            out += [(f"W{l}", (arch["d_model"], d_prev), "he"), (f"b{l}", (arch["d_model"],), "zero")]
            d_prev = arch["d_model"]
        out += [("Wout", (arch["n_out"], d_prev), "he"), ("bout", (arch["n_out"],), "zero")]
        return out
    d, F, V, S = arch["d_model"], arch["d_ffn"], arch["n_out"], arch["max_seq"]
    out += [("tok_emb", (V, d), "n02"), ("pos_emb", (S, d), "n02")]
    for l in range(arch["n_layers"]):
        p = f"L{l}."
        out += [(p + "ln1.g", (d,), "one"), (p + "ln1.b", (d,), "zero"),
                (p + "Wqkv", (3 * d, d), "n02"), (p + "bqkv", (3 * d,), "zero"),
                (p + "Wo", (d, d), "n02"), (p + "bo", (d,), "zero"),
                (p + "ln2.g", (d,), "one"), (p + "ln2.b", (d,), "zero"),
                (p + "W1", (F, d), "n02"), (p + "b1", (F,), "zero")]
        if arch["ffn_gated"]:
            out += [(p + "Wg", (F, d), "n02"), (p + "bg", (F,), "zero")]
        out += [(p + "W2", (d, F), "n02"), (p + "b2", (d,), "zero")]
    out += [("lnf.g", (d,), "one"), ("lnf.b", (d,), "zero"), ("Whead", (V, d), "n02"), ("bhead", (V,), "zero")]
    return out


def init_params(arch: Dict, seed: int, model: int) -> List[np.ndarray]:
    params = []
    for j, (_, shape, kind) in enumerate(tensor_specs(arch)):
        n = int(np.prod(shape))
        if kind == "zero":
            t = np.zeros(n, dtype=np.float32)
        elif kind == "one":
            t = np.ones(n, dtype=np.float32)
        else:
            a = np.float32(np.sqrt(6.0 / shape[-1])) if kind == "he" else np.float32(0.02 * np.sqrt(3.0))
            t = uniform_sym(seed, tensor_stream(model, j), n, a)
        params.append(t.reshape(shape))
    return params


def n_units(arch: Dict) -> int:
    return arch["n_layers"] + 1 if arch["kind"] == KIND_MLP else arch["n_layers"]


def unit_tensors(arch: Dict, u: int) -> List[int]:
    """Indices (canonical order) of the tensors unit u owns."""
    if arch["kind"] == KIND_MLP:
        return [2 * u, 2 * u + 1]
    per = 14 if arch["ffn_gated"] else 12
    idx = list(range(2 + per * u, 2 + per * (u + 1)))
    if u == 0:
        idx = [0, 1] + idx
    if u == arch["n_layers"] - 1:
        base = 2 + per * arch["n_layers"]
        idx += [base, base + 1, base + 2, base + 3]
    return idx


def _act(arch):
    return (L.relu, L.relu_grad) if arch["act"] == ACT_RELU else (L.gelu, L.gelu_grad)


def _f64(t):
    return t.astype(F64)


# ---- unit forward / adjoint -------------------------------------------------------------------
# batch: dict(inputs=..., target_pos=..., targets=...) for ONE step.
# fwd returns (output, cache); for the last unit the output is the scalar loss.
# bwd takes the gradient w.r.t. the unit's output (ignored for the last unit: d loss / d loss = 1)
# and returns (gradient w.r.t. the unit's input or None, {tensor index: fp64 gradient}).

def unit_fwd(arch, params, u, x, batch):
    if arch["kind"] == KIND_MLP:
        return _mlp_fwd(arch, params, u, x, batch)
    return _block_fwd(arch, params, u, x, batch)


def unit_bwd(arch, params, u, cache, dout):
    if arch["kind"] == KIND_MLP:
        return _mlp_bwd(arch, params, u, cache, dout)
    return _block_bwd(arch, params, u, cache, dout)


def _mlp_fwd(arch, params, u, x, batch):
    if u == 0:
        x = _f64(batch["inputs"])
    W, b = _f64(params[2 * u]), _f64(params[2 * u + 1])
    z = L.linear_fwd(x, W, b)
    if u == arch["n_layers"]:
        loss, dz = L.softmax_ce(z, batch["targets"])
        return loss, (x, dz)
    act, _ = _act(arch)
    return act(z), (x, z)


def _mlp_bwd(arch, params, u, cache, dout):
    W = _f64(params[2 * u])
    if u == arch["n_layers"]:
        x, dz = cache
    else:
        x, z = cache
        dz = dout * _act(arch)[1](z)
    dx, dW, db = L.linear_bwd(x, W, dz)
    return (dx if u > 0 else None), {2 * u: dW, 2 * u + 1: db}


def _split_heads(t, H):
    B, S, d = t.shape
    return t.reshape(B, S, H, d // H).transpose(0, 2, 1, 3)


def _merge_heads(t):
    B, H, S, dh = t.shape
    return t.transpose(0, 2, 1, 3).reshape(B, S, H * dh)


def _block_fwd(arch, params, u, x, batch):
    d, H, Lyr = arch["d_model"], arch["n_heads"], arch["n_layers"]
    idx = unit_tensors(arch, u)
    c = {}
    if u == 0:
        x = L.embed_fwd(batch["inputs"], _f64(params[0]), _f64(params[1]))
        c["ids"] = batch["inputs"]
        idx = idx[2:]
    p = [_f64(params[j]) for j in idx]
    gated = bool(arch["ffn_gated"])
    ln1g, ln1b, Wqkv, bqkv, Wo, bo, ln2g, ln2b, W1, b1 = p[:10]
    Wg, bg = (p[10], p[11]) if gated else (None, None)
    W2, b2 = p[12 if gated else 10], p[13 if gated else 11]
    B, S, _ = x.shape
    a, c["ln1"] = L.layernorm_fwd(x, ln1g, ln1b)
    qkv = L.linear_fwd(a.reshape(B * S, d), Wqkv, bqkv).reshape(B, S, 3 * d)
    q, k, v = (_split_heads(qkv[..., i * d:(i + 1) * d], H) for i in range(3))
    o, P = L.attention_fwd(q, k, v, bool(arch["causal"]))
    om = _merge_heads(o)
    x1 = x + L.linear_fwd(om.reshape(B * S, d), Wo, bo).reshape(B, S, d)
    f, c["ln2"] = L.layernorm_fwd(x1, ln2g, ln2b)
    f2 = f.reshape(B * S, d)
    z1 = L.linear_fwd(f2, W1, b1)
    if gated:
        zg = L.linear_fwd(f2, Wg, bg)
        hmid = L.gelu(zg) * z1
        c["zg"] = zg
    else:
        hmid = L.gelu(z1)
    x2 = x1 + L.linear_fwd(hmid, W2, b2).reshape(B, S, d)
    c.update(a=a, q=q, k=k, v=v, P=P, om=om, f2=f2, z1=z1, hmid=hmid)
    if u != Lyr - 1:
        return x2, c
    lnfg, lnfb, Wh, bh = (_f64(params[j]) for j in idx[-4:])
    xf, c["lnf"] = L.layernorm_fwd(x2, lnfg, lnfb)
    pos, tgt = batch["target_pos"], batch["targets"]
    rows = (np.arange(B)[:, None] * S + pos).reshape(-1)
    xt = xf.reshape(B * S, d)[rows]
    logits = L.linear_fwd(xt, Wh, bh)
    loss, dz = L.softmax_ce(logits, tgt.reshape(-1))
    c.update(rows=rows, xt=xt, dz=dz)
    return loss, c


def _block_bwd(arch, params, u, c, dout):
    d, H, Lyr = arch["d_model"], arch["n_heads"], arch["n_layers"]
    idx_all = unit_tensors(arch, u)
    idx = idx_all[2:] if u == 0 else idx_all
    p = [_f64(params[j]) for j in idx]
    gated = bool(arch["ffn_gated"])
    ln1g, _, Wqkv, _, Wo, _, ln2g, _, W1, _ = p[:10]
    Wg = p[10] if gated else None
    W2 = p[12 if gated else 10]
    B, _, S, _ = c["q"].shape
    g = {}
    if u == Lyr - 1:
        lnfg, _, Wh, _ = (_f64(params[j]) for j in idx[-4:])
        j0 = idx[-4]
        dxt, g[j0 + 2], g[j0 + 3] = L.linear_bwd(c["xt"], Wh, c["dz"])
        dxf = np.zeros((B * S, d), dtype=F64)
        np.add.at(dxf, c["rows"], dxt)
        dout, g[j0], g[j0 + 1] = L.layernorm_bwd(dxf.reshape(B, S, d), c["lnf"], lnfg)
    k0 = idx[0]                      # index of ln1.g
    o2 = 12 if gated else 10         # offset of W2 within the block's tensors
    dx2 = dout
    dh, g[k0 + o2], g[k0 + o2 + 1] = L.linear_bwd(c["hmid"], W2, dx2.reshape(B * S, d))
    if gated:
        dz1 = dh * L.gelu(c["zg"])
        dzg = dh * c["z1"] * L.gelu_grad(c["zg"])
        df_a, g[k0 + 8], g[k0 + 9] = L.linear_bwd(c["f2"], W1, dz1)
        df_b, g[k0 + 10], g[k0 + 11] = L.linear_bwd(c["f2"], Wg, dzg)
        df = df_a + df_b
    else:
        dz1 = dh * L.gelu_grad(c["z1"])
        df, g[k0 + 8], g[k0 + 9] = L.linear_bwd(c["f2"], W1, dz1)
    dx1, g[k0 + 6], g[k0 + 7] = L.layernorm_bwd(df.reshape(B, S, d), c["ln2"], ln2g)
    dx1 = dx1 + dx2
    dom, g[k0 + 4], g[k0 + 5] = L.linear_bwd(c["om"].reshape(B * S, d), Wo, dx1.reshape(B * S, d))
    do = _split_heads(dom.reshape(B, S, d), H)
    dq, dk, dv = L.attention_bwd(c["q"], c["k"], c["v"], c["P"], do)
    dqkv = np.concatenate([_merge_heads(t) for t in (dq, dk, dv)], axis=-1).reshape(B * S, 3 * d)
    da, g[k0 + 2], g[k0 + 3] = L.linear_bwd(c["a"].reshape(B * S, d), Wqkv, dqkv)
    dx, g[k0], g[k0 + 1] = L.layernorm_bwd(da.reshape(B, S, d), c["ln1"], ln1g)
    dx = dx + dx1
    if u == 0:
        g[0], g[1] = L.embed_bwd(c["ids"], dx, arch["n_out"], arch["max_seq"])
        return None, g
    return dx, g


def loss_and_grads(arch, params, batch):
    """One unsharded forward + backward: (loss, [fp64 gradient per tensor])."""
    caches, x = [], None
    for u in range(n_units(arch)):
        x, c = unit_fwd(arch, params, u, x, batch)
        caches.append(c)
    loss, grads, dx = x, {}, None
    for u in reversed(range(n_units(arch))):
        dx, g = unit_bwd(arch, params, u, caches[u], dx)
        grads.update(g)
    return loss, [grads[j].reshape(params[j].shape) for j in range(len(params))]
