"""Layer definitions of the oracle, forward and adjoint, all in fp64.

Every function is the textbook definition written out; matrix products use
numpy's matmul as a library step.  The paper gives no formulas (it speaks only
of forward inference and backpropagation passing features and gradients from
layer to layer; Introduction, "Motivation"), so each docstring states the
definition it implements.  Test infrastructure only.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf

F64 = np.float64
_SQRT2 = np.sqrt(2.0)
_INV_SQRT_2PI = 1.0 / np.sqrt(2.0 * np.pi)
LN_EPS = 1e-5


# ---- affine layer -----------------------------------------------------------------------------

def linear_fwd(x, W, b):
    """y[m,n] = sum_k x[m,k] W[n,k] + b[n]   (W stored [out, in])."""
    return x @ W.T + b


def linear_bwd(x, W, dy):
    """Adjoint of linear_fwd: dW = dy^T x, db = column sums of dy, dx = dy W."""
    return dy @ W, dy.T @ x, dy.sum(axis=0)


# ---- activations ------------------------------------------------------------------------------

def relu(z):
    return np.maximum(z, 0.0)


def relu_grad(z):
    """Derivative of max(z,0); taken as 0 at z = 0."""
    return (z > 0.0).astype(F64)


def gelu(z):
    """GeLU(z) = z * Phi(z), Phi the standard normal CDF (exact erf form)."""
    return 0.5 * z * (1.0 + erf(z / _SQRT2))


def gelu_grad(z):
    """d/dz [z Phi(z)] = Phi(z) + z phi(z), phi the standard normal density."""
    return 0.5 * (1.0 + erf(z / _SQRT2)) + z * np.exp(-0.5 * z * z) * _INV_SQRT_2PI


# ---- layer normalisation ----------------------------------------------------------------------

def layernorm_fwd(x, gamma, beta, eps=LN_EPS):
    """Per row: mu = mean, var = biased variance, xhat = (x-mu)/sqrt(var+eps), y = xhat*gamma + beta."""
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = xc * rstd
    return xhat * gamma + beta, (xhat, rstd)


def layernorm_bwd(dy, cache, gamma):
    """With g = dy*gamma: dx = rstd * (g - mean(g) - xhat * mean(g*xhat)); dgamma = sum dy*xhat; dbeta = sum dy."""
    xhat, rstd = cache
    g = dy * gamma
    dx = rstd * (g - g.mean(axis=-1, keepdims=True) - xhat * (g * xhat).mean(axis=-1, keepdims=True))
    red = tuple(range(dy.ndim - 1))
    return dx, (dy * xhat).sum(axis=red), dy.sum(axis=red)


# ---- scaled dot-product attention ------------------------------------------------------------

def attention_fwd(q, k, v, causal):
    """q,k,v: [B,H,S,dh].  P = softmax_rows(q k^T / sqrt(dh) + mask), o = P v.
    mask is -inf strictly above the diagonal when causal, else absent."""
    dh = q.shape[-1]
    s = np.matmul(q, np.swapaxes(k, -1, -2)) / np.sqrt(F64(dh))
    if causal:
        S = s.shape[-1]
        s = np.where(np.tril(np.ones((S, S), dtype=bool)), s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    P = e / e.sum(axis=-1, keepdims=True)
    return np.matmul(P, v), P


def attention_bwd(q, k, v, P, do):
    """Adjoint: dv = P^T do; dP = do v^T; dS = P o (dP - rowsum(dP o P)); dq = dS k / sqrt(dh); dk = dS^T q / sqrt(dh)."""
    dh = q.shape[-1]
    dv = np.matmul(np.swapaxes(P, -1, -2), do)
    dP = np.matmul(do, np.swapaxes(v, -1, -2))
    dS = P * (dP - (dP * P).sum(axis=-1, keepdims=True))
    scale = 1.0 / np.sqrt(F64(dh))
    dq = np.matmul(dS, k) * scale
    dk = np.matmul(np.swapaxes(dS, -1, -2), q) * scale
    return dq, dk, dv


# ---- softmax cross-entropy -------------------------------------------------------------------

def softmax_ce(logits, y):
    """loss = mean_i [ logsumexp(z_i) - z_i[y_i] ];  dz = (softmax(z) - onehot(y)) / N."""
    n = logits.shape[0]
    zmax = logits.max(axis=1, keepdims=True)
    e = np.exp(logits - zmax)
    se = e.sum(axis=1, keepdims=True)
    lse = np.log(se) + zmax
    loss = (lse[:, 0] - logits[np.arange(n), y]).mean()
    dz = e / se
    dz[np.arange(n), y] -= 1.0
    return F64(loss), dz / n


# ---- embedding -------------------------------------------------------------------------------

def embed_fwd(ids, tok, pos):
    """x[b,s,:] = tok[ids[b,s],:] + pos[s,:]."""
    S = ids.shape[1]
    return tok[ids] + pos[:S][None, :, :]


def embed_bwd(ids, dx, V, S_max):
    """dtok[v,:] = sum over (b,s) with ids[b,s]==v of dx[b,s,:];  dpos[s,:] = sum_b dx[b,s,:]."""
    d = dx.shape[-1]
    dtok = np.zeros((V, d), dtype=F64)
    np.add.at(dtok, ids.reshape(-1), dx.reshape(-1, d))
    dpos = np.zeros((S_max, d), dtype=F64)
    dpos[: ids.shape[1]] = dx.sum(axis=0)
    return dtok, dpos
