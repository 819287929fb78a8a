"""Pins of the oracle's layer functions: closed forms, invariants, brute force on tiny inputs."""
import math
import os

import numpy as np
import pytest

from oracle import layers as L
from oracle import rng as R

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read(name):
    with open(os.path.join(GOLD, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


# ---- counter RNG --------------------------------------------------------------------------------

def test_splitmix64_published_vectors():
    want = [int(r[0], 16) for r in _read("splitmix64_seed0.txt")]
    got = [int(x) for x in R.splitmix64_at(0, np.arange(len(want)))]
    assert got == want


def test_splitmix64_is_sequential_generator():
    # n-th output computed directly equals stepping the generator n times (state += golden; finalise)
    state, mask = 12345, (1 << 64) - 1
    seq = []
    for _ in range(5):
        state = (state + 0x9E3779B97F4A7C15) & mask
        z = state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
        seq.append(z ^ (z >> 31))
    assert [int(x) for x in R.splitmix64_at(12345, np.arange(5))] == seq


def test_uniform_ranges_and_moments():
    u = R.uniform24(42, R.tensor_stream(3, 7), 200000)
    assert u.min() >= 0.0 and u.max() < 1.0
    assert np.all(u * 2 ** 24 == np.floor(u * 2 ** 24))
    assert abs(u.mean() - 0.5) < 3e-3 and abs(u.var() - 1 / 12) < 2e-3
    a = np.float32(0.153)
    s = R.uniform_sym(42, 5, 100000, a)
    assert s.dtype == np.float32 and s.min() >= -a and s.max() < a
    assert abs(float(s.std()) - float(a) / math.sqrt(3)) < 1e-3
    # streams differ, same stream repeats, and `start` continues a stream
    assert not np.array_equal(R.uniform24(42, 5, 16), R.uniform24(42, 6, 16))
    assert np.array_equal(R.uniform24(42, 5, 16)[4:], R.uniform24(42, 5, 12, start=4))


# ---- affine layer -------------------------------------------------------------------------------

def test_linear_matches_scalar_loops():
    r = np.random.default_rng(0)
    x, W, b, dy = r.normal(size=(3, 5)), r.normal(size=(4, 5)), r.normal(size=4), r.normal(size=(3, 4))
    y = L.linear_fwd(x, W, b)
    dx, dW, db = L.linear_bwd(x, W, dy)
    for m in range(3):
        for n in range(4):
            assert y[m, n] == pytest.approx(sum(x[m, k] * W[n, k] for k in range(5)) + b[n], rel=1e-13)
    for n in range(4):
        assert db[n] == pytest.approx(sum(dy[m, n] for m in range(3)), rel=1e-13)
        for k in range(5):
            assert dW[n, k] == pytest.approx(sum(dy[m, n] * x[m, k] for m in range(3)), rel=1e-12)
    for m in range(3):
        for k in range(5):
            assert dx[m, k] == pytest.approx(sum(dy[m, n] * W[n, k] for n in range(4)), rel=1e-12)


def test_linear_least_squares_gradient_vanishes_at_solution():
    # for 0.5*||x W^T - T||^2 the gradient is (xW^T - T)^T x, which is zero at the least-squares solution
    r = np.random.default_rng(1)
    x, T = r.normal(size=(20, 4)), r.normal(size=(20, 3))
    Wls = np.linalg.lstsq(x, T, rcond=None)[0].T
    res = L.linear_fwd(x, Wls, np.zeros(3)) - T
    _, dW, _ = L.linear_bwd(x, Wls, res)
    assert np.abs(dW).max() < 1e-12


# ---- softmax cross-entropy ----------------------------------------------------------------------

@pytest.mark.parametrize("C", [10, 1000, 30522])
def test_ce_zero_logits_is_log_C(C):
    y = np.random.default_rng(2).integers(0, C, size=64)
    loss, dz = L.softmax_ce(np.zeros((64, C)), y)
    assert loss == pytest.approx(math.log(C), rel=1e-14)
    db = dz.sum(axis=0)
    freq = np.bincount(y, minlength=C) / 64.0
    assert np.allclose(db, 1.0 / C - freq, atol=1e-15)


def test_ce_invariants_and_definition():
    r = np.random.default_rng(3)
    z, y = r.normal(size=(7, 9)) * 4, r.integers(0, 9, size=7)
    loss, dz = L.softmax_ce(z, y)
    assert np.allclose(dz.sum(axis=1), 0.0, atol=1e-15)
    loss2, dz2 = L.softmax_ce(z + 1000.0 * r.normal(size=(7, 1)), y)
    assert loss2 == pytest.approx(loss, rel=1e-10) and np.allclose(dz, dz2, atol=1e-10)
    brute = 0.0
    for i in range(7):
        brute += -math.log(math.exp(z[i, y[i]]) / sum(math.exp(v) for v in z[i]))
    assert loss == pytest.approx(brute / 7, rel=1e-13)
    # gradient vs central differences
    h = 1e-6
    for (i, j) in [(0, 0), (3, int(y[3])), (6, 8)]:
        zp, zm = z.copy(), z.copy()
        zp[i, j] += h
        zm[i, j] -= h
        fd = (L.softmax_ce(zp, y)[0] - L.softmax_ce(zm, y)[0]) / (2 * h)
        assert dz[i, j] == pytest.approx(fd, rel=1e-6, abs=2e-9)


# ---- activations --------------------------------------------------------------------------------

def test_gelu_table_and_identities():
    for xs, ps in _read("normal_cdf.txt"):
        x, p = float(xs), float(ps)
        assert float(L.gelu(np.array([x]))[0]) == pytest.approx(x * p, rel=1e-14, abs=1e-16)
    x = np.linspace(-6, 6, 241)
    assert L.gelu(np.array([0.0]))[0] == 0.0 and L.gelu_grad(np.array([0.0]))[0] == 0.5
    assert np.allclose(L.gelu(x) - L.gelu(-x), x, atol=1e-14)
    assert np.allclose(L.gelu_grad(x) + L.gelu_grad(-x), 1.0, atol=1e-14)
    h = 1e-5
    assert np.allclose(L.gelu_grad(x), (L.gelu(x + h) - L.gelu(x - h)) / (2 * h), atol=1e-9)


def test_relu():
    z = np.array([-2.0, -0.0, 0.0, 1e-30, 3.0])
    assert np.array_equal(L.relu(z), [0, 0, 0, 1e-30, 3.0])
    assert np.array_equal(L.relu_grad(z), [0, 0, 0, 1, 1])


# ---- layer normalisation ------------------------------------------------------------------------

def test_layernorm_statistics_and_invariances():
    r = np.random.default_rng(4)
    x = r.normal(size=(5, 3, 64)) * 3 + 7
    y, (xhat, rstd) = L.layernorm_fwd(x, np.ones(64), np.zeros(64))
    assert np.allclose(y.mean(-1), 0, atol=1e-14)
    assert np.allclose(y.var(-1), 1.0, atol=1e-5)           # 1 - eps/(var+eps)
    assert np.allclose(y.var(-1), x.var(-1) / (x.var(-1) + L.LN_EPS), rtol=1e-12)
    y2, _ = L.layernorm_fwd(2.5 * x - 11.0, np.ones(64), np.zeros(64), eps=0.0)
    y3, _ = L.layernorm_fwd(x, np.ones(64), np.zeros(64), eps=0.0)
    assert np.allclose(y2, y3, atol=1e-11)
    g, b = r.normal(size=64), r.normal(size=64)
    y4, _ = L.layernorm_fwd(x, g, b)
    assert np.allclose(y4, y * g + b, atol=1e-13)
    # scalar definition on one row
    row = x[1, 2]
    mu = sum(row) / 64
    var = sum((v - mu) ** 2 for v in row) / 64
    assert np.allclose(y[1, 2], [(v - mu) / math.sqrt(var + 1e-5) for v in row], atol=1e-13)


def test_layernorm_backward_orthogonality_and_fd():
    r = np.random.default_rng(5)
    x, dy = r.normal(size=(4, 16)), r.normal(size=(4, 16))
    # with eps = 0 the rows of xhat have unit second moment, so dx is orthogonal to both 1 and xhat
    y, c = L.layernorm_fwd(x, np.ones(16), np.zeros(16), eps=0.0)
    dx, dg, db = L.layernorm_bwd(dy, c, np.ones(16))
    assert np.allclose(dx.sum(-1), 0, atol=1e-13)
    assert np.allclose((dx * c[0]).sum(-1), 0, atol=1e-13)
    g, b = r.normal(size=16), r.normal(size=16)

    def f(x_, g_, b_):
        return float((L.layernorm_fwd(x_, g_, b_)[0] * dy).sum())
    _, c = L.layernorm_fwd(x, g, b)
    dx, dg, db = L.layernorm_bwd(dy, c, g)
    h = 1e-6
    for idx in [(0, 0), (2, 7), (3, 15)]:
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        assert dx[idx] == pytest.approx((f(xp, g, b) - f(xm, g, b)) / (2 * h), rel=1e-6, abs=1e-9)
    for j in (0, 9):
        e = np.zeros(16)
        e[j] = h
        assert dg[j] == pytest.approx((f(x, g + e, b) - f(x, g - e, b)) / (2 * h), rel=1e-6, abs=1e-9)
        assert db[j] == pytest.approx((f(x, g, b + e) - f(x, g, b - e)) / (2 * h), rel=1e-6, abs=1e-9)


# ---- attention ----------------------------------------------------------------------------------

def test_attention_uniform_when_scores_are_zero():
    r = np.random.default_rng(6)
    v = r.normal(size=(2, 3, 6, 4))
    z = np.zeros_like(v)
    o, P = L.attention_fwd(z, z, v, causal=False)
    assert np.allclose(P, 1 / 6)
    assert np.allclose(o, np.broadcast_to(v.mean(axis=2, keepdims=True), v.shape))
    o, P = L.attention_fwd(z, z, v, causal=True)
    for i in range(6):
        assert np.allclose(o[:, :, i], v[:, :, : i + 1].mean(axis=2))
        assert np.allclose(P[:, :, i, i + 1:], 0.0)


def test_attention_scalar_brute_force():
    r = np.random.default_rng(7)
    q, k, v = (r.normal(size=(1, 2, 5, 3)) for _ in range(3))
    for causal in (False, True):
        o, P = L.attention_fwd(q, k, v, causal)
        for h in range(2):
            for i in range(5):
                js = range(i + 1) if causal else range(5)
                sc = {j: sum(q[0, h, i, c] * k[0, h, j, c] for c in range(3)) / math.sqrt(3) for j in js}
                den = sum(math.exp(s) for s in sc.values())
                for c in range(3):
                    want = sum(math.exp(sc[j]) / den * v[0, h, j, c] for j in js)
                    assert o[0, h, i, c] == pytest.approx(want, rel=1e-12)


def test_attention_causality_and_permutation_equivariance():
    r = np.random.default_rng(8)
    q, k, v = (r.normal(size=(1, 2, 6, 4)) for _ in range(3))
    o, _ = L.attention_fwd(q, k, v, True)
    k2, v2, q2 = k.copy(), v.copy(), q.copy()
    k2[:, :, 4:] += 3.0
    v2[:, :, 4:] -= 2.0
    q2[:, :, 4:] *= 0.3
    o2, _ = L.attention_fwd(q2, k2, v2, True)
    assert np.array_equal(o[:, :, :4], o2[:, :, :4])
    perm = r.permutation(6)
    o3, _ = L.attention_fwd(q, k, v, False)
    o4, _ = L.attention_fwd(q[:, :, perm], k[:, :, perm], v[:, :, perm], False)
    assert np.allclose(o3[:, :, perm], o4, atol=1e-13)


@pytest.mark.parametrize("causal", [False, True])
def test_attention_backward_fd(causal):
    r = np.random.default_rng(9)
    q, k, v, do = (r.normal(size=(2, 2, 5, 3)) for _ in range(4))
    _, P = L.attention_fwd(q, k, v, causal)
    dq, dk, dv = L.attention_bwd(q, k, v, P, do)

    def f(q_, k_, v_):
        return float((L.attention_fwd(q_, k_, v_, causal)[0] * do).sum())
    h = 1e-6
    for idx in [(0, 0, 0, 0), (1, 1, 4, 2), (0, 1, 2, 1)]:
        for which, grad in enumerate((dq, dk, dv)):
            args_p, args_m = [q.copy(), k.copy(), v.copy()], [q.copy(), k.copy(), v.copy()]
            args_p[which][idx] += h
            args_m[which][idx] -= h
            assert grad[idx] == pytest.approx((f(*args_p) - f(*args_m)) / (2 * h), rel=2e-6, abs=1e-9)


# ---- embedding ----------------------------------------------------------------------------------

def test_embedding_forward_and_duplicate_scatter():
    r = np.random.default_rng(10)
    tok, pos = r.normal(size=(7, 3)), r.normal(size=(5, 3))
    ids = np.array([[1, 1, 4, 0], [1, 6, 6, 6]])
    x = L.embed_fwd(ids, tok, pos)
    assert np.array_equal(x[1, 2], tok[6] + pos[2])
    dx = r.normal(size=(2, 4, 3))
    dtok, dpos = L.embed_bwd(ids, dx, 7, 5)
    assert np.allclose(dtok[1], dx[0, 0] + dx[0, 1] + dx[1, 0])
    assert np.allclose(dtok[6], dx[1, 1] + dx[1, 2] + dx[1, 3])
    assert np.array_equal(dtok[2], np.zeros(3)) and np.array_equal(dpos[4], np.zeros(3))
    assert np.allclose(dpos[:4], dx.sum(0))
