"""Pins of the oracle's models, optimizers and drivers: finite differences over every parameter of
tiny models, closed forms of SGD/Adam, exact replication under sharding, model independence."""
import math

import numpy as np
import pytest

from hydra_workloads import configs as C
from hydra_workloads import make_data, scaled_workload, workload
from oracle import model as M
from oracle import optim as O
from oracle import train as T


def _tiny_mlp(act):
    return C.mlp_arch(2, 3, 4, 2, act, C.DTYPE_F32)


def _tiny_tr(kind, gated):
    return C.transformer_arch(kind, 2, 8, 2, 16, 11, 4, gated, C.DTYPE_F32)


def _tiny_batch(arch, seed=0):
    r = np.random.default_rng(seed)
    if arch["kind"] == C.KIND_MLP:
        return dict(inputs=r.normal(size=(5, arch["d_in"])).astype(np.float32), target_pos=None,
                    targets=r.integers(0, arch["n_out"], size=5).astype(np.int32))
    B, S, V = 3, arch["max_seq"], arch["n_out"]
    ids = r.integers(0, V, size=(B, S)).astype(np.int32)
    ids[0, 1] = ids[0, 0]                                    # duplicate token: exercises scatter-add
    if arch["kind"] == C.KIND_DECODER:
        pos = np.broadcast_to(np.arange(S, dtype=np.int32), (B, S)).copy()
    else:
        pos = np.sort(np.stack([r.permutation(S)[:2] for _ in range(B)]), axis=1).astype(np.int32)
    return dict(inputs=ids, target_pos=pos, targets=r.integers(0, V, size=pos.shape).astype(np.int32))


def _loss64(arch, params64, batch):
    """Forward-only loss with fp64 parameters (the unit functions upcast whatever they are given)."""
    x = None
    for u in range(M.n_units(arch)):
        x, _ = M.unit_fwd(arch, params64, u, x, batch)
    return float(x)


@pytest.mark.parametrize("name", ["mlp_relu", "mlp_gelu", "encoder", "decoder_gated", "encoder_gated"])
def test_gradients_match_central_differences_on_every_parameter(name):
    arch = {"mlp_relu": _tiny_mlp(C.ACT_RELU), "mlp_gelu": _tiny_mlp(C.ACT_GELU),
            "encoder": _tiny_tr(C.KIND_ENCODER, 0), "decoder_gated": _tiny_tr(C.KIND_DECODER, 1),
            "encoder_gated": _tiny_tr(C.KIND_ENCODER, 1)}[name]
    r = np.random.default_rng(11)
    # random fp64 parameters incl. non-trivial biases / LN affine, so no gradient path is hidden by zeros
    params = [r.normal(size=s) * (0.5 if len(s) > 1 else 0.3) + (1.0 if nm.endswith(".g") else 0.0)
              for nm, s, _ in M.tensor_specs(arch)]
    batch = _tiny_batch(arch)
    loss, grads = M.loss_and_grads(arch, params, batch)
    assert loss == pytest.approx(_loss64(arch, params, batch), rel=1e-14)
    h = 1e-5
    worst = 0.0
    for j, p in enumerate(params):
        flat = p.reshape(-1)
        gflat = grads[j].reshape(-1)
        for i in range(flat.size):
            old = flat[i]
            flat[i] = old + h
            lp = _loss64(arch, params, batch)
            flat[i] = old - h
            lm = _loss64(arch, params, batch)
            flat[i] = old
            fd = (lp - lm) / (2 * h)
            # truncation error ~h^2, round-off ~1e-16*loss/h = few 1e-11 absolute
            err = abs(fd - gflat[i]) / (2e-6 * abs(gflat[i]) + 2e-9)
            worst = max(worst, err)
    assert worst < 1.0, worst


def test_unused_embedding_rows_get_zero_gradient():
    arch = _tiny_tr(C.KIND_ENCODER, 0)
    params = M.init_params(arch, 42, 0)
    batch = _tiny_batch(arch)
    _, grads = M.loss_and_grads(arch, params, batch)
    used = set(batch["inputs"].reshape(-1).tolist())
    for v in range(arch["n_out"]):
        assert (np.abs(grads[0][v]).max() > 0) == (v in used)


@pytest.mark.parametrize("kind", [C.KIND_ENCODER, C.KIND_DECODER])
def test_key_bias_gradient_is_zero(kind):
    # adding a constant to every key shifts all scores of a query equally: softmax, hence the loss, cannot see it
    arch = _tiny_tr(kind, 0)
    r = np.random.default_rng(3)
    params = [r.normal(size=s) * 0.5 for _, s, _ in M.tensor_specs(arch)]
    _, grads = M.loss_and_grads(arch, params, _tiny_batch(arch))
    d = arch["d_model"]
    for l in range(arch["n_layers"]):
        g = grads[2 + 12 * l + 3]
        assert np.abs(g[d:2 * d]).max() < 1e-15 and np.abs(g[:d]).max() > 1e-4 and np.abs(g[2 * d:]).max() > 1e-4


def test_tiny_encoder_forward_matches_scalar_loops():
    """Brute-force scalar forward of one pre-LN block + head (index-by-index, Python floats)."""
    arch = C.transformer_arch(C.KIND_ENCODER, 1, 4, 2, 6, 5, 3, 0, C.DTYPE_F32)
    r = np.random.default_rng(12)
    P = [r.normal(size=s) * 0.7 for _, s, _ in M.tensor_specs(arch)]
    tok, pos, l1g, l1b, Wqkv, bqkv, Wo, bo, l2g, l2b, W1, b1, W2, b2, lfg, lfb, Wh, bh = P
    ids = np.array([[2, 4, 2]], dtype=np.int32)
    batch = dict(inputs=ids, target_pos=np.array([[0, 2]], dtype=np.int32), targets=np.array([[1, 3]], dtype=np.int32))
    got = _loss64(arch, P, batch)
    d, H, S, dh = 4, 2, 3, 2

    def ln(row, g, b):
        mu = sum(row) / len(row)
        var = sum((v - mu) ** 2 for v in row) / len(row)
        return [(v - mu) / math.sqrt(var + 1e-5) * g[i] + b[i] for i, v in enumerate(row)]

    def lin(row, W, b):
        return [sum(row[k] * W[n][k] for k in range(len(row))) + b[n] for n in range(len(b))]

    def gelu(z):
        return 0.5 * z * (1 + math.erf(z / math.sqrt(2)))
    x = [[tok[ids[0, s]][c] + pos[s][c] for c in range(d)] for s in range(S)]
    a = [ln(x[s], l1g, l1b) for s in range(S)]
    qkv = [lin(a[s], Wqkv, bqkv) for s in range(S)]
    om = [[0.0] * d for _ in range(S)]
    for h in range(H):
        for i in range(S):
            sc = [sum(qkv[i][h * dh + c] * qkv[j][d + h * dh + c] for c in range(dh)) / math.sqrt(dh) for j in range(S)]
            den = sum(math.exp(s_) for s_ in sc)
            for c in range(dh):
                om[i][h * dh + c] = sum(math.exp(sc[j]) / den * qkv[j][2 * d + h * dh + c] for j in range(S))
    x1 = [[x[s][c] + v for c, v in enumerate(lin(om[s], Wo, bo))] for s in range(S)]
    f = [ln(x1[s], l2g, l2b) for s in range(S)]
    hm = [[gelu(z) for z in lin(f[s], W1, b1)] for s in range(S)]
    x2 = [[x1[s][c] + v for c, v in enumerate(lin(hm[s], W2, b2))] for s in range(S)]
    loss = 0.0
    for p_, t_ in ((0, 1), (2, 3)):
        z = lin(ln(x2[p_], lfg, lfb), Wh, bh)
        loss += math.log(sum(math.exp(v) for v in z)) - z[t_]
    assert got == pytest.approx(loss / 2, rel=1e-12)


# ---- optimizers ---------------------------------------------------------------------------------

def test_sgd_step_and_zero_lr():
    w = workload(0)
    data = make_data(w)
    arch = w.archs[0]
    p0 = M.init_params(arch, w.init_seed, 0)
    loss, g = M.loss_and_grads(arch, p0, T.batch_at(data, 1))
    _, p1, _ = T.train_model(arch, C.hparams(C.OPT_SGD, 0.05), data, 1, w.init_seed, 0)
    for a, b, gg in zip(p0, p1, g):
        assert np.array_equal(b, (a.astype(np.float64) - 0.05 * gg).astype(np.float32))
    one = {k: (v[:1] if v is not None else None) for k, v in data.items()}
    losses, p2, _ = T.train_model(arch, C.hparams(C.OPT_SGD, 0.0), one, 3, w.init_seed, 0)
    assert all(np.array_equal(a, b) for a, b in zip(p0, p2)) and losses[0] == losses[1] == losses[2]


def test_adam_first_step_and_constant_gradient():
    hp = C.hparams(C.OPT_ADAM, 1e-3)
    g = np.array([0.5, -2.0, 0.0, 1e-3, -7.0])
    p = np.zeros(5, dtype=np.float32)
    m, v = np.zeros_like(p), np.zeros_like(p)
    O.update_tensor(hp, 1, p, g, m, v)
    want = -1e-3 * g / (np.abs(g) + 1e-8)
    assert np.allclose(p, want, rtol=1e-6, atol=0) and p[2] == 0.0
    assert np.array_equal(np.sign(p), -np.sign(g).astype(np.float32))
    # constant gradient: bias correction is exact, so every step moves by the same amount
    prev = p.astype(np.float64).copy()
    for t in range(2, 8):
        O.update_tensor(hp, t, p, g, m, v)
        assert np.allclose(p.astype(np.float64) - prev, want, rtol=2e-5, atol=1e-10)
        prev = p.astype(np.float64).copy()


def test_adam_second_step_by_hand():
    hp = C.hparams(C.OPT_ADAM, 0.01)
    p = np.array([1.0], dtype=np.float32)
    m, v = np.zeros(1, np.float32), np.zeros(1, np.float32)
    O.update_tensor(hp, 1, p, np.array([2.0]), m, v)
    O.update_tensor(hp, 2, p, np.array([-1.0]), m, v)
    m2 = 0.9 * (0.1 * 2.0) + 0.1 * (-1.0)
    v2 = 0.999 * (0.001 * 4.0) + 0.001 * 1.0
    step2 = 0.01 * (m2 / (1 - 0.81)) / (math.sqrt(v2 / (1 - 0.999 ** 2)) + 1e-8)
    assert float(p[0]) == pytest.approx(1.0 - 0.01 - step2, rel=1e-6)


def test_warmup_schedule_table():
    hp = C.hparams(C.OPT_ADAM, 4e-4, warmup_steps=5)
    assert [O.lr_at(hp, t) for t in range(1, 8)] == pytest.approx([0.8e-4, 1.6e-4, 2.4e-4, 3.2e-4, 4e-4, 4e-4, 4e-4])
    assert O.lr_at(C.hparams(C.OPT_ADAM, 3e-4), 1) == 3e-4


# ---- drivers ------------------------------------------------------------------------------------

def _same(r1, r2):
    return all(np.array_equal(r1[k][0], r2[k][0]) and all(np.array_equal(a, b) for a, b in zip(r1[k][1], r2[k][1]))
               for k in r1)


@pytest.mark.parametrize("i", [0, 1, 2, 3, 4])
def test_sharded_interleaved_training_is_bit_identical(i):
    w = workload(0) if i == 0 else scaled_workload(i, steps=3)
    data = make_data(w)
    ref = T.train_all(w.archs, w.hparams, data, w.steps, w.init_seed)
    assert _same(ref, T.train_sharded_interleaved(w.archs, w.hparams, data, w.steps, w.init_seed, w.boundaries))
    # another legal order: model-major (one model at a time) and different cut points
    cuts = [[1] for _ in w.archs]
    order = []
    for k in reversed(range(w.K)):
        order += [(k, 0, T.PH_F), (k, 1, T.PH_F), (k, 1, T.PH_B), (k, 0, T.PH_B), (k, 0, T.PH_U), (k, 1, T.PH_U)]
    assert _same(ref, T.train_sharded_interleaved(w.archs, w.hparams, data, w.steps, w.init_seed, cuts, order))


def test_illegal_orders_are_refused():
    w = workload(0)
    data = make_data(w)
    a, h = w.archs[:1], w.hparams[:1]
    F, B, U = T.PH_F, T.PH_B, T.PH_U
    bad = [
        [(0, 1, F), (0, 0, F), (0, 1, B), (0, 0, B), (0, 0, U), (0, 1, U)],       # F out of order
        [(0, 0, F), (0, 1, F), (0, 0, B), (0, 1, B), (0, 0, U), (0, 1, U)],       # B before its successor's B
        [(0, 0, F), (0, 1, F), (0, 1, U), (0, 1, B), (0, 0, B), (0, 0, U)],       # U before B
        [(0, 0, F), (0, 1, F), (0, 1, B), (0, 0, B), (0, 0, U)],                  # task missing
    ]
    for order in bad:
        with pytest.raises(ValueError):
            T.train_sharded_interleaved(a, h, data, 1, w.init_seed, [[2]], order)


def test_models_are_independent_and_seeded_per_model():
    w = workload(0)
    data = make_data(w)
    full = T.train_all(w.archs, w.hparams, data, 3, w.init_seed)
    sub = T.train_all(w.archs, w.hparams, data, 3, w.init_seed, models=[2, 0])
    assert _same(sub, {k: full[k] for k in (2, 0)})
    p0, p1 = M.init_params(w.archs[0], 42, 0), M.init_params(w.archs[0], 42, 1)
    assert not np.array_equal(p0[0], p1[0])
    a = np.float32(math.sqrt(6.0 / 256))
    assert np.abs(p0[0]).max() < a and np.abs(p0[0]).max() > 0.99 * a and not p0[1].any()
    l1, q1, _ = T.train_model(w.archs[0], w.hparams[1], data, 3, w.init_seed, 5)
    l2, q2, _ = T.train_model(w.archs[1], w.hparams[1], data, 3, w.init_seed, 5)
    assert np.array_equal(l1, l2) and all(np.array_equal(x, y) for x, y in zip(q1, q2))


def test_memorisation_and_directional_derivative():
    arch = C.mlp_arch(2, 6, 16, 3, C.ACT_GELU, C.DTYPE_F32)
    r = np.random.default_rng(13)
    data = dict(inputs=r.normal(size=(1, 8, 6)).astype(np.float32), target_pos=None,
                targets=r.integers(0, 3, size=(1, 8)).astype(np.int32))
    losses, _, _ = T.train_model(arch, C.hparams(C.OPT_SGD, 0.2), data, 400, 7, 0)
    assert np.all(np.diff(losses) < 1e-12) and losses[-1] < 0.1 * math.log(3)
    p0 = M.init_params(arch, 7, 0)
    L0, g = M.loss_and_grads(arch, p0, T.batch_at(data, 1))
    gn2 = sum(float((x * x).sum()) for x in g)
    ratios = []
    for lr in (1e-2, 1e-3, 1e-4):
        p64 = [p.astype(np.float64) - lr * x for p, x in zip(p0, g)]
        x = None
        for u in range(M.n_units(arch)):
            x, _ = M.unit_fwd(arch, p64, u, x, T.batch_at(data, 1))
        ratios.append((float(x) - L0) / (-lr * gn2))
    assert abs(ratios[2] - 1) < abs(ratios[1] - 1) < abs(ratios[0] - 1) and abs(ratios[2] - 1) < 1e-3


def test_initial_loss_is_near_log_classes_for_transformers():
    # std-0.02 init gives near-uniform predictions: first loss within a few percent of ln V
    w = scaled_workload(2, steps=1)
    data = make_data(w)
    res = T.train_all(w.archs, w.hparams, data, 1, w.init_seed)
    for k in res:
        assert res[k][0][0] == pytest.approx(math.log(w.archs[k]["n_out"]), rel=0.03)


def _splitmix_python(state, n):
    """n-th output of SplitMix64 from `state` with Python integers (Steele, Lea, Flood 2014)."""
    mask = (1 << 64) - 1
    z = (state + (n + 1) * 0x9E3779B97F4A7C15) & mask
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
    return z ^ (z >> 31)


def test_transformer_initialisation_bound_moments_and_stream():
    """Matrices and embeddings of a Transformer start uniform on [-a, a) with a = fp32(0.02*sqrt(3)), i.e. standard
    deviation 0.02: the bound, the first two moments, the zero / one tensors and, value by value, the counter
    stream keyed by (seed, model, tensor) recomputed here with Python integers and exact rational arithmetic."""
    from fractions import Fraction
    arch = C.transformer_arch(C.KIND_ENCODER, 2, 64, 1, 256, 5000, 16, 0, C.DTYPE_BF16)
    seed, model = 42, 3
    params = M.init_params(arch, seed, model)
    specs = M.tensor_specs(arch)
    a = np.float32(0.02 * math.sqrt(3.0))
    assert abs(float(a) - 0.0346410162) < 1e-9
    for j, ((name, shape, kind), p) in enumerate(zip(specs, params)):
        assert p.dtype == np.float32 and p.shape == tuple(shape)
        if kind == "zero":
            assert not p.any(), name
        elif kind == "one":
            assert np.all(p == 1.0), name
        else:
            assert kind == "n02" and np.abs(p).max() <= a, name
            if p.size >= 1 << 14:   # sampling error of the moments of n uniform draws
                n = p.size
                assert abs(float(p.mean())) < 5 * 0.02 / math.sqrt(n), name
                assert float(p.std()) == pytest.approx(0.02, rel=5 * math.sqrt(0.8 / n) / 2 + 1e-4), name
                assert np.abs(p).max() > float(a) * (1 - 20.0 / n), name
            # the first values of the stream, exactly
            key = _splitmix_python(_splitmix_python(seed, 0) ^ ((model << 20) | j), 0)
            for i in range(3):
                u = Fraction(_splitmix_python(key, i) >> 40, 1 << 24)
                exact = u * 2 * Fraction(float(a)) - Fraction(float(a))
                assert p.reshape(-1)[i] == np.float32(float(exact)), (name, i)   # one rounding of the exact value
    # the largest embedding has 5000*64 = 320000 entries: the head matrix differs from it (another stream)
    assert not np.array_equal(params[0], params[-2])


def test_batches_cycle_through_the_data_set():
    """Step t (1-based) consumes batch (t-1) mod n_batches: a second pass over the data set reuses the batches in order."""
    arch = C.mlp_arch(1, 4, 6, 3, C.ACT_GELU, C.DTYPE_F32)
    r = np.random.default_rng(3)
    nb = 3
    data = dict(inputs=r.normal(size=(nb, 5, 4)).astype(np.float32), target_pos=None,
                targets=r.integers(0, 3, size=(nb, 5)).astype(np.int32))
    for t, want in zip(range(1, 9), [0, 1, 2, 0, 1, 2, 0, 1]):
        b = T.batch_at(data, t)
        assert np.array_equal(b["inputs"], data["inputs"][want]) and np.array_equal(b["targets"], data["targets"][want])
        assert b["target_pos"] is None
    # training 7 steps on 3 batches = training 7 steps on the 7 batches laid out in that order
    order = [0, 1, 2, 0, 1, 2, 0]
    flat = dict(inputs=data["inputs"][order], target_pos=None, targets=data["targets"][order])
    hp = C.hparams(C.OPT_ADAM, 1e-2, warmup_steps=3)
    l1, p1, _ = T.train_model(arch, hp, data, 7, 11, 0)
    l2, p2, _ = T.train_model(arch, hp, flat, 7, 11, 0)
    assert np.array_equal(l1, l2) and all(np.array_equal(x, y) for x, y in zip(p1, p2))
    assert len(set(np.round(l1, 12))) == 7                    # and the steps are not all the same batch
