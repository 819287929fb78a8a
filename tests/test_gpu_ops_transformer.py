"""Parity of the Transformer-side HIP operations (LayerNorm, attention, embedding) with the oracle's
layer functions (GPU only).  bf16 inputs are rounded once on the host and the oracle gets exactly those
values in fp64; tolerances are the bf16 output rounding (2^-8 relative) plus, for attention, the bf16
rounding of the probabilities that feed the second matrix product."""
import math

import numpy as np
import pytest

from oracle import layers as OL

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available(), "GPU tests need a HIP device"
    return t


@pytest.fixture(scope="module")
def ops():
    from paper_2107_06469_amd import ops as o
    return o


def _bf(torch, a):
    """fp array -> (bf16 cuda tensor, the rounded values as fp64)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.cuda(), t.to(torch.float64).numpy()


def _f32(torch, a):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.cuda(), t.to(torch.float64).numpy()


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("shape", [(37, 64), (130, 768), (9, 1024), (5, 2048 + 64), (6, 4096), (100, 1536), (70, 4096)])
def test_layernorm_forward_and_backward(torch, ops, dtype, shape):
    rows, d = shape
    r = np.random.default_rng(rows * d)
    mk = _bf if dtype else _f32
    tdt = torch.bfloat16 if dtype else torch.float32
    G = 2
    xs, ys, gs, bs, mus, rss, dys, adds, dxs, parts, dgs, dbs, ref = ([] for _ in range(13))
    for g in range(G):
        xd, xv = mk(torch, r.normal(size=(rows, d)) * 2 + 0.5)
        dyd, dyv = mk(torch, r.normal(size=(rows, d)))
        ad, av = mk(torch, r.normal(size=(rows, d)))
        gam, bet = (r.normal(size=d) * 0.3 + 1).astype(np.float32), (r.normal(size=d) * 0.2).astype(np.float32)
        xs.append(xd), dys.append(dyd), adds.append(ad)
        gs.append(torch.from_numpy(gam).cuda()), bs.append(torch.from_numpy(bet).cuda())
        ys.append(torch.zeros((rows, d), dtype=tdt, device="cuda"))
        dxs.append(torch.zeros((rows, d), dtype=tdt, device="cuda"))
        mus.append(torch.zeros(rows, device="cuda")), rss.append(torch.zeros(rows, device="cuda"))
        parts.append(torch.zeros(ops.hydra_op_layernorm_part_floats(rows, d), device="cuda"))
        dgs.append(torch.zeros(d, device="cuda")), dbs.append(torch.zeros(d, device="cuda"))
        y, cache = OL.layernorm_fwd(xv, gam.astype(np.float64), bet.astype(np.float64))
        dx, dg, db = OL.layernorm_bwd(dyv, cache, gam.astype(np.float64))
        ref.append((y, cache, dx + av, dg, db))
    ops.hydra_op_layernorm_fwd(dtype, rows, d, d, 1e-5, xs, ys, gs, bs, mus, rss)
    ops.hydra_op_layernorm_bwd(dtype, rows, d, d, xs, dys, adds, dxs, gs, mus, rss, parts, dgs, dbs)
    torch.cuda.synchronize()
    out_eps = 2.0 ** -8 if dtype else 2e-6
    for g in range(G):
        y, (xhat, rstd), dx, dg, db = ref[g]
        assert np.allclose(mus[g].cpu().numpy(), (xs[g].double().cpu().numpy()).mean(-1), atol=1e-5)
        assert np.allclose(rss[g].cpu().numpy(), rstd[:, 0], rtol=2e-5)
        assert np.all(np.abs(ys[g].double().cpu().numpy() - y) <= out_eps * np.abs(y) + 1e-5)
        assert np.all(np.abs(dxs[g].double().cpu().numpy() - dx) <= out_eps * np.abs(dx) + 2e-5)
        # column sums over `rows` terms in fp32
        assert np.allclose(dgs[g].cpu().numpy(), dg, rtol=1e-4, atol=1e-4 * math.sqrt(rows))
        assert np.allclose(dbs[g].cpu().numpy(), db, rtol=1e-4, atol=1e-4 * math.sqrt(rows))


def _attention_case(torch, ops, B, S, H, DH, causal, seed):
    r = np.random.default_rng(seed)
    d = H * DH
    G = 2
    qkvs, os_, lses, douts, deltas, dqkvs, refs = [], [], [], [], [], [], []
    scale = 1.0 / math.sqrt(DH)
    for g in range(G):
        qd, qv = _bf(torch, r.normal(size=(B * S, 3 * d)) * 1.5)
        dod, dov = _bf(torch, r.normal(size=(B * S, d)))
        qkvs.append(qd), douts.append(dod)
        os_.append(torch.zeros((B * S, d), dtype=torch.bfloat16, device="cuda"))
        lses.append(torch.zeros(B * H * S, device="cuda")), deltas.append(torch.zeros(B * H * S, device="cuda"))
        dqkvs.append(torch.full((B * S, 3 * d), 9.0, dtype=torch.bfloat16, device="cuda"))
        t = qv.reshape(B, S, 3, H, DH)
        q, k, v = (t[:, :, i].transpose(0, 2, 1, 3) for i in range(3))           # [B,H,S,DH]
        o, P = OL.attention_fwd(q, k, v, causal)
        do = dov.reshape(B, S, H, DH).transpose(0, 2, 1, 3)
        dq, dk, dv = OL.attention_bwd(q, k, v, P, do)
        sc = np.matmul(q, np.swapaxes(k, -1, -2)) * scale
        if causal:
            sc = np.where(np.tril(np.ones((S, S), dtype=bool)), sc, -np.inf)
        lse = np.log(np.exp(sc - sc.max(-1, keepdims=True)).sum(-1)) + sc.max(-1)
        refs.append((o, lse, dq, dk, dv))
    ops.hydra_op_attention_fwd(B, S, H, DH, 3 * d, d, causal, scale, qkvs, os_, lses)
    # the backward kernels read the forward's own (rounded) output, as they do in training
    ops.hydra_op_attention_bwd(B, S, H, DH, 3 * d, d, causal, scale, qkvs, os_, douts, lses, deltas, dqkvs)
    torch.cuda.synchronize()
    for g in range(G):
        o, lse, dq, dk, dv = refs[g]
        got_o = os_[g].double().cpu().numpy().reshape(B, S, H, DH).transpose(0, 2, 1, 3)
        # P is rounded to bf16 before P.v: error <= 2^-8 * sum_j P_ij |v_j| <= 2^-8 * max|v|; plus output rounding
        assert np.abs(got_o - o).max() <= 2.0 ** -7 * 8.0, f"o: {np.abs(got_o - o).max()}"
        assert np.sqrt(((got_o - o) ** 2).mean()) <= 4e-3 * np.sqrt((o ** 2).mean()), "o rms"
        assert np.allclose(lses[g].cpu().numpy().reshape(B, H, S), lse, rtol=1e-5, atol=1e-4)
        got = dqkvs[g].double().cpu().numpy().reshape(B, S, 3, H, DH)
        for name, i, ref in (("dq", 0, dq), ("dk", 1, dk), ("dv", 2, dv)):
            a = got[:, :, i].transpose(0, 2, 1, 3)
            rel = np.sqrt(((a - ref) ** 2).mean()) / np.sqrt((ref ** 2).mean())
            assert rel <= 1.5e-2, f"{name}: rel rms {rel}"
            assert np.abs(a - ref).max() <= 0.06 * np.abs(ref).max() + 1e-3, f"{name}: max {np.abs(a - ref).max()}"


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", [(2, 64, 2, 64), (1, 80, 3, 64), (2, 200, 1, 64), (1, 512, 2, 64), (1, 136, 2, 128),
                                   (1, 33, 1, 128)])
def test_attention_forward_and_backward(torch, ops, causal, shape):
    B, S, H, DH = shape
    _attention_case(torch, ops, B, S, H, DH, causal, seed=S * DH + int(causal))


@pytest.mark.parametrize("shape", [(32, 512, 12, 64, False), (2, 2048, 8, 128, True)])
def test_attention_at_the_workloads_shapes(torch, ops, shape):
    """The attention of workload 2 at its full per-model size (batch 32, 12 heads of 64, S = 512: 8 key tiles per
    query block, 384 x 4 workgroups per problem, two problems grouped) and of workload 4's decoders (S = 2048, heads
    of 128, causal: 32 key tiles, short and long causal blocks dealt over the XCDs), the latter on 2 sequences x 8
    heads instead of 8 x 32 so that the fp64 oracle's probability matrices fit a test."""
    B, S, H, DH, causal = shape
    _attention_case(torch, ops, B, S, H, DH, causal, seed=S + DH)


@pytest.mark.parametrize("causal", [False, True])
def test_attention_over_128_key_tiles(torch, ops, causal):
    """One head of 64 at S = 8192 (the longest sequence the kernel rates are quoted at): the running maximum and sum go
    through 128 key tiles per query block, the backward kernels through 128 query tiles per key block."""
    _attention_case(torch, ops, 1, 8192, 1, 64, causal, seed=8192 + int(causal))


def test_attention_uniform_scores_closed_form(torch, ops):
    """q = k = 0 gives uniform probabilities: o is the running (causal) or global mean of v; lse = log(count)."""
    B, S, H, DH = 1, 96, 1, 64
    r = np.random.default_rng(0)
    qkv = np.zeros((S, 3 * DH))
    qkv[:, 2 * DH:] = r.normal(size=(S, DH))
    qd, qv = _bf(torch, qkv)
    for causal in (False, True):
        o = torch.zeros((S, DH), dtype=torch.bfloat16, device="cuda")
        lse = torch.zeros(S, device="cuda")
        ops.hydra_op_attention_fwd(B, S, H, DH, 3 * DH, DH, causal, 0.125, [qd], [o], [lse])
        torch.cuda.synchronize()
        v = qv[:, 2 * DH:]
        want = np.cumsum(v, 0) / np.arange(1, S + 1)[:, None] if causal else np.broadcast_to(v.mean(0), (S, DH))
        cnt = np.arange(1, S + 1) if causal else np.full(S, S)
        assert np.abs(o.double().cpu().numpy() - want).max() <= 2.0 ** -7 * np.abs(v).max()
        assert np.allclose(lse.cpu().numpy(), np.log(cnt), atol=1e-5)


@pytest.mark.parametrize("dtype", [0, 1])
def test_embedding_forward_and_backward(torch, ops, dtype):
    r = np.random.default_rng(5)
    V, S_table, S, B, d = 50, 40, 33, 3, 72
    mk = _bf if dtype else _f32
    ids = r.integers(0, V, size=(B, S)).astype(np.int32)
    ids[0, :5] = 7                                           # duplicates
    order = np.argsort(ids.reshape(-1), kind="stable").astype(np.int32)
    row_ptr = np.concatenate([[0], np.cumsum(np.bincount(ids.reshape(-1), minlength=V))]).astype(np.int32)
    toks, poss, xs, dxs, dtoks, dposs, refs = [], [], [], [], [], [], []
    for g in range(2):
        td, tv = mk(torch, r.normal(size=(V, d)))
        pd, pv = mk(torch, r.normal(size=(S_table, d)))
        dd, dv = mk(torch, r.normal(size=(B * S, d)))
        toks.append(td), poss.append(pd), dxs.append(dd)
        xs.append(torch.zeros((B * S, d), dtype=td.dtype, device="cuda"))
        dtoks.append(torch.full((V, d), 3.0, device="cuda")), dposs.append(torch.full((S_table, d), 3.0, device="cuda"))
        x = OL.embed_fwd(ids, tv, pv)
        dtok, dpos = OL.embed_bwd(ids, dv.reshape(B, S, d), V, S_table)
        refs.append((x, dtok, dpos))
    idd = torch.from_numpy(ids.reshape(-1)).cuda()
    ops.hydra_op_embed_fwd(dtype, B * S, S, d, d, idd, toks, poss, xs)
    ops.hydra_op_embed_bwd(dtype, V, S, S_table, B, d, d, torch.from_numpy(row_ptr).cuda(), torch.from_numpy(order).cuda(),
                           dxs, dtoks, dposs)
    torch.cuda.synchronize()
    for g in range(2):
        x, dtok, dpos = refs[g]
        tol = 2.0 ** -8 if dtype else 1e-6
        assert np.all(np.abs(xs[g].double().cpu().numpy().reshape(B, S, d) - x) <= tol * np.abs(x) + 1e-7)
        assert np.allclose(dtoks[g].cpu().numpy(), dtok, rtol=1e-5, atol=1e-5)
        assert np.allclose(dposs[g].cpu().numpy(), dpos, rtol=1e-5, atol=1e-5)
