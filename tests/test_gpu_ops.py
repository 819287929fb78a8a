"""Parity of the individual HIP operations with the oracle's layer functions (GPU only).

Inputs are seeded; bf16 operands are rounded to bf16 once on the host and the oracle gets exactly
those values in fp64, so the only differences are fp32 accumulation order and output rounding.
Tolerance for a dot product of length K accumulated in fp32: |err| <= 2*K*2^-24 * sum|x||w| (the
standard forward bound), plus 2^-8 relative when the output is rounded to bf16.
"""
import math

import numpy as np
import pytest

from oracle import layers as OL
from oracle import rng as ORNG

pytestmark = pytest.mark.gpu

EPS32 = 2.0 ** -24


@pytest.fixture(scope="module")
def torch():
    import torch as t
    assert t.cuda.is_available(), "GPU tests need a HIP device"
    return t


@pytest.fixture(scope="module")
def ops():
    from paper_2107_06469_amd import ops as o
    return o


def _ld(n, e=8):
    return (n + e - 1) // e * e


def _dev(torch, a, dtype, ld=None):
    """host fp array [r,c] -> device tensor [r,ld] of dtype (zero padded); returns (tensor, values as fp64)."""
    r, c = a.shape
    ld = ld or _ld(c)
    t = torch.zeros((r, ld), dtype=torch.float32)
    t[:, :c] = torch.from_numpy(a.astype(np.float32))
    t = t.to(torch.bfloat16 if dtype == 1 else torch.float32)
    vals = t[:, :c].to(torch.float64).numpy().copy()
    return t.cuda(), vals


def _check(got, want, bound, out_bf16, what):
    tol = bound + (2.0 ** -8) * np.abs(want) * (1.0 if out_bf16 else 0.0) + 1e-30
    bad = np.abs(got - want) > tol
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} off, worst {np.abs(got - want).max()} vs tol {tol[bad].min()}"


SHAPES = [  # (M, N, K)
    (32, 256, 256), (96, 72, 320), (130, 200, 136), (512, 1000, 520), (257, 130, 72), (40, 10, 256),
]


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("tile", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("layout", ["fwd", "dgrad", "wgrad"])
def test_gemm_layouts_tiles_and_ragged_shapes(torch, ops, dtype, tile, layout):
    r = np.random.default_rng(100 * dtype + 10 * tile + len(layout))
    G = 3
    for (M, N, K) in SHAPES:
        Xs, Ws, outs, wants, bounds = [], [], [], [], []
        for g in range(G):
            x = r.normal(size=(M, K))
            w = r.normal(size=(N, K)) / math.sqrt(K)
            if layout == "fwd":      # out[M,N] = x w^T, both k-major
                xd, xv = _dev(torch, x, dtype)
                wd, wv = _dev(torch, w, dtype)
                kw = dict(x_kmajor=1, w_kmajor=1, ldx=xd.shape[1], ldw=wd.shape[1])
            elif layout == "dgrad":  # out[M,N] = x(m,k) * wt[k,n]: second operand stored [K,N]
                xd, xv = _dev(torch, x, dtype)
                wd, wtv = _dev(torch, w.T.copy(), dtype)
                wv = wtv.T
                kw = dict(x_kmajor=1, w_kmajor=0, ldx=xd.shape[1], ldw=wd.shape[1])
            else:                    # out[M,N] = xt[k,m]^T wt[k,n]: both stored with k slow
                xd, xtv = _dev(torch, x.T.copy(), dtype)
                wd, wtv = _dev(torch, w.T.copy(), dtype)
                xv, wv = xtv.T, wtv.T
                kw = dict(x_kmajor=0, w_kmajor=0, ldx=xd.shape[1], ldw=wd.shape[1])
            Xs.append(xd)
            Ws.append(wd)
            outs.append(torch.full((M, _ld(N)), 7.0, dtype=torch.float32, device="cuda"))
            wants.append(OL.linear_fwd(xv, wv, np.zeros(N)))
            bounds.append(2 * K * EPS32 * (np.abs(xv) @ np.abs(wv).T))
        ops.hydra_op_gemm(dtype, M, N, K, Xs, Ws, outs, ldo=_ld(N), out_f32=True, tile=tile, **kw)
        torch.cuda.synchronize()
        for g in range(G):
            o = outs[g].cpu().numpy().astype(np.float64)
            _check(o[:, :N], wants[g], bounds[g], False, f"{layout} dtype={dtype} tile={tile} {(M, N, K)} g={g}")
            assert np.all(o[:, N:] == 7.0), "columns beyond N were written"


# Linear layers of the measured workloads at their full size: (problems grouped, tokens, in, out).
FULL_SIZE_LAYERS = [(8, 512, 4096, 4096),      # workload 1: eight models' hidden layer in one launch
                    (2, 16384, 768, 2304),     # workload 2: the QKV projection (two of its four models)
                    (1, 16384, 4096, 11008)]   # workload 4: the FFN up-projection of a 4096-wide decoder


@pytest.mark.parametrize("layout", ["fwd", "dgrad", "wgrad"])
@pytest.mark.parametrize("layer", FULL_SIZE_LAYERS)
def test_gemm_at_the_workloads_full_size(torch, ops, layer, layout):
    """Element by element against the oracle's Linear at shapes that reach what the small cases cannot: more than 8
    tile rows (several bands of the tile order), grids whose tile count is not a multiple of the 8 XCDs, k-loops of
    128 to 512 sub-tiles, and the split sum over 16384 tokens of a weight gradient with few output tiles.
    The kernels add 16 products per MFMA step and chain K/16 steps in fp32 (K/(16 S) per range, then S partial sums,
    when split), so |error| <= (K/16 + 16) * 2^-24 * sum_k |x||w|; the test allows twice that with the sum bounded by
    |x_m| |w_n| (Cauchy-Schwarz), which costs no second matrix product."""
    G, T, d_in, d_out = layer
    r = np.random.default_rng(T + d_in + len(layout))
    if layout == "fwd":
        M, N, K = T, d_out, d_in
    elif layout == "dgrad":
        M, N, K = T, d_in, d_out
    else:
        M, N, K = d_out, d_in, T
    Xs, Ws, outs, wss, refs = [], [], [], [], []
    split = ops.hydra_op_gemm_split_k(M, N, K) if layout == "wgrad" else 1
    for g in range(G):
        # operands as the kernel reads them: X(m,k), W(n,k); stored k-major or k-slow depending on the layout
        x = r.standard_normal((M, K), dtype=np.float32)
        w = r.standard_normal((N, K), dtype=np.float32) * np.float32(1.0 / math.sqrt(K))
        xk, wk = layout != "wgrad", layout == "fwd"
        xt = torch.from_numpy(x if xk else np.ascontiguousarray(x.T)).to(torch.bfloat16)
        wt = torch.from_numpy(w if wk else np.ascontiguousarray(w.T)).to(torch.bfloat16)
        xv, wv = xt.to(torch.float64).numpy(), wt.to(torch.float64).numpy()
        xv, wv = (xv if xk else xv.T), (wv if wk else wv.T)
        refs.append((OL.linear_fwd(xv, wv, np.zeros(N)), np.linalg.norm(xv, axis=1), np.linalg.norm(wv, axis=1)))
        Xs.append(xt.cuda()), Ws.append(wt.cuda())
        outs.append(torch.full((M, N), 7.0, dtype=torch.float32, device="cuda"))
        if split > 1:
            wss.append(torch.zeros(ops.hydra_op_gemm_split_ws_bytes(M, N, K, N), dtype=torch.uint8, device="cuda"))
    assert (split > 1) == (layout == "wgrad" and layer[1] == 16384 and d_in == 768), "which shapes split is part of the design"
    ops.hydra_op_gemm(1, M, N, K, Xs, Ws, outs, x_kmajor=int(xk), w_kmajor=int(wk), ldx=Xs[0].shape[1], ldw=Ws[0].shape[1],
                      ldo=N, out_f32=True, ws=wss or None)
    torch.cuda.synchronize()
    for g in range(G):
        want, nx, nw = refs[g]
        got = outs[g].cpu().numpy().astype(np.float64)
        tol = 2 * (K / 16 + 16) * EPS32 * np.outer(nx, nw)
        bad = np.abs(got - want) > tol
        assert not bad.any(), f"{layout} {layer} g={g}: {bad.sum()} of {bad.size} off, worst {np.abs(got - want).max()}"
        # the tolerance is a small fraction of the values it guards: a dropped MFMA step would not pass
        assert np.median(tol) < 0.03 * np.sqrt((want ** 2).mean())


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("act", [1, 2])
def test_gemm_forward_epilogue_bias_activation_preactivation(torch, ops, dtype, act):
    r = np.random.default_rng(7 + dtype + act)
    M, N, K, G = 96, 200, 136, 2
    tdt = torch.bfloat16 if dtype else torch.float32
    Xs, Ws, Bs, outs, pres, want_h, want_z, bounds = [], [], [], [], [], [], [], []
    for g in range(G):
        xd, xv = _dev(torch, r.normal(size=(M, K)), dtype)
        wd, wv = _dev(torch, r.normal(size=(N, K)) / math.sqrt(K), dtype)
        b = r.normal(size=N).astype(np.float32)
        Xs.append(xd), Ws.append(wd), Bs.append(torch.from_numpy(b).cuda())
        outs.append(torch.zeros((M, _ld(N)), dtype=tdt, device="cuda"))
        pres.append(torch.zeros((M, _ld(N)), dtype=tdt, device="cuda"))
        z = OL.linear_fwd(xv, wv, b.astype(np.float64))
        want_z.append(z)
        want_h.append(OL.relu(z) if act == 1 else OL.gelu(z))
        bounds.append(2 * K * EPS32 * (np.abs(xv) @ np.abs(wv).T) + 1e-6)
    ops.hydra_op_gemm(dtype, M, N, K, Xs, Ws, outs, x_kmajor=1, w_kmajor=1, ldx=Xs[0].shape[1], ldw=Ws[0].shape[1],
                      ldo=_ld(N), bias=Bs, pre=pres, act=act)
    torch.cuda.synchronize()
    for g in range(G):
        _check(pres[g][:, :N].double().cpu().numpy(), want_z[g], bounds[g], dtype == 1, "pre-activation")
        # the activation is applied to the fp32 value before rounding; allow one more bf16 ulp of the input side
        _check(outs[g][:, :N].double().cpu().numpy(), want_h[g], 1.2 * bounds[g] + 1e-6, dtype == 1, "activation")


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("act", [1, 2])
def test_gemm_dgrad_epilogue_gate_and_residual(torch, ops, dtype, act):
    r = np.random.default_rng(17 + dtype + act)
    M, N, K, G = 72, 136, 200, 2
    tdt = torch.bfloat16 if dtype else torch.float32
    Xs, Ws, gates, resids, outs, wants, bounds = [], [], [], [], [], [], []
    for g in range(G):
        xd, xv = _dev(torch, r.normal(size=(M, K)), dtype)
        wd, wtv = _dev(torch, (r.normal(size=(N, K)) / math.sqrt(K)).T.copy(), dtype)
        zd, zv = _dev(torch, r.normal(size=(M, N)) + 0.3, dtype)
        rd, rv = _dev(torch, r.normal(size=(M, N)), dtype)
        Xs.append(xd), Ws.append(wd), gates.append(zd), resids.append(rd)
        outs.append(torch.zeros((M, _ld(N)), dtype=tdt, device="cuda"))
        grad = OL.relu_grad(zv) if act == 1 else OL.gelu_grad(zv)
        wants.append((xv @ wtv) * grad + rv)
        bounds.append(2 * K * EPS32 * (np.abs(xv) @ np.abs(wtv)) * np.abs(grad) + 2e-6)
    ops.hydra_op_gemm(dtype, M, N, K, Xs, Ws, outs, x_kmajor=1, w_kmajor=0, ldx=Xs[0].shape[1], ldw=Ws[0].shape[1],
                      ldo=_ld(N), gate=gates, ldg=_ld(N), resid=resids, ldr=_ld(N), act=act)
    torch.cuda.synchronize()
    for g in range(G):
        _check(outs[g][:, :N].double().cpu().numpy(), wants[g], bounds[g], dtype == 1, "dgrad epilogue")


def test_gelu_and_its_derivative_over_the_whole_range(torch, ops):
    """The kernels' GeLU (an exponential of a fitted polynomial) and GeLU' (rational erf) against the oracle's erf
    forms on a dense grid of arguments from -10 to 10: fp32 products with an identity weight (and, for the
    derivative, a product that is exactly 1), so that the epilogue's function is all that is measured."""
    M, N = 520, 64
    z = np.linspace(-10.0, 10.0, M * N).reshape(M, N)
    zd, zv = _dev(torch, z, 0)
    eye = torch.eye(N, dtype=torch.float32, device="cuda")
    out = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    ops.hydra_op_gemm(0, M, N, N, [zd], [eye], [out], x_kmajor=1, w_kmajor=1, ldx=N, ldw=N, ldo=N, act=2)
    torch.cuda.synchronize()
    want = OL.gelu(zv)
    err = np.abs(out.double().cpu().numpy() - want)
    assert (err <= 6e-7 + 2.0 ** -23 * np.abs(want)).all(), f"GeLU off by {err.max()} at z = {zv.flat[err.argmax()]}"
    ones = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    ones[:, 0] = 1.0
    w = torch.zeros((N, N), dtype=torch.float32, device="cuda")
    w[0, :] = 1.0                                          # (ones @ w)[m, n] = 1
    ops.hydra_op_gemm(0, M, N, N, [ones], [w], [out], x_kmajor=1, w_kmajor=0, ldx=N, ldw=N, ldo=N, gate=[zd], ldg=N, act=2)
    torch.cuda.synchronize()
    want = OL.gelu_grad(zv)
    err = np.abs(out.double().cpu().numpy() - want)
    assert (err <= 6e-7 + 2.0 ** -23 * np.abs(want)).all(), f"GeLU' off by {err.max()} at z = {zv.flat[err.argmax()]}"


@pytest.mark.parametrize("layout", ["fwd", "dgrad", "wgrad"])
def test_gemm_result_is_independent_of_tile_and_group(torch, ops, layout):
    """Bitwise: the same problem alone, inside a group, and with every tile shape gives the same bits (tile 1
    loads bf16 operands straight into LDS, tile 4 is the same tile staged through registers)."""
    r = np.random.default_rng(5)
    M, N, K = 160, 264, 328
    xk, wk = layout != "wgrad", layout == "fwd"

    def operands():
        x, w = r.normal(size=(M, K)), r.normal(size=(N, K))
        return _dev(torch, x if xk else x.T.copy(), 1)[0], _dev(torch, w if wk else w.T.copy(), 1)[0]
    xd, wd = operands()
    other_x, other_w = operands()
    ref = None
    for tile in (1, 2, 3, 4):
        for group in ([(xd, wd)], [(other_x, other_w), (xd, wd), (other_x, wd)]):
            outs = [torch.zeros((M, _ld(N)), dtype=torch.float32, device="cuda") for _ in group]
            ops.hydra_op_gemm(1, M, N, K, [g[0] for g in group], [g[1] for g in group], outs, x_kmajor=int(xk),
                              w_kmajor=int(wk), ldx=xd.shape[1], ldw=wd.shape[1], ldo=_ld(N), out_f32=True, tile=tile)
            torch.cuda.synchronize()
            mine = outs[[i for i, g in enumerate(group) if g[0] is xd and g[1] is wd][0]].cpu().numpy()
            if ref is None:
                ref = mine
            assert np.array_equal(ref, mine), f"{layout}: tile {tile}, group of {len(group)}"


@pytest.mark.parametrize("combo", ["bias", "bias_resid", "bias_gelu_pre", "bias_relu_pre", "none", "resid", "gate_gelu",
                                   "gate_relu_resid", "fwd_plain", "fwd_resid_only"])
def test_gemm_epilogue_variants_on_big_tiles_agree_with_the_general_path(torch, ops, combo):
    """256x256 tiles of the direct-to-LDS kernel (tile 1) run waves whose block lies inside the matrix through an
    epilogue without bounds checks, compiled as straight-line code for the operand combinations the trainers use (the
    last two combinations take its version that tests the operands at run time); the
    register-staged 256x256 tile (tile 4) runs every wave through the general epilogue.  Both must give the same bits
    for every element, also in the ragged last tiles (M = 600: rows 512.. of the third tile row; N = 520), and match the
    oracle's Linear with the same epilogue."""
    r = np.random.default_rng(100 + len(combo) + sum(map(ord, combo)))
    fwd = combo.startswith(("bias", "fwd"))   # forward layout (W k-contiguous) or input-gradient layout
    M, N, K, G = 600, 520, 264, 2
    act = 2 if "gelu" in combo else (1 if "relu" in combo else 0)
    Xs, Ws, want, extra = [], [], [], dict(bias=[], pre=[], gate=[], resid=[])
    for g in range(G):
        xd, xv = _dev(torch, r.normal(size=(M, K)), 1)
        w = r.normal(size=(N, K)) / math.sqrt(K)
        wd, wv = _dev(torch, w if fwd else w.T.copy(), 1)
        Xs.append(xd), Ws.append(wd)
        z = xv @ (wv.T if fwd else wv)
        if "bias" in combo:
            b = r.normal(size=N).astype(np.float32)
            extra["bias"].append(torch.from_numpy(b).cuda())
            z = z + b.astype(np.float64)
        v = z
        if "pre" in combo:
            extra["pre"].append(torch.zeros((M, _ld(N)), dtype=torch.bfloat16, device="cuda"))
        if "gate" in combo:
            gd, gv = _dev(torch, r.normal(size=(M, N)) + 0.3, 1)
            extra["gate"].append(gd)
            v = v * (OL.gelu_grad(gv) if act == 2 else OL.relu_grad(gv))
        elif act:
            v = OL.gelu(v) if act == 2 else OL.relu(v)
        if "resid" in combo:
            rd, rv = _dev(torch, r.normal(size=(M, N)), 1)
            extra["resid"].append(rd)
            v = v + rv
        want.append(v)
    kw = {k: v for k, v in extra.items() if v}
    got = {}
    for tile in (1, 4):
        outs = [torch.zeros((M, _ld(N)), dtype=torch.bfloat16, device="cuda") for _ in range(G)]
        if "pre" in kw:
            kw["pre"] = [torch.zeros((M, _ld(N)), dtype=torch.bfloat16, device="cuda") for _ in range(G)]
        ops.hydra_op_gemm(1, M, N, K, Xs, Ws, outs, x_kmajor=1, w_kmajor=int(fwd), ldx=Xs[0].shape[1], ldw=Ws[0].shape[1],
                          ldo=_ld(N), ldg=_ld(N), ldr=_ld(N), act=act, tile=tile, **kw)
        torch.cuda.synchronize()
        got[tile] = ([o[:, :N].float().cpu().numpy() for o in outs],
                     [p_[:, :N].float().cpu().numpy() for p_ in kw.get("pre", [])])
    for g in range(G):
        assert np.array_equal(got[1][0][g], got[4][0][g]), f"{combo}: outputs differ between the two epilogue paths"
        for a_, b_ in zip(got[1][1], got[4][1]):
            assert np.array_equal(a_, b_), f"{combo}: stored pre-activations differ between the two epilogue paths"
        scale = np.abs(want[g]).max()
        assert np.abs(got[1][0][g] - want[g]).max() <= 2 ** -7 * scale + 1e-3, combo   # bf16 output rounding + bf16 operands


def test_gemm_rejects_bad_arguments(torch, ops):
    from paper_2107_06469_amd.hydra import HydraError
    x = torch.zeros((8, 16), dtype=torch.bfloat16, device="cuda")
    o = torch.zeros((8, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(HydraError):   # ldx not a multiple of 8 elements
        ops.hydra_op_gemm(1, 8, 8, 12, [x], [x], [o], x_kmajor=1, w_kmajor=1, ldx=12, ldw=16, ldo=8, out_f32=True)
    with pytest.raises(HydraError):   # ldo smaller than N
        ops.hydra_op_gemm(1, 8, 16, 16, [x], [x], [o], x_kmajor=1, w_kmajor=1, ldx=16, ldw=16, ldo=8, out_f32=True)
    with pytest.raises(HydraError):   # group too large
        ops.hydra_op_gemm(1, 8, 8, 16, [x] * 17, [x] * 17, [o] * 17, x_kmajor=1, w_kmajor=1, ldx=16, ldw=16, ldo=8,
                          out_f32=True)


@pytest.mark.parametrize("dtype", [0, 1])
def test_colsum(torch, ops, dtype):
    r = np.random.default_rng(3)
    for (M, N) in [(32, 10), (512, 1000), (97, 130), (2000, 72)]:
        srcs, outs, wants, parts = [], [], [], []
        for g in range(2):
            d, v = _dev(torch, r.normal(size=(M, N)), dtype)
            srcs.append(d), wants.append(v.sum(axis=0))
            outs.append(torch.zeros(N, dtype=torch.float32, device="cuda"))
            parts.append(torch.zeros(max(1, ops.hydra_op_colsum_part_floats(M, N)), dtype=torch.float32, device="cuda"))
        ops.hydra_op_colsum(dtype, M, N, srcs[0].shape[1], srcs, outs, parts)
        torch.cuda.synchronize()
        for g in range(2):
            assert np.allclose(outs[g].cpu().numpy(), wants[g], rtol=0, atol=2 * M * EPS32 * 4)


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("shape", [(32, 10), (64, 1000), (24, 30522), (5, 8190), (7, 1003, "tight"), (3, 40000)])
def test_softmax_cross_entropy(torch, ops, dtype, shape):
    """Rows of up to 32768 padded logits with aligned storage take the register-resident kernel (three sizes of it:
    up to 1024, 8192, 32768); a row pitch that is not a multiple of 4 ("tight") and longer rows take the three-pass one."""
    M, Cn = shape[:2]
    r = np.random.default_rng(Cn)
    ldz = Cn if len(shape) > 2 else _ld(Cn)
    y = r.integers(0, Cn, size=M).astype(np.int32)
    yd = torch.from_numpy(y).cuda()
    logits, dzs, rls, ls, wants = [], [], [], [], []
    for g in range(2):
        z = (r.normal(size=(M, Cn)) * 3).astype(np.float32)
        zd = torch.zeros((M, ldz), dtype=torch.float32)
        zd[:, :Cn] = torch.from_numpy(z)
        logits.append(zd.cuda())
        dzs.append(torch.full((M, ldz), 5.0, dtype=torch.bfloat16 if dtype else torch.float32, device="cuda"))
        rls.append(torch.zeros(M, dtype=torch.float32, device="cuda"))
        ls.append(torch.zeros(1, dtype=torch.float32, device="cuda"))
        wants.append(OL.softmax_ce(z.astype(np.float64), y))
    ops.hydra_op_softmax_ce(dtype, M, Cn, ldz, ldz, 1.0 / M, logits, yd, dzs, rls, ls)
    torch.cuda.synchronize()
    for g in range(2):
        loss, dz = wants[g]
        assert float(ls[g].item()) == pytest.approx(loss, rel=5e-6)
        got = dzs[g].double().cpu().numpy()
        tol = 4e-7 / M + (2.0 ** -8 if dtype else 5e-6) * np.abs(dz)
        assert np.all(np.abs(got[:, :Cn] - dz) <= tol)
        assert np.all(got[:, Cn:] == 0.0)


@pytest.mark.parametrize("opt", [0, 1])
@pytest.mark.parametrize("w16", [False, True])
def test_optimizer_step_matches_oracle(torch, ops, opt, w16):
    from oracle import optim as OO
    r = np.random.default_rng(11 + opt)
    n, G = 4096 + 64, 3
    P, Gr, Ms, Vs, W16, hp_rows, want = [], [], [], [], [], [], []
    for g in range(G):
        p = r.normal(size=n).astype(np.float32)
        gr = (r.normal(size=n) * 0.1).astype(np.float32)
        gr[::7] = 0.0
        m = (r.normal(size=n) * 0.05).astype(np.float32)
        v = (r.random(size=n) * 0.01).astype(np.float32)
        t = 3 + g
        hp = dict(opt=opt, lr=1e-3 * (g + 1), beta1=0.9, beta2=0.999, eps=1e-8, warmup_steps=0)
        P.append(torch.from_numpy(p).cuda()), Gr.append(torch.from_numpy(gr).cuda())
        Ms.append(torch.from_numpy(m).cuda()), Vs.append(torch.from_numpy(v).cuda())
        W16.append(torch.zeros(n, dtype=torch.bfloat16, device="cuda"))
        hp_rows.append((hp["lr"], 0.9, 0.999, 1e-8, 1 / (1 - 0.9 ** t), 1 / (1 - 0.999 ** t)))
        pw, mw, vw = p.copy(), m.copy(), v.copy()
        OO.update_tensor(hp, t, pw, gr.astype(np.float64), mw, vw)
        want.append((pw, mw, vw))
    ops.hydra_op_optim(opt, n, P, Gr, Ms, Vs, W16 if w16 else None, hp_rows)
    torch.cuda.synchronize()
    for g in range(G):
        pw, mw, vw = want[g]
        assert np.allclose(P[g].cpu().numpy(), pw, rtol=3e-6, atol=1e-7)
        if opt == 1:
            assert np.allclose(Ms[g].cpu().numpy(), mw, rtol=1e-6, atol=2e-8)   # fp32 rounding of a two-term sum
            assert np.allclose(Vs[g].cpu().numpy(), vw, rtol=1e-6, atol=1e-10)
        if w16:
            assert torch.equal(W16[g], P[g].to(torch.bfloat16))


@pytest.mark.parametrize("opt", [0, 1])
@pytest.mark.parametrize("dtype_name,tile,M,N,K", [("bf16", 1, 384, 512, 200), ("bf16", 2, 200, 264, 96), ("bf16", 3, 72, 320, 50),
                                                   ("f32", 2, 136, 200, 64), ("f32", 0, 72, 40, 30)])
def test_update_in_the_gradient_kernel_equals_gradient_then_optimizer(torch, ops, opt, dtype_name, tile, M, N, K):
    # the same gradient GEMM, once stored and applied by the optimizer kernel, once applied in the epilogue:
    # parameters, moments and working copy must agree bit for bit (and the optimizer kernel is checked
    # against the oracle above)
    bf = dtype_name == "bf16"
    td = torch.bfloat16 if bf else torch.float32
    dt = ops.BF16 if bf else ops.F32
    r = np.random.default_rng(M + N + K + opt)
    G, E = 2, (8 if bf else 4)
    ldx, ldw = (M + E - 1) // E * E, (N + E - 1) // E * E
    n = M * N
    X = [torch.from_numpy(r.normal(size=(K, ldx)).astype(np.float32)).cuda().to(td) for _ in range(G)]
    W = [torch.from_numpy(r.normal(size=(K, ldw)).astype(np.float32)).cuda().to(td) for _ in range(G)]
    hp_rows = [(1e-3 * (g + 1), 0.9, 0.999, 1e-8, 1 / (1 - 0.9 ** (2 + g)), 1 / (1 - 0.999 ** (2 + g))) for g in range(G)]

    def state():
        rr = np.random.default_rng(5)
        return ([torch.from_numpy(rr.normal(size=n).astype(np.float32)).cuda() for _ in range(G)],
                [torch.from_numpy((rr.normal(size=n) * 0.05).astype(np.float32)).cuda() for _ in range(G)],
                [torch.from_numpy((rr.random(size=n) * 0.01).astype(np.float32)).cuda() for _ in range(G)],
                [torch.zeros(n, dtype=torch.bfloat16, device="cuda") for _ in range(G)] if bf else None)
    # two-kernel path
    P1, M1, V1, W1 = state()
    Gr = [torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(G)]
    ops.hydra_op_gemm(dt, M, N, K, X, W, Gr, x_kmajor=False, w_kmajor=False, ldx=ldx, ldw=ldw, ldo=N, out_f32=True, tile=tile)
    ops.hydra_op_optim(opt, n, P1, Gr, M1, V1, W1, hp_rows)
    # fused path, with and without storing the gradient
    P2, M2, V2, W2 = state()
    ops.hydra_op_gemm_update(dt, M, N, K, X, W, opt, P2, M2, V2, W2, hp_rows, ldx=ldx, ldw=ldw, ldo=N, tile=tile)
    P3, M3, V3, W3 = state()
    Gr3 = [torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(G)]
    ops.hydra_op_gemm_update(dt, M, N, K, X, W, opt, P3, M3, V3, W3, hp_rows, ldx=ldx, ldw=ldw, ldo=N, out=Gr3, tile=tile)
    torch.cuda.synchronize()
    for g in range(G):
        assert not torch.equal(P1[g], state()[0][g])
        for a, b, c in ((P1, P2, P3), (M1, M2, M3), (V1, V2, V3)) + (((W1, W2, W3),) if bf else ()):
            assert torch.equal(a[g], b[g]) and torch.equal(a[g], c[g])
        assert torch.equal(Gr[g], Gr3[g])


@pytest.mark.parametrize("dtype_name,tile,M,N,K", [("bf16", 1, 520, 264, 1000), ("bf16", 2, 200, 136, 300), ("bf16", 3, 72, 320, 70),
                                                   ("f32", 2, 136, 200, 90), ("f32", 1, 300, 256, 129)])
def test_weight_gradient_gemm_also_gives_the_bias_gradient(torch, ops, dtype_name, tile, M, N, K):
    # rowsum[m] = sum_k X(k, m): with X = dY this is the bias gradient.  Reference: fp64 sum of the operand
    # values; the result must also not depend on the tile shape.
    bf = dtype_name == "bf16"
    td = torch.bfloat16 if bf else torch.float32
    dt = ops.BF16 if bf else ops.F32
    r = np.random.default_rng(M + K)
    E = 8 if bf else 4
    ldx, ldw = (M + E - 1) // E * E, (N + E - 1) // E * E
    G = 2
    X = [torch.from_numpy(r.normal(size=(K, ldx)).astype(np.float32)).cuda().to(td) for _ in range(G)]
    W = [torch.from_numpy(r.normal(size=(K, ldw)).astype(np.float32)).cuda().to(td) for _ in range(G)]
    out = [torch.zeros(M, N, dtype=torch.float32, device="cuda") for _ in range(G)]
    got = {}
    for t in (tile, 3):
        rs = [torch.full((M,), 7.0, dtype=torch.float32, device="cuda") for _ in range(G)]
        ops.hydra_op_gemm(dt, M, N, K, X, W, out, x_kmajor=False, w_kmajor=False, ldx=ldx, ldw=ldw, ldo=N, out_f32=True,
                          tile=t, rowsum=rs)
        torch.cuda.synchronize()
        got[t] = [x.cpu().numpy() for x in rs]
    for g in range(G):
        xs = X[g].to(torch.float64).cpu().numpy()[:, :M]
        want = xs.sum(axis=0)
        bound = 2 * K * 2.0 ** -24 * np.abs(xs).sum(axis=0) + 1e-30
        assert np.all(np.abs(got[tile][g] - want) <= bound)
        assert np.array_equal(got[tile][g], got[3][g])
    from paper_2107_06469_amd.hydra import HydraError
    with pytest.raises(HydraError):   # only the weight-gradient layout has row sums
        ops.hydra_op_gemm(dt, M, N, K, X, W, out, x_kmajor=True, w_kmajor=True, ldx=ldx, ldw=ldw, ldo=N, out_f32=True, rowsum=rs)


def test_seeded_initialisation_is_bit_identical_to_the_oracle(torch, ops):
    for (seed, model, tensor, n, a) in [(42, 0, 0, 65536, math.sqrt(6 / 256)), (42, 7, 33, 1000, 0.02 * math.sqrt(3)),
                                        (2 ** 40 + 5, 15, 2, 4097, 1.0)]:
        d = torch.zeros(n, dtype=torch.float32, device="cuda")
        ops.hydra_op_init_uniform(d, n, seed, ORNG.tensor_stream(model, tensor), float(np.float32(a)))
        torch.cuda.synchronize()
        want = ORNG.uniform_sym(seed, ORNG.tensor_stream(model, tensor), n, np.float32(a))
        assert np.array_equal(d.cpu().numpy(), want)


def test_bf16_cast_rounds_to_nearest_even(torch, ops):
    r = np.random.default_rng(1)
    x = r.normal(size=5000).astype(np.float32)
    x[:4] = np.array([1.00390625, 1.01171875, -1.00390625, 3.0e38], dtype=np.float32)   # ties and a large value
    s = torch.from_numpy(x).cuda()
    d = torch.zeros(5000, dtype=torch.bfloat16, device="cuda")
    ops.hydra_op_cast_bf16(s, d, 5000)
    torch.cuda.synchronize()
    # reference rounding done with integer arithmetic on the host
    bits = x.view(np.uint32).astype(np.uint64)
    rounded = ((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16).astype(np.uint16)
    assert np.array_equal(d.view(torch.int16).cpu().numpy().view(np.uint16), rounded)


def test_split_weight_gradient_matches_oracle_and_ignores_tile_and_group(torch, ops):
    """A weight gradient with few output tiles and a long sum over the tokens is cut into S ranges of k (S from the
    shape alone) when scratch is given: the result stays within the fp32 dot-product bound of the oracle, equals the
    one-chain result up to that bound, and is bit-identical for every tile code, alone or inside a group; the update
    epilogue applied by the second launch equals gradient-then-optimizer bit for bit; the bias gradient (row sums) too."""
    r = np.random.default_rng(11)
    M, N, K = 264, 200, 4100            # weight [M, N], K tokens (ragged everywhere)
    S = ops.hydra_op_gemm_split_k(M, N, K)
    assert S > 1 and ops.hydra_op_gemm_split_k(4096, 4096, 512) == 1 and ops.hydra_op_gemm_split_k(M, N, 1000) == 1
    nbytes = ops.hydra_op_gemm_split_ws_bytes(M, N, K, _ld(N))
    assert nbytes == (S * M * _ld(N) + S * M) * 4

    def operands():
        dy, x = r.normal(size=(K, M)), r.normal(size=(K, N))
        a, av = _dev(torch, dy, 1)
        b, bv = _dev(torch, x, 1)
        return a, b, av, bv
    dyd, xd, dyv, xv = operands()
    o_dy, o_x, _, _ = operands()
    want = dyv.T @ xv
    bound = 2 * K * EPS32 * (np.abs(dyv).T @ np.abs(xv))

    def ws(n):
        return [torch.empty(nbytes, dtype=torch.uint8, device="cuda") for _ in range(n)]
    ref = None
    for tile in (0, 1, 2, 4):
        for group in ([(dyd, xd)], [(o_dy, o_x), (dyd, xd), (o_dy, xd)]):
            outs = [torch.zeros((M, _ld(N)), dtype=torch.float32, device="cuda") for _ in group]
            rs = [torch.zeros(M, dtype=torch.float32, device="cuda") for _ in group]
            ops.hydra_op_gemm(1, M, N, K, [g[0] for g in group], [g[1] for g in group], outs, x_kmajor=0, w_kmajor=0,
                              ldx=dyd.shape[1], ldw=xd.shape[1], ldo=_ld(N), out_f32=True, tile=tile, rowsum=rs, ws=ws(len(group)))
            torch.cuda.synchronize()
            i = [j for j, g in enumerate(group) if g[0] is dyd and g[1] is xd][0]
            mine = (outs[i].cpu().numpy(), rs[i].cpu().numpy())
            if ref is None:
                ref = mine
            assert np.array_equal(ref[0], mine[0]) and np.array_equal(ref[1], mine[1]), f"tile {tile}, group of {len(group)}"
    assert np.all(np.abs(ref[0][:, :N] - want) <= bound)
    assert np.all(np.abs(ref[1] - dyv.sum(axis=0)) <= 2 * K * EPS32 * np.abs(dyv).sum(axis=0))
    one = torch.zeros((M, _ld(N)), dtype=torch.float32, device="cuda")
    ops.hydra_op_gemm(1, M, N, K, [dyd], [xd], [one], x_kmajor=0, w_kmajor=0, ldx=dyd.shape[1], ldw=xd.shape[1], ldo=_ld(N),
                      out_f32=True)
    torch.cuda.synchronize()
    assert np.all(np.abs(one.cpu().numpy()[:, :N] - ref[0][:, :N]) <= 2 * bound)
    # update in the second launch == stored gradient followed by the optimizer kernel
    n = M * _ld(N)
    hp = [(1e-3, 0.9, 0.999, 1e-8, 10.0, 1000.0)]
    P0 = torch.randn(n, device="cuda")
    P1, P2 = P0.clone(), P0.clone()
    M1, V1 = torch.rand(n, device="cuda") * 1e-3, torch.rand(n, device="cuda") * 1e-6
    M2, V2 = M1.clone(), V1.clone()
    W1 = torch.zeros(n, dtype=torch.bfloat16, device="cuda")
    W2 = torch.zeros_like(W1)
    G1 = torch.from_numpy(ref[0]).cuda().reshape(-1).contiguous()
    ops.hydra_op_optim(1, n, [P1], [G1], [M1], [V1], [W1], hp)
    ops.hydra_op_gemm_update(1, M, N, K, [dyd], [xd], 1, [P2], [M2], [V2], [W2], hp, ldx=dyd.shape[1], ldw=xd.shape[1],
                             ldo=_ld(N), ws=ws(1))
    torch.cuda.synchronize()
    keep = np.zeros((M, _ld(N)), dtype=bool)
    keep[:, :N] = True
    keep = keep.reshape(-1)
    for a, b in ((P1, P2), (M1, M2), (V1, V2), (W1.float(), W2.float())):
        assert np.array_equal(a.cpu().numpy()[keep], b.cpu().numpy()[keep])
