"""Stand-alone rates of the library's kernels at the shapes of the measured workloads, each against the peak that
bounds it (HBM 8 TB/s for the streaming kernels, 2.5 PFLOP/s dense bf16 MFMA for the products).

    python3 -m paper_2107_06469_amd.kernel_rates            # all kernels
    python3 -m paper_2107_06469_amd.kernel_rates gemm adam  # only the kernels whose label contains a word

Every launch goes through the operator entry points of the C library on torch's current stream; a rate is the
algorithmic work of one launch (flops of the products, or bytes that must cross HBM once) over the best of five
timings of ten launches each (HIP events on that stream).  Inputs are random, outputs are not checked here.
"""
from __future__ import annotations

import sys

HBM_PEAK = 8.0e12
MFMA_PEAK = 2.5e15
ROUNDS, REPS = 5, 10


def _time(f):
    import torch
    f()
    torch.cuda.synchronize()
    best = float("inf")
    for _ in range(ROUNDS):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(REPS):
            f()
        b.record()
        torch.cuda.synchronize()
        best = min(best, a.elapsed_time(b) * 1e-3 / REPS)
    return best


def _report(label, seconds, flops=0.0, nbytes=0.0):
    if flops:
        rate, peak, unit = flops / seconds / 1e12, MFMA_PEAK / 1e12, "TFLOP/s"
    else:
        rate, peak, unit = nbytes / seconds / 1e9, HBM_PEAK / 1e9, "GB/s"
    print(f"{label:112s} {seconds * 1e6:9.1f} us {rate:9.0f} {unit:8s} {rate / peak:6.3f} of peak", flush=True)


def _gemms(want):
    import torch
    from . import ops
    bf = torch.bfloat16
    # (label, models in one launch, tokens, out features, in features, forward epilogue, input-gradient epilogue) with
    # the epilogues the trainers give these layers: "act" = bias, GeLU and the stored pre-activation; "resid" = bias and
    # the residual stream added; "gate" = the product times GeLU'(stored pre-activation of the layer before)
    shapes = [("workload 1 layer", 8, 512, 4096, 4096, "act", "gate"), ("workload 2 QKV", 4, 16384, 2304, 768, "bias", "plain"),
              ("workload 2 FFN in", 4, 16384, 3072, 768, "act", "plain"), ("workload 2 FFN out", 4, 16384, 768, 3072, "resid", "gate"),
              ("workload 3 FFN in", 16, 8192, 4096, 1024, "act", "plain"), ("workload 4 FFN in", 2, 16384, 11008, 4096, "act", "plain")]
    for name, G, M, N, K, fwd_epi, bwd_epi in shapes:
        if not want(f"gemm {name}"):
            continue
        X = [torch.randn(M, K, device="cuda").to(bf) for _ in range(G)]
        W = [(torch.randn(N, K, device="cuda") * 0.02).to(bf) for _ in range(G)]
        O = [torch.zeros(M, N, dtype=bf, device="cuda") for _ in range(G)]
        DY = [torch.randn(M, N, device="cuda").to(bf) for _ in range(G)]
        DX = [torch.zeros(M, K, dtype=bf, device="cuda") for _ in range(G)]
        GW = [torch.zeros(N, K, device="cuda") for _ in range(G)]
        bias = [torch.zeros(N, device="cuda") for _ in range(G)]
        ws = None
        if ops.hydra_op_gemm_split_k(N, K, M) > 1:
            ws = [torch.zeros(ops.hydra_op_gemm_split_ws_bytes(N, K, M, K), dtype=torch.uint8, device="cuda") for _ in range(G)]
        fl = 2.0 * M * N * K * G
        tag = f"gemm {name}: {G} x [{M} tokens, {K} -> {N}]"
        fkw, flabel = dict(bias=bias), " forward (+bias)"
        if fwd_epi == "act":
            PRE = [torch.zeros(M, N, dtype=bf, device="cuda") for _ in range(G)]
            fkw, flabel = dict(bias=bias, pre=PRE, act=ops.EPI_GELU), " forward (+bias, GeLU, pre-activation stored)"
        elif fwd_epi == "resid":
            RES = [torch.randn(M, N, device="cuda").to(bf) for _ in range(G)]
            fkw, flabel = dict(bias=bias, resid=RES, ldr=N), " forward (+bias, +residual)"
        bkw, blabel = dict(), " input gradient"
        if bwd_epi == "gate":
            GATE = [torch.randn(M, K, device="cuda").to(bf) for _ in range(G)]
            bkw, blabel = dict(gate=GATE, ldg=K, act=ops.EPI_GELU), " input gradient (x GeLU' of the stored pre-activation)"
        _report(tag + flabel, _time(lambda: ops.hydra_op_gemm(
            ops.BF16, M, N, K, X, W, O, x_kmajor=True, w_kmajor=True, ldx=K, ldw=K, ldo=N, **fkw)), flops=fl)
        _report(tag + blabel, _time(lambda: ops.hydra_op_gemm(
            ops.BF16, M, K, N, DY, W, DX, x_kmajor=True, w_kmajor=False, ldx=N, ldw=K, ldo=K, **bkw)), flops=fl)
        del fkw, bkw
        _report(tag + " weight gradient (fp32 out" + (", split over k)" if ws else ")"), _time(lambda: ops.hydra_op_gemm(
            ops.BF16, N, K, M, DY, X, GW, x_kmajor=False, w_kmajor=False, ldx=N, ldw=K, ldo=K, out_f32=True, ws=ws)), flops=fl)
        del X, W, O, DY, DX, GW, ws
        torch.cuda.empty_cache()


def _update(want):
    import torch
    from . import ops
    bf = torch.bfloat16
    G, d, B = 8, 4096, 512
    n = d * d
    hp = [(1e-3, 0.9, 0.999, 1e-8, 10.0, 1000.0)] * G
    if want("update gemm") or want("adam"):
        p = [torch.randn(n, device="cuda") for _ in range(G)]
        m = [torch.zeros(n, device="cuda") for _ in range(G)]
        v = [torch.zeros(n, device="cuda") for _ in range(G)]
        w16 = [t.to(bf) for t in p]
    if want("update gemm"):
        dz = [torch.randn(B, d, device="cuda").to(bf) for _ in range(G)]
        h = [torch.randn(B, d, device="cuda").to(bf) for _ in range(G)]
        t = _time(lambda: ops.hydra_op_gemm_update(ops.BF16, d, d, B, dz, h, 1, p, m, v, w16, hp, ldx=d, ldw=d, ldo=d))
        # p, m, v read and written in fp32, the bf16 copy written, the two operands read
        _report(f"update gemm workload 1: {G} x [{d} x {d}, {B} tokens], Adam in the epilogue", t,
                nbytes=G * (26.0 * n + 2.0 * B * 2 * d))
    if want("adam"):
        g = [torch.randn(n, device="cuda") for _ in range(G)]
        t = _time(lambda: ops.hydra_op_optim(1, n, p, g, m, v, w16, hp))
        _report(f"adam streaming: {G} x {n} parameters (fp32 p, g, m, v; bf16 copy)", t, nbytes=G * 30.0 * n)


def _layernorm(want):
    import torch
    from . import ops
    bf = torch.bfloat16
    for name, G, rows, d in [("workload 2", 4, 16384, 768), ("workload 3", 16, 8192, 1024), ("workload 4", 2, 16384, 4096)]:
        if not want(f"layernorm {name}"):
            continue
        x = [torch.randn(rows, d, device="cuda").to(bf) for _ in range(G)]
        y = [torch.zeros(rows, d, dtype=bf, device="cuda") for _ in range(G)]
        dy = [torch.randn(rows, d, device="cuda").to(bf) for _ in range(G)]
        add = [torch.randn(rows, d, device="cuda").to(bf) for _ in range(G)]
        dx = [torch.zeros(rows, d, dtype=bf, device="cuda") for _ in range(G)]
        gam = [torch.ones(d, device="cuda") for _ in range(G)]
        bet = [torch.zeros(d, device="cuda") for _ in range(G)]
        mu = [torch.zeros(rows, device="cuda") for _ in range(G)]
        rs = [torch.zeros(rows, device="cuda") for _ in range(G)]
        part = [torch.zeros(ops.hydra_op_layernorm_part_floats(rows, d), device="cuda") for _ in range(G)]
        dg = [torch.zeros(d, device="cuda") for _ in range(G)]
        db = [torch.zeros(d, device="cuda") for _ in range(G)]
        tag = f"layernorm {name}: {G} x [{rows} x {d}]"
        _report(tag + " forward", _time(lambda: ops.hydra_op_layernorm_fwd(ops.BF16, rows, d, d, 1e-5, x, y, gam, bet, mu, rs)),
                nbytes=4.0 * G * rows * d)
        _report(tag + " backward (+ residual gradient, + gamma/beta reduction)", _time(lambda: ops.hydra_op_layernorm_bwd(
            ops.BF16, rows, d, d, x, dy, add, dx, gam, mu, rs, part, dg, db)), nbytes=8.0 * G * rows * d)
        del x, y, dy, add, dx
        torch.cuda.empty_cache()


def _loss(want):
    import torch
    from . import ops
    for name, G, M, V in [("workload 1", 8, 512, 1000), ("workload 2", 4, 2432, 30522), ("workload 4", 2, 16384, 32000)]:
        if not want(f"softmax ce {name}"):
            continue
        ld = (V + 7) // 8 * 8            # the trainer pads rows to 8 elements
        z = [torch.randn(M, ld, device="cuda") for _ in range(G)]
        dz = [torch.zeros(M, ld, dtype=torch.bfloat16, device="cuda") for _ in range(G)]
        y = torch.randint(0, V, (M,), dtype=torch.int32, device="cuda")
        rl = [torch.zeros(M, device="cuda") for _ in range(G)]
        ls = [torch.zeros(1, device="cuda") for _ in range(G)]
        t = _time(lambda: ops.hydra_op_softmax_ce(ops.BF16, M, V, ld, ld, 1.0 / M, z, y, dz, rl, ls))
        _report(f"softmax ce {name}: {G} x [{M} x {V}] fp32 logits -> bf16 gradient", t, nbytes=6.0 * G * M * V)
        del z, dz
        torch.cuda.empty_cache()


def _attention(want):
    import torch
    from . import ops
    bf = torch.bfloat16
    for name, G, B, S, H, DH, causal in [("workload 2", 4, 32, 512, 12, 64, 0), ("workload 3", 16, 16, 512, 16, 64, 0),
                                         ("workload 4", 2, 8, 2048, 32, 128, 1)]:
        if not want(f"attention {name}"):
            continue
        d = H * DH
        qkv = [torch.randn(B * S, 3 * d, device="cuda").to(bf) for _ in range(G)]
        o = [torch.zeros(B * S, d, dtype=bf, device="cuda") for _ in range(G)]
        do = [torch.randn(B * S, d, device="cuda").to(bf) for _ in range(G)]
        lse = [torch.zeros(B * H * S, device="cuda") for _ in range(G)]
        delta = [torch.zeros(B * H * S, device="cuda") for _ in range(G)]
        dqkv = [torch.zeros(B * S, 3 * d, dtype=bf, device="cuda") for _ in range(G)]
        sc = DH ** -0.5
        fl = 4.0 * B * H * S * S * DH * (0.5 if causal else 1.0) * G
        tag = f"attention {name}: {G} x [{B} x {H} heads, S={S}, dh={DH}{', causal' if causal else ''}]"
        _report(tag + " forward", _time(lambda: ops.hydra_op_attention_fwd(B, S, H, DH, 3 * d, d, causal, sc, qkv, o, lse)), flops=fl)
        _report(tag + " backward (algorithmic 2.5 x forward)", _time(lambda: ops.hydra_op_attention_bwd(
            B, S, H, DH, 3 * d, d, causal, sc, qkv, o, do, lse, delta, dqkv)), flops=2.5 * fl)
        del qkv, o, do, dqkv
        torch.cuda.empty_cache()


def main(words):
    import torch
    if not torch.cuda.is_available():
        sys.exit("kernel_rates: no HIP device")
    want = (lambda label: any(w in label for w in words)) if words else (lambda label: True)
    print(f"# {torch.cuda.get_device_name(0)}; best of {ROUNDS} x {REPS} launches; peaks: HBM {HBM_PEAK / 1e12:.0f} TB/s, "
          f"bf16 MFMA {MFMA_PEAK / 1e15:.1f} PFLOP/s")
    _gemms(want)
    _update(want)
    _layernorm(want)
    _loss(want)
    _attention(want)


if __name__ == "__main__":
    main(sys.argv[1:])
