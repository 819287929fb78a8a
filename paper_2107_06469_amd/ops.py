"""ctypes binding of include/hydra_ops.h (argument marshalling only).

Arguments are torch CUDA tensors (device memory is PyTorch's job here); every
function enqueues the named C entry point on torch's current stream.
"""
from __future__ import annotations

import ctypes as C
from typing import Optional, Sequence

from .hydra import HydraError, lib

F32, BF16 = 0, 1
EPI_NONE, EPI_RELU, EPI_GELU = 0, 1, 2


class hydra_gemm_desc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("dtype", "M", "N", "K", "x_kmajor", "w_kmajor", "ldx", "ldw", "ldo", "ldg", "ldr",
                                       "act", "out_f32", "tile", "G")] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("X", "W", "bias", "out", "pre", "gate", "resid", "rowsum", "ws")] + \
               [("ws_bytes", C.c_size_t)]


_ready = False


def _L():
    global _ready
    L = lib()
    if not _ready:
        vp, pp = C.c_void_p, C.POINTER(C.c_void_p)
        L.hydra_op_gemm.argtypes = [C.POINTER(hydra_gemm_desc), vp]
        L.hydra_op_gemm_update.argtypes = [C.POINTER(hydra_gemm_desc), C.c_int, pp, pp, pp, pp, C.POINTER(C.c_double), vp]
        L.hydra_op_colsum.argtypes = [C.c_int] * 5 + [pp, pp, pp, vp]
        L.hydra_op_colsum_part_floats.argtypes = [C.c_int, C.c_int]
        L.hydra_op_colsum_part_floats.restype = C.c_size_t
        L.hydra_op_colsum_noalloc.argtypes = [C.c_int] * 5 + [pp, pp, vp]
        L.hydra_op_colsum_noalloc_max_floats.argtypes = []
        L.hydra_op_colsum_noalloc_max_floats.restype = C.c_size_t
        L.hydra_op_gemm_split_k.argtypes = [C.c_int] * 3
        L.hydra_op_gemm_split_ws_bytes.argtypes = [C.c_int] * 4
        L.hydra_op_gemm_split_ws_bytes.restype = C.c_size_t
        L.hydra_op_softmax_ce.argtypes = [C.c_int] * 5 + [C.c_float, C.c_int, pp, vp, pp, pp, pp, vp]
        L.hydra_op_optim.argtypes = [C.c_int, C.c_size_t, C.c_int, pp, pp, pp, pp, pp, C.POINTER(C.c_double), vp]
        L.hydra_op_init_uniform.argtypes = [vp, C.c_size_t, C.c_uint64, C.c_uint64, C.c_float, vp]
        L.hydra_op_cast_bf16.argtypes = [vp, vp, C.c_size_t, vp]
        L.hydra_op_layernorm_fwd.argtypes = [C.c_int] * 4 + [C.c_float, C.c_int] + [pp] * 6 + [vp]
        L.hydra_op_layernorm_bwd.argtypes = [C.c_int] * 5 + [pp] * 10 + [vp]
        L.hydra_op_layernorm_part_floats.argtypes = [C.c_int, C.c_int]
        L.hydra_op_layernorm_part_floats.restype = C.c_size_t
        L.hydra_op_attention_fwd.argtypes = [C.c_int] * 7 + [C.c_float, C.c_int, pp, pp, pp, vp]
        L.hydra_op_attention_bwd.argtypes = [C.c_int] * 7 + [C.c_float, C.c_int] + [pp] * 6 + [vp]
        L.hydra_op_embed_fwd.argtypes = [C.c_int] * 6 + [vp, pp, pp, pp, vp]
        L.hydra_op_embed_bwd.argtypes = [C.c_int] * 8 + [vp, vp, pp, pp, pp, vp]
        L.hydra_op_empty_launches.argtypes = [C.c_int, vp]
        L.hydra_ops_last_error.restype = C.c_char_p
        _ready = True
    return L


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _tab(ts: Optional[Sequence]):
    if ts is None:
        return None
    return (C.c_void_p * len(ts))(*[t.data_ptr() for t in ts])


def _check(st: int):
    if st != 0:
        raise HydraError(st, _L().hydra_ops_last_error().decode())


def hydra_op_gemm(dtype, M, N, K, X, W, out, *, x_kmajor, w_kmajor, ldx, ldw, ldo, bias=None, pre=None, gate=None,
                  resid=None, ldg=0, ldr=0, act=EPI_NONE, out_f32=False, tile=0, rowsum=None, ws=None):
    """ws: optional per-problem scratch tensors (uint8, hydra_op_gemm_split_ws_bytes bytes) that allow a split sum over k."""
    d = hydra_gemm_desc()
    d.dtype, d.M, d.N, d.K, d.x_kmajor, d.w_kmajor = dtype, M, N, K, int(x_kmajor), int(w_kmajor)
    d.ldx, d.ldw, d.ldo, d.ldg, d.ldr, d.act, d.out_f32, d.tile, d.G = ldx, ldw, ldo, ldg, ldr, act, int(out_f32), tile, len(X)
    tabs = [_tab(t) for t in (X, W, bias, out, pre, gate, resid, rowsum, ws)]
    for name, t in zip(("X", "W", "bias", "out", "pre", "gate", "resid", "rowsum", "ws"), tabs):
        if t is not None:
            setattr(d, name, C.cast(t, C.POINTER(C.c_void_p)))
    d.ws_bytes = 0 if ws is None else min(int(t.numel() * t.element_size()) for t in ws)
    _check(_L().hydra_op_gemm(C.byref(d), _stream()))


def hydra_op_gemm_split_k(M, N, K) -> int:
    return int(_L().hydra_op_gemm_split_k(M, N, K))


def hydra_op_gemm_split_ws_bytes(M, N, K, ldo) -> int:
    return int(_L().hydra_op_gemm_split_ws_bytes(M, N, K, ldo))


def hydra_op_gemm_update(dtype, M, N, K, X, W, opt, p, m, v, w16, hp_rows, *, ldx, ldw, ldo, out=None, tile=0, rowsum=None,
                         ws=None):
    """Weight gradient dW[M,N] = sum_k X(k,m) W(k,n) with the optimizer step of hydra_op_optim in its epilogue."""
    d = hydra_gemm_desc()
    d.dtype, d.M, d.N, d.K, d.x_kmajor, d.w_kmajor = dtype, M, N, K, 0, 0
    d.ldx, d.ldw, d.ldo, d.ldg, d.ldr, d.act, d.out_f32, d.tile, d.G = ldx, ldw, ldo, 0, 0, EPI_NONE, 1, tile, len(X)
    tabs = [_tab(t) for t in (X, W, out, rowsum, ws)]
    for name, t in zip(("X", "W", "out", "rowsum", "ws"), tabs):
        if t is not None:
            setattr(d, name, C.cast(t, C.POINTER(C.c_void_p)))
    d.ws_bytes = 0 if ws is None else min(int(t.numel() * t.element_size()) for t in ws)
    flat = (C.c_double * (6 * len(p)))(*[float(x) for row in hp_rows for x in row])
    _check(_L().hydra_op_gemm_update(C.byref(d), opt, _tab(p), _tab(m), _tab(v), _tab(w16), flat, _stream()))


def hydra_op_colsum_part_floats(M, N) -> int:
    return int(_L().hydra_op_colsum_part_floats(M, N))


def hydra_op_colsum(dtype, M, N, ld, src, out, part=None):
    _check(_L().hydra_op_colsum(dtype, M, N, ld, len(src), _tab(src), _tab(out), _tab(part), _stream()))


def hydra_op_empty_launches(n: int):
    _check(_L().hydra_op_empty_launches(n, _stream()))


def hydra_op_colsum_noalloc(dtype, M, N, ld, src, out):
    _check(_L().hydra_op_colsum_noalloc(dtype, M, N, ld, len(src), _tab(src), _tab(out), _stream()))


def hydra_op_colsum_noalloc_max_floats() -> int:
    return int(_L().hydra_op_colsum_noalloc_max_floats())


def hydra_op_softmax_ce(dtype, M, Cn, ldz, lddz, inv_n, logits, labels, dz, rowloss, loss):
    _check(_L().hydra_op_softmax_ce(dtype, M, Cn, ldz, lddz, inv_n, len(logits), _tab(logits), C.c_void_p(labels.data_ptr()),
                                    _tab(dz), _tab(rowloss), _tab(loss), _stream()))


def hydra_op_optim(opt, n, p, g, m, v, w16, hp_rows):
    """hp_rows: per problem (lr, b1, b2, eps, bc1, bc2)."""
    flat = (C.c_double * (6 * len(p)))(*[float(x) for row in hp_rows for x in row])
    _check(_L().hydra_op_optim(opt, n, len(p), _tab(p), _tab(g), _tab(m), _tab(v), _tab(w16), flat, _stream()))


def hydra_op_init_uniform(dst, n, seed, stream_id, a):
    _check(_L().hydra_op_init_uniform(C.c_void_p(dst.data_ptr()), n, C.c_uint64(seed), C.c_uint64(stream_id), a, _stream()))


def hydra_op_cast_bf16(src, dst, n):
    _check(_L().hydra_op_cast_bf16(C.c_void_p(src.data_ptr()), C.c_void_p(dst.data_ptr()), n, _stream()))


def hydra_op_layernorm_fwd(dtype, rows, d, ld, eps, x, y, gamma, beta, mean, rstd):
    _check(_L().hydra_op_layernorm_fwd(dtype, rows, d, ld, eps, len(x), _tab(x), _tab(y), _tab(gamma), _tab(beta),
                                       _tab(mean), _tab(rstd), _stream()))


def hydra_op_layernorm_part_floats(rows, d) -> int:
    return int(_L().hydra_op_layernorm_part_floats(rows, d))


def hydra_op_layernorm_bwd(dtype, rows, d, ld, x, dy, add, dx, gamma, mean, rstd, part, dgamma, dbeta):
    _check(_L().hydra_op_layernorm_bwd(dtype, rows, d, ld, len(x), _tab(x), _tab(dy), _tab(add), _tab(dx), _tab(gamma),
                                       _tab(mean), _tab(rstd), _tab(part), _tab(dgamma), _tab(dbeta), _stream()))


def hydra_op_attention_fwd(B, S, H, DH, ld_qkv, ld_o, causal, scale, qkv, o, lse):
    _check(_L().hydra_op_attention_fwd(B, S, H, DH, ld_qkv, ld_o, int(causal), scale, len(qkv), _tab(qkv), _tab(o),
                                       _tab(lse), _stream()))


def hydra_op_attention_bwd(B, S, H, DH, ld_qkv, ld_o, causal, scale, qkv, o, dout, lse, delta, dqkv):
    _check(_L().hydra_op_attention_bwd(B, S, H, DH, ld_qkv, ld_o, int(causal), scale, len(qkv), _tab(qkv), _tab(o),
                                       _tab(dout), _tab(lse), _tab(delta), _tab(dqkv), _stream()))


def hydra_op_embed_fwd(dtype, tokens, S, d, ld, ids, tok, pos, x):
    _check(_L().hydra_op_embed_fwd(dtype, tokens, S, d, ld, len(x), C.c_void_p(ids.data_ptr()), _tab(tok), _tab(pos),
                                   _tab(x), _stream()))


def hydra_op_embed_bwd(dtype, V, S, S_table, B, d, ld, row_ptr, positions, dx, dtok, dpos):
    _check(_L().hydra_op_embed_bwd(dtype, V, S, S_table, B, d, ld, len(dx), C.c_void_p(row_ptr.data_ptr()),
                                   C.c_void_p(positions.data_ptr()), _tab(dx), _tab(dtok), _tab(dpos), _stream()))
