"""Counter-based uniform numbers for weight initialisation (oracle side).

Generator: SplitMix64 (Steele, Lea, Flood, "Fast splittable pseudorandom
number generators", OOPSLA 2014): state advances by the 64-bit golden-ratio
constant, output is a three-round xor-shift-multiply finaliser of the state.
Because the state after n steps is key + n*GOLDEN, output n can be computed
directly from (key, n) with no sequential dependence.

  key(seed, stream)  = SM(SM(seed, 0) xor stream, 0)      SM(s, n) = n-th output from state s
  bits(seed,stream,i)= SM(key, i)
  u                  = (bits >> 40) * 2**-24               24-bit uniform in [0,1)
  sym(a)             = round_fp32(u * (2a) - a)            one rounding (a is an fp32 value)

Test infrastructure only; written independently of the GPU library's generator.
"""
from __future__ import annotations

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _finalise(z: np.ndarray) -> np.ndarray:
    z = z.astype(np.uint64, copy=True)
    z ^= z >> np.uint64(30)
    z *= _M1
    z ^= z >> np.uint64(27)
    z *= _M2
    z ^= z >> np.uint64(31)
    return z


def splitmix64_at(state, n) -> np.ndarray:
    """n-th output (n = 0 is the first) of SplitMix64 started from `state`."""
    with np.errstate(over="ignore"):
        s = np.asarray(state, dtype=np.uint64)
        n = np.asarray(n, dtype=np.uint64)
        return _finalise(s + (n + np.uint64(1)) * _GOLDEN)


def stream_key(seed: int, stream: int) -> np.uint64:
    a = splitmix64_at(np.uint64(seed), 0)
    return splitmix64_at(a ^ np.uint64(stream), 0)


def uniform24(seed: int, stream: int, n: int, start: int = 0) -> np.ndarray:
    """u[i] in [0,1) with 24 random bits, as fp64 (exactly representable)."""
    key = stream_key(seed, stream)
    idx = np.arange(start, start + n, dtype=np.uint64)
    bits = splitmix64_at(key, idx)
    return (bits >> np.uint64(40)).astype(np.float64) * 2.0 ** -24


def uniform_sym(seed: int, stream: int, n: int, a) -> np.ndarray:
    """fp32 values uniform on [-a, a): u*(2a) - a evaluated exactly, rounded once to fp32."""
    a32 = np.float32(a)
    u = uniform24(seed, stream, n)
    return (u * (2.0 * np.float64(a32)) - np.float64(a32)).astype(np.float32)


def tensor_stream(model: int, tensor: int) -> int:
    """Stream id of tensor `tensor` (canonical order) of model `model`."""
    return (model << 20) | tensor
