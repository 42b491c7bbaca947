"""Seeded synthetic inputs shaped like decode-time SwiGLU MLP layers.

This module serves both the CPU oracle's tests and the GPU path's tests and
benchmark, and holds none of the method's arithmetic: it only draws random
tensors and rounds them to the storage type.

Recipe (one MLP layer, ``layer`` = l):
    X      [M, d_model]     ~ N(0, 1)                seed_X     = seed
    W_gate [d_ff, d_model]  ~ N(0, 1/d_model)        seed_Wgate = seed + 1 + 3 l
    W_up   [d_ff, d_model]  ~ N(0, 1/d_model)        seed_Wup   = seed + 2 + 3 l
    W_down [d_ff, d_model]  ~ N(0, 1/d_ff)           seed_Wdown = seed + 3 + 3 l
(std = 1/sqrt(fan_in)), rounded to bfloat16 with round-to-nearest-even, or
kept as fp32 for the fp32 test mode.

Two generators:
  * ``mlp_inputs``: a counter-based generator (splitmix64 of (seed, index) ->
    Box-Muller) in numpy.  Bit-reproducible anywhere; used for every stored
    expected value and for small and medium shapes.
  * ``mlp_inputs_torch``: torch's seeded generator on a given device, for the
    multi-hundred-megabyte shapes where the numpy generator would take
    minutes.  Reproducible for a given torch build and device type; the host
    copy of the very same tensors is what the oracle is given.

bfloat16 tensors travel as uint16 bit patterns in numpy (numpy has no
bfloat16); ``to_torch``/``to_numpy`` convert without changing a bit.
"""
from __future__ import annotations

import math

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _splitmix64(x: np.ndarray) -> np.ndarray:
    """One splitmix64 output step applied elementwise to uint64 counters."""
    with np.errstate(over="ignore"):
        z = x + _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def standard_normal(seed: int, n: int, chunk: int = 1 << 22) -> np.ndarray:
    """n draws of N(0,1) as float64; draw i depends only on (seed, i)."""
    out = np.empty(n, np.float64)
    with np.errstate(over="ignore"):
        key = _splitmix64(np.array([seed], np.uint64))[0]
        for lo in range(0, n, chunk):
            hi = min(n, lo + chunk)
            idx = np.arange(lo, hi, dtype=np.uint64)
            a = _splitmix64(key ^ (idx * np.uint64(2)))
            b = _splitmix64(key ^ (idx * np.uint64(2) + np.uint64(1)))
            # 53-bit uniforms; u1 in (0, 1], u2 in [0, 1)
            u1 = ((a >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)
            u2 = (b >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)
            out[lo:hi] = np.sqrt(-2.0 * np.log(u1)) * np.cos((2.0 * math.pi) * u2)
    return out


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    quiet = (u >> np.uint32(16)) | np.uint32(0x0040)
    return np.where(nan, quiet, rounded).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float32, exact."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def as_f64(a: np.ndarray) -> np.ndarray:
    """Exact float64 view of a uint16 (bf16 bits), float16 or float32 array."""
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return np.asarray(a, dtype=np.float64)


def tensor(seed: int, shape, std: float, dtype: str = "bf16") -> np.ndarray:
    n = int(np.prod(shape))
    f = (standard_normal(seed, n) * std).astype(np.float32).reshape(shape)
    if dtype == "bf16":
        return f32_to_bf16_bits(f)
    if dtype == "fp32":
        return f
    if dtype == "fp16":
        return f.astype(np.float16)      # round-to-nearest-even
    raise ValueError("dtype must be 'bf16', 'fp16' or 'fp32'")


def layer_seeds(seed: int, layer: int):
    return {"X": seed, "Wg": seed + 1 + 3 * layer, "Wu": seed + 2 + 3 * layer,
            "Wd": seed + 3 + 3 * layer}


def mlp_inputs(M: int, d_model: int, d_ff: int, seed: int = 0, layer: int = 0,
               dtype: str = "bf16"):
    """Counter-based inputs of one MLP layer as numpy arrays (see module doc)."""
    s = layer_seeds(seed, layer)
    return {
        "X": tensor(s["X"], (M, d_model), 1.0, dtype),
        "Wg": tensor(s["Wg"], (d_ff, d_model), 1.0 / math.sqrt(d_model), dtype),
        "Wu": tensor(s["Wu"], (d_ff, d_model), 1.0 / math.sqrt(d_model), dtype),
        "Wd": tensor(s["Wd"], (d_ff, d_model), 1.0 / math.sqrt(d_ff), dtype),
    }


# ---- torch interchange (imported lazily so numpy-only users need no torch) ----

def to_torch(a: np.ndarray, device="cpu"):
    """numpy uint16 bf16 bits -> torch.bfloat16; float16 -> torch.float16; float32 -> torch.float32."""
    import torch
    if a.dtype == np.uint16:
        t = torch.from_numpy(np.ascontiguousarray(a).view(np.int16).copy()).view(torch.bfloat16)
    elif a.dtype == np.float16:
        t = torch.from_numpy(np.ascontiguousarray(a).copy())
    else:
        t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32).copy())
    return t.to(device)


def to_numpy(t) -> np.ndarray:
    """torch.bfloat16 -> numpy uint16 bit patterns; torch.float16 -> float16; torch.float32 -> float32."""
    import torch
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    if t.dtype == torch.float16:
        return t.numpy().copy()
    return t.to(torch.float32).numpy().copy()


def mlp_inputs_torch(M: int, d_model: int, d_ff: int, seed: int = 0, layer: int = 0,
                     dtype: str = "bf16", device="cuda"):
    """Same recipe from torch's seeded generator on ``device`` (large shapes)."""
    import torch
    tdt = {"bf16": torch.bfloat16, "fp16": torch.float16, "fp32": torch.float32}[dtype]
    s = layer_seeds(seed, layer)

    def draw(sd, shape, std):
        g = torch.Generator(device=device)
        g.manual_seed(int(sd))
        return (torch.randn(shape, generator=g, device=device, dtype=torch.float32) * std).to(tdt)

    return {
        "X": draw(s["X"], (M, d_model), 1.0),
        "Wg": draw(s["Wg"], (d_ff, d_model), 1.0 / math.sqrt(d_model)),
        "Wu": draw(s["Wu"], (d_ff, d_model), 1.0 / math.sqrt(d_model)),
        "Wd": draw(s["Wd"], (d_ff, d_model), 1.0 / math.sqrt(d_ff)),
    }
