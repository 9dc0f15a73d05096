"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module holds NONE of the method's arithmetic: it only produces the tensors
that stand in for the paper's workloads (linear-layer weights of LLaMA / OPT
shaped models, their input activations with a few large "outlier" channels, and
the calibration features captured on such activations, Section 2 and Section 5.1
of the paper).  Neither the CPU oracle nor the HIP library imports it; callers
hand the generated arrays to both.

Bulk tensors are produced by a counter-based generator (an integer hash of the
element index followed by a Box-Muller transform) written with torch ops, so any
sub-block (a few channels, a few rows) can be generated on its own and equals the
same block of the full tensor made on the same device.  Per-channel laws (a few
thousand numbers) come from numpy's Philox generator.
"""
from __future__ import annotations

import math
import zlib

import numpy as np
import torch

SEED = 20231015

_MASK64 = (1 << 64) - 1


def _s64(v: int) -> int:
    """Two's-complement view of an unsigned 64-bit constant as a Python int that fits int64."""
    v &= _MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


_C1 = _s64(0xBF58476D1CE4E5B9)
_C2 = _s64(0x94D049BB133111EB)
_GOLD = _s64(0x9E3779B97F4A7C15)


def stream_id(*parts) -> int:
    """Stable 31-bit stream number from a tuple of names / numbers."""
    text = "|".join(str(p) for p in parts).encode()
    return zlib.crc32(text) & 0x7FFFFFFF


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix64(x: torch.Tensor) -> torch.Tensor:
    """64-bit finaliser (xor-shift / multiply rounds) on wrapping int64 tensors."""
    x = x ^ _lsr(x, 30)
    x = x * _C1
    x = x ^ _lsr(x, 27)
    x = x * _C2
    x = x ^ _lsr(x, 31)
    return x


def _uniform(idx: torch.Tensor, stream: int, salt: int) -> torch.Tensor:
    """Uniform on (0, 1), 53 bits, as float64, a pure function of (idx, stream, salt)."""
    key = _s64((SEED * 0x1000003 + stream) * 0x9E3779B97F4A7C15 + salt * 0xD1B54A32D192ED03)
    h = _mix64(_mix64(idx * _GOLD + key) ^ key)
    return (_lsr(h, 11).to(torch.float64) + 0.5) * (2.0 ** -53)


def standard_normal(idx: torch.Tensor, stream: int) -> torch.Tensor:
    """N(0,1) deviates (float64) for int64 element indices `idx`."""
    u1 = _uniform(idx, stream, 1)
    u2 = _uniform(idx, stream, 2)
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)


def _index_grid(rows: torch.Tensor, cols: torch.Tensor, ncols_full: int) -> torch.Tensor:
    return rows.to(torch.int64)[:, None] * int(ncols_full) + cols.to(torch.int64)[None, :]


def _as_index(sel, n: int, device) -> torch.Tensor:
    if sel is None:
        return torch.arange(n, device=device, dtype=torch.int64)
    return torch.as_tensor(sel, device=device, dtype=torch.int64)


def normal_matrix(nrows: int, ncols: int, stream: int, *, col_scale=None, scale: float = 1.0,
                  dtype=torch.float16, device="cpu", rows=None, cols=None,
                  chunk_elems: int = 1 << 24) -> torch.Tensor:
    """dtype( z[r, c] * scale * col_scale[c] ) for the selected rows / cols of an
    [nrows, ncols] matrix of N(0,1) deviates; z depends only on (r, c, stream)."""
    device = torch.device(device)
    r = _as_index(rows, nrows, device)
    c = _as_index(cols, ncols, device)
    cs = None
    if col_scale is not None:
        cs_full = torch.as_tensor(np.asarray(col_scale, dtype=np.float64), device=device)
        cs = cs_full[c]
    out = torch.empty((r.numel(), c.numel()), dtype=dtype, device=device)
    step = max(1, chunk_elems // max(1, c.numel()))
    for lo in range(0, r.numel(), step):
        rr = r[lo:lo + step]
        z = standard_normal(_index_grid(rr, c, ncols), stream) * scale
        if cs is not None:
            z = z * cs[None, :]
        out[lo:lo + step] = z.to(dtype)
    return out


# ----------------------------------------------------------------------------------------
# per-channel laws
# ----------------------------------------------------------------------------------------
def _philox(stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[SEED, stream]))


def channel_scales(kind: str, K: int, stream: int) -> np.ndarray:
    """Per-input-channel activation scale (float64 [K]).

    'outlier20'  : 1 everywhere, x20 on round(0.01 K) random channels      (config 1)
    'lognormal'  : exp(g), g ~ N(0,1), x30 on round(0.005 K) random channels (configs 2-4)
    'student3'   : |t|, t ~ Student-t with 3 degrees of freedom              (config 5)
    'unit'       : 1
    """
    rng = _philox(stream)
    if kind == "unit":
        return np.ones(K)
    if kind == "outlier20":
        s = np.ones(K)
        n_out = int(round(0.01 * K))
        s[rng.choice(K, size=n_out, replace=False)] = 20.0
        return s
    if kind == "lognormal":
        s = np.exp(rng.standard_normal(K))
        n_out = int(round(0.005 * K))
        s[rng.choice(K, size=n_out, replace=False)] *= 30.0
        return s
    if kind == "student3":
        return np.abs(rng.standard_t(3.0, size=K))
    raise ValueError(kind)


# ----------------------------------------------------------------------------------------
# the five workload configurations
# ----------------------------------------------------------------------------------------
CONFIGS = {
    1: dict(name="single-512", dtype="f16", act="outlier20", T=256, block=64,
            layers={"linear": (512, 512)}, M=(16,)),
    2: dict(name="llama7b", dtype="f16", act="lognormal", T=128 * 2048, block=64,
            layers={"qkvo": (4096, 4096), "gate_up": (11008, 4096), "down": (4096, 11008)},
            M=(1, 8, 32)),
    3: dict(name="llama13b", dtype="f16", act="lognormal", T=128 * 2048, block=64,
            layers={"qkvo": (5120, 5120), "gate_up": (13824, 5120), "down": (5120, 13824)},
            M=(512, 2048)),
    4: dict(name="llama65b", dtype="bf16", act="lognormal", T=128 * 2048, block=64,
            layers={"qkvo": (8192, 8192), "gate_up": (22016, 8192), "down": (8192, 22016)},
            M=(1, 16, 128, 2048)),
    5: dict(name="opt66b", dtype="f16", act="student3", T=128 * 2048, block=64,
            layers={"qkv_out": (9216, 9216), "fc1": (36864, 9216), "fc2": (9216, 36864)},
            M=(1, 64, 1024)),
    # the GEMM shapes of the paper's own latency table (Table 5): decoder rows (16 tokens) and context rows
    # (16384 tokens); weights [N, K] = (output features, input features) of each "Input x Weights" row
    6: dict(name="table5", dtype="f16", act="lognormal", T=4096, block=64,
            layers={"qkv": (5376, 14336), "att_out": (14336, 1792), "ffn1": (7168, 14336), "ffn2": (14336, 7168)},
            M=(16, 16384)),
}

TORCH_DTYPE = {"f16": torch.float16, "bf16": torch.bfloat16}


def weights(cfg: int, layer: str, *, instance: int = 0, device="cpu", rows=None, cols=None,
            shape=None) -> torch.Tensor:
    """W[N, K] ~ N(0, std = K^-1/2), rounded once to the config dtype."""
    c = CONFIGS[cfg]
    N, K = shape if shape is not None else c["layers"][layer]
    return normal_matrix(N, K, stream_id("W", cfg, layer, instance), scale=K ** -0.5,
                         dtype=TORCH_DTYPE[c["dtype"]], device=device, rows=rows, cols=cols)


def act_scales(cfg: int, layer: str, K: int | None = None) -> np.ndarray:
    c = CONFIGS[cfg]
    if K is None:
        K = c["layers"][layer][1]
    return channel_scales(c["act"], K, stream_id("scale", cfg, layer))


def activations(cfg: int, layer: str, M: int, *, device="cpu", rows=None, cols=None,
                K: int | None = None) -> torch.Tensor:
    """Inference activations X[M, K]: z * per-channel scale (same law as the calibration set)."""
    c = CONFIGS[cfg]
    if K is None:
        K = c["layers"][layer][1]
    return normal_matrix(M, K, stream_id("X", cfg, layer), col_scale=act_scales(cfg, layer, K),
                         dtype=TORCH_DTYPE[c["dtype"]], device=device, rows=rows, cols=cols)


def calibration(cfg: int, layer: str, *, T: int | None = None, device="cpu", rows=None,
                cols=None, K: int | None = None) -> torch.Tensor:
    """Calibration features Xc[T, K] (all sequences pooled), same law as `activations`."""
    c = CONFIGS[cfg]
    if K is None:
        K = c["layers"][layer][1]
    if T is None:
        T = c["T"]
    return normal_matrix(T, K, stream_id("Xc", cfg, layer), col_scale=act_scales(cfg, layer, K),
                         dtype=TORCH_DTYPE[c["dtype"]], device=device, rows=rows, cols=cols)


def default_alpha(T: int) -> float:
    """The value of alpha used by the benchmarks: T^-1/2, which turns alpha * ||X_c||_2 into
    the channel RMS (the paper prints no value for alpha)."""
    return 1.0 / math.sqrt(float(T))
