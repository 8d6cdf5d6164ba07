"""Seeded synthetic inputs for the agent-attention forward pass.

This module holds no arithmetic of the method itself: it only produces random
tensors and rounds them to a storage type.  Both the GPU library's callers and
the CPU oracle's callers take their inputs from here, so the two sides consume
identical bits.

Generator: counter-based.  Element i of stream (seed, stream_id) uses
splitmix64 of two consecutive counters for a Box-Muller pair, so any element can
be regenerated independently of the others and the result does not depend on the
device, the torch version or the thread count.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 231208874

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix64(x: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        z = (x + np.uint64(0x9E3779B97F4A7C15)) & _M64
        z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
        z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
        return z ^ (z >> np.uint64(31))


def _stream_key(seed: int, stream: int) -> np.uint64:
    k = _splitmix64(np.array([seed & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64))
    k = _splitmix64(k ^ np.uint64((stream * 0xD1342543DE82EF95) & 0xFFFFFFFFFFFFFFFF))
    return k[0]


def uniform01(seed: int, stream: int, count: int, offset: int = 0) -> np.ndarray:
    """float64 uniforms in (0, 1), 53 bits, element i depends only on (seed, stream, offset+i)."""
    key = _stream_key(seed, stream)
    with np.errstate(over="ignore"):
        ctr = np.arange(offset, offset + count, dtype=np.uint64) + key
    bits = _splitmix64(ctr) >> np.uint64(11)
    return (bits.astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed: int, stream: int, count: int, std: float = 1.0, mean: float = 0.0) -> np.ndarray:
    """float32 N(mean, std^2) by Box-Muller on the counter-based uniforms."""
    half = (count + 1) // 2
    u = uniform01(seed, stream, 2 * half)
    r = np.sqrt(-2.0 * np.log(u[0::2]))
    th = (2.0 * np.pi) * u[1::2]
    z = np.empty(2 * half, dtype=np.float64)
    z[0::2] = r * np.cos(th)
    z[1::2] = r * np.sin(th)
    return (z[:count] * std + mean).astype(np.float32)


def uniform(seed: int, stream: int, count: int, lo: float, hi: float) -> np.ndarray:
    return (lo + (hi - lo) * uniform01(seed, stream, count)).astype(np.float32)


# ---------------------------------------------------------------------------
# storage types: values are rounded once (nearest even); `bits` is what the
# device consumes, `exact` is the same values as float64 for the oracle.
# ---------------------------------------------------------------------------
DTYPES = ("f32", "f16", "bf16")


def to_storage(x32: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 values to `dtype`; returns float32 / float16 / uint16(bf16 bits)."""
    x32 = np.ascontiguousarray(x32, dtype=np.float32)
    if dtype == "f32":
        return x32
    if dtype == "f16":
        return x32.astype(np.float16)
    if dtype == "bf16":
        b = x32.view(np.uint32)
        rounded = b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
        return (rounded >> np.uint32(16)).astype(np.uint16)
    raise ValueError(dtype)


def to_float64(stored: np.ndarray, dtype: str) -> np.ndarray:
    """Exact float64 image of stored values."""
    if dtype == "bf16":
        return (stored.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return stored.astype(np.float64)


@dataclass(frozen=True)
class Workload:
    name: str
    index: int          # position in the configuration list, used in stream ids
    batch: int
    heads: int
    grid: tuple         # (h, w) token grid, N = h*w
    d: int
    agent_grid: tuple   # (h_a, w_a) agent grid, n = h_a*w_a
    dtype: str
    std: float

    @property
    def N(self):
        return self.grid[0] * self.grid[1]

    @property
    def n(self):
        return self.agent_grid[0] * self.agent_grid[1]

    @property
    def units(self):
        return self.batch * self.heads


# The five evaluation shapes.  Shapes follow the paper's architecture tables
# (DeiT-T block, Swin-T stage 1 with 49 agents, Stable-Diffusion latent,
# high-resolution regime); values are i.i.d. Gaussians standing in for
# activations of trained networks.
WORKLOADS = {
    "tiny": Workload("tiny", 0, 1, 1, (14, 14), 32, (7, 7), "f32", 1.0),
    "deit_t": Workload("deit_t", 1, 64, 3, (14, 14), 64, (7, 7), "bf16", 0.5),
    "swin_t_s1": Workload("swin_t_s1", 2, 32, 3, (56, 56), 32, (7, 7), "bf16", 1.0),
    "sd_latent": Workload("sd_latent", 3, 2, 8, (64, 64), 40, (16, 16), "f16", 1.0),
    "highres": Workload("highres", 4, 1, 8, (128, 128), 64, (32, 32), "bf16", 1.0),
}

# tensor index inside a workload's stream id
T_Q, T_K, T_V = 0, 1, 2
T_B1_COL, T_B1_ROW, T_B1_BLK, T_B2_COL, T_B2_ROW, T_B2_BLK = 3, 4, 5, 6, 7, 8
T_DWC_W, T_DWC_B, T_A = 9, 10, 11


def make_tensor(shape, *, seed=BASE_SEED, stream=0, std=1.0, mean=0.0, dtype="f32"):
    count = int(np.prod(shape))
    x = normal(seed, stream, count, std=std, mean=mean).reshape(shape)
    return to_storage(x, dtype)


def make_qkv(wl: Workload, *, seed=BASE_SEED, units=None, scale_qk=1.0, v_mean=0.0):
    """Q, K, V of shape [units, N, d] in the workload's storage type.

    `units` truncates to the first units (batch*heads) -- the generator is
    counter based, so the first units of the full tensor are reproduced exactly.
    """
    u = wl.units if units is None else units
    shape = (u, wl.N, wl.d)
    out = {}
    for name, t in (("Q", T_Q), ("K", T_K), ("V", T_V)):
        std = wl.std * (scale_qk if name in ("Q", "K") else 1.0)
        mean = v_mean if name == "V" else 0.0
        out[name] = make_tensor(shape, seed=seed, stream=wl.index * 16 + t, std=std, mean=mean,
                                dtype=wl.dtype)
    return out


def make_module_params(heads, n, d, grid, *, blk=(7, 7), seed=BASE_SEED, index=0, bias_std=0.5):
    """Agent-bias components and DWC weights (float32).  The paper gives no
    initialisation; bias_std 0.5 makes the bias change the output measurably."""
    h, w = grid
    h0, w0 = blk
    s = index * 16

    def nrm(shape, t, std):
        return normal(seed, s + t, int(np.prod(shape)), std=std).reshape(shape)

    return {
        "b1_col": nrm((heads, n, w), T_B1_COL, bias_std),
        "b1_row": nrm((heads, n, h), T_B1_ROW, bias_std),
        "b1_blk": nrm((heads, n, h0, w0), T_B1_BLK, bias_std),
        "b2_col": nrm((heads, w, n), T_B2_COL, bias_std),
        "b2_row": nrm((heads, h, n), T_B2_ROW, bias_std),
        "b2_blk": nrm((heads, h0, w0, n), T_B2_BLK, bias_std),
        "dwc_w": uniform(seed, s + T_DWC_W, heads * d * 9, -1.0 / 3, 1.0 / 3).reshape(heads, d, 3, 3),
        "dwc_b": nrm((heads, d), T_DWC_B, 0.1),
    }
