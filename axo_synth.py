"""Seeded synthetic inputs for the 3D-tensor-parallel FC shard GEMMs.

This module only manufactures input bytes and names workloads.  It holds none
of the method's arithmetic: no matrix product, no epilogue, no shard
arithmetic beyond slicing a generated global tensor.  Both the CPU oracle's
tests and the HIP path's tests/bench draw their inputs from here, so both
sides always see the same bf16 bit patterns.

Generator: counter based.  Element `idx` of tensor stream `s` under `seed`
takes two 64-bit words from splitmix64 over the counter
`(seed, s, idx)`, maps them to uniforms, applies the Box-Muller transform in
fp64, scales by sigma, rounds to fp32 and then to bf16 (round to nearest,
ties to even).  Because every element is addressed by its global index, a
shard cut from a global tensor equals the same region generated on its own.

Workloads follow the paper's GPT shapes (Table 1 hidden sizes, sequence
length 2048; Section 3.2 for the grid decomposition); values stand in for
real activations / weights: X, dY ~ N(0,1), W, bias ~ N(0,0.02).
"""
from __future__ import annotations

import dataclasses
import os
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Optional, Tuple

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)

# tensor streams (fixed draw order X, W, dY, bias)
STREAM_X, STREAM_W, STREAM_DY, STREAM_BIAS = 0, 1, 2, 3
SIGMA_ACT = 1.0
SIGMA_W = 0.02


def _workers() -> int:
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    return max(1, min(16, n))


def _splitmix64(x: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser (Steele, Lea, Flood 2014), vectorised, wrap-around uint64."""
    with np.errstate(over="ignore"):
        z = (x + np.uint64(0x9E3779B97F4A7C15)) & _M64
        z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
        z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
        return z ^ (z >> np.uint64(31))


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 bit patterns, round-to-nearest-even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns exactly to fp64 (data conversion only)."""
    u = np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def _stream_base(seed: int, stream: int) -> np.uint64:
    s = np.array([(seed * 0x100000001B3 + stream * 0x9E3779B1 + 0x5851F42D4C957F2D) & 0xFFFFFFFFFFFFFFFF],
                 dtype=np.uint64)
    return _splitmix64(_splitmix64(s))[0]


def normal_bf16_region(seed: int, stream: int, global_cols: int, row0: int, rows: int,
                       col0: int, cols: int, sigma: float) -> np.ndarray:
    """bf16 bits of the [rows, cols] region at (row0, col0) of a global row-major
    tensor with `global_cols` columns, elements i.i.d. N(0, sigma^2)."""
    out = np.empty((rows, cols), dtype=np.uint16)
    if rows == 0 or cols == 0:
        return out
    base = _stream_base(seed, stream)
    two_pi = 2.0 * np.pi
    chunk = max(1, (1 << 20) // max(cols, 1))
    cidx = np.arange(col0, col0 + cols, dtype=np.uint64)

    def fill(r: int) -> None:
        rr = np.arange(row0 + r, row0 + min(rows, r + chunk), dtype=np.uint64)
        idx = rr[:, None] * np.uint64(global_cols) + cidx[None, :]
        with np.errstate(over="ignore"):
            c = (base + idx * np.uint64(2)) & _M64
            z1 = _splitmix64(c)
            z2 = _splitmix64((c + np.uint64(1)) & _M64)
        u1 = ((z1 >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)  # (0,1]
        u2 = (z2 >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)          # [0,1)
        g = np.sqrt(-2.0 * np.log(u1)) * np.cos(two_pi * u2) * sigma
        out[r:r + rr.shape[0]] = f32_to_bf16_bits(g.astype(np.float32))

    starts = list(range(0, rows, chunk))
    if len(starts) == 1:
        fill(0)
    else:  # numpy releases the GIL inside its loops; chunks are independent (counter based)
        with ThreadPoolExecutor(max_workers=_workers()) as ex:
            list(ex.map(fill, starts))
    return out


def normal_bf16(seed: int, stream: int, shape: Tuple[int, int], sigma: float) -> np.ndarray:
    return normal_bf16_region(seed, stream, shape[1], 0, shape[0], 0, shape[1], sigma)


# --------------------------------------------------------------------------
# Workloads
# --------------------------------------------------------------------------
EPI_NONE, EPI_BIAS, EPI_BIAS_GELU_TANH, EPI_BIAS_GELU_ERF = 0, 1, 2, 3


@dataclasses.dataclass(frozen=True)
class Layer:
    """One FC layer on a Gx x Gy x Gz grid; T, K, N are GLOBAL sizes."""
    name: str
    grid: Tuple[int, int, int]
    T: int
    K: int
    N: int
    epilogue: int = EPI_NONE
    seed: int = 0
    layer_index: int = 0  # separates the streams of the layers of a chain

    @property
    def shard(self) -> Tuple[int, int, int]:
        gx, gy, gz = self.grid
        return self.T // gz, self.K // gx, self.N // gy

    @property
    def flop_per_gemm(self) -> int:
        m, k, n = self.shard
        return 2 * m * k * n


def layer_inputs(layer: Layer, coord: Tuple[int, int, int] = (0, 0, 0),
                 want=("X", "W", "dY", "bias")) -> Dict[str, np.ndarray]:
    """The shard tensors GPU g_{ix,iy,iz} holds (K split over Gx, N over Gy, T over Gz),
    cut from the seeded global tensors.  bf16 bit patterns, C-contiguous uint16."""
    gx, gy, gz = layer.grid
    ix, iy, iz = coord
    m, kl, nl = layer.shard
    s = layer.layer_index * 8
    out: Dict[str, np.ndarray] = {}
    if "X" in want:
        out["X"] = normal_bf16_region(layer.seed, s + STREAM_X, layer.K, iz * m, m, ix * kl, kl, SIGMA_ACT)
    if "W" in want:
        out["W"] = normal_bf16_region(layer.seed, s + STREAM_W, layer.N, ix * kl, kl, iy * nl, nl, SIGMA_W)
    if "dY" in want:
        out["dY"] = normal_bf16_region(layer.seed, s + STREAM_DY, layer.N, iz * m, m, iy * nl, nl, SIGMA_ACT)
    if "bias" in want:
        out["bias"] = normal_bf16_region(layer.seed, s + STREAM_BIAS, layer.N, 0, 1, iy * nl, nl, SIGMA_W)[0]
    return out


def global_inputs(layer: Layer) -> Dict[str, np.ndarray]:
    """The unsharded tensors of a layer (same streams as layer_inputs)."""
    one = dataclasses.replace(layer, grid=(1, 1, 1))
    return layer_inputs(one)


# The five benchmark configurations and the paper's running example.  Each is a list of layers
# (a chain for cfg5 and gpt20b).
def configs() -> Dict[str, List[Layer]]:
    return {
        "cfg1": [Layer("fc", (1, 1, 1), 512, 1024, 1024)],
        "cfg1_grid222": [Layer("fc", (2, 2, 2), 512, 1024, 1024)],
        "cfg2": [Layer("qkv", (2, 2, 4), 16384, 4096, 12288)],
        "cfg3": [Layer("mlp_up", (4, 2, 8), 32768, 8192, 32768, EPI_BIAS_GELU_TANH)],
        "cfg4": [Layer("mlp_down", (2, 4, 8), 32768, 32768, 8192)],
        "cfg5": [
            Layer("qkv", (8, 8, 4), 16384, 12288, 36864, EPI_NONE, 0, 0),
            Layer("attn_out", (8, 8, 4), 16384, 12288, 12288, EPI_NONE, 0, 1),
            Layer("mlp_up", (8, 8, 4), 16384, 12288, 49152, EPI_BIAS_GELU_TANH, 0, 2),
            Layer("mlp_down", (8, 8, 4), 16384, 49152, 12288, EPI_NONE, 0, 3),
        ],
        # The running example of Section 4: a 20B-parameter GPT (Table 1: hidden size 7168), a
        # batch of 32k tokens, Gx = Gy = 2, Gz = 4 on 16 GPUs; the four FC layers of one block.
        "gpt20b": [
            Layer("qkv", (2, 2, 4), 32768, 7168, 21504, EPI_NONE, 0, 0),
            Layer("attn_out", (2, 2, 4), 32768, 7168, 7168, EPI_NONE, 0, 1),
            Layer("mlp_up", (2, 2, 4), 32768, 7168, 28672, EPI_BIAS_GELU_TANH, 0, 2),
            Layer("mlp_down", (2, 2, 4), 32768, 28672, 7168, EPI_NONE, 0, 3),
        ],
    }


def sample_rows(n_rows: int, tile: int, per_tile: int, seed: int) -> np.ndarray:
    """A stratified, sorted row sample: the first and last row of every `tile`-row
    block plus `per_tile` seeded rows inside it (covers every tile edge)."""
    rng = np.random.default_rng(seed)
    picks = set()
    for t0 in range(0, n_rows, tile):
        t1 = min(n_rows, t0 + tile)
        picks.add(t0)
        picks.add(t1 - 1)
        for r in rng.integers(t0, t1, size=per_tile):
            picks.add(int(r))
    return np.array(sorted(picks), dtype=np.int64)


def sample_rows_banded(n_rows: int, tile: int, band: int, seed: int) -> np.ndarray:
    """A stratified, sorted row sample: the first and last row of every `tile`-row block and one
    seeded row out of every `band` consecutive rows (with tile 256 and band 16: every row band of
    every matrix-core tile of every workgroup tile is hit)."""
    rng = np.random.default_rng(seed)
    picks = set()
    for t0 in range(0, n_rows, tile):
        picks.add(t0)
        picks.add(min(n_rows, t0 + tile) - 1)
    for b0 in range(0, n_rows, band):
        picks.add(int(rng.integers(b0, min(n_rows, b0 + band))))
    return np.array(sorted(picks), dtype=np.int64)
