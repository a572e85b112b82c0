"""Seeded, position-addressable synthetic inputs for the tensor-parallel linear layer.

This module only produces input bits.  It holds none of the layer's arithmetic
(no matmul, no GeLU, no partition map) and is the one module that both the CPU
oracle's tests and the GPU path's tests/bench may import.

Every element of a *full* (unpartitioned) tensor is a pure function of
``(seed, tensor_id, row, col, ncols_full)``: a 64-bit counter is hashed twice
(splitmix64 finaliser), the two words become two uniforms, Box-Muller turns
them into one N(0,1) sample, the sample is scaled by ``std`` and quantised to
the nearest bf16 (ties to even).  A rank's block is therefore generated without
materialising the full tensor, and every consumer sees identical bits.

Values are returned as ``uint16`` bf16 bit patterns (numpy, C-contiguous).

Stand-in statement: the paper trains ViT / BERT / GPT-style models on ImageNet
and Wikipedia; a linear layer's cost depends only on shapes and (weakly) on the
bit toggling of the operands, so activations are drawn N(0,1), weights and
biases N(0, 0.02^2), upstream gradients N(0,1).
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

BASE_SEED = 211014883

# tensor ids (any fixed distinct values)
T_X = 1
T_W1 = 2
T_B1 = 3
T_W2 = 4
T_G = 5
T_PEER_G = 6
T_PEER_A = 7

_U64 = np.uint64
_GOLD = _U64(0x9E3779B97F4A7C15)
_M1 = _U64(0xBF58476D1CE4E5B9)
_M2 = _U64(0x94D049BB133111EB)


def _mix(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function on a uint64 array (wrap-around arithmetic)."""
    z = (z ^ (z >> _U64(30))) * _M1
    z = (z ^ (z >> _U64(27))) * _M2
    return z ^ (z >> _U64(31))


def _key(seed: int, tensor_id: int) -> np.uint64:
    k = np.array([(seed * 0x632BE59BD9B4E019 + tensor_id * 0xD1342543DE82EF95) % (1 << 64)], dtype=np.uint64)
    return _mix(_mix(k) + _GOLD)[0]


def _f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Quantise finite float32 values to bf16 bit patterns, nearest, ties to even."""
    u = x.astype(np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    u = u + np.uint32(0x7FFF) + lsb
    return (u >> np.uint32(16)).astype(np.uint16)


def _normal_rows(key: np.uint64, ncols_full: int, row0: int, nrows: int, col0: int, ncols: int,
                 std: float) -> np.ndarray:
    with np.errstate(over="ignore"):
        rows = (np.arange(row0, row0 + nrows, dtype=np.uint64) * _U64(ncols_full))[:, None]
        cols = np.arange(col0, col0 + ncols, dtype=np.uint64)[None, :]
        ctr = (rows + cols) * _U64(2)
        h1 = _mix(key + ctr * _GOLD)
        h2 = _mix(key + (ctr + _U64(1)) * _GOLD)
    # 53-bit uniforms in (0,1): never 0, so the log is finite
    u1 = ((h1 >> _U64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)
    u2 = ((h2 >> _U64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return _f32_to_bf16_bits((z * std).astype(np.float32))


def normal_block_bf16(seed: int, tensor_id: int, ncols_full: int, row0: int, nrows: int,
                      col0: int, ncols: int, std: float, threads: int | None = None) -> np.ndarray:
    """bf16 bit patterns of rows [row0,row0+nrows) x cols [col0,col0+ncols) of the full
    tensor ``tensor_id`` whose row length is ``ncols_full``; entries ~ N(0, std^2)."""
    out = np.empty((nrows, ncols), dtype=np.uint16)
    if nrows == 0 or ncols == 0:
        return out
    key = _key(seed, tensor_id)
    # about 1M elements per task keeps the float64 temporaries small
    rows_per = max(1, (1 << 20) // max(1, ncols))
    spans = [(r, min(rows_per, nrows - r)) for r in range(0, nrows, rows_per)]
    if threads is None:
        threads = min(16, os.cpu_count() or 1)

    def work(span):
        r, n = span
        out[r:r + n] = _normal_rows(key, ncols_full, row0 + r, n, col0, ncols, std)

    if threads <= 1 or len(spans) == 1:
        for s in spans:
            work(s)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, spans))
    return out


def sample_rows(seed: int, nrows: int, count: int, tile: int = 256) -> np.ndarray:
    """A sorted set of distinct row indices: the first and last row, the last row of the
    first tile and the first row of the ragged tail tile (when there is one), one row in
    every ``tile``-row band while the budget lasts, and seeded random rows for the rest."""
    if nrows <= count:
        return np.arange(nrows, dtype=np.int64)
    rng = np.random.default_rng(seed)
    picks = {0, nrows - 1, min(tile - 1, nrows - 1), (nrows - 1) // tile * tile}
    bands = np.arange(0, nrows, tile)
    if len(bands) > count // 2:
        bands = rng.choice(bands, size=count // 2, replace=False)
    for b in bands:
        picks.add(int(b + rng.integers(0, min(tile, nrows - b))))
    while len(picks) < count:
        picks.add(int(rng.integers(0, nrows)))
    return np.array(sorted(picks), dtype=np.int64)
