"""Counter-based input generator.

value(seed, tensor_id, r, c) is a pure function of its arguments, so any
window of a logical tensor can be generated on its own (a sampled set of rows
for the oracle, the whole tensor for the GPU) and the two agree element for
element, whatever the sharding.

Recipe: 64-bit counter = r * cols + c, mixed with a per-tensor key through the
splitmix64 finaliser; the two 32-bit halves of the hash give two uniforms in
(0, 1); normals come from one Box-Muller branch in float64.  Values that a
workload stores as bfloat16 are rounded once here (nearest, ties to even), so
both sides see the same 16-bit words.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor

import numpy as np

SEED_BASE = 211015032

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z + np.uint64(0x9E3779B97F4A7C15))
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def _key(seed: int, tensor_id: int) -> np.uint64:
    with np.errstate(over="ignore"):
        return _mix(np.array([(seed * 0x100000001B3 + tensor_id * 0x9E3779B97F4A7C15) & 0xFFFFFFFFFFFFFFFF],
                             dtype=np.uint64))[0]


def _bits(seed, tensor_id, cols_total, r_idx, c_idx) -> np.ndarray:
    """hash words for the window rows r_idx x columns c_idx of a tensor with cols_total columns"""
    r = np.asarray(r_idx, dtype=np.uint64)[:, None]
    c = np.asarray(c_idx, dtype=np.uint64)[None, :]
    with np.errstate(over="ignore"):
        ctr = r * np.uint64(cols_total) + c
        return _mix(ctr ^ _key(seed, tensor_id))


def _window(shape, rows, cols):
    R, C = shape
    r_idx = np.arange(R) if rows is None else np.asarray(rows)
    c_idx = np.arange(C) if cols is None else np.asarray(cols)
    return r_idx, c_idx


def _blocked(fn, r_idx, c_idx, dtype, threads=8):
    """evaluate fn(row_index_block, c_idx) over row blocks on a few threads (numpy drops the GIL)"""
    out = np.empty((len(r_idx), len(c_idx)), dtype=dtype)
    if out.size == 0:
        return out
    step = max(1, (1 << 20) // max(1, len(c_idx)))
    blocks = [(s, min(s + step, len(r_idx))) for s in range(0, len(r_idx), step)]

    def work(b):
        out[b[0]:b[1]] = fn(r_idx[b[0]:b[1]], c_idx)

    if len(blocks) == 1:
        work(blocks[0])
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, blocks))
    return out


def uniform(seed: int, tensor_id: int, shape, lo=-1.0, hi=1.0, rows=None, cols=None) -> np.ndarray:
    """float64 uniform[lo, hi) window of a logical tensor of `shape`"""
    r_idx, c_idx = _window(shape, rows, cols)

    def fn(r, c):
        h = _bits(seed, tensor_id, shape[1], r, c)
        u = (h >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))
        return lo + (hi - lo) * u

    return _blocked(fn, r_idx, c_idx, np.float64)


def normal(seed: int, tensor_id: int, shape, std=1.0, rows=None, cols=None, dtype=np.float64) -> np.ndarray:
    """N(0, std^2) window of a logical tensor of `shape` (std = standard deviation)"""
    r_idx, c_idx = _window(shape, rows, cols)

    def fn(r, c):
        h = _bits(seed, tensor_id, shape[1], r, c)
        u1 = ((h >> np.uint64(32)).astype(np.float64) + 0.5) * (1.0 / (1 << 32))
        u2 = ((h & np.uint64(0xFFFFFFFF)).astype(np.float64) + 0.5) * (1.0 / (1 << 32))
        return (std * np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)).astype(dtype)

    return _blocked(fn, r_idx, c_idx, dtype)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float values -> bfloat16 words (uint16): torch's own fp32 -> bf16 cast (nearest, ties to even), so
    that this module holds no rounding arithmetic of its own"""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def pattern_u16(shape, rows=None, cols=None) -> np.ndarray:
    """integer pattern word(r, c) = (r * cols_total + c) mod 2^16, as uint16"""
    r_idx, c_idx = _window(shape, rows, cols)
    r = np.asarray(r_idx, dtype=np.uint64)[:, None]
    c = np.asarray(c_idx, dtype=np.uint64)[None, :]
    return ((r * np.uint64(shape[1]) + c) & np.uint64(0xFFFF)).astype(np.uint16)
