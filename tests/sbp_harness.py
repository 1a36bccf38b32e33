"""Glue between numpy inputs, torch device buffers, the HIP binding and the oracle.

Only plumbing: uploads shards, builds descriptors, downloads results.  The HIP path is reached
through paper_2110_15032_amd (C ABI); the oracle through oracle/.  The two never meet except in
the assertions of the tests that use this module."""
from __future__ import annotations

import numpy as np

import oracle as orc
import paper_2110_15032_amd as sbp

# oracle spelling <-> ABI spelling of a signature
TO_ABI = {orc.S0: sbp.S(0), orc.S1: sbp.S(1), orc.B: sbp.B, orc.P_SUM: sbp.P_SUM, orc.P_MAX: sbp.P_MAX}
FROM_NAME = {"S0": orc.S0, "S1": orc.S1, "B": orc.B, "Psum": orc.P_SUM, "Pmax": orc.P_MAX}


def torch_mod():
    import torch
    return torch


def upload(a: np.ndarray):
    """numpy (float32 | uint16 words | uint32 words) -> device tensor holding the same bytes"""
    torch = torch_mod()
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).cuda()
    assert a.dtype == np.float32, a.dtype
    return torch.from_numpy(a).cuda()


def download(t, like: np.dtype) -> np.ndarray:
    a = t.cpu().numpy()
    return a.view(like) if a.dtype != like else a


def empty_dev(shape, np_dtype):
    """poisoned device buffer (so unwritten outputs cannot pass)"""
    torch = torch_mod()
    td = {np.dtype(np.float32): torch.float32, np.dtype(np.uint16): torch.int16,
          np.dtype(np.uint32): torch.int32}[np.dtype(np_dtype)]
    n = int(np.prod(shape))
    t = torch.empty(max(n, 8), dtype=td, device="cuda")   # never a null pointer for tiny shards
    if td == torch.float32:
        t.fill_(float("nan"))
    else:
        t.fill_(0x7FC1 if td == torch.int16 else 0x7FC00001)
    return t[:n].view(*shape) if n else t[:0].view(*shape)


def abi_dtype(np_dtype) -> int:
    return sbp.BF16 if np.dtype(np_dtype) == np.uint16 else sbp.F32


POISON = {np.dtype(np.float32): np.float32(np.nan), np.dtype(np.uint16): np.uint16(0x7FC1), np.dtype(np.uint32): np.uint32(0x7FC00001)}


class DevTensor:
    """k device shards of one global tensor + the ABI descriptor.  ld > 0: every stored local buffer has that row
    pitch (elements); the padding is poisoned on upload and host() asserts that it still is (never written)."""

    def __init__(self, shards_dev, rows, cols, np_dtype, sbp_sig, trans=0, ld=0, stored_shapes=None):
        self.dev = list(shards_dev)
        self.rows, self.cols = rows, cols
        self.np_dtype = np.dtype(np_dtype)
        self.sig = sbp_sig
        self.trans = trans
        self.ld = ld
        self.stored_shapes = stored_shapes     # (rows, cols) of every stored buffer, needed with ld
        self.desc = sbp.SbpTensor(self.dev, rows, cols, abi_dtype(np_dtype), trans, ld)

    @property
    def k(self):
        return len(self.dev)

    @staticmethod
    def _padded(a: np.ndarray, ld: int) -> np.ndarray:
        a = np.ascontiguousarray(a)
        out = np.full((a.shape[0], ld), POISON[a.dtype], dtype=a.dtype)
        out[:, :a.shape[1]] = a
        return out

    @classmethod
    def from_host(cls, shards: list[np.ndarray], rows, cols, sig, trans=0, ld=0):
        """shards are the LOGICAL local tensors; trans=1 stores each transposed"""
        stored = [np.ascontiguousarray(s.T if trans else s) for s in shards]
        dev = [upload(cls._padded(s, ld) if ld else s) for s in stored]
        return cls(dev, rows, cols, shards[0].dtype, sig, trans, ld, [s.shape for s in stored])

    @classmethod
    def empty(cls, rows, cols, np_dtype, sig, k, ld=0):
        shapes = [orc.local_shape(rows, cols, sig, k, i) for i in range(k)]
        dev = [empty_dev((s[0], ld) if ld else s, np_dtype) for s in shapes]
        return cls(dev, rows, cols, np_dtype, sig, 0, ld, shapes)

    def host(self) -> list[np.ndarray]:
        out = [download(t, self.np_dtype) for t in self.dev]
        if self.ld:
            cut = []
            for o, (r, c) in zip(out, self.stored_shapes):
                o = o.reshape(r, self.ld) if r else o.reshape(0, self.ld)
                pad = o[:, c:]
                want = np.full(pad.shape, POISON[self.np_dtype], dtype=self.np_dtype)
                assert pad.tobytes() == want.tobytes(), "the padding between rows was written"
                cut.append(np.ascontiguousarray(o[:, :c]))
            out = cut
        return [o.T if self.trans else o for o in out]


def sync():
    torch_mod().cuda.synchronize()


def values(a: np.ndarray) -> np.ndarray:
    """stored words -> float64 values (bf16 words widened exactly)"""
    return orc.bf16_to_f64(a) if a.dtype == np.uint16 else a.astype(np.float64)


def gen(spec, seed, as_bf16: bool, rows=None, cols=None) -> np.ndarray:
    """one workload tensor (or a window of it) as stored words: float32, or uint16 bf16 words"""
    import workloads as wl
    shape, dist = spec["shape"], spec["dist"]
    if dist[0] == "pattern":
        return wl.pattern_u16(shape, rows, cols)
    if dist[0] == "uniform":
        x = wl.uniform(seed, spec["id"], shape, dist[1], dist[2], rows, cols)
    else:
        x = wl.normal(seed, spec["id"], shape, dist[1], rows, cols)
    return wl.to_bf16_bits(x) if as_bf16 else x.astype(np.float32)


# ------------------------------------------------------------------ tolerances (written out)
def assert_matmul_close(got: np.ndarray, ref: np.ndarray, rel: float, what=""):
    """|got - ref| <= rel * max(|ref|, rms(ref)) element-wise.
    rel = 2e-2 for bf16 inputs (fp32 accumulate), 1e-5 for fp32 inputs."""
    got = got.astype(np.float64)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    bound = rel * np.maximum(np.abs(ref), rms)
    err = np.abs(got - ref)
    bad = err > bound
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside tolerance, worst {err.max():.3e} (rms {rms:.3e})"
    return float((err / np.maximum(np.abs(ref), rms if rms else 1.0)).max()) if ref.size else 0.0


def assert_psum_close(got: np.ndarray, parts: list[np.ndarray], ref: np.ndarray, what=""):
    """fp32 partial-sum reduction: |got - ref| <= 1e-5 * sum_i |in_i| element-wise"""
    scale = np.sum([np.abs(p.astype(np.float64)) for p in parts], axis=0)
    err = np.abs(got.astype(np.float64) - ref)
    bad = err > 1e-5 * scale + 1e-30
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside 1e-5 * sum|in_i|, worst {err.max():.3e}"


def assert_bits_equal(got: np.ndarray, ref: np.ndarray, what=""):
    assert got.shape == ref.shape, f"{what}: shape {got.shape} vs {ref.shape}"
    assert got.dtype == ref.dtype, f"{what}: dtype {got.dtype} vs {ref.dtype}"
    if got.tobytes() != ref.tobytes():
        g = got.view(np.uint16 if got.itemsize == 2 else np.uint32)
        r = ref.view(g.dtype)
        n = int((g != r).sum())
        raise AssertionError(f"{what}: {n} of {g.size} words differ")
