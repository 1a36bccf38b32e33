"""Seeded random cases of sbp_matmul over every row of Table 1 (Sec. 3.1): shapes that fall on both sides of the
kernel-selection thresholds (persistent 256 x 256 tile, one-tile kernels, the 128 x 128 tile, the split kernel for an
fp32 partial next to bf16, the generic kernel), uneven splits, transposed storage, row pitches, k from 1 to 8, each
against the oracle at the usual bars; and seeded random boxing conversions of ragged tensors, bit-exact or within the
partial-sum bound."""
import numpy as np
import pytest

import oracle as orc
import paper_2110_15032_amd as sbp
import workloads as wl
from sbp_harness import DevTensor, TO_ABI, assert_bits_equal, assert_matmul_close, assert_psum_close, sync, values

pytestmark = pytest.mark.gpu
SEED = wl.SEED_BASE + 900
TABLE1 = [(orc.S0, orc.B), (orc.B, orc.S1), (orc.S1, orc.S0), (orc.P_SUM, orc.B), (orc.B, orc.P_SUM), (orc.B, orc.B)]


def partials_of(tid, T, k):
    parts = [wl.normal(SEED, tid + 1 + i, T.shape).astype(np.float32) for i in range(k - 1)]
    return parts + [(T - np.sum(parts, axis=0, dtype=np.float32)).astype(np.float32)]


def draw_case(rng):
    sx, sw = TABLE1[rng.integers(len(TABLE1))]
    k = int(rng.choice([1, 2, 3, 4, 5, 8]))
    bf16 = bool(rng.integers(4) != 0)
    kind = rng.integers(4)
    if kind == 0:      # large enough for the persistent kernels when the reduction length allows
        M, N = int(rng.integers(130, 700)), int(rng.integers(130, 900))
        K = int(rng.choice([128, 256, 384])) * (k if sx == orc.S1 else 1)
    elif kind == 1:    # reduction length a multiple of 64 or 32 only
        M, N = int(rng.integers(100, 500)), int(rng.integers(100, 600))
        K = int(rng.choice([64, 192, 96, 160])) * (k if sx == orc.S1 else 1)
    elif kind == 2:    # small and odd everywhere: generic kernel
        M, N, K = int(rng.integers(1, 90)), int(rng.integers(1, 90)), int(rng.integers(1, 200))
    else:              # 16-byte aligned but small: 128 x 128 tile
        M, N = 8 * int(rng.integers(1, 30)), 8 * int(rng.integers(1, 30))
        K = 64 * int(rng.integers(1, 6)) * (k if sx == orc.S1 else 1)
    if rng.integers(2):   # multiples of 8 on the split axes keep the MFMA paths reachable
        M, N = (M + 7) // 8 * 8 * (k if sx == orc.S0 else 1), (N + 7) // 8 * 8 * (k if sw == orc.S1 else 1)
    tx, tw = int(rng.integers(2)), int(rng.integers(2))
    pads = tuple(int(rng.choice([0, 0, 8, 16, 3])) for _ in range(3))
    return sx, sw, k, bf16, M, K, N, tx, tw, pads


CASES = [draw_case(np.random.default_rng(1000 + i)) for i in range(60)]


@pytest.mark.parametrize("case", CASES, ids=[f"{i}-{c[0]}{c[1]}-k{c[2]}-{'bf16' if c[3] else 'f32'}-{c[4]}x{c[5]}x{c[6]}-t{c[7]}{c[8]}-pad{c[9]}" for i, c in enumerate(CASES)])
def test_random_matmul_case(case):
    sx, sw, k, bf16, M, K, N, tx, tw, pads = case
    sy = orc.infer_matmul(sx, sw)
    X = wl.normal(SEED, 1, (M, K))
    W = wl.normal(SEED, 2, (K, N), 0.05)

    def operand(tid, T, sig):
        """local tensors as stored and their values"""
        if sig == orc.P_SUM:                                  # fp32 partials, next to bf16 or fp32 alike
            parts = partials_of(tid, T.astype(np.float32), k)
            return parts, parts
        if bf16:
            words = orc.scatter(wl.to_bf16_bits(T), sig, k)
            return words, [values(w) for w in words]
        f = orc.scatter(T.astype(np.float32), sig, k)
        return f, f

    Xs, Xv = operand(10, X, sx)
    Ws, Wv = operand(40, W, sw)
    ref, _ = orc.matmul_sbp(Xv, sx, Wv, sw)
    out_dt = np.float32 if (sy == orc.P_SUM or not bf16) else np.uint16

    def ld_of(shards, trans, pad):
        return 0 if not pad else max((s.shape[0] if trans else s.shape[1]) for s in shards) + pad

    dx = DevTensor.from_host(Xs, M, K, sx, trans=tx, ld=ld_of(Xs, tx, pads[0]))
    dw = DevTensor.from_host(Ws, K, N, sw, trans=tw, ld=ld_of(Ws, tw, pads[1]))
    ldy = 0 if not pads[2] else max(r.shape[1] for r in ref) + pads[2]
    dy = DevTensor.empty(M, N, out_dt, sy, k, ld=ldy)
    sbp.sbp_matmul(dx.desc, TO_ABI[sx], dw.desc, TO_ABI[sw], dy.desc, sbp.AUTO, k)
    sync()
    fp32_exact = not bf16 or sx == orc.P_SUM or sw == orc.P_SUM      # fp32 operands, or an fp32 partial kept exact next to bf16
    rel = 2e-2 if (bf16 and sy != orc.P_SUM and not fp32_exact) else (1e-5 if fp32_exact else 1e-4)
    for i, g in enumerate(dy.host()):
        gv = values(g) if out_dt == np.uint16 else g
        assert gv.shape == ref[i].shape
        assert_matmul_close(gv, ref[i], rel, f"shard {i}")


def draw_boxing(rng):
    sigs = [orc.S0, orc.S1, orc.B, orc.P_SUM, orc.P_MAX]
    si = sigs[rng.integers(5)]
    so = sigs[rng.integers(5)]
    k = int(rng.choice([1, 2, 3, 5, 7, 8, 16]))
    rows, cols = int(rng.integers(1, 300)), int(rng.integers(1, 300))
    if rng.integers(2):
        cols = (cols + 3) // 4 * 4          # 16-byte rows: vector paths
    return si, so, k, rows, cols


BOXINGS = [draw_boxing(np.random.default_rng(5000 + i)) for i in range(60)]


@pytest.mark.parametrize("case", BOXINGS, ids=[f"{i}-{c[0]}to{c[1]}-k{c[2]}-{c[3]}x{c[4]}" for i, c in enumerate(BOXINGS)])
def test_random_boxing_case(case):
    si, so, k, rows, cols = case
    partial_in = si in (orc.P_SUM, orc.P_MAX)
    partial_out = so in (orc.P_SUM, orc.P_MAX)
    if partial_in and partial_out and si != so:
        pytest.skip("P(sum) <-> P(max) is not a conversion of Table 2")
    T = wl.normal(SEED, 7, (rows, cols)).astype(np.float32)
    if si == orc.P_SUM:
        ins = partials_of(20, T, k)
    elif si == orc.P_MAX:
        ins = [(T - np.abs(wl.normal(SEED, 30 + i, T.shape).astype(np.float32)) * (i % 2)).astype(np.float32) for i in range(k)]
    else:
        ins = orc.scatter(T, si, k)
    ref = orc.boxing([a.astype(np.float64) for a in ins] if partial_in else ins, si, so, k)
    d_in = DevTensor.from_host(ins, rows, cols, si)
    d_out = DevTensor.empty(rows, cols, np.float32, so, k)
    sbp.sbp_boxing(d_in.desc, TO_ABI[si], d_out.desc, TO_ABI[so], k)
    sync()
    for j, (g, r) in enumerate(zip(d_out.host(), ref)):
        assert g.shape == r.shape
        if si == orc.P_SUM and not partial_out:
            parts = ins if so == orc.B else [orc.scatter(p, so, k)[j] for p in ins]
            assert_psum_close(g, parts, r, f"shard {j}")
        else:
            assert_bits_equal(g, np.asarray(r, dtype=np.float32), f"shard {j}")
