"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element, on
seeded inputs small enough for the oracle to finish in seconds but spanning several tiles and
ragged tails.  Bars: bit-exact for S/B relayout boxing and P(max); 1e-5 * sum|in_i| for fp32
P(sum) reductions; 2e-2 relative for bf16 matmuls (fp32 accumulate); 1e-5 for fp32 matmuls."""
import itertools

import numpy as np
import pytest

import oracle as orc
import paper_2110_15032_amd as sbp
import workloads as wl
from sbp_harness import (DevTensor, TO_ABI, assert_bits_equal, assert_matmul_close, assert_psum_close,
                         sync, values)

pytestmark = pytest.mark.gpu
SEED = wl.SEED_BASE


def rnd_f32(tid, shape):
    return wl.normal(SEED, tid, shape).astype(np.float32)


def rnd_bf16(tid, shape, std=1.0):
    return wl.to_bf16_bits(wl.normal(SEED, tid, shape, std))


def rnd_words(tid, shape):
    """arbitrary 16-bit words, NaN / Inf patterns included"""
    w = wl.uniform(SEED, tid, shape, 0.0, 65536.0).astype(np.uint32).astype(np.uint16)
    w.flat[:4] = [0x7F80, 0x7FC1, 0xFF80, 0xFFFF][: min(4, w.size)]
    return w


def random_partials(tid, T, k, op):
    if op == "sum":
        parts = [rnd_f32(tid + 1 + i, T.shape) for i in range(k - 1)]
        return parts + [(T - np.sum(parts, axis=0, dtype=np.float32)).astype(np.float32)]
    return [(T - np.abs(rnd_f32(tid + 1 + i, T.shape)) * (i % 2)).astype(np.float32) for i in range(k)]


# ------------------------------------------------------------------------------- boxing
RELAYOUT = [(a, b) for a, b in itertools.product((orc.S0, orc.S1, orc.B), repeat=2)]
SHAPES = [(64, 96), (37, 53), (16, 1024), (130, 24), (5, 3)]


@pytest.mark.parametrize("k", [1, 2, 3, 8, 16])
@pytest.mark.parametrize("si,so", RELAYOUT)
@pytest.mark.parametrize("words", ["u16", "f32"])
def test_relayout_boxing_is_bit_exact(k, si, so, words):
    for n, shape in enumerate(SHAPES):
        T = rnd_words(n, shape) if words == "u16" else rnd_f32(n, shape)
        ins = orc.scatter(T, si, k)
        if si == orc.B and so != orc.B:
            # make the k "copies" differ so that reading the wrong device's copy shows (B -> S)
            ins = [np.ascontiguousarray(T + (np.uint16(j) if words == "u16" else np.float32(j))) for j in range(k)]
        ref = orc.boxing(ins, si, so, k)
        d_in = DevTensor.from_host(ins, *shape, si)
        d_out = DevTensor.empty(*shape, T.dtype, so, k)
        sbp.sbp_boxing(d_in.desc, TO_ABI[si], d_out.desc, TO_ABI[so], k)
        sync()
        for j, (g, r) in enumerate(zip(d_out.host(), ref)):
            assert_bits_equal(g, r, f"{si}->{so} k={k} shape={shape} shard {j}")


@pytest.mark.parametrize("k", [1, 2, 3, 8, 16, 5])
@pytest.mark.parametrize("op", ["sum", "max"])
@pytest.mark.parametrize("so", [orc.B, orc.S0, orc.S1])
def test_partial_value_boxing(k, op, so):
    si = orc.P_SUM if op == "sum" else orc.P_MAX
    for n, shape in enumerate(SHAPES + [(256, 1030)]):
        T = rnd_f32(100 + n, shape)
        parts = random_partials(200 + 20 * n, T, k, op)
        ref = orc.boxing(parts, si, so, k)              # float64
        d_in = DevTensor.from_host(parts, *shape, si)
        d_out = DevTensor.empty(*shape, np.float32, so, k)
        sbp.sbp_boxing(d_in.desc, TO_ABI[si], d_out.desc, TO_ABI[so], k)
        sync()
        got = d_out.host()
        for j in range(k):
            what = f"P({op})->{so} k={k} shape={shape} shard {j}"
            assert got[j].shape == ref[j].shape, what
            if op == "max":
                assert_bits_equal(got[j], ref[j].astype(np.float32), what)      # max is exact
            else:
                local_parts = [orc.boxing([p] * k, orc.B, so, k)[j] for p in parts] if so != orc.B else parts
                assert_psum_close(got[j], local_parts, ref[j], what)
        if so == orc.B:
            for j in range(1, k):
                assert_bits_equal(got[j], got[0], f"B copies 0 and {j} of P({op})->B")


@pytest.mark.parametrize("so", [orc.B, orc.S0])
def test_partial_max_with_nan_and_signed_zero(so):
    """P(max) ignores a NaN next to a number, gives NaN only when every partial is NaN, and may give either
    sign for the maximum of +0 and -0 (the reading in sbp.h; the oracle takes the same one)."""
    k, shape = 3, (8, 64)
    nan = np.float32("nan")
    parts = [rnd_f32(900 + i, shape) for i in range(k)]
    parts[0][0, :8] = nan                      # NaN first, numbers after
    parts[2][1, :8] = nan                      # numbers first, NaN last
    for q in parts:
        q[2, :8] = nan                         # all NaN
    parts[0][3, :8], parts[1][3, :8], parts[2][3, :8] = 0.0, -0.0, -0.0
    parts[0][4, :8], parts[1][4, :8], parts[2][4, :8] = -0.0, -1.0, 0.0
    ref = orc.boxing(parts, orc.P_MAX, so, k)
    d_in = DevTensor.from_host(parts, *shape, orc.P_MAX)
    d_out = DevTensor.empty(*shape, np.float32, so, k)
    sbp.sbp_boxing(d_in.desc, sbp.P_MAX, d_out.desc, TO_ABI[so], k)
    sync()
    for j, (g, r) in enumerate(zip(d_out.host(), ref)):
        r = r.astype(np.float32)
        assert np.array_equal(np.isnan(g), np.isnan(r)), f"NaN positions, shard {j}"
        ok = ~np.isnan(r)
        assert np.array_equal(g[ok], r[ok]), f"values, shard {j}"           # -0 == +0 here: either sign passes
        nz = ok & (r != 0)
        assert np.array_equal(g[nz].view(np.uint32), r[nz].view(np.uint32)), f"bits, shard {j}"
    # the local row maximum of the model-parallel softmax takes the same reading
    L = rnd_f32(950, (16, 96))
    L[0, 5], L[1, :], L[2, 0] = nan, nan, nan
    Ls = orc.scatter(L, orc.S1, k)
    d_l = DevTensor.from_host(Ls, 16, 96, orc.S1)
    m_p = DevTensor.empty(16, 1, np.float32, orc.P_MAX, k)
    sbp.sbp_row_max(d_l.desc, sbp.S(1), m_p.desc, k)
    sync()
    for i, g in enumerate(m_p.host()):
        r = orc.row_max(Ls[i].astype(np.float64))[:, None].astype(np.float32)
        r[np.isnan(r)] = -np.inf               # an all-NaN row: the kernel starts from the identity of max
        assert np.array_equal(g, r), f"row max, shard {i}"


@pytest.mark.parametrize("k", [1, 2, 3, 8, 16])
@pytest.mark.parametrize("op", ["sum", "max"])
@pytest.mark.parametrize("si", [orc.S0, orc.S1, orc.B])
def test_boxing_into_partial_keeps_values_in_place(k, op, si):
    """S(a) -> P and B -> P (priced at zero in Table 2): every device keeps its own values inside a
    full-shape partial and holds the identity of the reduction elsewhere.  Bit-exact, and the
    partials must reduce back to the global tensor."""
    so = orc.P_SUM if op == "sum" else orc.P_MAX
    for n, shape in enumerate(SHAPES + [(256, 1030)]):
        T = rnd_f32(400 + n, shape)
        ins = orc.scatter(T, si, k)
        ref = orc.boxing(ins, si, so, k)                 # float64, exact images of the fp32 values
        d_in = DevTensor.from_host(ins, *shape, si)
        d_out = DevTensor.empty(*shape, np.float32, so, k)
        sbp.sbp_boxing(d_in.desc, TO_ABI[si], d_out.desc, TO_ABI[so], k)
        sync()
        got = d_out.host()
        for j in range(k):
            assert got[j].shape == shape
            assert np.array_equal(got[j].astype(np.float64), ref[j]), f"{si}->{so} k={k} shape={shape} shard {j}"
        assert np.array_equal(orc.assemble([g.astype(np.float64) for g in got], so), T.astype(np.float64))


@pytest.mark.parametrize("k", [1, 2, 3, 8, 16])
@pytest.mark.parametrize("axis", [0, 1])
def test_cast_fused_into_all_gather(k, axis):
    """Sec. 6.4 forward: fp32 S(a) -> bf16 B, one rounding to nearest even.  Bit-exact against the
    oracle's rounding of the assembled tensor; ties, values that round up into the next binade,
    subnormals and infinities planted."""
    si = orc.S0 if axis == 0 else orc.S1
    for n, shape in enumerate(SHAPES + [(256, 1032), (96, 8 * 16 * 5)]):
        T = rnd_f32(500 + n, shape)
        flat = T.reshape(-1)
        special = np.array([1.00390625, 1.01171875, -1.00390625, 3.3895313892515355e38, 1e-40, -0.0, np.inf, 255.5], np.float32)
        flat[: min(special.size, flat.size)] = special[: flat.size]
        ins = orc.scatter(T, si, k)
        d_in = DevTensor.from_host(ins, *shape, si)
        d_out = DevTensor.empty(*shape, np.uint16, orc.B, k)
        sbp.sbp_boxing_cast(d_in.desc, TO_ABI[si], d_out.desc, sbp.B, k)
        sync()
        ref = orc.bf16_round(T.astype(np.float64))
        for j, g in enumerate(d_out.host()):
            assert_bits_equal(g, ref, f"cast + all-gather S({axis})->B k={k} shape={shape} copy {j}")


@pytest.mark.parametrize("k", [1, 2, 3, 8, 5])
@pytest.mark.parametrize("axis", [0, 1])
def test_cast_fused_into_reduce_scatter(k, axis):
    """Sec. 6.4 backward: k bf16 partial gradients -> fp32 S(a): widened exactly, summed in fp32."""
    so = orc.S0 if axis == 0 else orc.S1
    for n, shape in enumerate(SHAPES + [(256, 1032), (96, 8 * 16 * 5)]):
        parts = [rnd_bf16(600 + 20 * n + i, shape) for i in range(k)]
        vals = [values(p) for p in parts]
        ref = orc.boxing(vals, orc.P_SUM, so, k)
        d_in = DevTensor.from_host(parts, *shape, orc.P_SUM)
        d_out = DevTensor.empty(*shape, np.float32, so, k)
        sbp.sbp_boxing_cast(d_in.desc, sbp.P_SUM, d_out.desc, TO_ABI[so], k)
        sync()
        for j, g in enumerate(d_out.host()):
            sl = [orc.scatter(v, so, k)[j] for v in vals]
            assert g.shape == ref[j].shape
            assert_psum_close(g, sl, ref[j], f"cast + reduce-scatter P->S({axis}) k={k} shape={shape} shard {j}")


def test_boxing_is_reproducible_run_to_run():
    k, shape = 8, (512, 640)
    parts = [rnd_f32(300 + i, shape) for i in range(k)]
    d_in = DevTensor.from_host(parts, *shape, orc.P_SUM)
    outs = []
    for _ in range(2):
        d_out = DevTensor.empty(*shape, np.float32, orc.B, k)
        sbp.sbp_boxing(d_in.desc, sbp.P_SUM, d_out.desc, sbp.B, k)
        sync()
        outs.append(d_out.host()[0])
    assert_bits_equal(outs[0], outs[1], "two runs of P(sum)->B")
    # fp32 sum in shard order is what the library documents: reproduce it exactly
    acc = parts[0].copy()
    for p in parts[1:]:
        acc = (acc + p).astype(np.float32)
    assert_bits_equal(outs[0], acc, "fp32 shard-order sum")


# ------------------------------------------------------------------------------- matmul
TABLE1 = [(orc.S0, orc.B), (orc.B, orc.S1), (orc.S1, orc.S0), (orc.P_SUM, orc.B), (orc.B, orc.P_SUM), (orc.B, orc.B)]


def shard_operand(tid, T, sig, k):
    if sig == orc.P_SUM:
        return random_partials(tid, T, k, "sum")
    return orc.scatter(T, sig, k)


def run_matmul(Xs, sx, Ws, sw, M, K, N, k, tx=0, tw=0, epilogue=sbp.EPI_NONE, variant=0):
    sy = orc.infer_matmul(sx, sw)
    out_dtype = np.float32 if (sy == orc.P_SUM or Xs[0].dtype == np.float32) else np.uint16
    dx = DevTensor.from_host(Xs, M, K, sx, trans=tx)
    dw = DevTensor.from_host(Ws, K, N, sw, trans=tw)
    dy = DevTensor.empty(M, N, out_dtype, sy, k)
    sbp.sbp_set_knob(sbp.KNOB_GEMM_VARIANT, variant)
    try:
        sbp.sbp_matmul_ex(dx.desc, TO_ABI[sx], dw.desc, TO_ABI[sw], dy.desc, sbp.AUTO, k, None, epilogue)
        sync()
    finally:
        sbp.sbp_set_knob(sbp.KNOB_GEMM_VARIANT, 0)
    return dy.host(), sy


@pytest.mark.parametrize("k", [1, 2, 3])
@pytest.mark.parametrize("sx,sw", TABLE1)
def test_matmul_fp32_every_table1_row(k, sx, sw):
    M, K, N = 37, 50, 29                       # uneven splits on every axis
    X, W = rnd_f32(1, (M, K)), rnd_f32(2, (K, N))
    Xs, Ws = shard_operand(10, X, sx, k), shard_operand(40, W, sw, k)
    ref, sy = orc.matmul_sbp(Xs, sx, Ws, sw)
    got, _ = run_matmul(Xs, sx, Ws, sw, M, K, N, k)
    for i in range(k):
        assert got[i].shape == ref[i].shape
        assert_matmul_close(got[i], ref[i], 1e-5, f"fp32 ({sx},{sw}) k={k} shard {i}")


@pytest.mark.parametrize("tx,tw", [(0, 0), (1, 0), (0, 1), (1, 1)])
@pytest.mark.parametrize("sx,sw", [(orc.S0, orc.B), (orc.B, orc.S1), (orc.S1, orc.S0), (orc.B, orc.B)])
@pytest.mark.parametrize("variant", [0, 1, 3, 4, 6, 7])
def test_matmul_bf16_mfma_shapes(sx, sw, tx, tw, variant):
    """several 256-tiles plus ragged M / N tails; K a multiple of 64 per shard.  variant 1 is the
    generic kernel on the same data, the others are MFMA kernel variants (256 x 256 tile with 2 x 64
    or 4 x 32 LDS stages, 128 x 128 tile); all must agree with the oracle."""
    k = 2
    M, K, N = 2 * 296, 2 * 192, 2 * 328        # per-shard 296 / 192 / 328 when split
    X, W = rnd_bf16(1, (M, K)), rnd_bf16(2, (K, N), 0.05)
    Xs, Ws = orc.scatter(X, sx, k), orc.scatter(W, sw, k)
    ref, sy = orc.matmul_sbp([values(x) for x in Xs], sx, [values(w) for w in Ws], sw)
    got, _ = run_matmul(Xs, sx, Ws, sw, M, K, N, k, tx, tw, variant=variant)
    for i in range(k):
        g = got[i] if sy == orc.P_SUM else values(got[i])
        assert_matmul_close(g, ref[i], 2e-2, f"bf16 ({sx},{sw}) trans=({tx},{tw}) v{variant} shard {i}")
        if sy == orc.P_SUM:
            # fp32 partials of exact bf16 products: only summation order differs from the oracle
            assert_matmul_close(g, ref[i], 1e-4, f"bf16->f32 partial, shard {i}")


@pytest.mark.parametrize("variant", [12, 16])
@pytest.mark.parametrize("tx,tw", [(0, 0), (1, 1), (1, 0), (0, 1)])
@pytest.mark.parametrize("sx,sw", [(orc.S0, orc.B), (orc.B, orc.S1), (orc.S1, orc.S0)])
@pytest.mark.parametrize("kshard", [128, 384])
def test_matmul_bf16_persistent_kernel(sx, sw, tx, tw, kshard, variant):
    """variants 12 and 16 (the 32x32x16 and the 16x16x32 matrix instruction) keep one workgroup per compute
    unit and walk it over several output tiles, the next tile's operand loads overlapping the current
    tile's stores.  270 tiles (more than one per workgroup), interior and ragged edge tiles, every
    operand layout, one and three rounds of four stages."""
    k = 3
    M, N = 2520, 2104                          # pitches must be multiples of 8 elements
    if sx == orc.S0:
        M *= k
    if sw == orc.S1:
        N *= k
    K = kshard * k if sx == orc.S1 else kshard
    X, W = rnd_bf16(3, (M, K)), rnd_bf16(4, (K, N), 0.05)
    Xs, Ws = orc.scatter(X, sx, k), orc.scatter(W, sw, k)
    ref, sy = orc.matmul_sbp([values(x) for x in Xs], sx, [values(w) for w in Ws], sw)
    got, _ = run_matmul(Xs, sx, Ws, sw, M, K, N, k, tx, tw, variant=variant)
    for i in range(k):
        g = got[i] if sy == orc.P_SUM else values(got[i])
        assert_matmul_close(g, ref[i], 2e-2, f"persistent v{variant} ({sx},{sw}) trans=({tx},{tw}) shard {i}")
        if sy == orc.P_SUM:
            assert_matmul_close(g, ref[i], 1e-4, f"persistent v{variant}: fp32 partial of exact products, shard {i}")


@pytest.mark.parametrize("tx,tw", [(0, 0), (1, 0), (0, 1), (1, 1)])
@pytest.mark.parametrize("row", [4, 5])
@pytest.mark.parametrize("shape,variant", [((296, 192, 328), 0), ((296, 192, 328), 32), ((600, 96, 536), 32), ((45, 100, 51), 0)])
def test_matmul_partial_fp32_times_bf16(row, tx, tw, shape, variant):
    """Table 1 rows 4 and 5 inside a bf16 graph: the P(sum) operand is k fp32 partials, its partner a
    bf16 B tensor, the result k fp32 partials Y_i = X_i W (or X W_i).  The first shape takes the
    MFMA kernel that splits the fp32 operand into three bf16 terms (several tiles, ragged edges), with
    its 128 x 128 tile (the choice for small shapes) and with the 128 x 256 tile forced (variant 32), which
    the third shape runs over several tiles in both directions and an odd number of reduction steps;
    the last shape takes the generic kernel.  All keep fp32-GEMM accuracy: the partial is never rounded."""
    k = 3
    M, K, N = shape
    X, W = rnd_f32(1, (M, K)), rnd_f32(2, (K, N))
    if row == 4:
        Xs = random_partials(10, X, k, "sum")
        Wb = rnd_bf16(2, (K, N), 0.05)
        Ws = orc.scatter(Wb, orc.B, k)
        sx, sw = orc.P_SUM, orc.B
        ref, sy = orc.matmul_sbp(Xs, sx, [values(w) for w in Ws], sw)
    else:
        Xb = rnd_bf16(1, (M, K))
        Xs = orc.scatter(Xb, orc.B, k)
        Ws = random_partials(40, W, k, "sum")
        sx, sw = orc.B, orc.P_SUM
        ref, sy = orc.matmul_sbp([values(x) for x in Xs], sx, Ws, sw)
    assert sy == orc.P_SUM
    got, _ = run_matmul(Xs, sx, Ws, sw, M, K, N, k, tx, tw, variant=variant)
    for i in range(k):
        assert got[i].dtype == np.float32 and got[i].shape == ref[i].shape
        assert_matmul_close(got[i], ref[i], 1e-5, f"row {row} trans=({tx},{tw}) shape={shape} variant={variant} partial {i}")


def test_fused_row_max_of_the_pingpong_kernel_across_tiles_rows_and_shards():
    """The ping-pong kernel carries the row maxima in registers from tile to tile and sends them to the P(max)
    vector only when a workgroup moves to other rows or to another shard, or ends (Sec. 6.3.1, local maximum).
    320 tiles over 256 workgroups: some walk two tiles, of the same rows or of different shards; the bottom tile
    row is cut by the matrix edge (rows past it must not reach the vector) and so is the right tile column."""
    k, M, K, N = 2, 3 * 256 + 40, 128, 2 * (39 * 256 + 24)
    X, W = rnd_bf16(31, (M, K)), rnd_bf16(32, (K, N), 0.05)
    X[M - 1, :] = np.uint16(0xBF80)              # last row -1: its maxima are negative in many column ranges
    Xs, Ws = orc.scatter(X, orc.B, k), orc.scatter(W, orc.S1, k)
    dx, dw = DevTensor.from_host(Xs, M, K, orc.B), DevTensor.from_host(Ws, K, N, orc.S1)
    torch = __import__("torch")
    res = {}
    for variant in (21, 16):
        y = DevTensor.empty(M, N, np.uint16, orc.S1, k)
        m_big = [torch.full((M + 256,), float("nan"), device="cuda") for _ in range(k)]     # 256 guard entries behind the vector
        m = sbp.SbpTensor(m_big, M, 1, sbp.F32)
        sbp.sbp_set_knob(sbp.KNOB_GEMM_VARIANT, variant)
        try:
            sbp.sbp_matmul_rowmax(dx.desc, sbp.B, dw.desc, sbp.S(1), y.desc, sbp.AUTO, m, k)
            sync()
        finally:
            sbp.sbp_set_knob(sbp.KNOB_GEMM_VARIANT, 0)
        for b in m_big:
            assert bool(torch.isnan(b[M:]).all()), f"variant {variant}: a row past the matrix edge reached the P(max) vector"
        res[variant] = (y.host(), [b[:M].cpu().numpy().reshape(M, 1) for b in m_big])
    ref, _ = orc.matmul_sbp([values(x) for x in Xs], orc.B, [values(w) for w in Ws], orc.S1)
    for i in range(k):
        assert_bits_equal(res[21][0][i], res[16][0][i], f"logits shard {i}: ping-pong against lockstep kernel")
        assert_matmul_close(values(res[21][0][i]), ref[i], 2e-2, f"logits shard {i} vs oracle")
        want = orc.row_max(values(res[21][0][i]))
        assert np.array_equal(res[21][1][i][:, 0].astype(np.float64), want), f"row max shard {i} vs oracle"
        assert np.array_equal(res[21][1][i], res[16][1][i]), f"row max shard {i}: ping-pong against lockstep kernel"


def test_matmul_bf16_persistent_kernel_uneven_shards():
    """S(0) x B with M = 5 * 256 + 3 over k = 5: three shards of 257 rows (two tile-rows, the second
    one row high), two of 256 (one tile-row), so the tile list has holes the persistent walk must
    skip; and k = 8 over 1100 rows with a 1024-deep reduction, eight rounds per tile."""
    for k, M, K, N in [(5, 1283, 256, 1304), (8, 1100, 1024, 520)]:
        X, W = rnd_bf16(5, (M, K)), rnd_bf16(6, (K, N), 0.05)
        Xs, Ws = orc.scatter(X, orc.S0, k), orc.scatter(W, orc.B, k)
        ref, sy = orc.matmul_sbp([values(x) for x in Xs], orc.S0, [values(w) for w in Ws], orc.B)
        for variant in (12, 16):
            got, _ = run_matmul(Xs, orc.S0, Ws, orc.B, M, K, N, k, variant=variant)
            for i in range(k):
                assert got[i].shape == ref[i].shape
                assert_matmul_close(values(got[i]), ref[i], 2e-2, f"uneven S(0) shards, v{variant}, k={k}, shard {i}")


def test_matmul_bf16_odd_shapes_fall_back():
    """pitches that are not multiples of 8 elements, K not a multiple of 64, uneven splits"""
    k = 3
    M, K, N = 45, 100, 51
    X, W = rnd_bf16(1, (M, K)), rnd_bf16(2, (K, N), 0.1)
    for sx, sw in [(orc.S0, orc.B), (orc.B, orc.S1), (orc.S1, orc.S0)]:
        Xs, Ws = orc.scatter(X, sx, k), orc.scatter(W, sw, k)
        ref, sy = orc.matmul_sbp([values(x) for x in Xs], sx, [values(w) for w in Ws], sw)
        got, _ = run_matmul(Xs, sx, Ws, sw, M, K, N, k)
        for i in range(k):
            g = got[i] if sy == orc.P_SUM else values(got[i])
            assert_matmul_close(g, ref[i], 2e-2, f"odd ({sx},{sw}) shard {i}")


def test_matmul_gelu_epilogue_and_single_rounding():
    k = 4
    M, K, N = 256, 128, 4 * 264
    X, W = rnd_bf16(1, (M, K)), rnd_bf16(2, (K, N), 0.1)
    Xs, Ws = orc.scatter(X, orc.B, k), orc.scatter(W, orc.S1, k)
    pre, sy = orc.matmul_sbp([values(x) for x in Xs], orc.B, [values(w) for w in Ws], orc.S1)
    got, _ = run_matmul(Xs, orc.B, Ws, orc.S1, M, K, N, k, epilogue=sbp.EPI_GELU)
    for i in range(k):
        ref = orc.bf16_to_f64(orc.bf16_round(orc.gelu(pre[i])))
        assert_matmul_close(values(got[i]), ref, 2e-2, f"gelu shard {i}")
        # Far tighter in fact, for EVERY element: the kernel's gelu is within 2.2e-5 relative of the erf form and
        # both sides round once, so the two bf16 results differ by at most one rounding step (2^-7 relative);
        # the floor covers the fp32 accumulation order of the 128 products in front of it (values near zero).
        err = np.abs(values(got[i]) - ref)
        bound = 2.0 ** -7 * np.abs(ref) + 2e-5
        assert (err <= bound).all(), f"gelu shard {i}: worst excess {np.max(err - bound):.3e} at ref {ref.flat[np.argmax(err - bound)]:.4e}"


def test_empty_and_degenerate_shards():
    # k larger than the split axis: trailing shards are empty
    k = 8
    M, K, N = 5, 64, 16
    X, W = rnd_f32(1, (M, K)), rnd_f32(2, (K, N))
    Xs, Ws = orc.scatter(X, orc.S0, k), orc.scatter(W, orc.B, k)
    ref, _ = orc.matmul_sbp(Xs, orc.S0, Ws, orc.B)
    got, _ = run_matmul(Xs, orc.S0, Ws, orc.B, M, K, N, k)
    for i in range(k):
        assert got[i].shape == ref[i].shape
        if ref[i].size:
            assert_matmul_close(got[i], ref[i], 1e-5, f"shard {i}")
    # boxing with empty shards
    T = rnd_words(5, (3, 40))
    for si, so in [(orc.S0, orc.S1), (orc.S0, orc.B), (orc.B, orc.S0)]:
        ins = orc.scatter(T, si, k)
        d_in = DevTensor.from_host(ins, 3, 40, si)
        d_out = DevTensor.empty(3, 40, np.uint16, so, k)
        sbp.sbp_boxing(d_in.desc, TO_ABI[si], d_out.desc, TO_ABI[so], k)
        sync()
        for g, r in zip(d_out.host(), orc.boxing(ins, si, so, k)):
            assert_bits_equal(g, r, f"{si}->{so} with empty shards")
    # zero-sized global tensor: a no-op that must not fail
    d_in = DevTensor.from_host(orc.scatter(np.zeros((0, 8), np.float32), orc.S0, 2), 0, 8, orc.S0)
    d_out = DevTensor.empty(0, 8, np.float32, orc.B, 2)
    sbp.sbp_boxing(d_in.desc, sbp.S(0), d_out.desc, sbp.B, 2)
    sync()


# ------------------------------------------------------------------------------- chains
def test_config1_tiny_chain():
    """k = 2, fp32: X[64,128] S(1) x W[128,96] S(0) -> P(sum); then P->B and P->S(0)."""
    from workloads import CONFIGS
    from sbp_harness import gen
    cfg = CONFIGS["tiny"]
    k = cfg["k"]
    X, W = gen(cfg["X"], SEED, False), gen(cfg["W"], SEED, False)
    Xs, Ws = orc.scatter(X, orc.S1, k), orc.scatter(W, orc.S0, k)
    ref_parts, sy = orc.matmul_sbp(Xs, orc.S1, Ws, orc.S0)
    assert sy == orc.P_SUM
    dx, dw = DevTensor.from_host(Xs, 64, 128, orc.S1), DevTensor.from_host(Ws, 128, 96, orc.S0)
    dy = DevTensor.empty(64, 96, np.float32, orc.P_SUM, k)
    sbp.sbp_matmul(dx.desc, sbp.S(1), dw.desc, sbp.S(0), dy.desc, sbp.P_SUM, k)
    d_b = DevTensor.empty(64, 96, np.float32, orc.B, k)
    d_s = DevTensor.empty(64, 96, np.float32, orc.S0, k)
    sbp.sbp_boxing(dy.desc, sbp.P_SUM, d_b.desc, sbp.B, k)
    sbp.sbp_boxing(dy.desc, sbp.P_SUM, d_s.desc, sbp.S(0), k)
    sync()
    parts = dy.host()
    for i in range(k):
        assert_matmul_close(parts[i], ref_parts[i], 1e-5, f"partial {i}")
    Y = orc.matmul(X, W)
    for j, g in enumerate(d_b.host()):
        assert_psum_close(g, ref_parts, Y, f"P->B copy {j}")
    for j, (g, r) in enumerate(zip(d_s.host(), orc.boxing(ref_parts, orc.P_SUM, orc.S0, k))):
        sl = slice(*orc.split_range(64, k, j))
        assert_psum_close(g, [p[sl] for p in ref_parts], r, f"P->S(0) shard {j}")
    # the boxing of the GPU's own partials, checked against the oracle's reduction of THOSE partials
    rb = orc.assemble([p.astype(np.float64) for p in parts], orc.P_SUM)
    assert_psum_close(d_b.host()[0], parts, rb, "P->B of the GPU partials")


def test_table4_program_on_gpu():
    """A0[4,5] S(0) x B0[5,8] B -> Y0 S(0); box to B; x B1[8,6] S(1) -> Y2 S(1); k = 2 (Table 4)."""
    k = 2
    A0, B0, B1 = rnd_f32(1, (4, 5)), rnd_f32(2, (5, 8)), rnd_f32(3, (8, 6))
    d_a = DevTensor.from_host(orc.scatter(A0, orc.S0, k), 4, 5, orc.S0)
    d_b0 = DevTensor.from_host(orc.scatter(B0, orc.B, k), 5, 8, orc.B)
    d_b1 = DevTensor.from_host(orc.scatter(B1, orc.S1, k), 8, 6, orc.S1)
    y0 = DevTensor.empty(4, 8, np.float32, orc.S0, k)
    y0b = DevTensor.empty(4, 8, np.float32, orc.B, k)
    y2 = DevTensor.empty(4, 6, np.float32, orc.S1, k)
    sbp.sbp_matmul(d_a.desc, sbp.S(0), d_b0.desc, sbp.B, y0.desc, sbp.AUTO, k)
    with pytest.raises(sbp.SbpError):           # Y0 as S(0) cannot feed MatMul_1: boxing is explicit
        sbp.sbp_matmul(y0.desc, sbp.S(0), d_b1.desc, sbp.S(1), y2.desc, sbp.AUTO, k)
    sbp.sbp_boxing(y0.desc, sbp.S(0), y0b.desc, sbp.B, k)
    sbp.sbp_matmul(y0b.desc, sbp.B, d_b1.desc, sbp.S(1), y2.desc, sbp.S(1), k)
    sync()
    Y2 = orc.assemble([g.astype(np.float64) for g in y2.host()], orc.S1)
    assert_matmul_close(Y2, orc.matmul(orc.matmul(A0, B0), B1), 1e-5, "Table 4 chain")


def test_uvw_deferred_boxing_on_gpu():
    """U S(1), V S(0), W B: (UV) stays P(sum) through the second matmul; one boxing at the end."""
    k = 4
    U, V, W = rnd_f32(1, (24, 32)), rnd_f32(2, (32, 20)), rnd_f32(3, (20, 28))
    d_u = DevTensor.from_host(orc.scatter(U, orc.S1, k), 24, 32, orc.S1)
    d_v = DevTensor.from_host(orc.scatter(V, orc.S0, k), 32, 20, orc.S0)
    d_w = DevTensor.from_host(orc.scatter(W, orc.B, k), 20, 28, orc.B)
    uv = DevTensor.empty(24, 20, np.float32, orc.P_SUM, k)
    uvw = DevTensor.empty(24, 28, np.float32, orc.P_SUM, k)
    out = DevTensor.empty(24, 28, np.float32, orc.B, k)
    sbp.sbp_matmul(d_u.desc, sbp.S(1), d_v.desc, sbp.S(0), uv.desc, sbp.AUTO, k)
    sbp.sbp_matmul(uv.desc, sbp.P_SUM, d_w.desc, sbp.B, uvw.desc, sbp.AUTO, k)
    sbp.sbp_boxing(uvw.desc, sbp.P_SUM, out.desc, sbp.B, k)
    sync()
    ref = orc.matmul(orc.matmul(U, V), W)
    for g in out.host():
        assert_matmul_close(g, ref, 1e-4, "U.V.W with one boxing at the end")


def test_uvw_bf16_graph_box_late_equals_box_early():
    """Sec. 3.3 with bf16 tensors: U S(1), V S(0), W B.  Deferred: (UV) stays k fp32 partials, each is
    multiplied by W (row 4, fp32 partial x bf16), one boxing at the end.  Immediate: (UV) is boxed to
    B first (fp32), then multiplied by W (row 6, fp32 B x bf16 B).  Both must give U V W; they differ
    only in where the fp32 additions happen."""
    k = 4
    M, K1, N1, N2 = 200, 4 * 96, 264, 136
    U, V, W = rnd_bf16(1, (M, K1)), rnd_bf16(2, (K1, N1), 0.05), rnd_bf16(3, (N1, N2), 0.05)
    d_u = DevTensor.from_host(orc.scatter(U, orc.S1, k), M, K1, orc.S1)
    d_v = DevTensor.from_host(orc.scatter(V, orc.S0, k), K1, N1, orc.S0)
    d_w = DevTensor.from_host(orc.scatter(W, orc.B, k), N1, N2, orc.B)
    uv = DevTensor.empty(M, N1, np.float32, orc.P_SUM, k)
    sbp.sbp_matmul(d_u.desc, sbp.S(1), d_v.desc, sbp.S(0), uv.desc, sbp.AUTO, k)
    # deferred boxing
    uvw_p = DevTensor.empty(M, N2, np.float32, orc.P_SUM, k)
    late = DevTensor.empty(M, N2, np.float32, orc.B, k)
    sbp.sbp_matmul(uv.desc, sbp.P_SUM, d_w.desc, sbp.B, uvw_p.desc, sbp.AUTO, k)
    sbp.sbp_boxing(uvw_p.desc, sbp.P_SUM, late.desc, sbp.B, k)
    # immediate boxing
    uv_b = DevTensor.empty(M, N1, np.float32, orc.B, k)
    early = DevTensor.empty(M, N2, np.float32, orc.B, k)
    sbp.sbp_boxing(uv.desc, sbp.P_SUM, uv_b.desc, sbp.B, k)
    sbp.sbp_matmul(uv_b.desc, sbp.B, d_w.desc, sbp.B, early.desc, sbp.AUTO, k)
    sync()
    ref = orc.matmul(orc.matmul(values(U), values(V)), values(W))
    for j in range(k):
        assert_matmul_close(late.host()[j], ref, 1e-4, f"box late, copy {j}")
        assert_matmul_close(early.host()[j], ref, 1e-4, f"box early, copy {j}")
    # the partials of the deferred form, each against the oracle's X_i W
    ref_uv, _ = orc.matmul_sbp([values(x) for x in orc.scatter(U, orc.S1, k)], orc.S1,
                               [values(x) for x in orc.scatter(V, orc.S0, k)], orc.S0)
    ref_p, sy = orc.matmul_sbp(ref_uv, orc.P_SUM, [values(W)] * k, orc.B)
    assert sy == orc.P_SUM
    for i, g in enumerate(uvw_p.host()):
        assert_matmul_close(g, ref_p[i], 1e-4, f"(U_i V_i) W partial {i}")


@pytest.mark.parametrize("k", [1, 4, 8])
@pytest.mark.parametrize("cols", [4 * 8 * 40, 1003])
def test_model_parallel_softmax_statistics(k, cols):
    """bf16 logits S(1) -> local row max P(max) -> B -> local sum exp P(sum) -> B (Sec. 6.3.1)."""
    rows = 33
    L = rnd_bf16(7, (rows, cols), 3.0)
    Ls = orc.scatter(L, orc.S1, k)
    d_l = DevTensor.from_host(Ls, rows, cols, orc.S1)
    m_p = DevTensor.empty(rows, 1, np.float32, orc.P_MAX, k)
    m_b = DevTensor.empty(rows, 1, np.float32, orc.B, k)
    s_p = DevTensor.empty(rows, 1, np.float32, orc.P_SUM, k)
    s_b = DevTensor.empty(rows, 1, np.float32, orc.B, k)
    sbp.sbp_row_max(d_l.desc, sbp.S(1), m_p.desc, k)
    sbp.sbp_boxing(m_p.desc, sbp.P_MAX, m_b.desc, sbp.B, k)
    sbp.sbp_row_sumexp(d_l.desc, sbp.S(1), m_b.desc, s_p.desc, k)
    sbp.sbp_boxing(s_p.desc, sbp.P_SUM, s_b.desc, sbp.B, k)
    sync()
    Lv = [values(s) for s in Ls]
    m_loc = [orc.row_max(s)[:, None] if s.shape[1] else np.full((rows, 1), -np.inf) for s in Lv]
    for i, g in enumerate(m_p.host()):
        assert_bits_equal(g, m_loc[i].astype(np.float32), f"local max {i}")      # bf16 values are exact in fp32
    m = orc.boxing(m_loc, orc.P_MAX, orc.B, k)
    for g in m_b.host():
        assert_bits_equal(g, m[0].astype(np.float32), "global max")
    s_loc = [orc.row_sumexp(s, m[0][:, 0])[:, None] if s.shape[1] else np.zeros((rows, 1)) for s in Lv]
    for i, g in enumerate(s_p.host()):
        assert np.allclose(g, s_loc[i], rtol=1e-5, atol=0), f"local sum-exp {i}"
    s = orc.boxing(s_loc, orc.P_SUM, orc.B, k)
    for g in s_b.host():
        assert np.allclose(g, s[0], rtol=1e-5, atol=0)
    for j in range(1, k):
        assert_bits_equal(s_b.host()[j], s_b.host()[0], "denominator copies")


@pytest.mark.parametrize("k", [1, 4, 8])
@pytest.mark.parametrize("cols,dtype", [(4 * 8 * 40, "bf16"), (1003, "bf16"), (8 * 4 * 30, "f32")])
def test_model_parallel_sparse_cross_entropy(k, cols, dtype):
    """Sec. 6.3.1 continued: softmax statistics (max -> B, sum exp -> B), then the loss partials
    (P(sum) -> B) and the gradient (S(1), elementwise), against the oracle's model-parallel forms and
    through them against the plain definitions."""
    rows = 37
    torch = __import__("torch")
    if dtype == "bf16":
        L = rnd_bf16(9, (rows, cols), 3.0)
    else:
        L = (rnd_f32(9, (rows, cols)) * 3.0).astype(np.float32)
    np_dt = L.dtype
    y = (wl.uniform(SEED, 11, (rows, 1), 0.0, float(cols)).astype(np.int64) % cols).astype(np.int32)
    y[3, 0] = -1                    # two ignored rows
    y[7, 0] = cols + 5
    g = rnd_f32(12, (rows, 1))
    Ls = orc.scatter(L, orc.S1, k)
    d_l = DevTensor.from_host(Ls, rows, cols, orc.S1)
    vec = lambda sig: DevTensor.empty(rows, 1, np.float32, sig, k)      # noqa: E731
    m_p, m_b, s_p, s_b, l_p, l_b = vec(orc.P_MAX), vec(orc.B), vec(orc.P_SUM), vec(orc.B), vec(orc.P_SUM), vec(orc.B)
    d_g = DevTensor.from_host([g] * k, rows, 1, orc.B)
    y_dev = [torch.from_numpy(y.copy()).cuda() for _ in range(k)]
    d_y = sbp.SbpTensor(y_dev, rows, 1, sbp.I32)
    d_dl = DevTensor.empty(rows, cols, np_dt, orc.S1, k)
    sbp.sbp_row_max(d_l.desc, sbp.S(1), m_p.desc, k)
    sbp.sbp_boxing(m_p.desc, sbp.P_MAX, m_b.desc, sbp.B, k)
    sbp.sbp_row_sumexp(d_l.desc, sbp.S(1), m_b.desc, s_p.desc, k)
    sbp.sbp_boxing(s_p.desc, sbp.P_SUM, s_b.desc, sbp.B, k)
    sbp.sbp_xent_loss(d_l.desc, sbp.S(1), d_y, m_b.desc, s_b.desc, l_p.desc, k)
    sbp.sbp_boxing(l_p.desc, sbp.P_SUM, l_b.desc, sbp.B, k)
    sbp.sbp_xent_grad(d_l.desc, sbp.S(1), d_y, m_b.desc, s_b.desc, d_g.desc, d_dl.desc, k)
    sync()
    Lv = [values(s) for s in Ls]
    m = m_b.host()[0][:, 0].astype(np.float64)
    s = s_b.host()[0][:, 0].astype(np.float64)
    # loss partials against the oracle's, fed with the GPU's own m and s (both fp32 images)
    ref_parts = orc.xent_loss_sbp(Lv, y[:, 0], m, s)
    for i, got in enumerate(l_p.host()):
        assert np.allclose(got[:, 0], ref_parts[i], rtol=2e-6, atol=2e-6), f"loss partial {i}"
    loss = l_b.host()[0][:, 0]
    plain = orc.softmax_xent_loss(values(L), y[:, 0])
    assert np.allclose(loss, plain, rtol=1e-5, atol=1e-5), "loss against the plain definition"
    assert loss[3] == 0.0 and loss[7] == 0.0
    for j in range(1, k):
        assert_bits_equal(l_b.host()[j], l_b.host()[0], "loss copies")
    # gradient
    ref_g = orc.xent_grad_sbp(Lv, y[:, 0], m, s, g[:, 0])
    plain_g = orc.scatter(orc.softmax_xent_grad(values(L), y[:, 0], g[:, 0]), orc.S1, k)
    for i, got in enumerate(d_dl.host()):
        gv = values(got)
        tol = 2.0 ** -7 if dtype == "bf16" else 2e-5       # one bf16 rounding step / fp32 exp
        assert gv.shape == ref_g[i].shape
        assert np.all(np.abs(gv - ref_g[i]) <= tol * np.abs(ref_g[i]) + 1e-12), f"gradient shard {i}"
        assert np.all(np.abs(gv - plain_g[i]) <= 2 * tol * np.abs(plain_g[i]) + 1e-7), f"gradient shard {i} vs plain"
        if gv.size:
            assert np.all(gv[3] == 0.0) and np.all(gv[7] == 0.0)


@pytest.mark.parametrize("shape,k", [((1000, 256, 3 * 1304), 3), ((300, 128, 2 * 520), 2), ((45, 100, 3 * 17), 3), ((64, 64, 8 * 16), 8)])
def test_matmul_with_fused_row_max(shape, k):
    """sbp_matmul_rowmax: (B, S(1)) -> S(1) bf16 logits plus their local row maxima (P(max)) in one
    call.  The first two shapes take the persistent kernel with the maximum folded into its stores
    (several tiles per workgroup, ragged right and bottom edges), the others the two-pass form.  The
    logits must be bit-identical to sbp_matmul's and the maxima bit-identical to sbp_row_max of them;
    both are then checked against the oracle."""
    M, K, N = shape
    X, W = rnd_bf16(21, (M, K)), rnd_bf16(22, (K, N), 0.05)
    X[5, :] = 0                                  # a row of zero logits (+0 / -0 products)
    W[:, 7] = np.uint16(0x8000)                  # a column of -0
    Xs, Ws = orc.scatter(X, orc.B, k), orc.scatter(W, orc.S1, k)
    dx, dw = DevTensor.from_host(Xs, M, K, orc.B), DevTensor.from_host(Ws, K, N, orc.S1)
    y_plain = DevTensor.empty(M, N, np.uint16, orc.S1, k)
    y_fused = DevTensor.empty(M, N, np.uint16, orc.S1, k)
    m_sep, m_fused = DevTensor.empty(M, 1, np.float32, orc.P_MAX, k), DevTensor.empty(M, 1, np.float32, orc.P_MAX, k)
    sbp.sbp_matmul(dx.desc, sbp.B, dw.desc, sbp.S(1), y_plain.desc, sbp.S(1), k)
    sbp.sbp_row_max(y_plain.desc, sbp.S(1), m_sep.desc, k)
    sbp.sbp_matmul_rowmax(dx.desc, sbp.B, dw.desc, sbp.S(1), y_fused.desc, sbp.AUTO, m_fused.desc, k)
    sync()
    ref, _ = orc.matmul_sbp([values(x) for x in Xs], orc.B, [values(w) for w in Ws], orc.S1)
    for i in range(k):
        assert_bits_equal(y_fused.host()[i], y_plain.host()[i], f"logits shard {i}")
        assert_matmul_close(values(y_fused.host()[i]), ref[i], 2e-2, f"logits shard {i} vs oracle")
        got_m, sep_m = m_fused.host()[i][:, 0], m_sep.host()[i][:, 0]
        assert np.array_equal(got_m, sep_m), f"row max shard {i}: fused vs separate"     # values (+0 == -0)
        assert np.array_equal(got_m.astype(np.float64), orc.row_max(values(y_fused.host()[i]))), f"row max shard {i} vs oracle"
    with pytest.raises(sbp.SbpError):           # a row-split result has no partial row maxima
        sbp.sbp_matmul_rowmax(DevTensor.from_host(orc.scatter(X, orc.S0, k), M, K, orc.S0).desc, sbp.S(0),
                              DevTensor.from_host(orc.scatter(W, orc.B, k), K, N, orc.B).desc, sbp.B,
                              DevTensor.empty(M, N, np.uint16, orc.S0, k).desc, sbp.AUTO, m_fused.desc, k)
