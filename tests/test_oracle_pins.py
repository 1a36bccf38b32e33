"""Pins for the CPU oracle: everything here checks oracle/ against something
other than itself -- the paper's printed tables (tests/golden/), closed forms,
invariants, numpy / scipy / torch library routines on special cases, and pure
Python brute force on tiny inputs.  CPU only."""
import itertools
import math
import os
import re

import numpy as np
import pytest

import oracle as orc
from oracle import B, P_MAX, P_SUM, S0, S1

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
RNG = np.random.default_rng(20211015)


def _parse_sbp(tok):
    return {"S(0)": S0, "S(1)": S1, "B": B, "P(sum)": P_SUM, "P(max)": P_MAX}[tok]


def _golden_rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


# ---------------------------------------------------------------- split rule
@pytest.mark.parametrize("n,k", [(10, 3), (7, 8), (0, 4), (64, 2), (125000, 8), (17, 16), (5, 1)])
def test_split_range_balanced(n, k):
    ranges = [orc.split_range(n, k, i) for i in range(k)]
    # contiguous, ordered, covering [0, n)
    assert ranges[0][0] == 0 and ranges[-1][1] == n
    for a, b in zip(ranges, ranges[1:]):
        assert a[1] == b[0]
    sizes = [e - b for b, e in ranges]
    assert max(sizes) - min(sizes) <= 1            # "balanced"
    assert sizes == sorted(sizes, reverse=True)    # the longer shards come first
    # numpy's array_split follows the same convention
    assert sizes == [len(a) for a in np.array_split(np.arange(n), k)]


# ------------------------------------------------------ scatter / assemble
@pytest.mark.parametrize("k", [1, 2, 3, 8])
@pytest.mark.parametrize("shape", [(8, 12), (7, 5), (3, 17)])
def test_scatter_assemble_roundtrip_bitwise(k, shape):
    T = RNG.integers(0, 2 ** 16, size=shape, dtype=np.uint16)   # raw words, NaN patterns included
    for sbp, axis in ((S0, 0), (S1, 1)):
        sh = orc.scatter(T, sbp, k)
        assert len(sh) == k
        ref = np.array_split(T, k, axis=axis)
        for a, b in zip(sh, ref):
            assert a.shape == b.shape and np.array_equal(a, b)
        assert np.array_equal(orc.assemble(sh, sbp), T)
    sh = orc.scatter(T, B, k)
    assert all(np.array_equal(s, T) for s in sh)
    assert np.array_equal(orc.assemble(sh, B), T)


def test_k1_is_identity():
    T = RNG.standard_normal((5, 6))
    for sbp in (S0, S1, B, P_SUM, P_MAX):
        assert np.array_equal(orc.assemble(orc.scatter(T, sbp, 1), sbp), T)


def test_assemble_broadcast_rejects_diverged_copies():
    T = RNG.standard_normal((4, 4))
    sh = orc.scatter(T, B, 3)
    sh[2][1, 1] += 1.0
    with pytest.raises(AssertionError):
        orc.assemble(sh, B)


def test_assemble_partial_is_elementwise_reduction():
    parts = [RNG.standard_normal((6, 5)) for _ in range(4)]
    assert np.allclose(orc.assemble(parts, P_SUM), np.sum(np.stack(parts), axis=0), rtol=0, atol=1e-14)
    assert np.array_equal(orc.assemble(parts, P_MAX), np.max(np.stack(parts), axis=0))
    # brute force, scalar loops
    ref = [[sum(p[r, c] for p in parts) for c in range(5)] for r in range(6)]
    assert np.allclose(orc.assemble(parts, P_SUM), np.array(ref), rtol=0, atol=1e-14)


# ----------------------------------------------------------- plain matmul
def test_matmul_against_numpy_and_python_loops():
    A = RNG.standard_normal((5, 7))
    W = RNG.standard_normal((7, 3))           # all three extents differ: a transposed operand cannot pass
    C = orc.matmul(A, W)
    assert C.shape == (5, 3)
    assert np.allclose(C, A @ W, rtol=0, atol=1e-13)
    ref = [[sum(A[m, q] * W[q, n] for q in range(7)) for n in range(3)] for m in range(5)]
    assert np.allclose(C, np.array(ref), rtol=0, atol=1e-13)


def test_matmul_exact_on_small_integers():
    A = RNG.integers(-8, 9, size=(33, 65)).astype(np.float64)
    W = RNG.integers(-8, 9, size=(65, 17)).astype(np.float64)
    assert np.array_equal(orc.matmul(A, W), (A.astype(np.int64) @ W.astype(np.int64)).astype(np.float64))


# ------------------------------------------------- Table 1 by brute force
def _local_products(Xs, Ws):
    out = []
    for x, w in zip(Xs, Ws):
        if x.shape[1] != w.shape[0]:
            return None
        out.append(x @ w)           # numpy here on purpose: independent of the oracle's matmul
    return out


def _random_partial(T, k, op):
    """k random local tensors that reduce to T under op"""
    if op == "sum":
        parts = [RNG.standard_normal(T.shape) for _ in range(k - 1)]
        return parts + [T - np.sum(parts, axis=0)]
    parts = [T - np.abs(RNG.standard_normal(T.shape)) for _ in range(k)]
    who = RNG.integers(0, k, size=T.shape)
    for i in range(k):
        parts[i] = np.where(who == i, T, parts[i])
    return parts


def _holds(Ys, sbp, Y):
    try:
        if sbp == B:
            return all(y.shape == Y.shape and np.allclose(y, Y, atol=1e-9) for y in Ys)
        got = orc.assemble(Ys, sbp)
    except (ValueError, AssertionError):
        return False
    return got.shape == Y.shape and np.allclose(got, Y, atol=1e-9)


@pytest.mark.parametrize("k", [2, 3])
def test_table1_is_exactly_what_the_mathematics_allows(k):
    """For every (sbp_X, sbp_W) in {S(0), S(1), B, P(sum)}^2 take local products on random
    inputs and ask under which 1-D signature, if any, they stand for XW.  The answer must
    be the paper's Table 1, row for row, and nothing else."""
    printed = {(_parse_sbp(a), _parse_sbp(b)): _parse_sbp(c)
               for a, b, c in _golden_rows("table1_matmul_sbp.txt")}
    assert len(printed) == 6
    M, K, N = 6 * k, 6 * k, 6 * k      # square and divisible so shapes alone never decide a value case
    X = RNG.standard_normal((M, K))
    W = RNG.standard_normal((K, N))
    Y = X @ W

    def shard(T, sbp):
        return _random_partial(T, k, "sum") if sbp == P_SUM else orc.scatter(T, sbp, k)

    derived = {}
    for sx, sw in itertools.product((S0, S1, B, P_SUM), repeat=2):
        Ys = _local_products(shard(X, sx), shard(W, sw))
        if Ys is None:
            continue
        fits = [s for s in (S0, S1, B, P_SUM) if _holds(Ys, s, Y)]
        if fits:
            assert len(fits) == 1
            derived[(sx, sw)] = fits[0]
    assert derived == printed
    # and the oracle's own table is the printed one
    for sx, sw in itertools.product((S0, S1, B, P_SUM, P_MAX), repeat=2):
        assert orc.infer_matmul(sx, sw) == printed.get((sx, sw))


@pytest.mark.parametrize("k", [1, 2, 4])
@pytest.mark.parametrize("row", range(6))
def test_matmul_sbp_rows_reassemble_to_XW(k, row):
    sx, sw, sy = [(_parse_sbp(a), _parse_sbp(b), _parse_sbp(c))
                  for a, b, c in _golden_rows("table1_matmul_sbp.txt")][row]
    M, K, N = 9, 10, 11                # uneven splits included
    X = RNG.standard_normal((M, K))
    W = RNG.standard_normal((K, N))
    Xs = _random_partial(X, k, "sum") if sx == P_SUM else orc.scatter(X, sx, k)
    Ws = _random_partial(W, k, "sum") if sw == P_SUM else orc.scatter(W, sw, k)
    Ys, got_sy = orc.matmul_sbp(Xs, sx, Ws, sw)
    assert got_sy == sy
    for i, y in enumerate(Ys):
        assert y.shape == orc.local_shape(M, N, sy, k, i)
    assert np.allclose(orc.assemble(Ys, sy), X @ W, rtol=0, atol=1e-12)


def test_matmul_sbp_rejects_invalid_pairs():
    X = [np.zeros((4, 4))] * 2
    for sx, sw in [(S0, S1), (S1, S1), (S0, S0), (S1, B), (B, S0), (P_SUM, P_SUM), (S0, P_SUM), (P_MAX, B)]:
        with pytest.raises(ValueError):
            orc.matmul_sbp(X, sx, X, sw)


# ------------------------------------------------------------ boxing
ALL = (S0, S1, B, P_SUM, P_MAX)


def _valid_boxing(si, so):
    if so in (P_SUM, P_MAX) and si in (P_SUM, P_MAX):
        return si == so
    return True


@pytest.mark.parametrize("k", [1, 2, 3, 5])
@pytest.mark.parametrize("si,so", [(a, b) for a in ALL for b in ALL if _valid_boxing(a, b)])
def test_boxing_never_changes_the_global_tensor(k, si, so):
    T = RNG.standard_normal((7, 11))
    if si in (P_SUM, P_MAX):
        shards = _random_partial(T, k, si[1])
    else:
        shards = orc.scatter(T, si, k)
    out = orc.boxing(shards, si, so, k)
    assert len(out) == k
    for j, o in enumerate(out):
        assert o.shape == orc.local_shape(7, 11, so, k, j)
    got = orc.assemble(out, so)
    if si in (S0, S1, B) and so in (S0, S1, B):
        assert got.tobytes() == T.tobytes()                     # pure moves: bitwise
    elif si == P_MAX or (si in (S0, S1, B) and so == P_MAX):
        assert np.array_equal(got, T)
    else:
        assert np.allclose(got, T, rtol=0, atol=1e-12)


def test_boxing_B_to_S_reads_the_copy_on_the_same_device():
    """Sec. 3.2: B->S is free because the output comes from the input on the same device.
    Give every device a *different* 'copy' and see which one each slice came from."""
    k = 4
    copies = [np.full((8, 8), float(j)) for j in range(k)]
    for so in (S0, S1):
        out = orc.boxing(copies, B, so, k)
        for j in range(k):
            assert np.all(out[j] == float(j))


def test_boxing_raw_words_survive():
    """relayout boxing must move NaN / Inf bit patterns untouched"""
    T = np.arange(16 * 24, dtype=np.uint32).reshape(16, 24).astype(np.uint16) * np.uint16(2731)
    T[0, :4] = [0x7F80, 0x7FC1, 0xFF80, 0xFFFF]
    for k in (2, 3, 8):
        for si, so in itertools.permutations((S0, S1, B), 2):
            out = orc.boxing(orc.scatter(T, si, k), si, so, k)
            assert out[0].dtype == np.uint16
            assert np.array_equal(orc.assemble(out, so), T)


@pytest.mark.parametrize("p", [2, 3, 4])
def test_table2_same_device_costs(p):
    """count moved elements by walking the routing and compare with the printed closed forms"""
    rows, cols = 2 * p, 3 * p
    T = rows * cols
    table = {(a, b): cost for a, b, cost, _ in _golden_rows("table2_transfer_cost.txt")}
    assert len(table) == 10

    def closed(expr):
        if expr == "0":
            return 0
        num, den = expr.rsplit("/", 1)
        return eval(num, {"p": p}) * T / eval(den, {"p": p})     # noqa: S307 - fixture arithmetic

    cases = {
        ("S(i)", "S(i)"): [(S0, S0), (S1, S1)],
        ("S(i)", "S(j)"): [(S0, S1), (S1, S0)],
        ("S", "B"): [(S0, B), (S1, B)],
        ("S", "P"): [(S0, P_SUM), (S1, P_SUM)],
        ("B", "S"): [(B, S0), (B, S1)],
        ("B", "B"): [(B, B)],
        ("B", "P"): [(B, P_SUM)],
        ("P", "S"): [(P_SUM, S0), (P_SUM, S1), (P_MAX, S0)],
        ("P", "B"): [(P_SUM, B), (P_MAX, B)],
        ("P", "P"): [(P_SUM, P_SUM)],
    }
    for key, pairs in cases.items():
        for si, so in pairs:
            assert orc.transfer_elems(si, so, rows, cols, p) == closed(table[key]), (key, si, so)


def test_zero_cost_boxings_keep_every_value_on_its_device():
    """S->P and B->P cost 0 in Table 2: what a device outputs must be computable from what it holds"""
    k = 3
    T = RNG.standard_normal((6, 9))
    for si in (S0, S1):
        shards = orc.scatter(T, si, k)
        out = orc.boxing(shards, si, P_SUM, k)
        for j in range(k):
            nz = out[j] != 0
            held = np.zeros_like(T, dtype=bool)
            b, e = orc.split_range(T.shape[si[1]], k, j)
            if si == S0:
                held[b:e, :] = True
            else:
                held[:, b:e] = True
            assert not np.any(nz & ~held)
    out = orc.boxing(orc.scatter(T, B, k), B, P_SUM, k)
    assert np.array_equal(out[0], T) and all(not o.any() for o in out[1:])


# ------------------------------------------------- chains the paper gives
def test_table4_program():
    spec = {r[0]: r[1:] for r in _golden_rows("table4_program.txt")}
    k = int(spec["k"][0])
    shp = lambda n: (int(spec[n][0]), int(spec[n][1]))     # noqa: E731
    A0 = RNG.standard_normal(shp("A0"))
    B0 = RNG.standard_normal(shp("B0"))
    B1 = RNG.standard_normal(shp("B1"))
    Y0s, s_y0 = orc.matmul_sbp(orc.scatter(A0, _parse_sbp(spec["A0"][2]), k), S0,
                               orc.scatter(B0, _parse_sbp(spec["B0"][2]), k), B)
    assert s_y0 == S0                                      # "inferred (as split(0))"
    with pytest.raises(ValueError):                        # MatMul_1 cannot take Y0 as S(0) with B1 S(1)
        orc.matmul_sbp(Y0s, S0, orc.scatter(B1, S1, k), S1)
    Y0b = orc.boxing(Y0s, S0, B, k)                        # to_global(..., broadcast): an all-gather
    Y2s, s_y2 = orc.matmul_sbp(Y0b, B, orc.scatter(B1, S1, k), S1)
    assert s_y2 == _parse_sbp(spec["Y2"][2])
    Y2 = orc.assemble(Y2s, s_y2)
    assert Y2.shape == shp("Y2")
    assert np.allclose(Y2, (A0 @ B0) @ B1, rtol=0, atol=1e-12)


@pytest.mark.parametrize("k", [2, 4])
def test_uvw_deferred_boxing(k):
    """Sec. 3.3: U S(1), V S(0), W B.  UV is P(sum); (UV)W is valid and P(sum); boxing once at the
    end gives what boxing in the middle gives."""
    U = RNG.standard_normal((6, 8))
    V = RNG.standard_normal((8, 5))
    W = RNG.standard_normal((5, 7))
    UVs, s1 = orc.matmul_sbp(orc.scatter(U, S1, k), S1, orc.scatter(V, S0, k), S0)
    assert s1 == P_SUM
    Ws = orc.scatter(W, B, k)
    late, s2 = orc.matmul_sbp(UVs, P_SUM, Ws, B)
    assert s2 == P_SUM
    late_B = orc.boxing(late, P_SUM, B, k)
    early, s3 = orc.matmul_sbp(orc.boxing(UVs, P_SUM, B, k), B, Ws, B)
    assert s3 == B
    ref = U @ V @ W
    for a, b in zip(late_B, early):
        assert np.allclose(a, b, rtol=0, atol=1e-12)
        assert np.allclose(a, ref, rtol=0, atol=1e-12)


# ------------------------------------------------------ bf16, GeLU, softmax
def test_bf16_round_matches_torch_cast_and_known_ties():
    import torch
    x32 = np.concatenate([
        RNG.standard_normal(20000).astype(np.float32),
        (RNG.standard_normal(2000) * 1e-39).astype(np.float32),          # bf16 subnormals
        np.float32([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 3.4e38, -3.4e38,
                    np.inf, -np.inf, 2.0 ** -133, 2.0 ** -134, 1.5 * 2.0 ** -133]),
    ])
    got = orc.bf16_round(x32.astype(np.float64))
    ref = torch.from_numpy(x32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, ref)
    # ties go to the even mantissa; values the format fixes
    assert list(orc.bf16_round([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, -2.0])) == [0x3F80, 0x3F80, 0x3F82, 0xC000]
    # a double just above a tie must round up even though it is a tie after a detour through fp32
    assert orc.bf16_round([1.0 + 2 ** -8 + 2 ** -40])[0] == 0x3F81
    # widening is exact
    bits = RNG.integers(0, 2 ** 16, size=5000, dtype=np.uint16)
    bits = bits[(bits & 0x7F80) != 0x7F80]
    back = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(orc.bf16_to_f64(bits), back)
    assert np.array_equal(orc.bf16_round(orc.bf16_to_f64(bits)), bits)


def test_gelu_erf_form():
    import torch
    x = np.linspace(-6, 6, 241)
    y = orc.gelu(x)
    assert y[120] == 0.0
    assert np.allclose(y - orc.gelu(-x), x, rtol=0, atol=1e-14)          # x Phi(x) + x Phi(-x) = x
    ref = np.array([0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0))) for v in x])
    assert np.allclose(y, ref, rtol=0, atol=1e-15)
    t = torch.nn.functional.gelu(torch.from_numpy(x))                    # default = erf form
    assert np.allclose(y, t.numpy(), rtol=0, atol=1e-14)
    # the tanh approximation is a different function: the oracle must not be it
    tanh = 0.5 * x * (1 + np.tanh(math.sqrt(2 / math.pi) * (x + 0.044715 * x ** 3)))
    assert np.max(np.abs(y - tanh)) > 1e-4


@pytest.mark.parametrize("k", [1, 4, 8])
def test_model_parallel_softmax_statistics(k):
    """Sec. 6.3.1: local max -> global max, local sum of exp -> global sum.  The result must not
    depend on k and must agree with scipy's logsumexp on the whole row."""
    from scipy.special import logsumexp
    L = RNG.standard_normal((5, 40)) * 3.0
    shards = orc.scatter(L, S1, k)
    m_loc = [orc.row_max(s)[:, None] for s in shards]                     # P(max)
    m = orc.boxing(m_loc, P_MAX, B, k)                                    # -> B
    assert np.array_equal(m[0][:, 0], L.max(axis=1))
    s_loc = [orc.row_sumexp(s, m[i][:, 0])[:, None] for i, s in enumerate(shards)]   # P(sum)
    s = orc.boxing(s_loc, P_SUM, B, k)
    assert np.allclose(np.log(s[0][:, 0]) + m[0][:, 0], logsumexp(L, axis=1), rtol=0, atol=1e-12)
    probs = np.exp(L - m[0]) / s[0]
    assert np.allclose(probs.sum(axis=1), 1.0, rtol=0, atol=1e-12)


# ------------------------------------------------ planted mistakes are caught
def test_pins_catch_a_transposed_or_missplit_oracle(monkeypatch):
    """sanity of the pins themselves: a wrong split rule fails the numpy cross-check"""
    import oracle.sbp_oracle as impl

    def bad_split(n, k, i):                      # remainder on the LAST shards instead of the first
        q, r = divmod(n, k)
        b = i * q + max(0, i - (k - r))
        return b, b + q + (1 if i >= k - r else 0)

    monkeypatch.setattr(impl, "split_range", bad_split)
    T = np.arange(70).reshape(10, 7)
    sh = impl.scatter(T, S0, 3)
    ref = np.array_split(T, 3, axis=0)
    assert any(a.shape != b.shape for a, b in zip(sh, ref))


# ------------------------------------------------------------ sparse cross entropy (Sec. 6.3.1)
def test_softmax_xent_against_scipy_and_finite_differences():
    from scipy.special import log_softmax, softmax
    R, C = 9, 23
    L = RNG.standard_normal((R, C)) * 3.0
    y = RNG.integers(0, C, size=R)
    y[2] = -1                                        # ignored row
    g = RNG.standard_normal(R)
    loss = orc.softmax_xent_loss(L, y)
    ref = -log_softmax(L, axis=1)[np.arange(R), np.where(y >= 0, y, 0)]
    ref[2] = 0.0
    assert np.allclose(loss, ref, rtol=1e-13, atol=1e-13)
    grad = orc.softmax_xent_grad(L, y, g)
    onehot = np.zeros((R, C))
    onehot[np.arange(R)[y >= 0], y[y >= 0]] = 1.0
    gg = np.where(y >= 0, g, 0.0)
    assert np.allclose(grad, (softmax(L, axis=1) - onehot) * gg[:, None], rtol=1e-12, atol=1e-14)
    assert np.allclose(grad.sum(axis=1), 0.0, atol=1e-14)          # softmax sums to one
    assert np.all(grad[2] == 0.0)
    # central differences of sum_r g[r] loss[r]
    eps = 1e-6
    for r, c in [(0, int(y[0])), (1, 5), (4, 0), (8, C - 1)]:
        Lp, Lm = L.copy(), L.copy()
        Lp[r, c] += eps
        Lm[r, c] -= eps
        num = (np.dot(gg, orc.softmax_xent_loss(Lp, y)) - np.dot(gg, orc.softmax_xent_loss(Lm, y))) / (2 * eps)
        assert abs(num - grad[r, c]) < 1e-8


@pytest.mark.parametrize("k", [1, 3, 8])
def test_model_parallel_xent_is_the_plain_one_for_every_shard_count(k):
    R, C = 7, 41
    L = RNG.standard_normal((R, C)) * 2.0
    y = RNG.integers(0, C, size=R)
    y[5] = C + 3                                     # ignored row
    g = RNG.standard_normal(R)
    Ls = orc.scatter(L, S1, k)
    m = orc.assemble([orc.row_max(s)[:, None] if s.shape[1] else np.full((R, 1), -np.inf) for s in Ls], P_MAX)[:, 0]
    s = orc.assemble([orc.row_sumexp(x, m)[:, None] if x.shape[1] else np.zeros((R, 1)) for x in Ls], P_SUM)[:, 0]
    parts = orc.xent_loss_sbp(Ls, y, m, s)
    assert len(parts) == k
    assert np.allclose(orc.assemble([p[:, None] for p in parts], P_SUM)[:, 0], orc.softmax_xent_loss(L, y), atol=1e-12)
    # exactly one device contributes per (non-ignored) row
    assert np.array_equal(sum((p != 0).astype(int) for p in parts), (np.arange(R) != 5).astype(int))
    grads = orc.xent_grad_sbp(Ls, y, m, s, g)
    assert np.allclose(orc.assemble(grads, S1), orc.softmax_xent_grad(L, y, g), atol=1e-13)


def test_partial_max_ignores_nan_next_to_a_number():
    """Reading for P(max) and the row maximum (the paper names the operation only): a NaN counts as
    missing, whatever its position; only all-NaN gives NaN.  numpy's fmax is that rule."""
    nan = float("nan")
    parts = [np.array([[nan, 1.0, -2.0, nan, -0.0]]), np.array([[3.0, nan, -5.0, nan, 0.0]]), np.array([[2.0, 0.5, nan, nan, -0.0]])]
    got = orc.assemble(parts, orc.P_MAX)
    want = np.fmax(np.fmax(parts[0], parts[1]), parts[2])
    assert np.array_equal(got[:, :3], want[:, :3]) and np.array_equal(got[:, :3], np.array([[3.0, 1.0, -2.0]]))
    assert np.isnan(got[0, 3]) and got[0, 4] == 0.0
    L = np.array([[nan, -1.0, -3.0], [-7.0, nan, -6.0], [nan, nan, nan]])
    m = orc.row_max(L)
    assert m[0] == -1.0 and m[1] == -6.0 and np.isnan(m[2])
