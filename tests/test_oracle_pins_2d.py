"""Pins for the oracle's two-dimensional SBP functions (Sec. 3.3, Table 3).  CPU only.

What the paper and the mathematics fix: the two rows Table 3 prints; that local products under a
2-D signature pair stand for XW exactly when each grid axis on its own is a row of Table 1 (found
here by brute force with numpy's matmul over all 256 pairs, not read from the oracle's table);
round trips; the reassembly invariant of boxing along either grid axis; k0 = 1 or k1 = 1 reducing
to the one-dimensional functions.
"""
import itertools
import os
import re

import numpy as np
import pytest

import oracle as orc
from oracle import B, P_SUM, S0, S1

RNG = np.random.default_rng(2110150323)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
SIG = {"S(0)": S0, "S(1)": S1, "B": B, "P(sum)": P_SUM, "P": P_SUM}


def _rows():
    out = []
    for line in open(os.path.join(GOLDEN, "table3_matmul_2d_sbp.txt")):
        if line.startswith("#") or not line.strip():
            continue
        pairs = re.findall(r"\(([^,()]+(?:\(\d\))?),\s*([^()]+?(?:\([^)]*\))?)\)", line)
        assert len(pairs) == 3, line
        out.append(tuple((SIG[a.strip()], SIG[b.strip()]) for a, b in pairs))
    return out


def _partials(T, k):
    parts = [RNG.standard_normal(T.shape) for _ in range(k - 1)]
    return parts + [T - np.sum(parts, axis=0)]


def _scatter2_random(T, sbp2, k0, k1):
    """like orc.scatter2, but a P position gets random partials (so that nothing passes by luck)"""
    nodes = _partials(T, k0) if sbp2[0] == P_SUM else orc.scatter(T, sbp2[0], k0)
    if sbp2 == (B, P_SUM):
        # replicated nodes must stay bit-identical after reduction: the same partials on every node
        ps = _partials(T, k1)
        return [p.copy() for _ in range(k0) for p in ps]
    out = []
    for n in nodes:
        out.extend(_partials(n, k1) if sbp2[1] == P_SUM else orc.scatter(n, sbp2[1], k1))
    return out


def test_table3_rows_as_printed():
    rows = _rows()
    assert len(rows) == 2
    for sx, sw, sy in rows:
        assert orc.infer_matmul2(sx, sw) == sy
    k0, k1 = 2, 3
    M, K, N = 8, 9, 10
    X, W = RNG.standard_normal((M, K)), RNG.standard_normal((K, N))
    for sx, sw, sy in rows:
        Ys, got = orc.matmul_sbp2(_scatter2_random(X, sx, k0, k1), sx, _scatter2_random(W, sw, k0, k1), sw)
        assert got == sy
        for a in range(k0):
            for b in range(k1):
                assert Ys[a * k1 + b].shape == orc.local_shape2(M, N, sy, k0, k1, a, b)
        assert np.allclose(orc.assemble2(Ys, sy, k0, k1), X @ W, atol=1e-12)


def test_valid_2d_pairs_are_exactly_the_per_axis_products_of_table1():
    """Brute force over all 4^4 signature pairs on a 2 x 3 grid: local numpy products either have
    mismatched shapes, or stand for XW under exactly one 2-D signature, or under none.  The pairs
    that work, and their results, must be what Table 1 gives axis by axis: 36 of them, Table 3's two
    among them."""
    k0, k1 = 2, 3
    n = 12                                  # divisible by 2, 3 and 6: shapes alone never decide
    X, W = RNG.standard_normal((n, n)), RNG.standard_normal((n, n))
    Y = X @ W
    sigs = (S0, S1, B, P_SUM)
    found = {}
    for sx in itertools.product(sigs, repeat=2):
        for sw in itertools.product(sigs, repeat=2):
            Xs, Ws = _scatter2_random(X, sx, k0, k1), _scatter2_random(W, sw, k0, k1)
            if any(x.shape[1] != w.shape[0] for x, w in zip(Xs, Ws)):
                continue
            Ys = [x @ w for x, w in zip(Xs, Ws)]
            fits = []
            for sy in itertools.product(sigs, repeat=2):
                try:
                    got = orc.assemble2(Ys, sy, k0, k1)
                except (ValueError, AssertionError):
                    continue
                if got.shape == Y.shape and np.allclose(got, Y, atol=1e-9):
                    fits.append(sy)
            if fits:
                assert len(fits) == 1, (sx, sw, fits)
                found[(sx, sw)] = fits[0]
    table1 = {(S0, B): S0, (B, S1): S1, (S1, S0): P_SUM, (P_SUM, B): P_SUM, (B, P_SUM): P_SUM, (B, B): B}
    expect = {((x0, x1), (w0, w1)): (y0, y1)
              for (x0, w0), y0 in table1.items() for (x1, w1), y1 in table1.items()}
    assert found == expect
    assert len(found) == 36
    for sx, sw, sy in _rows():
        assert found[(sx, sw)] == sy
    for key, sy in expect.items():
        assert orc.infer_matmul2(*key) == sy
    assert orc.infer_matmul2((S0, S1), (B, S1)) is None and orc.infer_matmul2((S1, B), (B, B)) is None


@pytest.mark.parametrize("k0,k1", [(1, 1), (2, 2), (3, 2), (2, 5)])
def test_scatter2_assemble2_round_trip(k0, k1):
    T = RNG.standard_normal((11, 13))
    for sbp2 in itertools.product((S0, S1, B), repeat=2):
        sh = orc.scatter2(T, sbp2, k0, k1)
        assert len(sh) == k0 * k1
        for a in range(k0):
            for b in range(k1):
                assert sh[a * k1 + b].shape == orc.local_shape2(11, 13, sbp2, k0, k1, a, b)
        assert orc.assemble2(sh, sbp2, k0, k1).tobytes() == T.tobytes()
    for sbp2 in [(S0, P_SUM), (P_SUM, S1), (P_SUM, P_SUM), (B, P_SUM)]:
        assert np.allclose(orc.assemble2(_scatter2_random(T, sbp2, k0, k1), sbp2, k0, k1), T, atol=1e-12)


def test_nested_split_of_one_axis_is_a_finer_balanced_split_only_when_even():
    # (S(0), S(0)) on 2 x 2 devices over 8 rows is the 4-way split; over 7 rows it is 4 = 2+2, 3 = 2+1
    T = np.arange(8 * 3).reshape(8, 3)
    assert [s.shape[0] for s in orc.scatter2(T, (S0, S0), 2, 2)] == [2, 2, 2, 2]
    T = np.arange(7 * 3).reshape(7, 3)
    assert [s.shape[0] for s in orc.scatter2(T, (S0, S0), 2, 2)] == [2, 2, 2, 1]
    assert [s[0, 0] // 3 for s in orc.scatter2(T, (S0, S0), 2, 2)] == [0, 2, 4, 6]


def test_degenerate_grids_reduce_to_one_dimension():
    T = RNG.standard_normal((9, 10))
    for s in (S0, S1, B):
        for k in (1, 3):
            a = orc.scatter2(T, (s, B), k, 1)
            b = orc.scatter(T, s, k)
            assert all(x.tobytes() == y.tobytes() for x, y in zip(a, b))
            a = orc.scatter2(T, (B, s), 1, k)
            assert all(x.tobytes() == y.tobytes() for x, y in zip(a, b))


ALL2 = [s for s in itertools.product((S0, S1, B, P_SUM), repeat=2)]


@pytest.mark.parametrize("k0,k1", [(2, 3), (3, 2)])
def test_boxing2_never_changes_the_global_tensor(k0, k1):
    T = RNG.standard_normal((12, 18))
    n_checked = 0
    for si in ALL2:
        shards = _scatter2_random(T, si, k0, k1)
        for so in ALL2:
            changed = [si[0] != so[0], si[1] != so[1]]
            if sum(changed) != 1:
                continue
            try:
                out = orc.boxing2(shards, si, so, k0, k1)
            except ValueError:
                # the only refusals: outer conversion along the axis the inner position splits
                assert changed[0] and si[1] in (S0, S1) and si[1] in (si[0], so[0])
                continue
            for a in range(k0):
                for b in range(k1):
                    assert out[a * k1 + b].shape == orc.local_shape2(12, 18, so, k0, k1, a, b)
            assert np.allclose(orc.assemble2(out, so, k0, k1), T, atol=1e-12), (si, so)
            n_checked += 1
    assert n_checked > 60


def test_boxing2_inner_all_reduce_of_table3_row2():
    """(S(0), P(sum)) -> (S(0), B): every node all-reduces its own row block."""
    k0, k1 = 2, 3
    T = RNG.standard_normal((8, 6))
    sh = _scatter2_random(T, (S0, P_SUM), k0, k1)
    out = orc.boxing2(sh, (S0, P_SUM), (S0, B), k0, k1)
    for a in range(k0):
        block = T[slice(*orc.split_range(8, k0, a))]
        for b in range(k1):
            assert np.allclose(out[a * k1 + b], block, atol=1e-12)


def test_boxing2_refuses_to_reduce_an_outer_partial_under_an_inner_partial_of_the_other_op():
    """Sec. 3.3: (outer, inner) = outer-op over nodes of (inner-op over a node's devices).  With
    X_ab on device (a, b), (P(sum), P(max)) stands for sum_a max_b X_ab; summing over a per device
    would leave max_b sum_a X_ab, another tensor."""
    k0, k1 = 2, 2
    X = [np.array([[1.0]]), np.array([[5.0]]), np.array([[4.0]]), np.array([[2.0]])]   # X_00, X_01, X_10, X_11
    glob = orc.assemble2(X, (P_SUM, orc.P_MAX), k0, k1)
    assert glob.item() == max(1.0, 5.0) + max(4.0, 2.0) == 9.0
    naive = max(1.0 + 4.0, 5.0 + 2.0)          # outer sum first, device by device: 7, not 9
    assert naive != glob.item()
    for outer_out in (B, S0, S1):
        with pytest.raises(ValueError):
            orc.boxing2(X, (P_SUM, orc.P_MAX), (outer_out, orc.P_MAX), k0, k1)
        with pytest.raises(ValueError):
            orc.boxing2(X, (orc.P_MAX, P_SUM), (outer_out, P_SUM), k0, k1)
    # the inner position of the same signature may be reduced: every node takes its own max
    inner = orc.boxing2(X, (P_SUM, orc.P_MAX), (P_SUM, B), k0, k1)
    assert [x.item() for x in inner] == [5.0, 5.0, 4.0, 4.0]
    assert orc.assemble2(inner, (P_SUM, B), k0, k1).item() == 9.0
    # equal operations commute and stay allowed
    same = orc.boxing2(X, (P_SUM, P_SUM), (B, P_SUM), k0, k1)
    assert orc.assemble2(same, (B, P_SUM), k0, k1).item() == 12.0
