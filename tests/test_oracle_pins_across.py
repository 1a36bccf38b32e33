"""Pins for the oracle's boxing between disjoint placements (Sec. 3.2, Table 2, column "disjoint"):
the printed costs, the reassembly invariant, the same-placement routine where the two must agree,
and numpy's own split / concatenate on the S and B outputs.  CPU only."""
import itertools
import os

import numpy as np
import pytest

import oracle as orc
from oracle import B, P_MAX, P_SUM, S0, S1

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
RNG = np.random.default_rng(2110150322)
ALL = (S0, S1, B, P_SUM, P_MAX)


def _golden_rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def _shards(T, sbp, k):
    """k local tensors of T under sbp; partial ones random with the right reduction"""
    if sbp == P_SUM:
        parts = [RNG.standard_normal(T.shape) for _ in range(k - 1)]
        return parts + [T - np.sum(parts, axis=0)]
    if sbp == P_MAX:
        parts = [T - np.abs(RNG.standard_normal(T.shape)) - 0.5 for _ in range(k)]
        who = RNG.integers(0, k, size=T.shape)
        return [np.where(who == i, T, parts[i]) for i in range(k)]
    return orc.scatter(T, sbp, k)


def _valid(si, so):
    return not (si in (P_SUM, P_MAX) and so in (P_SUM, P_MAX) and si != so)   # the reduction cannot change


@pytest.mark.parametrize("p1,p2", [(2, 3), (3, 2), (4, 4), (1, 3), (4, 1), (2, 6)])
def test_table2_disjoint_costs(p1, p2):
    """count what travels by walking the routing and compare with the printed column"""
    rows, cols = 2 * p1 * p2, 3 * p1 * p2
    T = rows * cols
    table = {(a, b): expr for a, b, expr in _golden_rows("table2_transfer_cost_disjoint.txt")}
    assert len(table) == 10
    cases = {
        ("S(i)", "S(i)"): [(S0, S0), (S1, S1)],
        ("S(i)", "S(j)"): [(S0, S1), (S1, S0)],
        ("S", "B"): [(S0, B), (S1, B)],
        ("S", "P"): [(S0, P_SUM), (S1, P_SUM), (S0, P_MAX)],
        ("B", "S"): [(B, S0), (B, S1)],
        ("B", "B"): [(B, B)],
        ("B", "P"): [(B, P_SUM), (B, P_MAX)],
        ("P", "S"): [(P_SUM, S0), (P_SUM, S1), (P_MAX, S0)],
        ("P", "B"): [(P_SUM, B), (P_MAX, B)],
        ("P", "P"): [(P_SUM, P_SUM), (P_MAX, P_MAX)],
    }
    for key, pairs in cases.items():
        want = eval(table[key], {"p1": p1, "p2": p2}) * T     # noqa: S307 - fixture arithmetic
        for si, so in pairs:
            assert orc.transfer_elems_across(si, p1, so, p2, rows, cols) == want, (key, si, so)


@pytest.mark.parametrize("k_in,k_out", [(2, 3), (3, 2), (4, 4), (1, 5), (5, 1), (3, 8), (8, 3)])
@pytest.mark.parametrize("shape", [(12, 18), (7, 5), (1, 9)])
def test_reassembly_invariant_across(k_in, k_out, shape):
    """the global tensor is the same before and after, whatever the two device counts"""
    T = RNG.standard_normal(shape)
    for si, so in itertools.product(ALL, repeat=2):
        if not _valid(si, so):
            continue
        out = orc.boxing_across(_shards(T, si, k_in), si, so, k_out)
        assert len(out) == k_out
        for j in range(k_out):
            assert out[j].shape == orc.local_shape(shape[0], shape[1], so, k_out, j)
        np.testing.assert_allclose(orc.assemble(out, so), T, rtol=0, atol=1e-12, err_msg=f"{si}->{so}")


def test_across_is_numpy_split_for_split_outputs():
    """S and B outputs against numpy's own array_split / copies of the assembled tensor"""
    T = RNG.standard_normal((11, 13))
    for k_in, k_out in ((3, 4), (4, 3)):
        for si in (S0, S1, B, P_SUM):
            ins = _shards(T, si, k_in)
            G = orc.assemble(ins, si)
            for axis, so in ((0, S0), (1, S1)):
                out = orc.boxing_across(ins, si, so, k_out)
                for a, b in zip(out, np.array_split(G, k_out, axis=axis)):
                    np.testing.assert_allclose(a, b, rtol=0, atol=1e-12)
            for o in orc.boxing_across(ins, si, B, k_out):
                np.testing.assert_allclose(o, G, rtol=0, atol=1e-12)


@pytest.mark.parametrize("k", [1, 2, 3, 8])
def test_across_with_equal_counts_matches_same_placement_boxing(k):
    """with k_in = k_out the values every device ends up with are those of boxing on one device
    set (the routine pinned elsewhere) -- except B -> S, where the source copy differs but the
    copies are identical, and P -> P, which is a plain copy in both."""
    T = RNG.standard_normal((8, 12))
    for si, so in itertools.product(ALL, repeat=2):
        if not _valid(si, so):
            continue
        ins = _shards(T, si, k)
        a = orc.boxing_across(ins, si, so, k)
        b = orc.boxing(ins, si, so, k)
        for x, y in zip(a, b):
            np.testing.assert_allclose(np.asarray(x, dtype=np.float64), np.asarray(y, dtype=np.float64), rtol=0, atol=1e-12,
                                       err_msg=f"{si}->{so}")


def test_partial_to_partial_folds_in_input_order():
    """P -> P onto fewer devices: device j holds the combination of partials j, j + k_out, ...;
    onto more devices: the extra ones hold the identity"""
    T = RNG.standard_normal((4, 6))
    ins = _shards(T, P_SUM, 5)
    out = orc.boxing_across(ins, P_SUM, P_SUM, 2)
    np.testing.assert_allclose(out[0], ins[0] + ins[2] + ins[4], rtol=0, atol=1e-12)
    np.testing.assert_allclose(out[1], ins[1] + ins[3], rtol=0, atol=1e-12)
    out = orc.boxing_across(ins[:2], P_SUM, P_SUM, 4)
    assert np.array_equal(out[0], ins[0]) and np.array_equal(out[1], ins[1])
    assert not out[2].any() and not out[3].any()
    mx = _shards(T, P_MAX, 3)
    out = orc.boxing_across(mx, P_MAX, P_MAX, 2)
    assert np.array_equal(out[0], np.maximum(mx[0], mx[2])) and np.array_equal(out[1], mx[1])
    out = orc.boxing_across(mx[:1], P_MAX, P_MAX, 2)
    assert np.all(np.isneginf(out[1]))


def test_raw_words_survive_across():
    """relayout between placements moves NaN / Inf bit patterns untouched and keeps the dtype"""
    T = (np.arange(10 * 12, dtype=np.uint32).reshape(10, 12) * 2731).astype(np.uint16)
    T[0, :4] = [0x7F80, 0x7FC1, 0xFF80, 0xFFFF]
    for k_in, k_out in ((2, 3), (4, 2)):
        for si, so in itertools.product((S0, S1, B), repeat=2):
            out = orc.boxing_across(orc.scatter(T, si, k_in), si, so, k_out)
            assert out[0].dtype == np.uint16
            assert np.array_equal(orc.assemble(out, so), T)


def test_mixing_reductions_is_refused():
    T = RNG.standard_normal((4, 4))
    with pytest.raises(ValueError):
        orc.boxing_across(_shards(T, P_SUM, 2), P_SUM, P_MAX, 3)


def test_reassembly_invariant_on_random_geometry():
    """property test: any shape, any two device counts, any valid pair of signatures"""
    from hypothesis import given, settings, strategies as st

    @settings(max_examples=150, deadline=None)
    @given(st.integers(0, 23), st.integers(0, 23), st.integers(1, 9), st.integers(1, 9), st.integers(0, 4), st.integers(0, 4),
           st.integers(0, 2 ** 31 - 1))
    def check(rows, cols, k_in, k_out, a, b, seed):
        si, so = ALL[a], ALL[b]
        if not _valid(si, so):
            return
        rng = np.random.default_rng(seed)
        T = rng.standard_normal((rows, cols))
        if si == P_SUM:
            parts = [rng.standard_normal(T.shape) for _ in range(k_in - 1)]
            ins = parts + [T - np.sum(parts, axis=0) if parts else T.copy()]
        elif si == P_MAX:
            who = rng.integers(0, k_in, size=T.shape)
            ins = [np.where(who == i, T, T - 1.0 - np.abs(rng.standard_normal(T.shape))) for i in range(k_in)]
        else:
            ins = orc.scatter(T, si, k_in)
        out = orc.boxing_across(ins, si, so, k_out)
        assert len(out) == k_out
        for j in range(k_out):
            assert out[j].shape == orc.local_shape(rows, cols, so, k_out, j)
        np.testing.assert_allclose(orc.assemble(out, so), T, rtol=0, atol=1e-11)
        if k_in == k_out and so not in (P_SUM, P_MAX):
            same = orc.boxing(ins, si, so, k_in)
            for x, y in zip(out, same):
                np.testing.assert_allclose(x, y, rtol=0, atol=1e-11)

    check()
