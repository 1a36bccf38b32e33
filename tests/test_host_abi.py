"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares, and
its host logic (Table 1, split geometry, argument validation) behaves as documented.  No kernel is
launched here: every call either is host-only or must fail validation before any launch."""
import ctypes
import itertools
import os
import re

import numpy as np
import pytest

import oracle as orc
import paper_2110_15032_amd as sbp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(ROOT, "tests", "golden")
SIG = {"S(0)": sbp.S(0), "S(1)": sbp.S(1), "B": sbp.B, "P(sum)": sbp.P_SUM, "P(max)": sbp.P_MAX}


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "sbp.h")).read()
    declared = set(re.findall(r"\b(sbp_[a-z_0-9]+)\s*\(", hdr))
    assert declared, "no declarations found"
    assert declared == set(sbp.EXPORTS)
    raw = ctypes.CDLL(sbp.lib_path())
    for name in declared:
        assert hasattr(raw, name), f"{name} not exported"


def test_strerror_covers_every_code():
    seen = set()
    for code in range(0, -11, -1):
        msg = sbp.sbp_strerror(code)
        assert msg and msg != "unknown status"
        seen.add(msg)
    assert len(seen) == 11
    assert sbp.sbp_strerror(-99) == "unknown status"


def test_table1_through_the_abi_matches_the_printed_table():
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "table1_matmul_sbp.txt"))
            if ln.strip() and not ln.startswith("#")]
    printed = {(SIG[a], SIG[b]): SIG[c] for a, b, c in rows}
    for sx, sw in itertools.product(SIG.values(), repeat=2):
        if (sx, sw) in printed:
            assert sbp.sbp_infer_matmul(sx, sw) == printed[(sx, sw)]
        else:
            with pytest.raises(sbp.SbpError) as e:
                sbp.sbp_infer_matmul(sx, sw)
            assert e.value.status == -6
    with pytest.raises(sbp.SbpError) as e:
        sbp.sbp_infer_matmul(2, sbp.B)          # split axis 2 is not a signature of a matrix
    assert e.value.status == -5


@pytest.mark.parametrize("n,k", [(10, 3), (7, 8), (125000, 8), (1000000, 8), (5, 1), (0, 2)])
def test_local_shape_uses_the_balanced_split(n, k):
    for i in range(k):
        b, e = orc.split_range(n, k, i)
        assert sbp.sbp_local_shape(n, 3, sbp.S(0), k, i) == (e - b, 3)
        assert sbp.sbp_local_shape(3, n, sbp.S(1), k, i) == (3, e - b)
        assert sbp.sbp_local_shape(n, 3, sbp.B, k, i) == (n, 3)
        assert sbp.sbp_local_shape(n, 3, sbp.P_SUM, k, i) == (n, 3)


# ----------------------------------------------------------------------------- validation
def fake(k, rows, cols, dtype=sbp.F32, base=0x10000000, step=0x1000000, trans=0, ld=0):
    """descriptor over made-up, well-aligned, non-overlapping addresses (never dereferenced:
    every call below must be rejected before a launch)"""
    return sbp.SbpTensor([base + i * step for i in range(k)], rows, cols, dtype, trans, ld)


def status_of(fn, *a, **kw):
    with pytest.raises(sbp.SbpError) as e:
        fn(*a, **kw)
    return e.value.status


def test_row_pitch_validation_errors():
    """sbp_tensor_t::ld: at least the longest stored row, never negative, and only where the header allows it"""
    k = 2
    S0, S1, B_, P = sbp.S(0), sbp.S(1), sbp.B, sbp.P_SUM
    x = fake(k, 8, 16)                                   # S(1): local [8, 8]
    w = fake(k, 16, 8, base=0x20000000)                  # S(0): local [8, 8]
    y = fake(k, 8, 8, base=0x30000000)
    assert status_of(sbp.sbp_matmul, fake(k, 8, 16, ld=7), S1, w, S0, y, P, k, 0) == -3       # shorter than a stored row
    assert status_of(sbp.sbp_matmul, x, S1, fake(k, 16, 8, base=0x20000000, ld=-8), S0, y, P, k, 0) == -3
    assert status_of(sbp.sbp_matmul, x, S1, w, S0, fake(k, 8, 8, base=0x30000000, ld=4), P, k, 0) == -3
    xt = fake(k, 8, 16, trans=1, ld=7)                   # stored [8 kk][8 m]: the stored row is the m extent
    assert status_of(sbp.sbp_matmul, xt, S1, w, S0, y, P, k, 0) == -3
    # a pitched output that would run into the next shard's buffer is an alias
    tight = sbp.SbpTensor([0x30000000, 0x30000000 + 8 * 8 * 4], 8, 8, sbp.F32, 0, 12)
    assert status_of(sbp.sbp_matmul, x, S1, w, S0, tight, P, k, 0) == -7
    # boxing and the two-dimensional entry points take dense tensors only
    t_in, t_out = fake(k, 8, 8, ld=16), fake(k, 8, 8, base=0x40000000)
    assert status_of(sbp.sbp_boxing, t_in, S0, t_out, B_, k, 0) == -9
    assert status_of(sbp.sbp_boxing, fake(k, 8, 8), S0, fake(k, 8, 8, base=0x40000000, ld=16), B_, k, 0) == -9
    assert status_of(sbp.sbp_boxing_across, t_in, S0, k, t_out, B_, k, 0) == -9
    assert status_of(sbp.sbp_boxing_cast, t_in, S0, fake(k, 8, 8, dtype=sbp.BF16, base=0x40000000), B_, k, 0) == -9


def test_matmul_validation_errors():
    k = 2
    x = fake(k, 8, 16)
    w = fake(k, 16, 8, base=0x20000000)
    y = fake(k, 8, 8, base=0x30000000)
    S0, S1, B_, P = sbp.S(0), sbp.S(1), sbp.B, sbp.P_SUM
    st = 0  # a stream value; never used because validation fails first
    assert status_of(sbp.sbp_matmul, x, S0, w, S1, y, sbp.AUTO, k, st) == -6          # not in Table 1
    assert status_of(sbp.sbp_matmul, x, S1, w, S0, y, B_, k, st) == -6                # would need implicit boxing
    assert status_of(sbp.sbp_matmul, x, S1, w, S0, y, P, 0, st) == -2                 # k
    assert status_of(sbp.sbp_matmul, x, S1, w, S0, y, P, 65, st) == -2
    assert status_of(sbp.sbp_matmul, x, 7, w, S0, y, P, k, st) == -5                  # axis
    bad_w = fake(k, 15, 8, base=0x20000000)
    assert status_of(sbp.sbp_matmul, x, S1, bad_w, S0, y, P, k, st) == -3             # inner extents differ
    bf_w = fake(k, 16, 8, dtype=sbp.BF16, base=0x20000000)
    assert status_of(sbp.sbp_matmul, x, S1, bf_w, S0, y, P, k, st) == -4              # mixed input dtypes
    y_bf = fake(k, 8, 8, dtype=sbp.BF16, base=0x30000000)
    assert status_of(sbp.sbp_matmul, x, S1, w, S0, y_bf, P, k, st) == -4              # P(sum) must be f32
    x_bf = fake(k, 8, 16, dtype=sbp.BF16)
    assert status_of(sbp.sbp_matmul, x_bf, P, bf_w, B_, y, P, k, st) == -4            # P operand must be f32
    y_alias = fake(k, 8, 8, base=0x10000000)
    assert status_of(sbp.sbp_matmul, x, S1, w, S0, y_alias, P, k, st) == -7           # y over x
    y_self = sbp.SbpTensor([0x30000000, 0x30000000], 8, 8, sbp.F32)
    assert status_of(sbp.sbp_matmul, x, S1, w, S0, y_self, P, k, st) == -7            # two outputs, one buffer
    y_mis = sbp.SbpTensor([0x30000000, 0x31000004], 8, 8, sbp.F32)
    assert status_of(sbp.sbp_matmul, x, S1, w, S0, y_mis, P, k, st) == -8             # alignment
    y_null = sbp.SbpTensor([0x30000000, None], 8, 8, sbp.F32)
    assert status_of(sbp.sbp_matmul, x, S1, w, S0, y_null, P, k, st) == -1            # null shard
    assert status_of(sbp.sbp_matmul_ex, x, S1, w, S0, y, P, k, st, sbp.EPI_GELU) == -6   # GeLU of a partial
    assert status_of(sbp.sbp_matmul_ex, x, S0, fake(k, 16, 8, base=0x20000000), B_, y, S0, k, st, 7) == -9
    y_t = fake(k, 8, 8, base=0x30000000, trans=1)
    assert status_of(sbp.sbp_matmul, x, S1, w, S0, y_t, P, k, st) == -9


def test_boxing_validation_errors():
    k = 2
    a = fake(k, 8, 8)
    b = fake(k, 8, 8, base=0x20000000)
    st = 0
    assert status_of(sbp.sbp_boxing, a, sbp.P_SUM, fake(k, 8, 9, base=0x20000000), sbp.B, k, st) == -3
    assert status_of(sbp.sbp_boxing, a, sbp.P_SUM, fake(k, 8, 8, sbp.BF16, base=0x20000000), sbp.B, k, st) == -4
    a_bf = fake(k, 8, 8, sbp.BF16)
    b_bf = fake(k, 8, 8, sbp.BF16, base=0x20000000)
    assert status_of(sbp.sbp_boxing, a_bf, sbp.P_SUM, b_bf, sbp.B, k, st) == -4        # P must be f32
    assert status_of(sbp.sbp_boxing, a, sbp.P_SUM, b, sbp.P_MAX, k, st) == -6          # changes the reduction
    assert status_of(sbp.sbp_boxing, a, sbp.S(0), a, sbp.S(1), k, st) == -7            # in place
    assert status_of(sbp.sbp_boxing, a, 5, b, sbp.B, k, st) == -5
    assert status_of(sbp.sbp_boxing, a, sbp.S(0), b, sbp.B, 0, st) == -2
    # a B input may name one buffer k times
    same = sbp.SbpTensor([0x10000000] * k, 8, 8, sbp.F32)
    assert status_of(sbp.sbp_boxing, same, sbp.B, same, sbp.S(0), k, st) == -7         # ...but not as its own output


def test_boxing_cast_validation_errors():
    k = 2
    f32_in, bf_out = fake(k, 8, 16), fake(k, 8, 16, sbp.BF16, base=0x20000000)
    bf_in, f32_out = fake(k, 8, 16, sbp.BF16), fake(k, 8, 16, base=0x20000000)
    st = 0
    assert status_of(sbp.sbp_boxing_cast, f32_in, sbp.S(0), f32_out, sbp.B, k, st) == -4       # forward writes bf16
    assert status_of(sbp.sbp_boxing_cast, bf_in, sbp.S(0), bf_out, sbp.B, k, st) == -4         # forward reads fp32
    assert status_of(sbp.sbp_boxing_cast, f32_in, sbp.P_SUM, f32_out, sbp.S(0), k, st) == -4   # backward reads bf16
    assert status_of(sbp.sbp_boxing_cast, f32_in, sbp.B, bf_out, sbp.S(0), k, st) == -6        # not a cast pattern
    assert status_of(sbp.sbp_boxing_cast, bf_in, sbp.P_MAX, f32_out, sbp.S(0), k, st) == -6
    assert status_of(sbp.sbp_boxing_cast, f32_in, sbp.S(0), fake(k, 8, 8, sbp.BF16, base=0x20000000), sbp.B, k, st) == -3
    assert status_of(sbp.sbp_boxing_cast, f32_in, sbp.S(0), bf_out, sbp.B, 0, st) == -2
    over = fake(k, 8, 16, sbp.BF16, base=0x10000000)
    assert status_of(sbp.sbp_boxing_cast, f32_in, sbp.S(0), over, sbp.B, k, st) == -7          # output over the input


def test_boxing_across_validation_errors():
    st = 0
    a3, b5 = fake(3, 8, 16), fake(5, 8, 16, base=0x20000000)
    assert status_of(sbp.sbp_boxing_across, a3, sbp.S(0), 3, b5, sbp.B, 0, st) == -2            # k_out out of range
    assert status_of(sbp.sbp_boxing_across, a3, sbp.S(0), 65, b5, sbp.B, 5, st) == -2           # k_in out of range
    assert status_of(sbp.sbp_boxing_across, a3, sbp.P_SUM, 3, b5, sbp.P_MAX, 5, st) == -6       # the reduction cannot change
    assert status_of(sbp.sbp_boxing_across, a3, sbp.S(0), 3, fake(5, 8, 8, base=0x20000000), sbp.B, 5, st) == -3
    assert status_of(sbp.sbp_boxing_across, a3, sbp.S(0), 3, fake(5, 8, 16, sbp.BF16, base=0x20000000), sbp.B, 5, st) == -4
    assert status_of(sbp.sbp_boxing_across, fake(3, 8, 16, sbp.BF16), sbp.P_SUM, 3, fake(5, 8, 16, sbp.BF16, base=0x20000000),
                     sbp.B, 5, st) == -4                                                        # partial values are fp32
    assert status_of(sbp.sbp_boxing_across, a3, 7, 3, b5, sbp.B, 5, st) == -5                   # not a signature
    over = fake(5, 8, 16, base=0x10000000)
    assert status_of(sbp.sbp_boxing_across, a3, sbp.S(0), 3, over, sbp.B, 5, st) == -7          # output over the input


def test_2d_validation_errors():
    k0, k1 = 2, 2
    S0, S1, B_, P = sbp.S(0), sbp.S(1), sbp.B, sbp.P_SUM
    x, w, y = fake(4, 8, 8), fake(4, 8, 8, base=0x20000000), fake(4, 8, 8, base=0x30000000)
    st = 0
    assert status_of(sbp.sbp_matmul_2d, x, (S0, S1), w, (B_, S1), y, None, k0, k1, st) == -6        # inner pair not in Table 1
    assert status_of(sbp.sbp_matmul_2d, x, (S0, B_), w, (B_, S1), y, (S0, B_), k0, k1, st) == -6    # deduced is (S0, S1)
    assert status_of(sbp.sbp_matmul_2d, x, (S0, B_), w, (B_, S1), y, None, 9, 9, st) == -2          # 81 devices
    assert status_of(sbp.sbp_matmul_2d, x, (S0, S1), w, (B_, S0), fake(4, 8, 8, sbp.BF16, base=0x30000000), None, k0, k1, st) == -4
    assert status_of(sbp.sbp_matmul_2d, x, (S0, B_), w, (B_, S1), x, None, k0, k1, st) == -7        # y over x
    assert status_of(sbp.sbp_boxing_2d, x, (S0, P), y, (B_, B_), k0, k1, st) == -9                  # both entries change
    assert status_of(sbp.sbp_boxing_2d, x, (S0, S0), y, (B_, S0), k0, k1, st) == -9                 # along the inner split's axis
    assert status_of(sbp.sbp_boxing_2d, x, (P, sbp.P_MAX), y, (B_, sbp.P_MAX), k0, k1, st) == -9    # outer sum under an inner max
    assert status_of(sbp.sbp_boxing_2d, x, (sbp.P_MAX, P), y, (S0, P), k0, k1, st) == -9            # outer max under an inner sum
    assert status_of(sbp.sbp_boxing_2d, fake(4, 8, 8, sbp.BF16), (S0, P), fake(4, 8, 8, sbp.BF16, base=0x30000000), (S0, B_), k0, k1, st) == -4
    assert status_of(sbp.sbp_boxing_2d, x, (S0, B_), x, (S0, S1), k0, k1, st) == -7
    assert sbp.sbp_infer_matmul_2d((S0, S1), (B_, S0)) == (S0, P)
    assert sbp.sbp_local_shape_2d(10, 7, (S0, S0), 2, 2, 1, 1) == (2, 7)


def test_xent_validation_errors():
    k = 4
    L = fake(k, 16, 64, sbp.BF16)
    vec = lambda base, dt=sbp.F32: fake(k, 16, 1, dt, base=base)      # noqa: E731
    y, m, s, g, loss = vec(0x20000000, sbp.I32), vec(0x30000000), vec(0x40000000), vec(0x50000000), vec(0x60000000)
    dl = fake(k, 16, 64, sbp.BF16, base=0x70000000)
    st = 0
    assert status_of(sbp.sbp_xent_loss, L, sbp.S(0), y, m, s, loss, k, st) == -9
    assert status_of(sbp.sbp_xent_loss, L, sbp.S(1), vec(0x20000000), m, s, loss, k, st) == -4      # labels must be I32
    assert status_of(sbp.sbp_xent_loss, L, sbp.S(1), y, fake(k, 15, 1, base=0x30000000), s, loss, k, st) == -3
    assert status_of(sbp.sbp_xent_loss, L, sbp.S(1), y, m, s, m, k, st) == -7                       # loss over gmax
    assert status_of(sbp.sbp_xent_grad, L, sbp.S(1), y, m, s, g, fake(k, 16, 64, base=0x70000000), k, st) == -3   # dtype of logits
    assert status_of(sbp.sbp_xent_grad, L, sbp.S(1), y, m, s, g, L, k, st) == -7                    # in place
    big = 40
    assert status_of(sbp.sbp_xent_loss, fake(big, 16, 64, sbp.BF16, step=0x10000), sbp.S(1), fake(big, 16, 1, sbp.I32, base=0x20000000, step=0x1000),
                     fake(big, 16, 1, base=0x30000000, step=0x1000), fake(big, 16, 1, base=0x40000000, step=0x1000),
                     fake(big, 16, 1, base=0x60000000, step=0x1000), big, st) == -9                 # more than 32 devices
    del dl


def test_sizes_beyond_the_kernels_index_range_are_refused_not_wrapped():
    """the boxing kernels index with 32 bits; a tensor of 2^40 elements must come back as
    SBP_ERR_UNSUPPORTED before anything is launched (made-up addresses, never dereferenced)"""
    k = 2
    big = 1 << 20
    step = 1 << 44
    a = sbp.SbpTensor([1 << 46, (1 << 46) + step], big, big, sbp.F32)
    b = sbp.SbpTensor([1 << 48, (1 << 48) + step], big, big, sbp.F32)
    st = 0
    for si, so in [(sbp.P_SUM, sbp.B), (sbp.S(0), sbp.B), (sbp.S(0), sbp.S(1)), (sbp.B, sbp.P_SUM)]:
        assert status_of(sbp.sbp_boxing, a, si, b, so, k, st) == -9, (si, so)
    a16 = sbp.SbpTensor([1 << 46, (1 << 46) + step], big, big, sbp.BF16)
    assert status_of(sbp.sbp_boxing_cast, a, sbp.S(0), sbp.SbpTensor([1 << 48, (1 << 48) + step], big, big, sbp.BF16), sbp.B, k, st) == -9
    assert status_of(sbp.sbp_boxing_cast, a16, sbp.P_SUM, b, sbp.S(0), k, st) == -9
    wide = sbp.SbpTensor([1 << 46, (1 << 46) + step], 8, (1 << 31) + 8, sbp.F32)
    assert status_of(sbp.sbp_matmul, a, sbp.B, wide, sbp.B, wide, sbp.B, k, st) in (-3, -9)


def test_row_stat_validation_errors():
    k = 4
    L = fake(k, 16, 64, sbp.BF16)
    out = fake(k, 16, 1, base=0x20000000)
    gm = fake(k, 16, 1, base=0x30000000)
    st = 0
    assert status_of(sbp.sbp_row_max, L, sbp.B, out, k, st) == -9
    assert status_of(sbp.sbp_row_max, L, sbp.P_SUM, out, k, st) == -6
    assert status_of(sbp.sbp_row_max, L, sbp.S(1), fake(k, 16, 2, base=0x20000000), k, st) == -3
    assert status_of(sbp.sbp_row_sumexp, L, sbp.S(1), fake(k, 15, 1, base=0x30000000), out, k, st) == -3
    assert status_of(sbp.sbp_row_sumexp, L, sbp.S(1), gm, gm, k, st) == -7


def test_knob_rejects_unknown():
    sbp.sbp_set_knob(sbp.KNOB_GEMM_VARIANT, 0)
    assert status_of(sbp.sbp_set_knob, 99, 0) == -9
    assert status_of(sbp.sbp_set_knob, sbp.KNOB_GEMM_VARIANT, -1) == -9


def test_local_shapes_agree_with_the_oracle_on_random_geometry():
    """property test: the library's split geometry (1-D and on a grid) against the oracle's, which is pinned to
    numpy's array_split elsewhere"""
    from hypothesis import given, settings, strategies as st

    sigs = [(sbp.S(0), orc.S0), (sbp.S(1), orc.S1), (sbp.B, orc.B), (sbp.P_SUM, orc.P_SUM), (sbp.P_MAX, orc.P_MAX)]

    @settings(max_examples=300, deadline=None)
    @given(st.integers(0, 5000), st.integers(0, 5000), st.integers(1, 64), st.integers(0, 4), st.data())
    def one_d(rows, cols, k, which, data):
        i = data.draw(st.integers(0, k - 1))
        abi, o = sigs[which]
        assert sbp.sbp_local_shape(rows, cols, abi, k, i) == orc.local_shape(rows, cols, o, k, i)

    @settings(max_examples=300, deadline=None)
    @given(st.integers(0, 3000), st.integers(0, 3000), st.integers(1, 8), st.integers(1, 8), st.integers(0, 4), st.integers(0, 4), st.data())
    def two_d(rows, cols, k0, k1, w0, w1, data):
        a, b = data.draw(st.integers(0, k0 - 1)), data.draw(st.integers(0, k1 - 1))
        abi2, o2 = (sigs[w0][0], sigs[w1][0]), (sigs[w0][1], sigs[w1][1])
        assert sbp.sbp_local_shape_2d(rows, cols, abi2, k0, k1, a, b) == orc.local_shape2(rows, cols, o2, k0, k1, a, b)

    one_d()
    two_d()


def test_binding_refuses_a_shard_array_shorter_than_k():
    """The library reads k pointers from every shard array; the binding must not let a short array through."""
    x, w, y = fake(2, 8, 8), fake(2, 8, 8, base=0x20000000), fake(2, 8, 8, base=0x30000000)
    with pytest.raises(ValueError):
        sbp.sbp_matmul(x, sbp.S(0), w, sbp.B, y, sbp.S(0), 4, 0)
    with pytest.raises(ValueError):
        sbp.sbp_boxing(x, sbp.S(0), y, sbp.B, 3, 0)
    with pytest.raises(ValueError):
        sbp.sbp_boxing_across(x, sbp.S(0), 2, y, sbp.B, 5, 0)
    with pytest.raises(ValueError):
        sbp.sbp_boxing_2d(x, (sbp.S(0), sbp.B), y, (sbp.S(0), sbp.S(1)), 2, 2, 0)
    # a count the library rejects by itself still reaches it
    assert status_of(sbp.sbp_boxing, x, sbp.S(0), y, sbp.B, 65, 0) == -2
