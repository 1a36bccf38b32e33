"""CPU oracle for the SBP matmul + boxing path.  TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64, written from the definitions in the OneFlow paper
(arXiv 2110.15032).  Only tests, the smoke check and the bench's cpu_baseline
leg may import this module; it shares nothing with the HIP library and never
imports it.  Layout work (scatter / assemble / boxing) is numpy slicing here;
arithmetic (matmul, reductions, GeLU, exp, bf16 rounding) is the C file next
to this one, loaded through ctypes.

Notation follows the paper: a *global* (logical) tensor is mapped onto k
*local* tensors by an SBP signature (Sec. 3.1):
    S(a)    split along axis a in a balanced manner,
    B       every local tensor is an exact copy,
    P(op)   locals have the global shape; global = element-wise op over them.
Signatures are spelled here as tuples: ("S", 0), ("S", 1), ("B",),
("P", "sum"), ("P", "max").

Pins (tests/test_oracle_*.py): Table 1 derived by brute force, the reassembly
invariant under every boxing, Table 2's closed forms, numpy float64 matmul on
the k = 1 case, torch's fp32->bf16 cast, the Table 4 program and the U.V.W
deferred-boxing example; for the two-dimensional signatures of Sec. 3.3, Table 3
as printed plus a brute-force derivation of every valid 2-D MatMul pair, and
the reassembly invariant of boxing along either grid axis; for boxing between
disjoint placements, Table 2's other column, the reassembly invariant and the
same-placement routine at k_in = k_out.  Parity unpinned by the paper (fixed by a stated
reading only): the uneven-split rule, the GeLU variant, and which sign a
P(max) of +0 and -0 yields.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

S0 = ("S", 0)
S1 = ("S", 1)
B = ("B",)
P_SUM = ("P", "sum")
P_MAX = ("P", "max")

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sbp_oracle.c")
_LIB = os.path.join(_HERE, "libsbp_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C half with gcc (OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"])
    return _LIB


def _c():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, i32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
        lib.orc_split_range.argtypes = [i64, i32, i32, ctypes.POINTER(i64), ctypes.POINTER(i64)]
        lib.orc_matmul.argtypes = [vp, vp, vp, i64, i64, i64]
        lib.orc_reduce_sum.argtypes = [vp, i32, vp, i64]
        lib.orc_reduce_max.argtypes = [vp, i32, vp, i64]
        lib.orc_gelu.argtypes = [vp, vp, i64]
        lib.orc_row_max.argtypes = [vp, i64, i64, vp]
        lib.orc_row_sumexp.argtypes = [vp, vp, i64, i64, vp]
        lib.orc_bf16_from_f64.argtypes = [vp, vp, i64]
        lib.orc_bf16_to_f64.argtypes = [vp, vp, i64]
        for f in ("orc_split_range", "orc_matmul", "orc_reduce_sum", "orc_reduce_max", "orc_gelu",
                  "orc_row_max", "orc_row_sumexp", "orc_bf16_from_f64", "orc_bf16_to_f64"):
            getattr(lib, f).restype = None
        _lib = lib
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


# ----------------------------------------------------------------------------
# dtype helpers
# ----------------------------------------------------------------------------
def bf16_round(x) -> np.ndarray:
    """float64 values -> nearest bfloat16 (ties to even), as uint16 bit patterns."""
    x = _f64(x)
    out = np.empty(x.shape, dtype=np.uint16)
    _c().orc_bf16_from_f64(_ptr(x), _ptr(out), x.size)
    return out


def bf16_to_f64(bits) -> np.ndarray:
    """uint16 bfloat16 patterns -> float64, exactly."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, dtype=np.float64)
    _c().orc_bf16_to_f64(_ptr(bits), _ptr(out), bits.size)
    return out


# ----------------------------------------------------------------------------
# Sec. 3.1: global tensor <-> k local tensors
# ----------------------------------------------------------------------------
def split_range(n: int, k: int, i: int) -> tuple[int, int]:
    """(begin, end) of the indices shard i owns on an axis of length n."""
    b, l = ctypes.c_int64(), ctypes.c_int64()
    _c().orc_split_range(n, k, i, ctypes.byref(b), ctypes.byref(l))
    return b.value, b.value + l.value


def local_shape(rows: int, cols: int, sbp, k: int, i: int) -> tuple[int, int]:
    if sbp == S0:
        b, e = split_range(rows, k, i)
        return e - b, cols
    if sbp == S1:
        b, e = split_range(cols, k, i)
        return rows, e - b
    return rows, cols


def scatter(T: np.ndarray, sbp, k: int) -> list[np.ndarray]:
    """Global 2-D tensor -> its k local tensors.  Works on any dtype (raw words
    included).  For P the choice is not unique; the one taken is the zero-cost
    one of Table 2 (B->P, S->P cost 0 on the same devices): device 0 keeps the
    value and every other device holds the identity of the reduction (0 for
    sum, -inf for max)."""
    assert T.ndim == 2
    rows, cols = T.shape
    if sbp == S0:
        return [T[slice(*split_range(rows, k, i)), :].copy() for i in range(k)]
    if sbp == S1:
        return [T[:, slice(*split_range(cols, k, i))].copy() for i in range(k)]
    if sbp == B:
        return [T.copy() for _ in range(k)]
    if sbp == P_SUM:
        return [T.copy()] + [np.zeros_like(T) for _ in range(k - 1)]
    if sbp == P_MAX:
        return [T.copy()] + [np.full_like(T, -np.inf) for _ in range(k - 1)]
    raise ValueError(f"bad sbp {sbp}")


def assemble(shards: list[np.ndarray], sbp) -> np.ndarray:
    """k local tensors -> the global tensor they stand for.
    S: concatenate; B: all copies must be bit-identical, take one;
    P(sum) / P(max): element-wise reduction in float64."""
    k = len(shards)
    if sbp == S0:
        return np.concatenate(shards, axis=0)
    if sbp == S1:
        return np.concatenate(shards, axis=1)
    if sbp == B:
        for i in range(1, k):
            if shards[i].shape != shards[0].shape or \
               shards[i].tobytes() != shards[0].tobytes():
                raise AssertionError(f"broadcast copies 0 and {i} differ")
        return shards[0].copy()
    if sbp in (P_SUM, P_MAX):
        parts = [_f64(s) for s in shards]
        for p in parts:
            assert p.shape == parts[0].shape
        out = np.empty(parts[0].shape, dtype=np.float64)
        arr = (ctypes.c_void_p * k)(*[_ptr(p) for p in parts])
        fn = _c().orc_reduce_sum if sbp == P_SUM else _c().orc_reduce_max
        fn(ctypes.cast(arr, ctypes.c_void_p), k, _ptr(out), out.size)
        return out
    raise ValueError(f"bad sbp {sbp}")


# ----------------------------------------------------------------------------
# Sec. 3.1, Table 1: MatMul under SBP
# ----------------------------------------------------------------------------
#: The six valid rows as the paper prints them: (sbp of X, sbp of W) -> sbp of Y.
MATMUL_TABLE = {
    (S0, B): S0,
    (B, S1): S1,
    (S1, S0): P_SUM,
    (P_SUM, B): P_SUM,
    (B, P_SUM): P_SUM,
    (B, B): B,
}


def infer_matmul(sbp_x, sbp_w):
    """Signature of Y = XW, or None when the pair is not in Table 1."""
    return MATMUL_TABLE.get((sbp_x, sbp_w))


def matmul(A, Bm) -> np.ndarray:
    """Plain float64 product of two 2-D arrays (triple loop in C)."""
    A, Bm = _f64(A), _f64(Bm)
    assert A.ndim == 2 and Bm.ndim == 2 and A.shape[1] == Bm.shape[0], (A.shape, Bm.shape)
    C = np.empty((A.shape[0], Bm.shape[1]), dtype=np.float64)
    _c().orc_matmul(_ptr(A), _ptr(Bm), _ptr(C), A.shape[0], A.shape[1], Bm.shape[1])
    return C


def matmul_sbp(Xs: list[np.ndarray], sbp_x, Ws: list[np.ndarray], sbp_w):
    """Every device multiplies the two local tensors it holds; the list of
    local products is Y under the signature Table 1 gives.  Returns
    (list of float64 local products, sbp_y)."""
    sbp_y = infer_matmul(sbp_x, sbp_w)
    if sbp_y is None:
        raise ValueError(f"({sbp_x}, {sbp_w}) is not a valid MatMul signature")
    assert len(Xs) == len(Ws)
    return [matmul(x, w) for x, w in zip(Xs, Ws)], sbp_y


# ----------------------------------------------------------------------------
# Sec. 3.3: two-dimensional SBP (Table 3)
# ----------------------------------------------------------------------------
# The logical devices form a k0 x k1 grid (k0 nodes of k1 devices).  A signature is a pair
# (outer, inner): `outer` maps the global tensor onto the k0 nodes, `inner` maps each node's
# tensor onto that node's k1 devices.  Device (a, b) is entry a * k1 + b of every list below.
def local_shape2(rows: int, cols: int, sbp2, k0: int, k1: int, a: int, b: int) -> tuple[int, int]:
    r, c = local_shape(rows, cols, sbp2[0], k0, a)
    return local_shape(r, c, sbp2[1], k1, b)


def scatter2(T: np.ndarray, sbp2, k0: int, k1: int) -> list[np.ndarray]:
    """Global tensor -> k0 * k1 local tensors: scatter over the nodes, then each
    node's tensor over its devices."""
    out = []
    for node in scatter(T, sbp2[0], k0):
        out.extend(scatter(node, sbp2[1], k1))
    return out


def assemble2(shards: list[np.ndarray], sbp2, k0: int, k1: int) -> np.ndarray:
    """The inverse: every node's tensor from its k1 devices, then the global one."""
    assert len(shards) == k0 * k1
    nodes = [assemble(shards[a * k1:(a + 1) * k1], sbp2[1]) for a in range(k0)]
    return assemble(nodes, sbp2[0])


def infer_matmul2(sbp_x2, sbp_w2):
    """Table 1 applied to each grid axis on its own (the two rows printed in
    Table 3 are two instances); None when either axis is not a Table 1 row."""
    y0, y1 = infer_matmul(sbp_x2[0], sbp_w2[0]), infer_matmul(sbp_x2[1], sbp_w2[1])
    return None if y0 is None or y1 is None else (y0, y1)


def matmul_sbp2(Xs: list[np.ndarray], sbp_x2, Ws: list[np.ndarray], sbp_w2):
    """Every device multiplies the two local tensors it holds."""
    sbp_y2 = infer_matmul2(sbp_x2, sbp_w2)
    if sbp_y2 is None:
        raise ValueError(f"({sbp_x2}, {sbp_w2}) is not a valid 2-D MatMul signature")
    assert len(Xs) == len(Ws)
    return [matmul(x, w) for x, w in zip(Xs, Ws)], sbp_y2


def boxing2(shards: list[np.ndarray], sbp_in2, sbp_out2, k0: int, k1: int) -> list[np.ndarray]:
    """Boxing along ONE grid axis (the other position of the signature stays).
    Inner position: each node re-arranges its own tensor (1-D boxing per node).
    Outer position: the devices with the same inner index b hold, between
    them, one tensor under the outer signature (the whole tensor when inner is
    B or P, its b-th slice when inner is S and the outer conversion leaves that
    axis alone); each such group is boxed on its own.  An outer P(op) is not
    reduced while the inner position is a partial of the OTHER operation."""
    assert len(shards) == k0 * k1
    if sbp_in2[0] == sbp_out2[0]:
        out = []
        for a in range(k0):
            out.extend(boxing(shards[a * k1:(a + 1) * k1], sbp_in2[1], sbp_out2[1], k1))
        return out
    if sbp_in2[1] != sbp_out2[1]:
        raise ValueError("boxing2 changes one position of the signature at a time")
    inner = sbp_in2[1]
    if inner in (S0, S1) and inner in (sbp_in2[0], sbp_out2[0]):
        raise ValueError("outer boxing along the axis the inner position splits is not a per-slice operation")
    # The nested signature means outer-op over the nodes of (inner-op over a node's devices) (Sec. 3.3:
    # the outer entry places the tensor on the nodes, the inner entry each node's tensor on its devices).
    # Reducing the outer partial first, device by device, would compute inner-op of outer-op instead,
    # and sum and max do not commute.
    if inner in (P_SUM, P_MAX) and sbp_in2[0] in (P_SUM, P_MAX) and sbp_in2[0] != inner:
        raise ValueError("an outer partial cannot be reduced underneath an inner partial of another operation")
    out = [None] * (k0 * k1)
    for b in range(k1):
        plane = boxing([shards[a * k1 + b] for a in range(k0)], sbp_in2[0], sbp_out2[0], k0)
        for a in range(k0):
            out[a * k1 + b] = plane[a]
    return out


# ----------------------------------------------------------------------------
# Sec. 3.2: boxing
# ----------------------------------------------------------------------------
def boxing(shards: list[np.ndarray], sbp_in, sbp_out, k: int | None = None) -> list[np.ndarray]:
    """Re-arrange the local tensors of one global tensor from sbp_in to sbp_out
    on the same k devices: by definition the global tensor is unchanged, so
    this is scatter(assemble(.)).  S/B -> S/B keeps the input dtype (raw moves);
    anything that starts from P yields float64.
    B -> S takes slice j from copy j (the copy on the same device), not copy 0."""
    k = len(shards) if k is None else k
    assert k == len(shards)
    if sbp_in == B and sbp_out in (S0, S1):
        rows, cols = shards[0].shape
        out = []
        for j in range(k):
            if sbp_out == S0:
                out.append(shards[j][slice(*split_range(rows, k, j)), :].copy())
            else:
                out.append(shards[j][:, slice(*split_range(cols, k, j))].copy())
        return out
    if sbp_out in (P_SUM, P_MAX):
        # Table 2 prices S->P, B->P and P->P at zero on the same devices, so no
        # value may leave its device: every device keeps what it already holds
        # and pads with the identity of the reduction.  (The paper does not say
        # how; this is the only zero-cost reading.)
        ident = 0.0 if sbp_out == P_SUM else -np.inf
        if sbp_in == sbp_out:
            return [_f64(s).copy() for s in shards]
        if sbp_in == B:
            return [_f64(shards[0]).copy()] + \
                   [np.full(shards[0].shape, ident, dtype=np.float64) for _ in range(k - 1)]
        if sbp_in in (S0, S1):
            G = assemble(shards, sbp_in)
            rows, cols = G.shape
            out = []
            for j in range(k):
                o = np.full((rows, cols), ident, dtype=np.float64)
                if sbp_in == S0:
                    b, e = split_range(rows, k, j)
                    o[b:e, :] = shards[j]
                else:
                    b, e = split_range(cols, k, j)
                    o[:, b:e] = shards[j]
                out.append(o)
            return out
        raise ValueError(f"boxing {sbp_in} -> {sbp_out} changes the reduction")
    return scatter(assemble(shards, sbp_in), sbp_out, k)


def transfer_elems(sbp_in, sbp_out, rows: int, cols: int, k: int) -> int:
    """Elements that cross between devices when boxing on the SAME k devices,
    counted by walking a routing: for every output device j and every element
    it must end up holding, look at which devices hold a contribution to that
    element under sbp_in and count the contributions that are not already on j.
    P -> B is routed the way Table 2 prices it, as P -> S(0) followed by
    S(0) -> B.  (Sec. 3.2, Table 2, "same" column.)"""
    def owner(sbp, r, c):
        if sbp == S0:
            return next(i for i in range(k) if split_range(rows, k, i)[0] <= r < split_range(rows, k, i)[1])
        if sbp == S1:
            return next(i for i in range(k) if split_range(cols, k, i)[0] <= c < split_range(cols, k, i)[1])
        raise ValueError

    if sbp_in in (P_SUM, P_MAX) and sbp_out == B:
        return transfer_elems(sbp_in, S0, rows, cols, k) + transfer_elems(S0, B, rows, cols, k)
    moved = 0
    for j in range(k):
        for r in range(rows):
            for c in range(cols):
                if sbp_out in (S0, S1):
                    needed = owner(sbp_out, r, c) == j
                elif sbp_out == B:
                    needed = True
                else:  # -> P: device 0 / the owner keeps the value, others hold the identity
                    needed = False
                if not needed:
                    continue
                if sbp_in in (S0, S1):
                    moved += 0 if owner(sbp_in, r, c) == j else 1
                elif sbp_in == B:
                    moved += 0           # own copy
                else:                    # P: one contribution per device, own one is local
                    moved += k - 1
    return moved


# ----------------------------------------------------------------------------
# Sec. 3.2, Table 2, column "disjoint": the input lives on k_in devices and the
# output on k_out OTHER devices, so every value the output holds has to travel.
# ----------------------------------------------------------------------------
def boxing_across(shards: list[np.ndarray], sbp_in, sbp_out, k_out: int) -> list[np.ndarray]:
    """Boxing from a placement of k_in = len(shards) devices to a disjoint one of
    k_out devices.  The global tensor is unchanged, so S and B outputs are
    scatter(assemble(.)) with the output's own device count.  For a P output the
    paper only prices the move (Table 2); the readings below are the ones that
    move exactly the priced amount (parity unpinned by the paper):
      S(a) -> P: output device j receives slice j of the balanced split of axis a
                 over k_out devices and pads with the identity        (|T| moves)
      B    -> P: output device 0 receives one copy, the rest hold the identity
                                                                      (|T| moves)
      P    -> P: partial i goes, whole, to output device i mod k_out; a device
                 that receives several combines them in input order, one that
                 receives none holds the identity                (k_in |T| move)"""
    k_in = len(shards)
    if sbp_out in (P_SUM, P_MAX):
        ident = 0.0 if sbp_out == P_SUM else -np.inf
        comb = np.add if sbp_out == P_SUM else np.maximum
        if sbp_in in (P_SUM, P_MAX):
            if sbp_in != sbp_out:
                raise ValueError(f"boxing {sbp_in} -> {sbp_out} changes the reduction")
            out = [None] * k_out
            for i in range(k_in):
                j = i % k_out
                out[j] = _f64(shards[i]).copy() if out[j] is None else comb(out[j], _f64(shards[i]))
            return [np.full(shards[0].shape, ident, dtype=np.float64) if o is None else o for o in out]
        G = _f64(assemble(shards, sbp_in))
        rows, cols = G.shape
        out = [np.full((rows, cols), ident, dtype=np.float64) for _ in range(k_out)]
        if sbp_in == B:
            out[0][:, :] = G
            return out
        for j in range(k_out):
            if sbp_in == S0:
                b, e = split_range(rows, k_out, j)
                out[j][b:e, :] = G[b:e, :]
            else:
                b, e = split_range(cols, k_out, j)
                out[j][:, b:e] = G[:, b:e]
        return out
    return scatter(assemble(shards, sbp_in), sbp_out, k_out)


def transfer_elems_across(sbp_in, k_in: int, sbp_out, k_out: int, rows: int, cols: int) -> int:
    """Elements that travel when boxing between DISJOINT device sets, counted by
    walking a routing: for every output device and every position where it ends
    up holding a real value (not the padding identity of a P output), count the
    contributions it receives; nothing is local.  P -> B is routed as Table 2
    prices it: P -> S(0) onto the k_out output devices, then S(0) -> B among
    them (there only the k_out - 1 other devices need each slice)."""
    T = rows * cols
    if sbp_in in (P_SUM, P_MAX) and sbp_out == B:
        inner = transfer_elems(S0, B, rows, cols, k_out)
        return transfer_elems_across(sbp_in, k_in, S0, k_out, rows, cols) + inner
    if sbp_in in (P_SUM, P_MAX) and sbp_out in (P_SUM, P_MAX):
        # walk the routing with tagged partials: partial i is 2^i everywhere, so the value an output device ends
        # up with spells out which partials it received; each of those travelled whole
        assert k_in <= 52, "tags must stay exact in float64"
        tagged = [np.full((rows, cols), float(1 << i)) for i in range(k_in)]
        held = boxing_across(tagged, P_SUM, P_SUM, k_out)
        moved = 0
        for h in held:
            assert (h == h.flat[0]).all(), "a partial arrives whole or not at all"
            moved += bin(int(h.flat[0])).count("1") * T
        return moved
    moved = 0
    probe = np.arange(T, dtype=np.float64).reshape(rows, cols) + 1.0   # no zeros: padding is visible
    held = boxing_across(scatter(probe, sbp_in, k_in) if sbp_in not in (P_SUM, P_MAX)
                         else [probe] + [np.zeros_like(probe)] * (k_in - 1), sbp_in, sbp_out, k_out)
    for j in range(k_out):
        if sbp_out in (P_SUM, P_MAX):
            real = int(np.count_nonzero(np.isfinite(held[j]) & (held[j] != 0)))
        else:
            real = held[j].size
        per_value = k_in if sbp_in in (P_SUM, P_MAX) else 1   # a P value has one contribution per input device
        moved += real * per_value
    return moved


# ----------------------------------------------------------------------------
# Workload element-wise / row ops
# ----------------------------------------------------------------------------
def gelu(x) -> np.ndarray:
    x = _f64(x)
    y = np.empty_like(x)
    _c().orc_gelu(_ptr(x), _ptr(y), x.size)
    return y


def row_max(L) -> np.ndarray:
    """m[r] = max over the columns of L (Sec. 6.3.1, local max)."""
    L = _f64(L)
    m = np.empty(L.shape[0], dtype=np.float64)
    _c().orc_row_max(_ptr(L), L.shape[0], L.shape[1], _ptr(m))
    return m


def row_sumexp(L, m) -> np.ndarray:
    """s[r] = sum over the columns of exp(L[r, c] - m[r]) (Sec. 6.3.1, local sum)."""
    L, m = _f64(L), _f64(m)
    assert m.shape == (L.shape[0],)
    s = np.empty(L.shape[0], dtype=np.float64)
    _c().orc_row_sumexp(_ptr(L), _ptr(m), L.shape[0], L.shape[1], _ptr(s))
    return s


# ----------------------------------------------------------------------------
# Sec. 6.3.1 continued: sparse cross entropy on model-parallel (S(1)) logits.
# The figure that details the operators is lost in the source text; what is
# computed is the textbook definition, loss[r] = -log softmax(L[r, :])[y[r]],
# and its gradient, decomposed over the column shards the way the softmax is:
# every device works on the columns it holds, using the global max m and
# the global denominator s obtained by boxing (parity unpinned by the paper).
# ----------------------------------------------------------------------------
def softmax_xent_loss(L, labels) -> np.ndarray:
    """loss[r] = log(sum_c exp(L[r, c])) - L[r, y[r]]; a label outside [0, C) marks an ignored row (0)."""
    L = _f64(L)
    labels = np.asarray(labels, dtype=np.int64)
    m = L.max(axis=1)
    lse = m + np.log(np.exp(L - m[:, None]).sum(axis=1))
    ok = (labels >= 0) & (labels < L.shape[1])
    picked = L[np.arange(L.shape[0]), np.where(ok, labels, 0)]
    return np.where(ok, lse - picked, 0.0)


def softmax_xent_grad(L, labels, g) -> np.ndarray:
    """d loss[r] / d L[r, c] * g[r] = (softmax(L[r, :])[c] - [c == y[r]]) * g[r]; ignored rows get 0."""
    L, g = _f64(L), _f64(g)
    labels = np.asarray(labels, dtype=np.int64)
    m = L.max(axis=1)
    e = np.exp(L - m[:, None])
    p = e / e.sum(axis=1)[:, None]
    ok = (labels >= 0) & (labels < L.shape[1])
    p[np.arange(L.shape[0])[ok], labels[ok]] -= 1.0
    return p * np.where(ok, g, 0.0)[:, None]


def xent_loss_sbp(Ls: list[np.ndarray], labels, m, s) -> list[np.ndarray]:
    """Model-parallel form: Ls are the S(1) shards of the logits, m and s the global row max and
    denominator.  The device that holds column y[r] contributes log s[r] + m[r] - L[r, y[r]], every
    other device 0: k partial vectors, P(sum)."""
    labels = np.asarray(labels, dtype=np.int64)
    m, s = _f64(m), _f64(s)
    out, begin = [], 0
    for Li in Ls:
        Li = _f64(Li)
        mine = (labels >= begin) & (labels < begin + Li.shape[1])
        v = np.zeros(Li.shape[0], dtype=np.float64)
        rows = np.arange(Li.shape[0])[mine]
        v[rows] = np.log(s[rows]) + m[rows] - Li[rows, labels[rows] - begin]
        out.append(v)
        begin += Li.shape[1]
    return out


def xent_grad_sbp(Ls: list[np.ndarray], labels, m, s, g) -> list[np.ndarray]:
    """Model-parallel gradient: elementwise on every S(1) shard, no communication."""
    labels = np.asarray(labels, dtype=np.int64)
    m, s, g = _f64(m), _f64(s), _f64(g)
    total = sum(Li.shape[1] for Li in Ls)
    ok = (labels >= 0) & (labels < total)
    out, begin = [], 0
    for Li in Ls:
        Li = _f64(Li)
        p = np.exp(Li - m[:, None]) / s[:, None]
        mine = (labels >= begin) & (labels < begin + Li.shape[1])
        rows = np.arange(Li.shape[0])[mine]
        p[rows, labels[rows] - begin] -= 1.0
        out.append(p * np.where(ok, g, 0.0)[:, None])
        begin += Li.shape[1]
    return out
