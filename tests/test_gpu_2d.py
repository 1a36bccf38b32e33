"""GPU parity for two-dimensional SBP (Sec. 3.3, Table 3): matmul on a k0 x k1 grid of logical
devices and boxing along one grid axis, through the C ABI, against the CPU oracle."""
import itertools

import numpy as np
import pytest

import oracle as orc
import paper_2110_15032_amd as sbp
import workloads as wl
from sbp_harness import TO_ABI, assert_bits_equal, assert_matmul_close, assert_psum_close, empty_dev, download, sync, upload, values

pytestmark = pytest.mark.gpu
SEED = wl.SEED_BASE + 2
S0, S1, B, P = orc.S0, orc.S1, orc.B, orc.P_SUM


def abi2(s2):
    return (TO_ABI[s2[0]], TO_ABI[s2[1]])


def rnd_f32(tid, shape):
    return wl.normal(SEED, tid, shape).astype(np.float32)


def rnd_bf16(tid, shape, std=1.0):
    return wl.to_bf16_bits(wl.normal(SEED, tid, shape, std))


class Dev2:
    """k0 * k1 device buffers of one global tensor"""

    def __init__(self, dev, rows, cols, np_dtype):
        self.dev, self.np_dtype = dev, np.dtype(np_dtype)
        self.desc = sbp.SbpTensor(dev, rows, cols, sbp.F32 if self.np_dtype == np.float32 else sbp.BF16)

    @classmethod
    def from_host(cls, shards, rows, cols):
        return cls([upload(s) for s in shards], rows, cols, shards[0].dtype)

    @classmethod
    def empty(cls, rows, cols, np_dtype, sig2, k0, k1):
        shapes = [orc.local_shape2(rows, cols, sig2, k0, k1, a, b) for a in range(k0) for b in range(k1)]
        return cls([empty_dev(s, np_dtype) for s in shapes], rows, cols, np_dtype)

    def host(self):
        return [download(t, self.np_dtype) for t in self.dev]


def partials(tid, T, k):
    parts = [rnd_f32(tid + 1 + i, T.shape) for i in range(k - 1)]
    return parts + [(T - np.sum(parts, axis=0, dtype=np.float32)).astype(np.float32)]


def scatter2_random(tid, T, s2, k0, k1):
    """orc.scatter2 with random partials in P positions (fp32 tensors only)"""
    nodes = partials(tid, T, k0) if s2[0] == P else orc.scatter(T, s2[0], k0)
    if s2 == (B, P):
        ps = partials(tid + 50, T, k1)
        return [p.copy() for _ in range(k0) for p in ps]
    out = []
    for a, n in enumerate(nodes):
        out.extend(partials(tid + 100 * (a + 1), n, k1) if s2[1] == P else orc.scatter(n, s2[1], k1))
    return out


TABLE3 = [((S0, B), (B, S1)), ((S0, S1), (B, S0))]


def test_infer_and_local_shape_2d_follow_the_oracle():
    for sx, sw in TABLE3 + [((S1, S1), (S0, S0)), ((B, P), (B, B))]:
        assert sbp.sbp_infer_matmul_2d(abi2(sx), abi2(sw)) == abi2(orc.infer_matmul2(sx, sw))
    with pytest.raises(sbp.SbpError):
        sbp.sbp_infer_matmul_2d(abi2((S0, S1)), abi2((B, S1)))
    for s2 in itertools.product((S0, S1, B, P), repeat=2):
        for a in range(3):
            for b in range(2):
                assert sbp.sbp_local_shape_2d(10, 7, abi2(s2), 3, 2, a, b) == orc.local_shape2(10, 7, s2, 3, 2, a, b)


@pytest.mark.parametrize("k0,k1", [(2, 2), (2, 3), (3, 1)])
@pytest.mark.parametrize("sx,sw", TABLE3 + [((S1, B), (S0, S1)), ((B, S0), (P, B)), ((S1, S1), (S0, S0))])
def test_matmul_2d_fp32(k0, k1, sx, sw):
    M, K, N = 37, 30, 29
    X, W = rnd_f32(1, (M, K)), rnd_f32(2, (K, N))
    Xs, Ws = scatter2_random(10, X, sx, k0, k1), scatter2_random(500, W, sw, k0, k1)
    ref, sy = orc.matmul_sbp2(Xs, sx, Ws, sw)
    dx, dw = Dev2.from_host(Xs, M, K), Dev2.from_host(Ws, K, N)
    dy = Dev2.empty(M, N, np.float32, sy, k0, k1)
    sbp.sbp_matmul_2d(dx.desc, abi2(sx), dw.desc, abi2(sw), dy.desc, None, k0, k1)
    sync()
    got = dy.host()
    for i, (g, r) in enumerate(zip(got, ref)):
        assert g.shape == r.shape
        if r.size:
            assert_matmul_close(g, r, 1e-5, f"2-D ({sx},{sw}) grid {k0}x{k1} device {i}")
    Y = orc.assemble2([g.astype(np.float64) for g in got], sy, k0, k1) if sy[0] != B and sy[1] != B else None
    if Y is not None:
        assert_matmul_close(Y, orc.matmul(X, W), 1e-5, "assembled")
    with pytest.raises(sbp.SbpError):       # the deduced signature is not negotiable
        wrong = (sbp.B, sbp.B) if abi2(sy) != (sbp.B, sbp.B) else (sbp.S(0), sbp.B)
        sbp.sbp_matmul_2d(dx.desc, abi2(sx), dw.desc, abi2(sw), dy.desc, wrong, k0, k1)


@pytest.mark.parametrize("sx,sw", TABLE3)
def test_matmul_2d_bf16_table3_on_the_matrix_cores(sx, sw):
    """2 x 4 grid; local products of several 256-tiles with ragged edges, K a multiple of 128 per device"""
    k0, k1 = 2, 4
    M, K, N = 2 * 520, 4 * 256, 4 * 328
    X, W = rnd_bf16(3, (M, K)), rnd_bf16(4, (K, N), 0.05)
    Xs, Ws = orc.scatter2(X, sx, k0, k1), orc.scatter2(W, sw, k0, k1)
    ref, sy = orc.matmul_sbp2([values(x) for x in Xs], sx, [values(w) for w in Ws], sw)
    dx, dw = Dev2.from_host(Xs, M, K), Dev2.from_host(Ws, K, N)
    out_dtype = np.float32 if P in sy else np.uint16
    dy = Dev2.empty(M, N, out_dtype, sy, k0, k1)
    sbp.sbp_matmul_2d(dx.desc, abi2(sx), dw.desc, abi2(sw), dy.desc, abi2(sy), k0, k1)
    sync()
    got = dy.host()
    for i, (g, r) in enumerate(zip(got, ref)):
        assert_matmul_close(values(g), r, 2e-2, f"bf16 2-D ({sx},{sw}) device {i}")
    assert_matmul_close(orc.assemble2([values(g) for g in got], sy, k0, k1), orc.matmul(values(X), values(W)), 2e-2, "assembled")


@pytest.mark.parametrize("sx,sw", TABLE3)
def test_matmul_2d_bf16_with_row_pitch_equals_the_dense_call(sx, sw):
    """the same products with every local buffer padded to a row pitch: bit-identical results, padding untouched"""
    k0, k1 = 2, 4
    M, K, N = 2 * 520, 4 * 256, 4 * 328
    X, W = rnd_bf16(3, (M, K)), rnd_bf16(4, (K, N), 0.05)
    Xs, Ws = orc.scatter2(X, sx, k0, k1), orc.scatter2(W, sw, k0, k1)
    _, sy = orc.matmul_sbp2([values(x) for x in Xs], sx, [values(w) for w in Ws], sw)
    out_dtype = np.float32 if P in sy else np.uint16
    dx, dw = Dev2.from_host(Xs, M, K), Dev2.from_host(Ws, K, N)
    dy = Dev2.empty(M, N, out_dtype, sy, k0, k1)
    sbp.sbp_matmul_2d(dx.desc, abi2(sx), dw.desc, abi2(sw), dy.desc, abi2(sy), k0, k1)
    sync()
    dense = dy.host()

    def padded(shards, pad, poison):
        ld = max(s.shape[1] for s in shards) + pad
        bufs = []
        for s in shards:
            b = np.full((s.shape[0], ld), poison, dtype=s.dtype)
            b[:, :s.shape[1]] = s
            bufs.append(upload(b))
        return bufs, ld

    xb, ldx = padded(Xs, 8, np.uint16(0x7FC1))
    wb, ldw = padded(Ws, 24, np.uint16(0x7FC1))
    yb, ldy = padded([np.zeros(d.shape, d.dtype) for d in dense], 16, np.float32(np.nan) if out_dtype == np.float32 else np.uint16(0x7FC1))
    abi_dt = sbp.F32 if out_dtype == np.float32 else sbp.BF16
    sbp.sbp_matmul_2d(sbp.SbpTensor(xb, M, K, sbp.BF16, 0, ldx), abi2(sx), sbp.SbpTensor(wb, K, N, sbp.BF16, 0, ldw), abi2(sw),
                      sbp.SbpTensor(yb, M, N, abi_dt, 0, ldy), abi2(sy), k0, k1)
    sync()
    for i, (t, d) in enumerate(zip(yb, dense)):
        full = download(t, np.dtype(out_dtype)).reshape(-1, ldy)
        assert_bits_equal(np.ascontiguousarray(full[:, :d.shape[1]]), d, f"device {i}: pitched against dense")
        pad = full[:, d.shape[1]:]
        assert bool(np.isnan(pad).all()) if out_dtype == np.float32 else bool((pad == 0x7FC1).all()), f"device {i}: padding written"


CONVERSIONS = [((S0, P), (S0, B)), ((S0, P), (S0, S1)), ((S0, S1), (S0, B)), ((S0, S1), (S0, S0)), ((S0, B), (S0, S1)),
               ((S0, B), (B, B)), ((B, S1), (S0, S1)), ((P, S1), (B, S1)), ((P, B), (S0, B)), ((S1, S0), (B, S0)),
               ((P, P), (P, B)), ((S0, B), (S0, P)), ((S1, B), (S0, B))]


@pytest.mark.parametrize("k0,k1", [(2, 3), (4, 2)])
@pytest.mark.parametrize("si,so", CONVERSIONS)
def test_boxing_2d_along_one_axis(k0, k1, si, so):
    for n, shape in enumerate([(24, 36), (13, 10), (64, 128)]):
        T = rnd_f32(40 + n, shape)
        ins = scatter2_random(60 + n, T, si, k0, k1)
        ref = orc.boxing2(ins, si, so, k0, k1)
        d_in = Dev2.from_host(ins, *shape)
        d_out = Dev2.empty(*shape, np.float32, so, k0, k1)
        sbp.sbp_boxing_2d(d_in.desc, abi2(si), d_out.desc, abi2(so), k0, k1)
        sync()
        got = d_out.host()
        reduces = P in si
        for i, (g, r) in enumerate(zip(got, ref)):
            assert g.shape == r.shape
            if not reduces:
                assert np.array_equal(g.astype(np.float64), np.asarray(r, dtype=np.float64)), f"{si}->{so} device {i}"
            else:
                assert np.allclose(g, r, rtol=0, atol=1e-5 * (1 + np.abs(r).max())), f"{si}->{so} device {i}"
        assert np.allclose(orc.assemble2([g.astype(np.float64) for g in got], so, k0, k1), T, atol=1e-4)


def test_boxing_2d_refusals():
    k0, k1 = 2, 2
    T = rnd_f32(70, (8, 8))
    d_in = Dev2.from_host(orc.scatter2(T, (S0, S0), k0, k1), 8, 8)
    d_out = Dev2.empty(8, 8, np.float32, (B, S0), k0, k1)
    with pytest.raises(sbp.SbpError) as e:      # outer conversion along the inner split's own axis
        sbp.sbp_boxing_2d(d_in.desc, abi2((S0, S0)), d_out.desc, abi2((B, S0)), k0, k1)
    assert e.value.status == -9
    d_out2 = Dev2.empty(8, 8, np.float32, (B, B), k0, k1)
    with pytest.raises(sbp.SbpError) as e:      # both positions at once
        sbp.sbp_boxing_2d(d_in.desc, abi2((S0, S0)), d_out2.desc, abi2((B, B)), k0, k1)
    assert e.value.status == -9


def test_table3_row2_then_all_reduce_inside_every_group():
    """((S0,S1),(B,S0)) -> (S0,P), then the inner boxing P -> B: every group holds its row block of XW"""
    k0, k1 = 2, 4
    M, K, N = 96, 4 * 64, 72
    X, W = rnd_bf16(5, (M, K)), rnd_bf16(6, (K, N), 0.05)
    sx, sw = TABLE3[1]
    dx = Dev2.from_host(orc.scatter2(X, sx, k0, k1), M, K)
    dw = Dev2.from_host(orc.scatter2(W, sw, k0, k1), K, N)
    dy = Dev2.empty(M, N, np.float32, (S0, P), k0, k1)
    db = Dev2.empty(M, N, np.float32, (S0, B), k0, k1)
    sbp.sbp_matmul_2d(dx.desc, abi2(sx), dw.desc, abi2(sw), dy.desc, None, k0, k1)
    sbp.sbp_boxing_2d(dy.desc, abi2((S0, P)), db.desc, abi2((S0, B)), k0, k1)
    sync()
    Y = orc.matmul(values(X), values(W))
    got = db.host()
    for a in range(k0):
        block = Y[slice(*orc.split_range(M, k0, a))]
        for b in range(k1):
            assert_matmul_close(got[a * k1 + b], block, 2e-2, f"group {a} device {b}")
            assert_bits_equal(got[a * k1 + b], got[a * k1], "copies inside a group")


@pytest.mark.parametrize("k0,k1", [(2, 4), (4, 2), (3, 5)])
@pytest.mark.parametrize("pm", ["sum", "max"])
def test_group_reductions_in_one_launch_equal_one_boxing_per_group(k0, k1, pm):
    """Reductions of equally shaped groups leave sbp_boxing_2d as ONE launch (the group in the grid's third
    dimension); uneven groups go one by one.  Either way every group's result must be, bit for bit, what
    sbp_boxing gives for that group alone (same kernels, same shard order), and match the oracle.  Sizes span
    many workgroups, even and uneven group shapes, inner and outer conversions, both partial operations."""
    PX = P if pm == "sum" else orc.P_MAX
    cases = [((S0, PX), (S0, B)), ((S0, PX), (S0, S1)), ((PX, S1), (B, S1)), ((PX, B), (S0, B)), ((B, PX), (B, S0))]
    for n, shape in enumerate([(k0 * 96, k1 * 256), (k0 * 96 + 1, k1 * 256 + 8)]):
        for c, (si, so) in enumerate(cases):
            T = rnd_f32(300 + 10 * n + c, shape)
            rng = np.random.default_rng(1000 + 10 * n + c)
            ins = []
            if pm == "sum":
                ins = scatter2_random(400 + 10 * n + c, T, si, k0, k1)
            else:
                # random locals; the tensor they stand for is whatever the oracle assembles
                for a in range(k0):
                    for b in range(k1):
                        ins.append(rng.standard_normal(orc.local_shape2(*shape, si, k0, k1, a, b)).astype(np.float32))
                if si[0] == B:      # every group holds the same tensor
                    ins = [ins[b].copy() for _ in range(k0) for b in range(k1)]
                if si[1] == B:      # the devices of a group hold copies
                    ins = [ins[a * k1].copy() for a in range(k0) for _ in range(k1)]
            ref = orc.boxing2(ins, si, so, k0, k1)
            d_in = Dev2.from_host(ins, *shape)
            d_out = Dev2.empty(*shape, np.float32, so, k0, k1)
            sbp.sbp_boxing_2d(d_in.desc, abi2(si), d_out.desc, abi2(so), k0, k1)
            sync()
            got = d_out.host()
            for i, (g, r) in enumerate(zip(got, ref)):
                assert g.shape == r.shape
                if pm == "max":
                    assert np.array_equal(g.astype(np.float64), np.asarray(r, dtype=np.float64)), f"{si}->{so} device {i}"
                else:
                    assert np.allclose(g, r, rtol=0, atol=1e-5 * (1 + np.abs(r).max())), f"{si}->{so} device {i}"
            # the same conversion group by group through the 1-D entry point
            inner = si[0] == so[0]
            parts, kk = (k0, k1) if inner else (k1, k0)
            keep = si[0] if inner else si[1]
            a1, b1 = (si[1], so[1]) if inner else (si[0], so[0])
            for g in range(parts):
                devs = [g * k1 + i if inner else i * k1 + g for i in range(kk)]
                lr, lc = orc.local_shape(*shape, keep, parts, g) if keep in (S0, S1) else shape
                if lr * lc == 0:
                    continue
                t_in = sbp.SbpTensor([d_in.dev[d] for d in devs], lr, lc, sbp.F32)
                outs = [empty_dev(got[d].shape, np.float32) for d in devs]
                sbp.sbp_boxing(t_in, TO_ABI[a1], sbp.SbpTensor(outs, lr, lc, sbp.F32), TO_ABI[b1], kk)
                sync()
                for d, o in zip(devs, outs):
                    assert_bits_equal(got[d], download(o, np.dtype(np.float32)).reshape(got[d].shape), f"{si}->{so} group {g} device {d}")
