"""Row pitch (sbp_tensor_t::ld) of the local buffers: the matmul entry points and the model-parallel softmax /
cross-entropy steps (Sec. 3.1 Table 1, Sec. 6.3.1) on shards whose rows are `ld` elements apart.  Every case is
compared with the oracle at the bar of the dense case, the padding between rows must come back untouched (the
harness poisons it and checks), and where the same kernel runs on dense buffers the results must agree bit for bit."""
import numpy as np
import pytest

import oracle as orc
import paper_2110_15032_amd as sbp
import workloads as wl
from sbp_harness import DevTensor, TO_ABI, assert_bits_equal, assert_matmul_close, sync, values

pytestmark = pytest.mark.gpu
SEED = wl.SEED_BASE + 5


def bf16(tid, shape, std=1.0):
    return wl.to_bf16_bits(wl.normal(SEED, tid, shape, std))


def f32(tid, shape):
    return wl.normal(SEED, tid, shape).astype(np.float32)


def stored_cols(shape, sig, k, trans):
    """longest stored row over the k shards"""
    loc = [orc.local_shape(shape[0], shape[1], sig, k, i) for i in range(k)]
    return max((l[0] if trans else l[1]) for l in loc)


# (dtype, sx, sw, (M, K, N), k, tx, tw, pad of X / W / Y rows in elements, kernel variant, epilogue)
CASES = [
    ("bf16", orc.B, orc.S1, (600, 256, 2 * 500), 2, 0, 0, (8, 12, 76), 0, sbp.EPI_NONE),      # Y pitch 576: whole cache lines, streaming stores
    ("bf16", orc.B, orc.S1, (600, 256, 2 * 500), 2, 0, 0, (0, 0, 4), 0, sbp.EPI_GELU),       # Y pitch 504: 16-byte aligned rows only
    ("bf16", orc.B, orc.S1, (600, 256, 2 * 500), 2, 0, 0, (8, 12, 76), 21, sbp.EPI_GELU),    # ping-pong kernel
    ("bf16", orc.B, orc.S1, (600, 256, 2 * 512), 2, 0, 0, (8, 64, 64), 0, sbp.EPI_GELU),     # dense form takes the same kernel: bit-identical
    ("bf16", orc.B, orc.S1, (600, 256, 2 * 512), 2, 0, 0, (8, 64, 64), 21, sbp.EPI_NONE),
    ("bf16", orc.B, orc.S1, (520, 128, 3 * 264), 3, 0, 0, (0, 8, 3), 0, sbp.EPI_NONE),       # odd Y pitch: guarded element-wise stores
    ("bf16", orc.S1, orc.S0, (520, 2 * 384, 300), 2, 0, 0, (16, 4, 20), 0, sbp.EPI_NONE),    # fp32 partials, pitch 320
    ("bf16", orc.S1, orc.S0, (520, 2 * 384, 300), 2, 0, 0, (16, 4, 20), 21, sbp.EPI_NONE),
    ("bf16", orc.S1, orc.S0, (300, 2 * 256, 520), 2, 1, 1, (4, 8, 8), 0, sbp.EPI_NONE),      # both operands stored transposed
    ("bf16", orc.S0, orc.B, (3 * 100, 192, 136), 3, 0, 0, (8, 8, 8), 0, sbp.EPI_NONE),       # small tile kernel
    ("f32", orc.S1, orc.S0, (37, 50, 29), 2, 0, 0, (3, 5, 1), 0, sbp.EPI_NONE),              # generic kernel, odd pitches
    ("f32", orc.B, orc.S1, (37, 50, 29), 3, 1, 0, (2, 0, 7), 0, sbp.EPI_NONE),
]


@pytest.mark.parametrize("case", CASES, ids=[f"{c[0]}-{c[1]}{c[2]}-{c[3]}-v{c[8]}-e{c[9]}-t{c[5]}{c[6]}-pad{c[7]}" for c in CASES])
def test_matmul_with_row_pitch(case):
    dt, sx, sw, (M, K, N), k, tx, tw, (px, pw, py), variant, epi = case
    if dt == "bf16":
        X, W = bf16(1, (M, K)), bf16(2, (K, N), 0.05)
    else:
        X, W = f32(1, (M, K)), f32(2, (K, N))
    Xs, Ws = orc.scatter(X, sx, k), orc.scatter(W, sw, k)
    sy = orc.infer_matmul(sx, sw)
    out_dt = np.float32 if (sy == orc.P_SUM or dt == "f32") else np.uint16
    ldx = stored_cols((M, K), sx, k, tx) + px if px else 0
    ldw = stored_cols((K, N), sw, k, tw) + pw if pw else 0
    ldy = stored_cols((M, N), sy, k, 0) + py if py else 0
    got = {}
    dense_rows = (stored_cols((M, K), sx, k, tx), stored_cols((K, N), sw, k, tw), stored_cols((M, N), sy, k, 0))
    # the dense form takes the same kernel, with the same order of operations, when its rows are 16-byte multiples too
    same_kernel = dt == "bf16" and all(v % 8 == 0 for v in dense_rows + (ldx, ldw, ldy))
    sbp.sbp_set_knob(sbp.KNOB_GEMM_VARIANT, variant)
    try:
        for name, lds in (("pitched", (ldx, ldw, ldy)), ("dense", (0, 0, 0))):
            if name == "dense" and not same_kernel:
                continue
            dx = DevTensor.from_host(Xs, M, K, sx, trans=tx, ld=lds[0])
            dw = DevTensor.from_host(Ws, K, N, sw, trans=tw, ld=lds[1])
            dy = DevTensor.empty(M, N, out_dt, sy, k, ld=lds[2])
            sbp.sbp_matmul_ex(dx.desc, TO_ABI[sx], dw.desc, TO_ABI[sw], dy.desc, sbp.AUTO, k, None, epi)
            sync()
            got[name] = dy.host()          # asserts that the padding is untouched
    finally:
        sbp.sbp_set_knob(sbp.KNOB_GEMM_VARIANT, 0)
    ref, _ = orc.matmul_sbp([values(x) for x in Xs], sx, [values(w) for w in Ws], sw)
    for i in range(k):
        r = orc.gelu(ref[i]) if epi == sbp.EPI_GELU else ref[i]
        g = values(got["pitched"][i]) if out_dt == np.uint16 else got["pitched"][i]
        assert g.shape == r.shape
        assert_matmul_close(g, r, 2e-2 if dt == "bf16" else 1e-5, f"pitched shard {i}")
        if same_kernel:
            assert_bits_equal(got["pitched"][i], got["dense"][i], f"shard {i}: pitched against dense")


@pytest.mark.parametrize("k,cols,pad,dtype", [(4, 4 * 8 * 40, 64, "bf16"), (3, 1003, 5, "bf16"), (8, 8 * 4 * 30, 8, "f32"), (2, 2 * 300, 84, "bf16")])
def test_fused_row_max_softmax_and_cross_entropy_with_row_pitch(k, cols, pad, dtype):
    """The classifier chain of Sec. 6.3.1 on padded logits: logits GEMM with the fused row maximum into a pitched
    S(1) tensor (bf16 cases), then row max, sum of exponentials, loss partials and the gradient written into a
    pitched tensor as well."""
    torch = __import__("torch")
    rows, D = 300, 128
    ld = -(-cols // k) + pad
    if dtype == "bf16":
        X, W = bf16(3, (rows, D)), bf16(4, (D, cols), 0.3)
        dx = DevTensor.from_host(orc.scatter(X, orc.B, k), rows, D, orc.B)
        dw = DevTensor.from_host(orc.scatter(W, orc.S1, k), D, cols, orc.S1)
        d_l = DevTensor.empty(rows, cols, np.uint16, orc.S1, k, ld=ld)
        m_f = DevTensor.empty(rows, 1, np.float32, orc.P_MAX, k)
        sbp.sbp_matmul_rowmax(dx.desc, sbp.B, dw.desc, sbp.S(1), d_l.desc, sbp.AUTO, m_f.desc, k)
        sync()
        Ls = d_l.host()
        ref, _ = orc.matmul_sbp([values(x) for x in orc.scatter(X, orc.B, k)], orc.B, [values(w) for w in orc.scatter(W, orc.S1, k)], orc.S1)
        for i in range(k):
            assert_matmul_close(values(Ls[i]), ref[i], 2e-2, f"logits shard {i}")
            assert np.array_equal(m_f.host()[i][:, 0].astype(np.float64), orc.row_max(values(Ls[i]))), f"fused row max shard {i}"
    else:
        L = (f32(9, (rows, cols)) * 3.0).astype(np.float32)
        Ls = orc.scatter(L, orc.S1, k)
        d_l = DevTensor.from_host(Ls, rows, cols, orc.S1, ld=ld)
    np_dt = Ls[0].dtype
    y = (wl.uniform(SEED, 11, (rows, 1), 0.0, float(cols)).astype(np.int64) % cols).astype(np.int32)
    y[3, 0] = -1
    g = f32(12, (rows, 1))
    vec = lambda sig: DevTensor.empty(rows, 1, np.float32, sig, k)      # noqa: E731
    m_p, m_b, s_p, s_b, l_p = vec(orc.P_MAX), vec(orc.B), vec(orc.P_SUM), vec(orc.B), vec(orc.P_SUM)
    d_g = DevTensor.from_host([g] * k, rows, 1, orc.B)
    d_y = sbp.SbpTensor([torch.from_numpy(y.copy()).cuda() for _ in range(k)], rows, 1, sbp.I32)
    d_dl = DevTensor.empty(rows, cols, np_dt, orc.S1, k, ld=ld + 8)
    sbp.sbp_row_max(d_l.desc, sbp.S(1), m_p.desc, k)
    sbp.sbp_boxing(m_p.desc, sbp.P_MAX, m_b.desc, sbp.B, k)
    sbp.sbp_row_sumexp(d_l.desc, sbp.S(1), m_b.desc, s_p.desc, k)
    sbp.sbp_boxing(s_p.desc, sbp.P_SUM, s_b.desc, sbp.B, k)
    sbp.sbp_xent_loss(d_l.desc, sbp.S(1), d_y, m_b.desc, s_b.desc, l_p.desc, k)
    sbp.sbp_xent_grad(d_l.desc, sbp.S(1), d_y, m_b.desc, s_b.desc, d_g.desc, d_dl.desc, k)
    sync()
    Lv = [values(s) for s in Ls]
    for i, got in enumerate(m_p.host()):
        assert_bits_equal(got, orc.row_max(Lv[i])[:, None].astype(np.float32), f"local max {i}")
    m = m_b.host()[0][:, 0].astype(np.float64)
    s = s_b.host()[0][:, 0].astype(np.float64)
    for i, got in enumerate(s_p.host()):
        assert np.allclose(got[:, 0], orc.row_sumexp(Lv[i], m), rtol=1e-5, atol=0), f"local sum-exp {i}"
    ref_parts = orc.xent_loss_sbp(Lv, y[:, 0], m, s)
    for i, got in enumerate(l_p.host()):
        assert np.allclose(got[:, 0], ref_parts[i], rtol=2e-6, atol=2e-6), f"loss partial {i}"
    ref_g = orc.xent_grad_sbp(Lv, y[:, 0], m, s, g[:, 0])
    tol = 2.0 ** -7 if dtype == "bf16" else 2e-5
    for i, got in enumerate(d_dl.host()):
        gv = values(got)
        assert gv.shape == ref_g[i].shape
        assert np.all(np.abs(gv - ref_g[i]) <= tol * np.abs(ref_g[i]) + 1e-12), f"gradient shard {i}"


def test_row_pitch_is_validated():
    k, M, K, N = 2, 64, 64, 64
    X, W = bf16(1, (M, K)), bf16(2, (K, N))
    dx = DevTensor.from_host(orc.scatter(X, orc.B, k), M, K, orc.B)
    dw = DevTensor.from_host(orc.scatter(W, orc.S1, k), K, N, orc.S1)
    dy = DevTensor.empty(M, N, np.uint16, orc.S1, k, ld=40)
    short = sbp.SbpTensor(dy.dev, M, N, sbp.BF16, 0, 24)            # local rows have 32 elements
    with pytest.raises(sbp.SbpError) as e:
        sbp.sbp_matmul(dx.desc, sbp.B, dw.desc, sbp.S(1), short, sbp.AUTO, k)
    assert e.value.status == -3      # SBP_ERR_SHAPE
    out = DevTensor.empty(M, N, np.uint16, orc.B, k)
    with pytest.raises(sbp.SbpError) as e:                          # boxing takes dense tensors only
        sbp.sbp_boxing(dy.desc, sbp.S(1), out.desc, sbp.B, k)
    assert e.value.status == -9      # SBP_ERR_UNSUPPORTED
