"""GPU parity at the FULL sizes of the five workloads, in the launch configuration bench.py times.

The oracle cannot recompute whole outputs at these sizes in seconds, so each test checks
  (a) sampled outputs the oracle computes one by one (rows chosen to hit every output tile), to the
      same bars as the small tests, and
  (b) properties that hold at any size, evaluated over the whole output on the device with plain
      torch ops (used as plumbing): all B copies bit-identical, reductions equal to the fp32
      shard-order sum of the partials the GPU itself produced, relayouts equal to slices of the
      uploaded global tensor.
Inputs come from the seeded generator only; nothing the HIP path produced is fed to the oracle.

The MLP block and the classifier head send ALL rows through the oracle (every element of every
output; about a minute of host time on the GPU machine), like the weight gradient; SBP_SAMPLED_ORACLE=1
in the environment cuts that down to a few rows per output tile for quick runs.  Inputs are cut
into shards with the oracle's split rule, never with a rule of the harness's own.
"""
import os

import numpy as np
import pytest

import oracle as orc
import paper_2110_15032_amd as sbp
import workloads as wl
from sbp_harness import assert_bits_equal, assert_matmul_close, assert_psum_close, sync, torch_mod
from workloads import CONFIGS

pytestmark = pytest.mark.gpu
SEED = wl.SEED_BASE
SAMPLED = os.environ.get("SBP_SAMPLED_ORACLE") == "1"
FULL = not SAMPLED


def bf16_window(spec, rows=None, cols=None):
    x = wl.normal(SEED, spec["id"], spec["shape"], spec["dist"][1], rows, cols, dtype=np.float32)
    return wl.to_bf16_bits(x)


def dev_u16(a):
    torch = torch_mod()
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()


def host_u16(t):
    return t.cpu().numpy().view(np.uint16)


def tile_rows(n, tile, per_tile, seed):
    """a few row indices inside every tile of `tile` rows (first, last and random ones)"""
    rng = np.random.default_rng(seed)
    out = []
    for t0 in range(0, n, tile):
        hi = min(t0 + tile, n)
        pick = {t0, hi - 1} | set(int(x) for x in rng.integers(t0, hi, size=max(0, per_tile - 2)))
        out.extend(sorted(pick))
    return np.array(sorted(set(out)))


# ----------------------------------------------------------------------------------------------
def test_config2_mlp_block_full_size():
    torch = torch_mod()
    cfg = CONFIGS["mlp"]
    k = cfg["k"]
    T, D = cfg["X"]["shape"]
    F = cfg["W1"]["shape"][1]
    x = dev_u16(bf16_window(cfg["X"]))
    x_sh = [x] + [x.clone() for _ in range(k - 1)]
    w1_sh = [dev_u16(bf16_window(cfg["W1"], cols=np.arange(*orc.split_range(F, k, i)))) for i in range(k)]
    w2_sh = [dev_u16(bf16_window(cfg["W2"], rows=np.arange(*orc.split_range(F, k, i)))) for i in range(k)]
    h_sh = [torch.full((T, F // k), 0x7FC1, dtype=torch.int16, device="cuda") for _ in range(k)]
    y_sh = [torch.full((T, D), float("nan"), device="cuda") for _ in range(k)]
    yb_sh = [torch.full((T, D), float("nan"), device="cuda") for _ in range(k)]
    X, W1, W2 = sbp.SbpTensor(x_sh, T, D, sbp.BF16), sbp.SbpTensor(w1_sh, D, F, sbp.BF16), sbp.SbpTensor(w2_sh, F, D, sbp.BF16)
    H, Y, Yb = sbp.SbpTensor(h_sh, T, F, sbp.BF16), sbp.SbpTensor(y_sh, T, D, sbp.F32), sbp.SbpTensor(yb_sh, T, D, sbp.F32)
    sbp.sbp_matmul_ex(X, sbp.B, W1, sbp.S(1), H, sbp.S(1), k, None, sbp.EPI_GELU)
    sbp.sbp_matmul(H, sbp.S(1), W2, sbp.S(0), Y, sbp.P_SUM, k)
    sbp.sbp_boxing(Y, sbp.P_SUM, Yb, sbp.B, k)
    sync()

    # (b) whole-output properties
    acc = y_sh[0].clone()
    for i in range(1, k):
        acc += y_sh[i]                       # fp32, shard order: what the library documents
    for j in range(k):
        assert torch.equal(yb_sh[j], acc), f"P->B copy {j} is not the fp32 shard-order sum of the partials"
    assert not torch.isnan(acc).any()

    # (a) sampled token rows through the oracle, every 256-row tile hit
    rows = np.arange(T) if FULL else tile_rows(T, 256, 3, 7)
    print(f"config 2: {len(rows)} of {T} token rows through the oracle", flush=True)
    Xr = orc.bf16_to_f64(bf16_window(cfg["X"], rows=rows))
    W1h = [orc.bf16_to_f64(host_u16(w)) for w in w1_sh]     # the uploaded words themselves (generator output)
    W2h = [orc.bf16_to_f64(host_u16(w)) for w in w2_sh]
    Hs, s_h = orc.matmul_sbp([Xr] * k, orc.B, W1h, orc.S1)
    assert s_h == orc.S1
    Hq = [orc.bf16_round(orc.gelu(h)) for h in Hs]
    Ys, s_y = orc.matmul_sbp([orc.bf16_to_f64(h) for h in Hq], orc.S1, W2h, orc.S0)
    assert s_y == orc.P_SUM
    Yref = orc.assemble(Ys, orc.P_SUM)
    ridx = torch.from_numpy(rows).cuda()
    worst = 0.0
    for i in range(k):
        got_h = orc.bf16_to_f64(host_u16(h_sh[i][ridx]))
        assert_matmul_close(got_h, orc.bf16_to_f64(Hq[i]), 2e-2, f"H shard {i}")
        got_y = y_sh[i][ridx].cpu().numpy()
        worst = max(worst, assert_matmul_close(got_y, Ys[i], 2e-2, f"Y partial {i}"))
    got = yb_sh[0][ridx].cpu().numpy()
    assert_matmul_close(got, Yref, 2e-2, "Y after P->B")
    parts_gpu = [y_sh[i][ridx].cpu().numpy() for i in range(k)]
    assert_psum_close(got, parts_gpu, orc.assemble(parts_gpu, orc.P_SUM), "P->B against the oracle's sum of the same partials")
    print(f"config 2: worst relative error of the fp32 partials {worst:.2e}")


# ----------------------------------------------------------------------------------------------
def test_config3_dp_weight_gradient_full_size():
    torch = torch_mod()
    cfg = CONFIGS["dp_grad"]
    k = cfg["k"]
    Tk, Din = cfg["X"]["shape"]       # 16384 tokens, 1024
    Dout = cfg["dY"]["shape"][1]      # 4096
    Xw, dYw = bf16_window(cfg["X"]), bf16_window(cfg["dY"])
    # X is S(0) by tokens; the operand of dW = X^T dY is X^T [1024, 16384], split S(1), stored transposed
    x_sh = [dev_u16(Xw[slice(*orc.split_range(Tk, k, i))]) for i in range(k)]
    dy_sh = [dev_u16(dYw[slice(*orc.split_range(Tk, k, i))]) for i in range(k)]
    dw_sh = [torch.full((Din, Dout), float("nan"), device="cuda") for _ in range(k)]
    dws_sh = [torch.full((Din // k, Dout), float("nan"), device="cuda") for _ in range(k)]
    dwb_sh = [torch.full((Din, Dout), float("nan"), device="cuda") for _ in range(k)]
    XT = sbp.SbpTensor(x_sh, Din, Tk, sbp.BF16, trans=1)
    DY = sbp.SbpTensor(dy_sh, Tk, Dout, sbp.BF16)
    DW = sbp.SbpTensor(dw_sh, Din, Dout, sbp.F32)
    DWS = sbp.SbpTensor(dws_sh, Din, Dout, sbp.F32)
    DWB = sbp.SbpTensor(dwb_sh, Din, Dout, sbp.F32)
    sbp.sbp_matmul(XT, sbp.S(1), DY, sbp.S(0), DW, sbp.P_SUM, k)
    sbp.sbp_boxing(DW, sbp.P_SUM, DWS, sbp.S(0), k)
    sbp.sbp_boxing(DW, sbp.P_SUM, DWB, sbp.B, k)
    sync()
    # the oracle does this one in full: 8 local products X_i^T dY_i in float64
    Xs = [orc.bf16_to_f64(Xw[slice(*orc.split_range(Tk, k, i))]).T.copy() for i in range(k)]
    dYs = [orc.bf16_to_f64(dYw[slice(*orc.split_range(Tk, k, i))]) for i in range(k)]
    parts, sy = orc.matmul_sbp(Xs, orc.S1, dYs, orc.S0)
    assert sy == orc.P_SUM
    got_parts = [t.cpu().numpy() for t in dw_sh]
    for i in range(k):
        assert_matmul_close(got_parts[i], parts[i], 2e-2, f"dW partial {i}")
        assert_matmul_close(got_parts[i], parts[i], 1e-4, f"dW partial {i} (fp32 accumulation of exact products)")
    ref_gpu_sum = orc.assemble(got_parts, orc.P_SUM)          # float64 sum of the GPU's partials
    for j, t in enumerate(dwb_sh):
        assert_psum_close(t.cpu().numpy(), got_parts, ref_gpu_sum, f"P->B copy {j}")
        assert torch.equal(t, dwb_sh[0])
    ref_s = orc.boxing(got_parts, orc.P_SUM, orc.S0, k)
    for j, t in enumerate(dws_sh):
        sl = slice(*orc.split_range(Din, k, j))
        assert_psum_close(t.cpu().numpy(), [p[sl] for p in got_parts], ref_s[j], f"P->S(0) shard {j}")
        assert torch.equal(t, dwb_sh[0][sl]), "reduce-scatter slice differs from the all-reduce result"
    assert_matmul_close(dwb_sh[0].cpu().numpy(), orc.assemble(parts, orc.P_SUM), 2e-2, "dW")


# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("layout", ["pitch128", "dense"])
def test_config4_classifier_head_full_size(layout):
    """layout pitch128: the logits and their gradient have a row pitch of 125056 elements (whole 128-byte lines,
    what bench.py times); dense: 125000, seven of eight rows straddle cache lines.  The padded form sends every
    row through the oracle, the dense one a sample."""
    torch = torch_mod()
    cfg = CONFIGS["classifier"]
    k = cfg["k"]
    R, Dm = cfg["F"]["shape"]         # 1024, 512
    C = cfg["W"]["shape"][1]          # 1,000,000 classes
    Fw = bf16_window(cfg["F"])
    f = dev_u16(Fw)
    f_sh = [f] + [f.clone() for _ in range(k - 1)]
    w_host = [bf16_window(cfg["W"], cols=np.arange(*orc.split_range(C, k, i))) for i in range(k)]   # [512, 125000] each
    w_sh = [dev_u16(w) for w in w_host]
    Ci = C // k
    P = (Ci + 63) // 64 * 64 if layout == "pitch128" else Ci      # row pitch in elements
    LD = P if P != Ci else 0

    def logits_buffers():
        store = [torch.full((R, P), 0x7FC1, dtype=torch.int16, device="cuda") for _ in range(k)]
        return store, [s[:, :Ci] for s in store]                  # the views start at the buffers' first element

    l_store, l_sh = logits_buffers()
    vec = lambda: [torch.full((R, 1), float("nan"), device="cuda") for _ in range(k)]      # noqa: E731
    mp, mb, sp, sb = vec(), vec(), vec(), vec()
    Ft, Wt = sbp.SbpTensor(f_sh, R, Dm, sbp.BF16), sbp.SbpTensor(w_sh, Dm, C, sbp.BF16)
    L = sbp.SbpTensor(l_sh, R, C, sbp.BF16, 0, LD)
    MP, MB, SP, SB = (sbp.SbpTensor(v, R, 1, sbp.F32) for v in (mp, mb, sp, sb))
    sbp.sbp_matmul(Ft, sbp.B, Wt, sbp.S(1), L, sbp.S(1), k)
    sbp.sbp_row_max(L, sbp.S(1), MP, k)
    sbp.sbp_boxing(MP, sbp.P_MAX, MB, sbp.B, k)
    sbp.sbp_row_sumexp(L, sbp.S(1), MB, SP, k)
    sbp.sbp_boxing(SP, sbp.P_SUM, SB, sbp.B, k)
    sync()

    # (b) whole-output properties on the device
    lf = [t.view(torch.bfloat16).float() for t in l_sh]
    for i in range(k):
        assert torch.equal(mp[i][:, 0], lf[i].max(dim=1).values), f"local row max {i}"
    gmax = torch.stack([m[:, 0] for m in mp]).max(dim=0).values
    for j in range(k):
        assert torch.equal(mb[j][:, 0], gmax), "global max copy"
        ref_s = torch.exp(lf[j].double() - gmax.double()[:, None]).sum(dim=1)
        assert torch.allclose(sp[j][:, 0].double(), ref_s, rtol=2e-5, atol=0), f"local sum-exp {j}"
    tot = sp[0].clone()
    for i in range(1, k):
        tot += sp[i]
    for j in range(k):
        assert torch.equal(sb[j], tot), "denominator copy"
    del lf

    # (a) sampled feature rows through the oracle (all 10^6 classes of each), shard by shard
    rows = np.arange(R) if (FULL and layout == "pitch128") else tile_rows(R, 256, 3, 11)
    print(f"config 4: {len(rows)} of {R} feature rows through the oracle", flush=True)
    Fr = orc.bf16_to_f64(Fw[rows])
    ridx = torch.from_numpy(rows).cuda()
    m_loc, logits_q = [], []
    for i in range(k):
        ref = orc.matmul(Fr, orc.bf16_to_f64(w_host[i]))
        got = orc.bf16_to_f64(host_u16(l_sh[i][ridx]))
        assert_matmul_close(got, ref, 2e-2, f"logits shard {i}")
        q = orc.bf16_to_f64(orc.bf16_round(ref))
        logits_q.append(q)
        m_loc.append(orc.row_max(q)[:, None])
    m = orc.boxing(m_loc, orc.P_MAX, orc.B, k)[0][:, 0]
    got_m = mb[0][ridx, 0].cpu().numpy().astype(np.float64)
    # the two sides round the same accumulations to bf16 independently: at most one bf16 step apart
    assert np.all(np.abs(got_m - m) <= 2.0 ** -7 * np.abs(m)), "global max vs oracle"
    s_loc = [orc.row_sumexp(q, m)[:, None] for q in logits_q]
    s = orc.boxing(s_loc, orc.P_SUM, orc.B, k)[0][:, 0]
    got_s = sb[0][ridx, 0].cpu().numpy().astype(np.float64)
    # softmax denominator: s * exp(m) is what does not depend on which of two adjacent bf16 values the max took
    assert np.allclose(np.log(got_s) + got_m, np.log(s) + m, rtol=0, atol=2e-2), "softmax denominator vs oracle"

    # ---- the form bench.py times: row max folded into the logits GEMM; then the sparse cross entropy ----
    print("config 4: fused row max, cross entropy loss and gradient at full size", flush=True)
    l2_store, l2_sh = logits_buffers()
    mp2 = vec()
    L2, MP2 = sbp.SbpTensor(l2_sh, R, C, sbp.BF16, 0, LD), sbp.SbpTensor(mp2, R, 1, sbp.F32)
    sbp.sbp_matmul_rowmax(Ft, sbp.B, Wt, sbp.S(1), L2, sbp.S(1), MP2, k)
    sync()
    for i in range(k):
        assert torch.equal(l2_sh[i], l_sh[i]), f"logits of the fused call, shard {i}"
        assert torch.equal(mp2[i], mp[i]), f"fused row max, shard {i}"
        assert bool((l2_store[i][:, Ci:] == 0x7FC1).all()), f"padding of the logits, shard {i}"
    del l2_sh, l2_store, L2

    y_host = (wl.uniform(SEED, 40, (R, 1), 0.0, float(C)).astype(np.int64) % C).astype(np.int32)
    y_host[5, 0] = -1                                   # ignored rows
    y_host[700, 0] = C
    g_host = wl.normal(SEED, 41, (R, 1), 1.0, dtype=np.float32)
    y_dev = torch.from_numpy(y_host).cuda()
    g_dev = torch.from_numpy(g_host).cuda()
    lp, lb = vec(), vec()
    dl_store, dl_sh = logits_buffers()
    Y = sbp.SbpTensor([y_dev] * k, R, 1, sbp.I32)
    G = sbp.SbpTensor([g_dev] * k, R, 1, sbp.F32)
    LP, LB = sbp.SbpTensor(lp, R, 1, sbp.F32), sbp.SbpTensor(lb, R, 1, sbp.F32)
    DL = sbp.SbpTensor(dl_sh, R, C, sbp.BF16, 0, LD)
    sbp.sbp_xent_loss(L, sbp.S(1), Y, MB, SB, LP, k)
    sbp.sbp_boxing(LP, sbp.P_SUM, LB, sbp.B, k)
    sbp.sbp_xent_grad(L, sbp.S(1), Y, MB, SB, G, DL, k)
    sync()

    for i in range(k):
        assert bool((l_store[i][:, Ci:] == 0x7FC1).all()) and bool((dl_store[i][:, Ci:] == 0x7FC1).all()), f"padding, shard {i}"

    # (b) over the whole output on the device: loss = log s + m - L[r, y], gradient = g (exp(L - m) / s - onehot)
    valid = (y_dev[:, 0] >= 0) & (y_dev[:, 0] < C)
    picked = torch.zeros(R, dtype=torch.float64, device="cuda")
    for i in range(k):
        lo = i * Ci
        mine = valid & (y_dev[:, 0] >= lo) & (y_dev[:, 0] < lo + Ci)
        idx = (y_dev[:, 0].long() - lo).clamp(0, Ci - 1)
        li = l_sh[i].view(torch.bfloat16).gather(1, idx[:, None])[:, 0].double()
        picked += torch.where(mine, li, torch.zeros_like(li))
    want_loss = torch.where(valid, torch.log(sb[0][:, 0].double()) + mb[0][:, 0].double() - picked, torch.zeros_like(picked))
    for j in range(k):
        assert torch.equal(lb[j], lb[0]), "loss copies"
    assert torch.allclose(lb[0][:, 0].double(), want_loss, rtol=1e-5, atol=1e-5), "loss over all rows"
    assert float(lb[0][5, 0]) == 0.0 and float(lb[0][700, 0]) == 0.0
    for i in range(k):
        lo = i * Ci
        pr = torch.exp(l_sh[i].view(torch.bfloat16).double() - mb[0].double()) / sb[0].double()
        mine = valid & (y_dev[:, 0] >= lo) & (y_dev[:, 0] < lo + Ci)
        r_idx = torch.nonzero(mine)[:, 0]
        pr[r_idx, (y_dev[r_idx, 0].long() - lo)] -= 1.0
        pr *= torch.where(valid, g_dev[:, 0], torch.zeros_like(g_dev[:, 0])).double()[:, None]
        got = dl_sh[i].view(torch.bfloat16).double()
        bad = (got - pr).abs() > 2.0 ** -7 * pr.abs() + 1e-30
        assert not bool(bad.any()), f"gradient shard {i}: {int(bad.sum())} entries more than one bf16 step off"
        del pr, got, bad

    # (a) the sampled rows through the oracle, from its own logits
    q_all = np.concatenate(logits_q, axis=1)
    yr = y_host[rows, 0]
    ref_loss = orc.softmax_xent_loss(q_all, yr)
    got_loss = lb[0][ridx, 0].cpu().numpy().astype(np.float64)
    assert np.allclose(got_loss, ref_loss, rtol=0, atol=2e-2), "loss vs oracle on sampled rows"
    ref_grad = orc.softmax_xent_grad(q_all, yr, g_host[rows, 0].astype(np.float64))
    for i in range(k):
        got = orc.bf16_to_f64(host_u16(dl_sh[i][ridx]))
        ref = ref_grad[:, i * Ci:(i + 1) * Ci]
        assert np.all(np.abs(got - ref) <= 2.0 ** -5 * np.abs(ref) + 1e-12), f"gradient vs oracle on sampled rows, shard {i}"


# ----------------------------------------------------------------------------------------------
def test_config5_relayout_full_size():
    torch = torch_mod()
    cfg = CONFIGS["relayout"]
    k = cfg["k"]
    R, C = cfg["T"]["shape"]          # 65536 x 8192 16-bit words
    Rk, Ck = R // k, C // k
    s0 = [dev_u16(wl.pattern_u16((R, C), rows=np.arange(i * Rk, (i + 1) * Rk))) for i in range(k)]
    G = torch.cat(s0, dim=0)          # the global tensor, for whole-output checks by slicing
    s1 = [torch.full((R, Ck), 0x7FC1, dtype=torch.int16, device="cuda") for _ in range(k)]
    T0, T1 = sbp.SbpTensor(s0, R, C, sbp.BF16), sbp.SbpTensor(s1, R, C, sbp.BF16)
    sbp.sbp_boxing(T0, sbp.S(0), T1, sbp.S(1), k)            # all2all
    sync()
    for j in range(k):
        assert torch.equal(s1[j], G[:, j * Ck:(j + 1) * Ck]), f"S(0)->S(1) shard {j}"
    # The oracle's own S(0) -> S(1) conversion of a sub-tensor made of the first and last row of every input
    # shard: scattered S(0) over k devices it gives device i exactly those two rows of shard i, so the oracle
    # routes the same words between the same devices as the full-size call.
    rows = np.array([r for i in range(k) for r in (i * Rk, (i + 1) * Rk - 1)])
    sub = wl.pattern_u16((R, C), rows=rows)
    sub_s0 = orc.scatter(sub, orc.S0, k)
    assert all(np.array_equal(sub_s0[i], host_u16(s0[i][[0, Rk - 1]])) for i in range(k))
    ref = orc.boxing(sub_s0, orc.S0, orc.S1, k)
    ridx = torch.from_numpy(rows).cuda()
    for j in range(k):
        assert_bits_equal(host_u16(s1[j][ridx]), ref[j], f"S(0)->S(1) first/last rows of every shard, shard {j}")
    del s0

    b = [torch.full((R, C), 0x7FC1, dtype=torch.int16, device="cuda") for _ in range(k)]     # 16 x 1 GiB
    TB = sbp.SbpTensor(b, R, C, sbp.BF16)
    sbp.sbp_boxing(T1, sbp.S(1), TB, sbp.B, k)               # all-gather
    sync()
    for j in range(k):
        assert torch.equal(b[j], G), f"S(1)->B copy {j}"
    refB = orc.boxing(orc.scatter(sub, orc.S1, k), orc.S1, orc.B, k)
    assert_bits_equal(host_u16(b[k - 1][ridx]), refB[k - 1], "S(1)->B sampled rows")
    del s1, T1

    # B -> S(0) reads device j's OWN copy: make the copies differ in one word each to see that
    for j in range(k):
        b[j][j * Rk, 0] = j + 1
    out = [torch.full((Rk, C), 0x7FC1, dtype=torch.int16, device="cuda") for _ in range(k)]
    TO = sbp.SbpTensor(out, R, C, sbp.BF16)
    sbp.sbp_boxing(TB, sbp.B, TO, sbp.S(0), k)               # local slice
    sync()
    for j in range(k):
        assert torch.equal(out[j], b[j][j * Rk:(j + 1) * Rk]), f"B->S(0) shard {j}"
        assert int(out[j][0, 0]) == j + 1


# ----------------------------------------------------------------------------------------------
def test_cast_fused_boxing_full_size():
    """The sharded-optimizer-state workload bench.py times (Sec. 6.4): 2^28 parameters, k = 8.  Forward:
    fp32 S(0) -> bf16 B; backward: bf16 P(sum) -> fp32 S(0)."""
    torch = torch_mod()
    k, R, C = 8, 16384, 16384
    Rk = R // k
    w32 = []
    for i in range(k):
        rows = np.arange(i * Rk, (i + 1) * Rk)
        w32.append(torch.from_numpy(wl.normal(SEED, 200, (R, C), 0.02, rows, None, dtype=np.float32)).cuda())
    w16 = [torch.full((R, C), 0x7FC1, dtype=torch.int16, device="cuda") for _ in range(k)]
    W32, W16 = sbp.SbpTensor(w32, R, C, sbp.F32), sbp.SbpTensor(w16, R, C, sbp.BF16)
    print("cast + all-gather, 16384 x 16384", flush=True)
    sbp.sbp_boxing_cast(W32, sbp.S(0), W16, sbp.B, k)
    sync()
    # (b) whole output: every copy equals the round-to-nearest-even cast of the assembled tensor (torch's cast as calculator)
    want = torch.cat(w32, dim=0).to(torch.bfloat16).view(torch.int16)
    for j in range(k):
        assert torch.equal(w16[j], want), f"bf16 copy {j}"
    # (a) sampled rows through the oracle's rounding
    rows = tile_rows(R, Rk, 3, 21)
    src = wl.normal(SEED, 200, (R, C), 0.02, rows, None, dtype=np.float32)
    ridx = torch.from_numpy(rows).cuda()
    assert_bits_equal(host_u16(w16[3][ridx]), orc.bf16_round(src), "sampled rows vs the oracle's bf16 rounding")
    del want, w32, W32

    print("cast + reduce-scatter, 8 x 16384 x 16384 bf16 partials", flush=True)
    g16 = w16                                            # reuse the buffers: k partial gradients, N(0, 1) rounded to bf16
    gen = torch.Generator(device="cuda").manual_seed(2110150329)
    for i in range(k):
        g16[i].view(torch.bfloat16).normal_(0.0, 1.0, generator=gen)
    g32 = [torch.full((Rk, C), float("nan"), device="cuda") for _ in range(k)]
    G16, G32 = sbp.SbpTensor(g16, R, C, sbp.BF16), sbp.SbpTensor(g32, R, C, sbp.F32)
    sbp.sbp_boxing_cast(G16, sbp.P_SUM, G32, sbp.S(0), k)
    sync()
    # (b) whole output: fp32 sum in shard order of the exactly widened partials
    for j in range(k):
        acc = g16[0][j * Rk:(j + 1) * Rk].view(torch.bfloat16).float()
        for i in range(1, k):
            acc = acc + g16[i][j * Rk:(j + 1) * Rk].view(torch.bfloat16).float()
        assert torch.equal(g32[j], acc), f"fp32 slice {j}"
    # (a) sampled rows through the oracle (fp64 sum of the widened partials), to the P(sum) bar
    for j in (0, 5):
        loc = np.array([0, 17, Rk - 1])
        parts = [orc.bf16_to_f64(host_u16(g16[i][j * Rk + torch.from_numpy(loc).cuda()])) for i in range(k)]
        ref = orc.assemble(parts, orc.P_SUM)
        assert_psum_close(g32[j][torch.from_numpy(loc).cuda()].cpu().numpy(), parts, ref, f"sampled rows of slice {j}")


# ----------------------------------------------------------------------------------------------
def test_uvw_deferred_boxing_full_size():
    """The Y = U V W workload bench.py times (Sec. 3.3): U[4096,16384] S(1), V[16384,4096] S(0), W[4096,1024] B,
    bf16, k = 8.  Deferred: (UV) stays 8 fp32 partials, each times W (Table 1 row 4), one P->B on Y.
    Immediate: P->B on (UV), then row 6.  Sampled rows of both against the oracle's U V W."""
    torch = torch_mod()
    k, M, K1, N1, N2 = 8, 4096, 16384, 4096, 1024

    def bits(tid, shape, std, rows=None, cols=None):
        return wl.to_bf16_bits(wl.normal(SEED, tid, shape, std, rows, cols, dtype=np.float32))

    u_host = [bits(100, (M, K1), 1.0, cols=np.arange(*orc.split_range(K1, k, i))) for i in range(k)]
    v_host = [bits(101, (K1, N1), 0.02, rows=np.arange(*orc.split_range(K1, k, i))) for i in range(k)]
    w_host = bits(102, (N1, N2), 0.02)
    u_sh, v_sh = [dev_u16(x) for x in u_host], [dev_u16(x) for x in v_host]
    w_sh = [dev_u16(w_host)] * k
    U, V, W = sbp.SbpTensor(u_sh, M, K1, sbp.BF16), sbp.SbpTensor(v_sh, K1, N1, sbp.BF16), sbp.SbpTensor(w_sh, N1, N2, sbp.BF16)
    f32 = lambda r, c: [torch.full((r, c), float("nan"), device="cuda") for _ in range(k)]      # noqa: E731
    uv, uvb, yp, yl, ye = f32(M, N1), f32(M, N1), f32(M, N2), f32(M, N2), f32(M, N2)
    UV, UVB = sbp.SbpTensor(uv, M, N1, sbp.F32), sbp.SbpTensor(uvb, M, N1, sbp.F32)
    YP, YL, YE = (sbp.SbpTensor(t, M, N2, sbp.F32) for t in (yp, yl, ye))
    print("U V W: deferred and immediate boxing at full size", flush=True)
    sbp.sbp_matmul(U, sbp.S(1), V, sbp.S(0), UV, sbp.P_SUM, k)
    sbp.sbp_matmul(UV, sbp.P_SUM, W, sbp.B, YP, sbp.P_SUM, k)
    sbp.sbp_boxing(YP, sbp.P_SUM, YL, sbp.B, k)
    sbp.sbp_boxing(UV, sbp.P_SUM, UVB, sbp.B, k)
    sbp.sbp_matmul(UVB, sbp.B, W, sbp.B, YE, sbp.B, k)
    sync()
    # (b) whole output: copies identical; the two orders of boxing agree to accumulation-order noise
    for j in range(1, k):
        assert torch.equal(yl[j], yl[0]) and torch.equal(ye[j], ye[0]) and torch.equal(uvb[j], uvb[0])
    scale = float(yl[0].abs().max())
    assert float((yl[0] - ye[0]).abs().max()) <= 1e-4 * scale, "deferred vs immediate boxing"
    # (a) sampled rows through the oracle: the partial products one by one, then the whole chain
    rows = tile_rows(M, 256, 3, 31)
    ridx = torch.from_numpy(rows).cuda()
    Wd = orc.bf16_to_f64(w_host)
    chain = np.zeros((len(rows), N2))
    for i in range(k):
        part = orc.matmul(orc.bf16_to_f64(u_host[i][rows]), orc.bf16_to_f64(v_host[i]))          # (UV)_i, fp64
        assert_matmul_close(uv[i][ridx].cpu().numpy(), part, 2e-2, f"partial {i} of U V")
        yi = orc.matmul(part, Wd)
        assert_matmul_close(yp[i][ridx].cpu().numpy(), yi, 2e-2, f"partial {i} of (U V) W")
        chain += yi
    assert_matmul_close(yl[0][ridx].cpu().numpy(), chain, 2e-2, "Y, boxing deferred")
    assert_matmul_close(ye[0][ridx].cpu().numpy(), chain, 2e-2, "Y, boxing immediate")


# ----------------------------------------------------------------------------------------------
def test_boxing_between_placements_full_size():
    """The placement-boundary workload bench.py times (Table 2, column "disjoint"): 8 -> 4 logical devices.
    T[16384,16384] 16-bit words S(0) -> S(0) and S(0) -> B; [8192,4096] fp32 partials P(sum) -> B and
    P(sum) -> S(0)."""
    torch = torch_mod()
    ki, ko, R, C = 8, 4, 16384, 16384
    a8 = [dev_u16(wl.pattern_u16((R, C), rows=np.arange(i * (R // ki), (i + 1) * (R // ki))) ^ np.uint16(257 * i)) for i in range(ki)]
    whole = torch.cat(a8, dim=0)
    a4 = [torch.full((R // ko, C), 0x7FC1, dtype=torch.int16, device="cuda") for _ in range(ko)]
    b4 = [torch.full((R, C), 0x7FC1, dtype=torch.int16, device="cuda") for _ in range(ko)]
    A8, A4, B4 = (sbp.SbpTensor(x, R, C, sbp.BF16) for x in (a8, a4, b4))
    print("between placements: relayout of 512 MiB", flush=True)
    sbp.sbp_boxing_across(A8, sbp.S(0), ki, A4, sbp.S(0), ko)
    sbp.sbp_boxing_across(A8, sbp.S(0), ki, B4, sbp.B, ko)
    sync()
    for j in range(ko):
        assert torch.equal(a4[j], whole[j * (R // ko):(j + 1) * (R // ko)]), f"S(0) slice {j}"
        assert torch.equal(b4[j], whole), f"B copy {j}"
    # the oracle's own conversions of the sub-tensor made of the first and last row of every input shard (8 devices
    # hold two rows each; S(0) over 4 devices gives output device j the rows of input shards 2 j and 2 j + 1)
    Rk8 = R // ki
    rows = np.array([r for i in range(ki) for r in (i * Rk8, (i + 1) * Rk8 - 1)])
    sub = np.stack([wl.pattern_u16((R, C), rows=np.array([r]))[0] ^ np.uint16(257 * (r // Rk8)) for r in rows])
    sub_in = orc.scatter(sub, orc.S0, ki)
    ridx = torch.from_numpy(rows).cuda()
    ref_b = orc.boxing_across(sub_in, orc.S0, orc.B, ko)
    ref_s = orc.boxing_across(sub_in, orc.S0, orc.S0, ko)
    local = torch.from_numpy(np.array([0, Rk8 - 1, Rk8, 2 * Rk8 - 1])).cuda()
    for j in range(ko):
        assert_bits_equal(host_u16(b4[j][ridx]), ref_b[j], f"S(0) x 8 -> B x 4, first/last rows of every shard, copy {j}")
        assert_bits_equal(host_u16(a4[j][local]), ref_s[j], f"S(0) x 8 -> S(0) x 4, first/last rows of every shard, slice {j}")
    del a8, a4, b4, whole

    print("between placements: 8 x 128 MiB partials", flush=True)
    PR, PC = 8192, 4096
    gen = torch.Generator(device="cuda").manual_seed(2110150330)
    p8 = [torch.empty(PR, PC, device="cuda").normal_(0.0, 0.02, generator=gen) for _ in range(ki)]
    pb4 = [torch.full((PR, PC), float("nan"), device="cuda") for _ in range(ko)]
    ps4 = [torch.full((PR // ko, PC), float("nan"), device="cuda") for _ in range(ko)]
    P8, PB4, PS4 = (sbp.SbpTensor(x, PR, PC, sbp.F32) for x in (p8, pb4, ps4))
    sbp.sbp_boxing_across(P8, sbp.P_SUM, ki, PB4, sbp.B, ko)
    sbp.sbp_boxing_across(P8, sbp.P_SUM, ki, PS4, sbp.S(0), ko)
    sync()
    acc = p8[0].clone()
    for i in range(1, ki):
        acc += p8[i]                                               # fp32, input order
    for j in range(ko):
        assert torch.equal(pb4[j], acc), f"all-reduce copy {j}"
        assert torch.equal(ps4[j], acc[j * (PR // ko):(j + 1) * (PR // ko)]), f"reduce-scatter slice {j}"
    # the oracle's all-reduce and reduce-scatter from 8 to 4 devices of four sampled rows (one per output slice)
    rows = np.array([0, PR // ko + 5, 2 * (PR // ko) + 4097 % (PR // ko), PR - 1])
    loc = torch.from_numpy(rows).cuda()
    parts = [p[loc].cpu().numpy() for p in p8]
    ref_b = orc.boxing_across([x.astype(np.float64) for x in parts], orc.P_SUM, orc.B, ko)
    ref_s = orc.boxing_across([x.astype(np.float64) for x in parts], orc.P_SUM, orc.S0, ko)
    for j in range(ko):
        assert_psum_close(pb4[j][loc].cpu().numpy(), parts, ref_b[j], f"sampled rows of the all-reduce vs the oracle, copy {j}")
        r = rows[j] - j * (PR // ko)
        assert_psum_close(ps4[j][r:r + 1].cpu().numpy(), [q[j:j + 1] for q in parts], ref_s[j], f"sampled row of reduce-scatter slice {j}")


# ----------------------------------------------------------------------------------------------
def test_grid_2x4_full_size():
    """The two-dimensional workload bench.py times (Sec. 3.3, Table 3) on a 2 x 4 grid at the MLP block's sizes:
    row 1 (S0,B) x (B,S1) -> (S0,S1), row 2 (S0,S1) x (B,S0) -> (S0,P), then the all-reduce inside each group."""
    torch = torch_mod()
    k0, k1, M, D, F = 2, 4, 8192, 4096, 16384
    k = k0 * k1
    S0, S1, B_, P = sbp.S(0), sbp.S(1), sbp.B, sbp.P_SUM
    Mg, Fd = M // k0, F // k1

    def bits(tid, shape, std, rows=None, cols=None):
        return wl.to_bf16_bits(wl.normal(SEED, tid, shape, std, rows, cols, dtype=np.float32))

    # row 1: X1[M,D] rows by group, W1[D,F] columns by device
    x1_h = [bits(300, (M, D), 1.0, rows=np.arange(a * Mg, (a + 1) * Mg)) for a in range(k0)]
    w1_h = [bits(301, (D, F), 0.02, cols=np.arange(b * Fd, (b + 1) * Fd)) for b in range(k1)]
    x1_d, w1_d = [dev_u16(x) for x in x1_h], [dev_u16(w) for w in w1_h]
    x1 = [x1_d[a] for a in range(k0) for b in range(k1)]
    w1 = [w1_d[b] for a in range(k0) for b in range(k1)]
    y1 = [torch.full((Mg, Fd), 0x7FC1, dtype=torch.int16, device="cuda") for _ in range(k)]
    # row 2: X2[M,F] rows by group and columns by device, W2[F,D] rows by device
    x2_h = [[bits(302, (M, F), 1.0, rows=np.arange(a * Mg, (a + 1) * Mg), cols=np.arange(b * Fd, (b + 1) * Fd)) for b in range(k1)]
            for a in range(k0)]
    w2_h = [bits(303, (F, D), 0.02, rows=np.arange(b * Fd, (b + 1) * Fd)) for b in range(k1)]
    w2_d = [dev_u16(w) for w in w2_h]
    x2 = [dev_u16(x2_h[a][b]) for a in range(k0) for b in range(k1)]
    w2 = [w2_d[b] for a in range(k0) for b in range(k1)]
    y2 = [torch.full((Mg, D), float("nan"), device="cuda") for _ in range(k)]
    y2b = [torch.full((Mg, D), float("nan"), device="cuda") for _ in range(k)]
    X1, W1, Y1 = sbp.SbpTensor(x1, M, D, sbp.BF16), sbp.SbpTensor(w1, D, F, sbp.BF16), sbp.SbpTensor(y1, M, F, sbp.BF16)
    X2, W2 = sbp.SbpTensor(x2, M, F, sbp.BF16), sbp.SbpTensor(w2, F, D, sbp.BF16)
    Y2, Y2B = sbp.SbpTensor(y2, M, D, sbp.F32), sbp.SbpTensor(y2b, M, D, sbp.F32)
    print("grid 2 x 4: Table 3 rows 1 and 2 at full size, inner all-reduce", flush=True)
    sbp.sbp_matmul_2d(X1, (S0, B_), W1, (B_, S1), Y1, (S0, S1), k0, k1)
    sbp.sbp_matmul_2d(X2, (S0, S1), W2, (B_, S0), Y2, (S0, P), k0, k1)
    sbp.sbp_boxing_2d(Y2, (S0, P), Y2B, (S0, B_), k0, k1)
    sync()
    # (b) whole output: inside each group the copies are identical and equal the fp32 sum of its partials in device order
    for a in range(k0):
        acc = y2[a * k1].clone()
        for b in range(1, k1):
            acc += y2[a * k1 + b]
        for b in range(k1):
            assert torch.equal(y2b[a * k1 + b], acc), f"group {a} copy {b}"
    # (a) sampled rows of every device's local product through the oracle
    rows = tile_rows(Mg, 256, 3, 41)
    ridx = torch.from_numpy(rows).cuda()
    for a in range(k0):
        Xr = orc.bf16_to_f64(x1_h[a][rows])
        total = np.zeros((len(rows), D))
        for b in range(k1):
            ref1 = orc.matmul(Xr, orc.bf16_to_f64(w1_h[b]))
            got1 = orc.bf16_to_f64(host_u16(y1[a * k1 + b][ridx]))
            assert_matmul_close(got1, orc.bf16_to_f64(orc.bf16_round(ref1)), 2e-2, f"row 1, device ({a},{b})")
            ref2 = orc.matmul(orc.bf16_to_f64(x2_h[a][b][rows]), orc.bf16_to_f64(w2_h[b]))
            assert_matmul_close(y2[a * k1 + b][ridx].cpu().numpy(), ref2, 2e-2, f"row 2 partial, device ({a},{b})")
            total += ref2
        assert_matmul_close(y2b[a * k1][ridx].cpu().numpy(), total, 2e-2, f"row 2 after the inner all-reduce, group {a}")
