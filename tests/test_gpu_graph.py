"""The path under HIP graph capture: every entry point only enqueues kernels on the caller's stream (no
allocation, no synchronisation, no memset node), so a caller may record a whole step once and replay it.
A small MLP block (Table 1 rows 2 and 3 + the all-reduce of Table 2) and a classifier-style logits GEMM with
the fused row maximum (Sec. 6.3.1) are captured into one graph and replayed several times on new inputs,
with eager work and synchronisations between the replays; every replay must equal, bit for bit, what the
same calls give eagerly on the same inputs, and the first one is checked against the oracle as well."""
import numpy as np
import pytest

import oracle as orc
import paper_2110_15032_amd as sbp
import workloads as wl
from sbp_harness import DevTensor, assert_matmul_close, assert_psum_close, sync, upload, values

pytestmark = pytest.mark.gpu
SEED = wl.SEED_BASE + 77


def bf16(tid, shape, std=1.0):
    return wl.to_bf16_bits(wl.normal(SEED, tid, shape, std))


def test_step_replays_from_a_hip_graph_equal_eager_calls():
    import torch
    k, M, D, F = 2, 512, 256, 1024          # local W1 [256, 512], local W2 [512, 256]: the persistent kernels
    C = 768                                  # classes of the logits GEMM, 384 per device

    def inputs(r):
        X, W1, W2, Wc = bf16(10 * r + 1, (M, D)), bf16(10 * r + 2, (D, F), 0.05), bf16(10 * r + 3, (F, D), 0.05), bf16(10 * r + 4, (D, C), 0.05)
        return X, W1, W2, Wc

    X0, W10, W20, Wc0 = inputs(0)
    dX = DevTensor.from_host(orc.scatter(X0, orc.B, k), M, D, orc.B)
    dW1 = DevTensor.from_host(orc.scatter(W10, orc.S1, k), D, F, orc.S1)
    dW2 = DevTensor.from_host(orc.scatter(W20, orc.S0, k), F, D, orc.S0)
    dWc = DevTensor.from_host(orc.scatter(Wc0, orc.S1, k), D, C, orc.S1)

    def outputs():
        return (DevTensor.empty(M, F, np.uint16, orc.S1, k), DevTensor.empty(M, D, np.float32, orc.P_SUM, k),
                DevTensor.empty(M, D, np.float32, orc.B, k), DevTensor.empty(M, C, np.uint16, orc.S1, k),
                DevTensor.empty(M, 1, np.float32, orc.P_MAX, k), DevTensor.empty(M, 1, np.float32, orc.B, k))

    def step(o, stream=None):
        H, Y, Yb, L, MP, MB = o
        sbp.sbp_matmul_ex(dX.desc, sbp.B, dW1.desc, sbp.S(1), H.desc, sbp.S(1), k, stream, sbp.EPI_GELU)
        sbp.sbp_matmul(H.desc, sbp.S(1), dW2.desc, sbp.S(0), Y.desc, sbp.P_SUM, k, stream)
        sbp.sbp_boxing(Y.desc, sbp.P_SUM, Yb.desc, sbp.B, k, stream)
        sbp.sbp_matmul_rowmax(dX.desc, sbp.B, dWc.desc, sbp.S(1), L.desc, sbp.S(1), MP.desc, k, stream)
        sbp.sbp_boxing(MP.desc, sbp.P_MAX, MB.desc, sbp.B, k, stream)

    def load(r):
        X, W1, W2, Wc = inputs(r)
        for d, full, sig in ((dX, X, orc.B), (dW1, W1, orc.S1), (dW2, W2, orc.S0), (dWc, Wc, orc.S1)):
            for t, h in zip(d.dev, orc.scatter(full, sig, k)):
                t.copy_(upload(h))
        return X, W1, W2, Wc

    eager, graphed = outputs(), outputs()
    step(eager)                                # warm-up outside the capture (first-use queries of the library)
    sync()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(graphed)                          # binding default: torch's current stream = the capturing stream
    sync()

    for r in range(4):
        X, W1, W2, Wc = load(r)
        for o in graphed:                      # poison what the replay must rewrite
            for t in o.dev:
                t.fill_(float("nan") if t.dtype == torch.float32 else 0x7FC1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        step(eager)                            # the program's own eager work between replays
        sync()
        for name, a, b in zip(("H", "Y", "Yb", "L", "Pmax", "max"), graphed, eager):
            for i, (x, y) in enumerate(zip(a.host(), b.host())):
                assert np.array_equal(x.view(np.uint8), y.view(np.uint8)), f"replay {r}: {name} shard {i} differs from the eager call"
        if r == 0:
            Hs, _ = orc.matmul_sbp([values(x) for x in orc.scatter(X, orc.B, k)], orc.B, [values(w) for w in orc.scatter(W1, orc.S1, k)], orc.S1)
            for i, h in enumerate(graphed[0].host()):
                assert_matmul_close(values(h), orc.gelu(Hs[i]), 2e-2, f"graph replay: H shard {i}")
            Hq = [values(h) for h in graphed[0].host()]
            Ys, sy = orc.matmul_sbp(Hq, orc.S1, [values(w) for w in orc.scatter(W2, orc.S0, k)], orc.S0)
            assert sy == orc.P_SUM
            parts = graphed[1].host()
            for i in range(k):
                assert_matmul_close(parts[i], Ys[i], 2e-2, f"graph replay: partial {i}")
            ref = orc.boxing([p.astype(np.float64) for p in parts], orc.P_SUM, orc.B, k)
            for i, y in enumerate(graphed[2].host()):
                assert_psum_close(y, parts, ref[i], f"graph replay: all-reduce copy {i}")
            logits = graphed[3].host()
            rowmax = np.max(np.concatenate([values(l) for l in logits], axis=1), axis=1)
            for i, m in enumerate(graphed[5].host()):
                assert np.array_equal(m.reshape(-1).astype(np.float64), rowmax), f"graph replay: row maximum copy {i}"
