"""sbp_probe_mfma_static: the probe for callers that cannot allocate (staging memory in a static device array of
the library) against sbp_probe_mfma (staging memory in the caller's workspace).

Both run the same kernels; what they leave behind, apart from cycle counts, is one float per thread: the sum of
the thread's accumulators, a pure function of (mode, iters, zero_operands).  The two entry points must agree on
it bit for bit, on two calls in a row (the second with fewer rounds: the array keeps the first call's contents),
in mode 6, the one that stages operands through the array, and in a mode that does not touch it."""
import numpy as np
import pytest

import paper_2110_15032_amd as sbp

pytestmark = pytest.mark.gpu


def _sums(torch, buf, cus):
    torch.cuda.synchronize()
    return buf[64:64 + cus * 512 * 4].cpu().numpy().view(np.uint32).copy()


def test_static_probe_matches_workspace_probe():
    import torch
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert cus * 512 * 4 + 64 <= 1 << 20
    work = torch.zeros(16 << 20, dtype=torch.uint8, device="cuda")     # sbp_probe_mfma: 1 MiB of results + 15 MiB of staging
    out = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")       # sbp_probe_mfma_static: results only
    for mode, iters in ((6, 300), (6, 100), (4, 50)):                  # the second call is the smaller one
        print(f"probe mode {mode} iters {iters}", flush=True)
        work[:1 << 20].fill_(0xAB)
        out.fill_(0xCD)
        sbp.sbp_probe_mfma(mode, iters, 0, work)
        want = _sums(torch, work, cus)
        sbp.sbp_probe_mfma_static(mode, iters, 0, out)
        got = _sums(torch, out, cus)
        assert np.array_equal(got, want), (mode, iters, int((got != want).sum()))
        assert len(np.unique(got)) > 1                                  # not a buffer that nobody wrote
        # the words behind the results stay as they were
        assert bool((out[64 + cus * 512 * 4:] == 0xCD).all())
        cyc = out[:64].cpu().numpy().view(np.uint64)
        assert (cyc > 0).all() and (cyc < (1 << 40)).all()


def test_static_probe_refuses_what_the_array_cannot_hold():
    import torch
    out = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    for mode in (7, 8, -1, 9):
        with pytest.raises(sbp.SbpError) as e:
            sbp.sbp_probe_mfma_static(mode, 10, 0, out)
        assert "without a kernel" in str(e.value)
    with pytest.raises(sbp.SbpError):
        sbp.sbp_probe_mfma_static(6, 0, 0, out)
    with pytest.raises(sbp.SbpError):
        sbp.sbp_probe_mfma_static(6, 10, 0, out.data_ptr() + 4)
    torch.cuda.synchronize()
