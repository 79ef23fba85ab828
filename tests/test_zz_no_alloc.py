"""dlcx_average_static, the entry point for callers that cannot allocate: its output must be
bitwise that of dlcx_average (same kernels, scratch in the library's fixed device array instead of
a caller's workspace), on two calls in a row, the second on a smaller input (the array keeps the
first call's contents), and the allocator must not be touched while it runs."""
import numpy as np
import pytest
import torch

import paper_2506_21263_amd as dlcx
from gpu_util import DEV, payload_buffers, to_np, ws_for

pytestmark = pytest.mark.gpu


def _payloads(d, K, seed):
    """K quantised P factors of a well-conditioned random m x r matrix (library quantiser)."""
    rng = np.random.default_rng(seed)
    codes, scales = payload_buffers(d, dlcx.PHASE_P, K)
    base = rng.standard_normal((d.r, d.m))
    for k in range(K):
        f = (base + 0.1 * rng.standard_normal((d.r, d.m))).astype(np.float32)
        dlcx.dlcx_quantize(torch.from_numpy(f).to(DEV), d.qbits, d.group, codes[k], scales[k])
    return codes, scales


def _both(d, K, seed):
    codes, scales = _payloads(d, K, seed)
    want = torch.empty(d.r, d.m, device=DEV)
    got = torch.full((d.r, d.m), float("nan"), device=DEV)
    ws = ws_for(d, K)
    dlcx.dlcx_average(d, dlcx.PHASE_P, codes, scales, want, ws)
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    dlcx.dlcx_average_static(d, dlcx.PHASE_P, codes, scales, got)
    after = torch.cuda.memory_stats()["allocation.all.allocated"]
    torch.cuda.synchronize()
    assert after == before
    return to_np(got), to_np(want)


def test_static_scratch_average_matches_workspace_average_twice():
    big = dlcx.desc(4096, 512, 96, 4, 128, dlcx.MMA_BF16)     # 8 Gram chunks, r x r in LDS
    small = dlcx.desc(640, 256, 24, 8, 64, dlcx.MMA_BF16)     # 2 chunks, ragged second chunk
    for d, K, seed in ((big, 4, 1), (small, 3, 2)):
        got, want = _both(d, K, seed)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (d.m, d.r)
        gram = want.astype(np.float64) @ want.astype(np.float64).T
        assert np.abs(gram - np.eye(d.r)).max() < 1e-5
    # phase Q needs no scratch: plain mean, same bits
    d = small
    codes, scales = payload_buffers(d, dlcx.PHASE_Q, 2)
    for k in range(2):
        x = torch.randn(d.r, d.n, device=DEV)
        dlcx.dlcx_quantize(x, d.qbits, d.group, codes[k], scales[k])
    a, b = torch.empty(d.r, d.n, device=DEV), torch.empty(d.r, d.n, device=DEV)
    dlcx.dlcx_average(d, dlcx.PHASE_Q, codes, scales, a, ws_for(d, 2))
    dlcx.dlcx_average_static(d, dlcx.PHASE_Q, codes, scales, b)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_static_scratch_rejects_what_does_not_fit():
    d = dlcx.desc(65536, 256, 256, 4, 128, dlcx.MMA_BF16)
    assert dlcx.dlcx_static_scratch_need(d, dlcx.PHASE_P) > dlcx.dlcx_static_scratch_bytes()
    codes, scales = payload_buffers(d, dlcx.PHASE_P, 1)
    out = torch.empty(d.r, d.m, device=DEV)
    with pytest.raises(dlcx.DlcxError) as e:
        dlcx.dlcx_average_static(d, dlcx.PHASE_P, codes, scales, out)
    assert e.value.code == dlcx.ETOOBIG
