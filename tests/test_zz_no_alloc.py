"""The allocation-free entry point biq_gemm_noalloc (workspace = a fixed buffer inside the
library) against biq_gemm (workspace passed by the caller): same kernels, so the results must be
the same bits, on calls in a row that reuse the buffer, the later ones with smaller inputs."""
import sys

import numpy as np
import pytest

from gpu_util import assert_within_tolerance, device_inputs, gpu_gemm, gpu_pack

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def biq():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2005_09904_amd as biq

    biq.load_library()
    return biq


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _inputs(m, n, q, b, seed):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((b, n), dtype=np.float32)
    B = (rng.integers(0, 2, size=(q, m, n), dtype=np.int8) * 2 - 1).astype(np.int8)
    alpha = rng.uniform(0.05, 1.0, size=(q, m)).astype(np.float32)
    return B, alpha, X


def test_noalloc_matches_gemm_on_consecutive_calls(biq, oracle):
    import torch

    limit = biq.biq_noalloc_scratch_bytes()
    assert limit == 32 << 20
    biq.biq_init()
    # shapes whose default plans use the workspace: matrix cores with split input and partial sums
    # (7 MiB), then smaller ones: the same path with less of it (4 MiB), batched table kernels with a
    # chunk split, a GEMV whose chunks are split over workgroups, and one that needs no workspace
    shapes = [(4096, 2048, 2, 96), (4096, 4096, 3, 32), (1024, 2048, 2, 128), (1024, 16384, 2, 1),
              (600, 3000, 3, 6), (512, 512, 1, 1)]
    used = []
    for i, (m, n, q, b) in enumerate(shapes):
        need = biq.biq_workspace_bytes(m, n, q, b, 8)
        used.append(need)
        _say("noalloc call %d: m=%d n=%d q=%d b=%d workspace=%d" % (i, m, n, q, b, need))
        assert need <= limit
        B, alpha, X = _inputs(m, n, q, b, 12000 + i)
        Bd, ad, Xd = device_inputs(B, alpha, X)
        K = gpu_pack(biq, Bd)
        want = gpu_gemm(biq, K, ad, Xd, m, n, q, 8)
        Y = torch.full((b, m), float("nan"), dtype=torch.float32, device="cuda")
        free_before = torch.cuda.mem_get_info()[0]
        biq.biq_gemm_noalloc(K, ad, Xd, Y, m, n, q, b, 8)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free_before, "device memory in use changed during the call"
        assert torch.equal(Y, want), "call %d differs from biq_gemm" % i
        assert_within_tolerance(Y.cpu().numpy(), oracle.gemm_dense(B, alpha, X), alpha, X, "noalloc call %d" % i)
    assert used[0] > used[1] > used[2] > used[3] > 0, used   # the buffer was really reused by smaller calls


def test_noalloc_rejects_what_does_not_fit(biq):
    import torch

    m, n, q, b = 16384, 16384, 2, 512
    assert biq.biq_workspace_bytes(m, n, q, b, 8) > biq.biq_noalloc_scratch_bytes()
    dummy = torch.zeros(64, dtype=torch.float32, device="cuda")   # never touched: the call fails its checks
    with pytest.raises(biq.BiqError) as e:
        biq.biq_gemm_noalloc(dummy, dummy, dummy, dummy, m, n, q, b, 8)
    assert e.value.status == biq.BIQ_EWORKSPACE
    with pytest.raises(biq.BiqError) as e:
        biq.biq_gemm_noalloc(dummy, dummy, dummy, dummy, 16, 16, 0, 1, 8)
    assert e.value.status == biq.BIQ_EINVAL
