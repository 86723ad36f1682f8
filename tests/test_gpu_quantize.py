"""GPU parity of biq_quantize (greedy binary-coding quantisation, Eq. 1) against the CPU oracle.
Scales within fp32 rounding; signs bit for bit wherever the oracle's residual is farther from zero
than fp32 rounding can move it (closer than that both signs are valid greedy choices, and the
element's later planes follow from that choice); bit-exact everywhere on inputs whose arithmetic
is exact.

The rounding bound.  u = 2^-24.  The kernel sums |r| over a row in fp32 along a fixed tree: per
lane over at most ceil(n / 64) elements, 6 butterfly steps, at most 3 more additions over the
waves of a long row; with the division by n that is at most d + 1 roundings on any path,
d = ceil(n / 64) + 9, so alpha_i carries a relative error of at most (d + 1) u on top of what the
residuals it is computed from already carry.  With e_i a bound on |r_gpu - r_ref| in plane i
(elements whose earlier signs agree): e_1 = 0 (the first residual is w itself) and
    |alpha_gpu_i - alpha_ref_i| <= e_i + (d + 1) u alpha_i
    e_(i+1) <= e_i + |alpha_gpu_i - alpha_ref_i| + u max|r| <= 2 e_i + (d + 1) u alpha_i + u max|w|.
A factor 1.1 covers the second-order terms.  For n = 4096 this is e_2 = 5e-6 alpha_1, e_3 = 1.2e-5
alpha_1: a sign may differ only where the oracle's residual is that close to zero."""
import sys

import numpy as np
import pytest

from gpu_util import assert_within_tolerance, gpu_gemm

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


def _gpu_quantize(biq, W, q):
    import torch

    m, n = W.shape
    Wd = torch.from_numpy(W).cuda()
    K = torch.full((biq.biq_packed_bytes(m, n, q),), 0xA5, dtype=torch.uint8, device="cuda")  # poison
    alpha = torch.full((q, m), float("nan"), dtype=torch.float32, device="cuda")
    biq.biq_quantize(Wd, K, alpha, m, n, q)
    torch.cuda.synchronize()
    return K, alpha


U = 2.0 ** -24


def _rounding_bounds(W, alpha_ref):
    """(e [q][m], dalpha [q][m]): the bounds derived in the module docstring, per plane and row."""
    m, n = W.shape
    q = alpha_ref.shape[0]
    d = -(-n // 64) + 9
    wmax = np.abs(W.astype(np.float64)).max(axis=1)
    e = np.zeros((q, m))
    dalpha = np.zeros((q, m))
    for i in range(q):
        dalpha[i] = 1.1 * (e[i] + (d + 1) * U * alpha_ref[i])
        if i + 1 < q:
            e[i + 1] = 1.1 * (2 * e[i] + (d + 1) * U * alpha_ref[i] + U * wmax)
    return e, dalpha


def _check_against_oracle(W, q, B_gpu, alpha_gpu, B_ref, alpha_ref, R):
    e, dalpha = _rounding_bounds(W, alpha_ref)
    assert np.all(np.abs(alpha_gpu - alpha_ref) <= dalpha + 1e-300), np.abs(alpha_gpu - alpha_ref).max()
    assert np.array_equal(B_gpu[0], B_ref[0]), "the first plane is sign(w): no rounding is involved"
    unsure = np.abs(R) <= e[:, :, None]
    tainted = np.logical_or.accumulate(unsure, axis=0)
    differs = (B_gpu != B_ref) & ~tainted
    assert not differs.any(), "%d sign(s) differ where the residual is not within rounding of zero" % differs.sum()
    # the residual's density near zero is below 1 / alpha_1 and the window is about 1e-5 alpha_1 wide:
    # a few elements per 100000 can be undecided, not more
    assert tainted.sum() <= 4 + 1e-4 * tainted.size, tainted.mean()


def _signs_from_bitmap(Kh, q, m, n):
    """+1/-1 int8 [q][m][n] from packed rows (bit j of a row <-> element j), plus the padding bits."""
    rows = Kh.reshape(q, m, -1)
    bits = np.unpackbits(rows, axis=2, bitorder="little")
    return (bits[:, :, :n].astype(np.int8) * 2 - 1), bits[:, :, n:]


SHAPES = [(1, 1, 1), (3, 7, 2), (37, 100, 3), (64, 128, 1), (130, 1000, 3), (20, 4100, 4), (257, 2056, 2),
          (5, 32768, 2), (700, 513, 3), (6, 8192, 2), (6, 8200, 2), (3, 449, 1), (3, 16384, 2), (2, 20001, 3)]


@pytest.mark.parametrize("m,n,q", SHAPES)
def test_quantize_parity(biq, oracle, m, n, q):
    _say("quantize m=%d n=%d q=%d" % (m, n, q))
    rng = np.random.default_rng(8100 + m + n + q)
    W = (rng.standard_normal((m, n)) * rng.uniform(0.05, 2.0, size=(m, 1))).astype(np.float32)
    B_ref, alpha_ref, R = oracle.quantize_greedy(W, q, with_residuals=True)
    K, alpha = _gpu_quantize(biq, W, q)
    B_gpu, padding = _signs_from_bitmap(K.cpu().numpy(), q, m, n)
    alpha_gpu = alpha.cpu().numpy().astype(np.float64)
    assert not padding.any(), "padding bits of the packed rows must be 0"
    # scales and signs to the rounding bound derived at the top of this file
    _check_against_oracle(W, q, B_gpu, alpha_gpu, B_ref, alpha_ref, R)
    # validity of the whole code: reconstruction error per row equals the oracle's
    W64 = W.astype(np.float64)
    err_gpu = ((W64 - np.einsum("im,imn->mn", alpha_gpu, B_gpu.astype(np.float64))) ** 2).sum(axis=1)
    err_ref = ((W64 - np.einsum("im,imn->mn", alpha_ref, B_ref.astype(np.float64))) ** 2).sum(axis=1)
    np.testing.assert_allclose(err_gpu, err_ref, rtol=1e-3, atol=1e-12)


def test_quantize_bit_exact_on_exact_inputs(biq, oracle):
    """Integer weights and n a power of two: every sum, mean and residual is exact in fp32, so
    signs (including sign(0) = +1) and scales must equal the oracle's bit for bit."""
    rng = np.random.default_rng(8200)
    for (m, n, q) in [(50, 64, 3), (9, 1024, 2), (300, 256, 3)]:
        _say("quantize exact m=%d n=%d q=%d" % (m, n, q))
        W = rng.integers(-8, 9, size=(m, n)).astype(np.float32)
        W[0, :] = 0.0          # a row of zeros: alpha = 0, all signs +1
        W[1, :] = 3.0          # constant row: exactly representable with one plane
        W[2, ::3] = -0.0       # negative zeros (a pruned weight computed as negative * 0): sign +1, r = -alpha
        W[3, :] = -0.0
        assert np.signbit(W[3]).all()
        B_ref, alpha_ref = oracle.quantize_greedy(W, q)
        K, alpha = _gpu_quantize(biq, W, q)
        B_gpu, padding = _signs_from_bitmap(K.cpu().numpy(), q, m, n)
        assert not padding.any()
        assert np.array_equal(B_gpu, B_ref)
        assert np.array_equal(alpha.cpu().numpy().astype(np.float64), alpha_ref)
        assert np.array_equal(K.cpu().numpy().reshape(q, m, -1), oracle.pack_bitmap(B_ref))


def test_quantized_layer_feeds_gemm(biq, oracle):
    """W -> biq_quantize -> biq_gemm: equals Eq. 2 on the code the quantiser produced (oracle, fp64),
    and approaches the unquantised product as q grows."""
    import torch

    rng = np.random.default_rng(8300)
    m, n, b = 384, 1536, 3
    W = rng.standard_normal((m, n)).astype(np.float32) * 0.05
    X = rng.standard_normal((b, n)).astype(np.float32)
    Xd = torch.from_numpy(X).cuda()
    exact = X.astype(np.float64) @ W.astype(np.float64).T
    prev = np.inf
    for q in (1, 2, 3, 4):
        _say("quantize + gemm q=%d" % q)
        K, alpha = _gpu_quantize(biq, W, q)
        B_gpu, _ = _signs_from_bitmap(K.cpu().numpy(), q, m, n)
        alpha_h = alpha.cpu().numpy()
        Y = gpu_gemm(biq, K, alpha, Xd, m, n, q, 8).cpu().numpy()
        assert_within_tolerance(Y, oracle.gemm_dense(B_gpu, alpha_h, X), alpha_h, X, "quantized q=%d" % q)
        rel = np.linalg.norm(Y - exact) / np.linalg.norm(exact)
        assert rel < prev
        prev = rel
    assert prev < 0.2   # 4 planes of a Gaussian row: a few per cent of relative error per weight


def test_quantize_is_deterministic_and_checks_arguments(biq):
    import torch

    W = torch.randn((64, 2000), device="cuda")
    K1 = torch.empty(biq.biq_packed_bytes(64, 2000, 3), dtype=torch.uint8, device="cuda")
    K2 = torch.empty_like(K1)
    a1 = torch.empty((3, 64), device="cuda")
    a2 = torch.empty_like(a1)
    biq.biq_quantize(W, K1, a1, 64, 2000, 3)
    biq.biq_quantize(W, K2, a2, 64, 2000, 3)
    torch.cuda.synchronize()
    assert torch.equal(K1, K2) and torch.equal(a1, a2)
    with pytest.raises(biq.BiqError) as e:
        biq.biq_quantize(W, K1, a1, 1, 32769, 1)      # row longer than the LDS residual buffer
    assert e.value.status == biq.BIQ_EUNSUPPORTED
    with pytest.raises(biq.BiqError):
        biq.biq_quantize(W, K1, a1, 64, 2000, 0)


def test_quantize_full_size_sampled_rows(biq, oracle):
    """The launch bench.py times (16384 x 4096, q = 2, wave-per-row kernel): the oracle quantises
    a sample of rows; rows are independent, so those rows of the GPU result must match."""
    import torch

    m, n, q = 16384, 4096, 2
    _say("quantize full size m=%d n=%d q=%d" % (m, n, q))
    gen = torch.Generator(device="cuda")
    gen.manual_seed(8400)
    Wd = torch.randn((m, n), device="cuda", generator=gen)
    K = torch.full((biq.biq_packed_bytes(m, n, q),), 0xA5, dtype=torch.uint8, device="cuda")
    alpha = torch.empty((q, m), dtype=torch.float32, device="cuda")
    biq.biq_quantize(Wd, K, alpha, m, n, q)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 1, m - 1], np.random.default_rng(8400).integers(0, m, size=60)]))
    W = Wd[torch.from_numpy(rows).cuda()].cpu().numpy()
    B_ref, alpha_ref, R = oracle.quantize_greedy(W, q, with_residuals=True)
    Kh = K.cpu().numpy().reshape(q, m, -1)[:, rows, :]
    B_gpu, padding = _signs_from_bitmap(np.ascontiguousarray(Kh), q, len(rows), n)
    assert not padding.any()
    _check_against_oracle(W, q, B_gpu, alpha.cpu().numpy()[:, rows].astype(np.float64), B_ref, alpha_ref, R)
