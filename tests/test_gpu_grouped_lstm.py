"""GPU parity of the grouped launch (several small multiplies in one dispatch) and of the fused
LSTM cell step, through the C ABI, against the CPU oracle."""
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


def _rand_inputs(m, n, q, b, seed, alpha_hi=1.0):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((b, n), dtype=np.float32)
    B = (rng.integers(0, 2, size=(q, m, n), dtype=np.int8) * 2 - 1).astype(np.int8)
    alpha = rng.uniform(0.05 * alpha_hi, alpha_hi, size=(q, m)).astype(np.float32)
    return B, alpha, X


def _group(biq, shapes, seed):
    import torch

    host, dev = [], []
    for i, (m, n, q, b) in enumerate(shapes):
        B, alpha, X = _rand_inputs(m, n, q, b, seed + i)
        Bd, ad, Xd = device_inputs(B, alpha, X)
        K = gpu_pack(biq, Bd)
        Y = torch.full((b, m), float("nan"), dtype=torch.float32, device="cuda")
        host.append((B, alpha, X))
        dev.append((K, ad, Xd, Y, m, n, q, b))
    return host, dev


def _same_family_plan(biq, m, n, q, b):
    """The single-call plan of the kernel family and row mode the grouped launch uses for this shape."""
    C = -(-n // 8)
    plan = biq.BiqPlan()
    plan.threads, plan.tiles_per_split, plan.row_mode, plan.rows_per_wg = 1024, 1, 1, 8
    if b == 1 and C <= 128:
        plan.kernel, plan.chunks_per_tile, plan.batch_tile = 1, 128, 1
    elif b == 1:
        plan.kernel, plan.chunks_per_tile, plan.batch_tile = 4, 256, 1
    else:
        plan.kernel, plan.chunks_per_tile, plan.batch_tile = 5, 128, 2
    return plan


GROUPS = [
    # eight equal fully connected layers (cfg 1's shape): one dispatch
    [(512, 512, 1, 1)] * 8,
    # eight LSTM-cell-shaped layers (cfg 3's shape, smaller m to keep the oracle quick)
    [(1024, 1024, 3, 8)] * 8,
    # the projections of a Transformer block: equal shapes, wider rows (half-table GEMV kernel)
    [(2048, 2048, 2, 1)] * 4,
    # mixed families, plane counts, ragged sizes: several dispatches
    [(37, 100, 2, 1), (300, 1000, 2, 1), (64, 1300, 2, 1), (129, 2048, 3, 1), (70, 513, 3, 9), (45, 800, 3, 2),
     (5, 7, 1, 1), (1, 1, 4, 3)],
    # more problems than fit one dispatch
    [(40 + 3 * i, 256 + 8 * i, 1, 1) for i in range(21)],
]


@pytest.mark.parametrize("gi", range(len(GROUPS)))
def test_grouped_launch_matches_oracle_and_single_calls(biq, oracle, gi):
    import torch

    shapes = GROUPS[gi]
    _say("grouped launch %d: %d problems, first %s" % (gi, len(shapes), shapes[0]))
    host, dev = _group(biq, shapes, 21000 + 100 * gi)
    biq.biq_gemm_grouped(dev, 8)
    torch.cuda.synchronize()
    for (B, alpha, X), (K, ad, Xd, Y, m, n, q, b) in zip(host, dev):
        assert_within_tolerance(Y.cpu().numpy(), oracle.gemm_dense(B, alpha, X), alpha, X, "grouped %s" % ((m, n, q, b),))
        # the same kernel family run on the problem alone: same arithmetic per row, same bits
        single = gpu_gemm(biq, K, ad, Xd, m, n, q, 8, plan=_same_family_plan(biq, m, n, q, b))
        assert torch.equal(single, Y), (m, n, q, b)


def test_grouped_launch_refuses_what_needs_a_second_kernel(biq):
    import torch

    _, dev = _group(biq, [(64, 512, 1, 1), (64, 4096, 1, 1)], 22000)     # the second one is wider than a tile
    with pytest.raises(biq.BiqError) as e:
        biq.biq_gemm_grouped(dev, 8)
    assert e.value.status == biq.BIQ_EUNSUPPORTED
    torch.cuda.synchronize()
    assert torch.isnan(dev[0][3]).all() and torch.isnan(dev[1][3]).all(), "nothing may have been launched"
    with pytest.raises(biq.BiqError) as e:
        biq.biq_gemm_grouped(dev[:1], 4)                                  # mu other than 8
    assert e.value.status == biq.BIQ_EUNSUPPORTED
    with pytest.raises(biq.BiqError) as e:
        biq.biq_gemm_grouped([], 8)
    assert e.value.status == biq.BIQ_EINVAL


LSTM_SHAPES = [
    # hidden, n, q, batch
    (1024, 1024, 3, 8),     # cfg 3: 4 gates x 1024 hidden, batch 8
    (256, 512, 2, 1),       # one input vector, rows of one full-table tile width
    (512, 2048, 3, 1),      # one input vector, widest rows served
    (37, 100, 2, 3),        # ragged everything, odd batch
    (1, 9, 1, 1),
    (300, 1000, 4, 5),
    (700, 333, 1, 2),
]


@pytest.mark.parametrize("H,n,q,b", LSTM_SHAPES)
def test_lstm_cell_parity(biq, oracle, H, n, q, b):
    """Tolerance.  z = W [x ; h] + bias is a sum of q * n / 8 table entries per row, added along a
    tree of depth < 64 (16 per lane, 3 or 4 butterfly steps, the planes, the bias), each entry itself
    4 roundings deep: |dz| <= 64 u * sum_i |alpha_i| * ||x||_1, u = 2^-24.  The cell update has
    slopes |dc'/dz| <= 1 + |c| / 4 and |dh'/dz| <= 1.25 + |c| / 4 (sigma' <= 1/4, tanh' <= 1), and
    expf / tanhf add a few units in the last place of values below 1 + |c|."""
    import torch

    _say("lstm cell H=%d n=%d q=%d b=%d" % (H, n, q, b))
    rng = np.random.default_rng(23000 + H + n)
    B = (rng.integers(0, 2, size=(q, 4 * H, n), dtype=np.int8) * 2 - 1).astype(np.int8)
    alpha = rng.uniform(0.01, 0.08, size=(q, 4 * H)).astype(np.float32)
    bias = rng.uniform(-0.5, 0.5, size=4 * H).astype(np.float32)
    X = rng.standard_normal((b, n)).astype(np.float32)
    C = rng.standard_normal((b, H)).astype(np.float32)
    Bd, ad, Xd = device_inputs(B, alpha, X)
    K = gpu_pack(biq, Bd)
    h = torch.full((b, H), float("nan"), dtype=torch.float32, device="cuda")
    c = torch.full((b, H), float("nan"), dtype=torch.float32, device="cuda")
    biq.biq_lstm_cell(K, ad, torch.from_numpy(bias).cuda(), Xd, torch.from_numpy(C).cuda(), h, c, H, n, q, b, 8)
    torch.cuda.synchronize()
    h_ref, c_ref = oracle.lstm_cell(B, alpha, bias, X, C)
    dz = 64 * 2.0 ** -24 * np.abs(alpha).sum(axis=0).max() * np.abs(X.astype(np.float64)).sum(axis=1)[:, None]
    tol = (1.25 + np.abs(C) / 4) * dz + 8 * 2.0 ** -24 * (1 + np.abs(C))
    assert np.all(np.abs(c.cpu().numpy() - c_ref) <= tol), np.abs(c.cpu().numpy() - c_ref).max()
    assert np.all(np.abs(h.cpu().numpy() - h_ref) <= tol), np.abs(h.cpu().numpy() - h_ref).max()


def test_lstm_cell_closed_form_and_unfused_path(biq, oracle):
    """alpha = 0, bias = 0: h = tanh(c / 2) / 2, c' = c / 2 to rounding.  And the fused step agrees
    with biq_gemm followed by the cell update on the host."""
    import torch

    H, n, q, b = 128, 640, 2, 4
    rng = np.random.default_rng(23900)
    B = (rng.integers(0, 2, size=(q, 4 * H, n), dtype=np.int8) * 2 - 1).astype(np.int8)
    alpha = rng.uniform(0.01, 0.08, size=(q, 4 * H)).astype(np.float32)
    bias = rng.uniform(-0.5, 0.5, size=4 * H).astype(np.float32)
    X = rng.standard_normal((b, n)).astype(np.float32)
    C = rng.standard_normal((b, H)).astype(np.float32)
    Bd, ad, Xd = device_inputs(B, alpha, X)
    K = gpu_pack(biq, Bd)
    Cd = torch.from_numpy(C).cuda()
    h = torch.empty((b, H), dtype=torch.float32, device="cuda")
    c = torch.empty((b, H), dtype=torch.float32, device="cuda")
    zero_a = torch.zeros_like(ad)
    zero_b = torch.zeros(4 * H, dtype=torch.float32, device="cuda")
    biq.biq_lstm_cell(K, zero_a, zero_b, Xd, Cd, h, c, H, n, q, b, 8)
    torch.cuda.synchronize()
    np.testing.assert_allclose(c.cpu().numpy(), C.astype(np.float64) / 2, rtol=0, atol=1e-7)
    np.testing.assert_allclose(h.cpu().numpy(), np.tanh(C.astype(np.float64) / 2) / 2, rtol=0, atol=2e-7)
    # unfused: Z from biq_gemm, cell update in fp64 on the host
    biq.biq_lstm_cell(K, ad, torch.from_numpy(bias).cuda(), Xd, Cd, h, c, H, n, q, b, 8)
    Z = gpu_gemm(biq, K, ad, Xd, 4 * H, n, q, 8).cpu().numpy().astype(np.float64) + bias
    sig = lambda z: 1 / (1 + np.exp(-z))
    c2 = sig(Z[:, H:2 * H]) * C + sig(Z[:, :H]) * np.tanh(Z[:, 2 * H:3 * H])
    h2 = sig(Z[:, 3 * H:]) * np.tanh(c2)
    np.testing.assert_allclose(c.cpu().numpy(), c2, rtol=0, atol=2e-5)
    np.testing.assert_allclose(h.cpu().numpy(), h2, rtol=0, atol=2e-5)


def test_lstm_cell_refuses_unsupported_shapes(biq):
    import torch

    d = torch.zeros(64, dtype=torch.float32, device="cuda")   # never touched: the calls fail their checks
    for (H, n, q, b, mu, status) in [(64, 4096, 2, 1, 8, biq.BIQ_EUNSUPPORTED), (64, 2048, 2, 2, 8, biq.BIQ_EUNSUPPORTED),
                                     (64, 512, 5, 1, 8, biq.BIQ_EUNSUPPORTED), (64, 512, 2, 1, 4, biq.BIQ_EUNSUPPORTED),
                                     (0, 512, 2, 1, 8, biq.BIQ_EINVAL)]:
        with pytest.raises(biq.BiqError) as e:
            biq.biq_lstm_cell(d, d, d, d, d, d, d, H, n, q, b, mu)
        assert e.value.status == status, (H, n, q, b, mu)
