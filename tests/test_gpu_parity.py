"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Keys and table indices bit-exact; fp32 outputs within the stated tolerance;
bit-exact on inputs whose partial sums are all exactly representable."""
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

    biq.load_library()  # raises if the HIP library is missing: there is no fallback
    return biq


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _rand_inputs(m, n, q, b, seed):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((b, n), dtype=np.float32)
    B = (rng.integers(0, 2, size=(q, m, n), dtype=np.int8) * 2 - 1).astype(np.int8)
    alpha = rng.uniform(0.05, 1.0, size=(q, m)).astype(np.float32)
    return B, alpha, X


RAGGED_SHAPES = [
    # m, n, q, batch
    (1, 1, 1, 1),
    (3, 7, 1, 1),
    (37, 100, 2, 1),
    (64, 128, 1, 2),
    (130, 1000, 3, 3),
    (257, 2056, 2, 1),
    (33, 4100, 1, 5),
    (500, 300, 2, 8),
    (70, 513, 3, 9),
    (45, 1300, 2, 33),
]


@pytest.mark.parametrize("m,n,q,b", RAGGED_SHAPES)
def test_pack_bit_exact(biq, oracle, m, n, q, b):
    _say("pack m=%d n=%d q=%d" % (m, n, q))
    B, _, _ = _rand_inputs(m, n, q, 1, 1000 + m + n)
    import torch

    K = gpu_pack(biq, torch.from_numpy(B).cuda())
    torch.cuda.synchronize()
    ref = oracle.pack_bitmap(B)
    assert np.array_equal(K.cpu().numpy().reshape(ref.shape), ref)


@pytest.mark.parametrize("mu", [1, 2, 3, 4, 5, 6, 7, 8, 9, 10])
def test_table_indices_bit_exact(biq, oracle, mu):
    import torch

    for (m, n, q) in [(5, 77, 2), (16, 1024, 1), (9, 4099, 1)]:
        _say("unpack_keys mu=%d m=%d n=%d q=%d" % (mu, m, n, q))
        B, _, _ = _rand_inputs(m, n, q, 1, 2000 + mu + n)
        K = gpu_pack(biq, torch.from_numpy(B).cuda(), mu)
        C = biq.biq_num_chunks(n, mu)
        ref = oracle.pack_keys(B, mu)
        keys16 = torch.full((q, m, C), 0x7EEE, dtype=torch.int16, device="cuda")   # uint16 storage
        biq.biq_unpack_keys16(K, keys16, m, n, q, mu)
        torch.cuda.synchronize()
        assert np.array_equal(keys16.cpu().numpy().view(np.uint16), ref)
        keys = torch.full((q, m, C), 0xEE, dtype=torch.uint8, device="cuda")
        if mu <= 8:
            biq.biq_unpack_keys(K, keys, m, n, q, mu)
            torch.cuda.synchronize()
            assert np.array_equal(keys.cpu().numpy().astype(np.uint16), ref)
        else:   # a key wider than a byte does not fit the 8-bit form
            with pytest.raises(biq.BiqError) as e:
                biq.biq_unpack_keys(K, keys, m, n, q, mu)
            assert e.value.status == biq.BIQ_EUNSUPPORTED


@pytest.mark.parametrize("mu", [1, 2, 3, 4, 5, 6, 7, 8, 9, 10])
def test_build_lut_parity_and_antisymmetry(biq, oracle, mu):
    import torch

    for (n, b) in [(1, 1), (50, 3), (1024, 1), (333, 8), (700, 12), (64, 4), (129, 6)]:
        _say("build_lut mu=%d n=%d b=%d" % (mu, n, b))
        X = np.random.default_rng(3000 + mu + n).standard_normal((b, n), dtype=np.float32)
        C = biq.biq_num_chunks(n, mu)
        E = 1 << mu
        assert biq.biq_lut_bytes(n, b, mu) == C * E * b * 4
        LUT = torch.full((C, E, b), float("nan"), dtype=torch.float32, device="cuda")
        biq.biq_build_lut(torch.from_numpy(X).cuda(), LUT, n, b, mu)
        torch.cuda.synchronize()
        got = LUT.cpu().numpy()
        ref = oracle.build_lut(X, mu)
        # fp32 pair sums and a chain over them: at most 4 roundings for mu <= 8, 5 for mu = 9, 10
        Xp = np.zeros((b, C * mu), dtype=np.float64)
        Xp[:, :n] = np.abs(X)
        l1 = Xp.reshape(b, C, mu).sum(axis=2).T  # [C][b]
        assert np.all(np.abs(got - ref) <= (5 if mu > 8 else 4) * 2.0 ** -24 * l1[:, None, :] + 1e-45)
        # LUT[~k] = -LUT[k] exactly (Algorithm 1 builds the upper half by negation)
        assert np.array_equal(got[:, ::-1, :], -got)


CONFIG_NAMES = ["cfg1_fc512_b1", "cfg2_gemv2048_q2_b1", "cfg3_lstm4096x1024_q3_b8"]


@pytest.mark.parametrize("name", CONFIG_NAMES)
def test_gemm_parity_full_configs(biq, oracle, name):
    from paper_2005_09904_amd.workloads import CONFIGS, make_inputs

    w = CONFIGS[name]
    _say("gemm %s" % name)
    B, alpha, X = make_inputs(w)
    Bd, ad, Xd = device_inputs(B, alpha, X)
    K = gpu_pack(biq, Bd, w.mu)
    assert np.array_equal(K.cpu().numpy().reshape(w.q, w.m, -1), oracle.pack_bitmap(B))
    Y = gpu_gemm(biq, K, ad, Xd, w.m, w.n, w.q, w.mu).cpu().numpy()
    ref = oracle.gemm_dense(B, alpha, X)
    assert_within_tolerance(Y, ref, alpha, X, name)
    # the method's own oracle (Algorithm 2) gives the same reference
    ref_lut = oracle.gemm_lut(oracle.pack_keys(B, w.mu), alpha, X, w.mu)
    assert_within_tolerance(Y, ref_lut, alpha, X, name + " vs lut oracle")


LARGE = [("cfg4_sq4096_q3_b32", [8]), ("cfg5_ffn_up_q2_b128", [4, 6, 8]), ("cfg5_ffn_down_q2_b128", [8])]


@pytest.mark.parametrize("name,mus", LARGE)
def test_gemm_parity_large_configs_every_element(biq, oracle, name, mus):
    """Full-size launches of the three large configurations, every element of Y and of K against
    the oracle (Eq. 2 with W reconstructed, all rows: seconds to tens of seconds on one core,
    computed once per configuration), for the library's default plan and for the lookup-table
    kernels, for every mu of the sweep, in the launch configuration bench.py times."""
    import torch
    from paper_2005_09904_amd.workloads import CONFIGS, make_inputs

    w = CONFIGS[name]
    B, alpha, X = make_inputs(w)
    Bd, ad, Xd = device_inputs(B, alpha, X)
    K = gpu_pack(biq, Bd, w.mu)
    del Bd
    _say("oracle gemm_dense %s, all %d rows" % (name, w.m))
    ref = oracle.gemm_dense(B, alpha, X)
    assert np.array_equal(K.cpu().numpy().reshape(w.q, w.m, -1), oracle.pack_bitmap(B))
    for mu in mus:
        default = biq.biq_plan_get(w.m, w.n, w.q, w.batch, mu)
        lut = biq.biq_plan_get_lut(w.m, w.n, w.q, w.batch, mu)
        for plan in ([None, lut] if default.kernel != lut.kernel else [None]):
            kname = biq.biq_kernel_name((plan or default).kernel)
            _say("gemm %s mu=%d %s (every element)" % (name, mu, kname))
            Y = gpu_gemm(biq, K, ad, Xd, w.m, w.n, w.q, mu, plan=plan).cpu().numpy()
            assert_within_tolerance(Y, ref, alpha, X, "%s mu=%d %s" % (name, mu, kname))
    torch.cuda.empty_cache()


@pytest.mark.parametrize("m,n,q,b", RAGGED_SHAPES)
@pytest.mark.parametrize("mu", [8, 4, 6, 1, 2, 3, 5, 7, 9, 10])
def test_gemm_parity_ragged_shapes(biq, oracle, m, n, q, b, mu):
    _say("gemm ragged m=%d n=%d q=%d b=%d mu=%d" % (m, n, q, b, mu))
    B, alpha, X = _rand_inputs(m, n, q, b, 4000 + m + n + mu)
    Bd, ad, Xd = device_inputs(B, alpha, X)
    K = gpu_pack(biq, Bd, mu)
    Y = gpu_gemm(biq, K, ad, Xd, m, n, q, mu).cpu().numpy()
    assert_within_tolerance(Y, oracle.gemm_dense(B, alpha, X), alpha, X, "ragged")


@pytest.mark.parametrize("mu", [8, 4, 6, 3, 9, 10])
def test_gemm_bit_exact_on_exact_inputs(biq, oracle, mu):
    """Small-integer x and power-of-two alpha: every fp32 partial sum is exact, so any table
    width, tiling and reduction order must reproduce the oracle bit for bit."""
    from paper_2005_09904_amd.workloads import Workload, make_exact_inputs

    for (m, n, q, b) in [(300, 2048, 2, 1), (129, 1000, 3, 4), (64, 4096, 1, 9)]:
        _say("gemm exact m=%d n=%d q=%d b=%d mu=%d" % (m, n, q, b, mu))
        w = Workload("exact", m, n, q, b, mu, "uniform", seed=500 + m)
        B, alpha, X = make_exact_inputs(w)
        Bd, ad, Xd = device_inputs(B, alpha, X)
        K = gpu_pack(biq, Bd, mu)
        Y = gpu_gemm(biq, K, ad, Xd, m, n, q, mu).cpu().numpy()
        ref = oracle.gemm_dense(B, alpha, X)
        assert np.array_equal(Y.astype(np.float64), ref)


def test_query_with_tables_from_memory_matches_fused(biq, oracle):
    import torch

    for (m, n, q, b, mu) in [(200, 1500, 2, 1, 8), (100, 700, 3, 6, 8), (90, 1000, 2, 3, 4), (50, 600, 1, 2, 6)]:
        _say("query m=%d n=%d q=%d b=%d mu=%d" % (m, n, q, b, mu))
        B, alpha, X = _rand_inputs(m, n, q, b, 6000 + m + mu)
        Bd, ad, Xd = device_inputs(B, alpha, X)
        K = gpu_pack(biq, Bd, mu)
        C = biq.biq_num_chunks(n, mu)
        LUT = torch.empty((C, 1 << mu, b), dtype=torch.float32, device="cuda")
        biq.biq_build_lut(Xd, LUT, n, b, mu)
        Y = torch.full((b, m), float("nan"), dtype=torch.float32, device="cuda")
        ws_bytes = biq.biq_workspace_bytes(m, n, q, b, mu)
        ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
        biq.biq_query(K, ad, LUT, Y, m, n, q, b, mu, workspace=ws)
        torch.cuda.synchronize()
        Yf = gpu_gemm(biq, K, ad, Xd, m, n, q, mu)
        assert torch.equal(Y, Yf)  # same tables, same order of sums
        assert_within_tolerance(Y.cpu().numpy(), oracle.gemm_dense(B, alpha, X), alpha, X, "query")


def _plan(biq, kernel, threads, ct, bt, tps, rows, row_mode=0):
    plan = biq.BiqPlan()
    plan.kernel, plan.threads, plan.chunks_per_tile, plan.batch_tile = kernel, threads, ct, bt
    plan.tiles_per_split, plan.rows_per_wg, plan.row_mode = tps, rows, row_mode
    return plan


def test_explicit_plans_give_the_same_result(biq, oracle):
    """Tile width, chunk splits, rows per workgroup and threads do not change the result
    beyond rounding (Algorithm 2's tiling is free)."""
    m, n, q, b, mu = 700, 3000, 2, 3, 8
    B, alpha, X = _rand_inputs(m, n, q, b, 7000)
    Bd, ad, Xd = device_inputs(B, alpha, X)
    K = gpu_pack(biq, Bd, mu)
    ref = oracle.gemm_dense(B, alpha, X)
    plans = [(0, 64, 16, 1, 1, 5), (0, 256, 32, 4, 3, 64), (0, 512, 64, 2, 100, 700),
             (0, 1024, 128, 1, 2, 33), (0, 128, 16, 8, 7, 1),
             # batched mu=8 kernel: 64-chunk tiles of 2 vectors
             (2, 1024, 64, 2, 1, 64), (2, 512, 64, 2, 2, 128), (2, 256, 64, 2, 6, 704), (2, 64, 64, 2, 3, 100),
             # half-table batched kernel: 128-chunk tiles of 2 vectors, 8 rows per wave step
             (5, 1024, 128, 2, 1, 64, 1), (5, 256, 128, 2, 1, 700, 1), (5, 64, 128, 2, 1, 9, 1),
             # ... in latency mode (one step of 16 rows per wave)
             (2, 1024, 64, 2, 1, 256, 1), (2, 256, 64, 2, 1, 700, 1), (2, 64, 64, 2, 1, 17, 1)]
    for spec in plans:
        _say("plan " + str(spec))
        Y = gpu_gemm(biq, K, ad, Xd, m, n, q, mu, plan=_plan(biq, *spec)).cpu().numpy()
        assert_within_tolerance(Y, ref, alpha, X, "plan")
    # GEMV kernel plans (batch 1)
    B, alpha, X = _rand_inputs(m, n, 3, 1, 7001)
    Bd, ad, Xd = device_inputs(B, alpha, X)
    K = gpu_pack(biq, Bd, mu)
    ref = oracle.gemm_dense(B, alpha, X)
    for spec in [(1, 1024, 128, 1, 1, 64), (1, 512, 128, 1, 3, 700), (1, 64, 128, 1, 2, 130),
                 (0, 256, 64, 1, 1, 50), (1, 1024, 128, 1, 1, 128, 1), (1, 128, 128, 1, 1, 700, 1),
                 (1, 64, 128, 1, 1, 9, 1),
                 # half-table kernel: 256-chunk tiles, 4 rows per wave step
                 (4, 1024, 256, 1, 1, 64, 1), (4, 256, 256, 1, 1, 700, 1), (4, 64, 256, 1, 1, 5, 1),
                 (4, 512, 256, 1, 1, 130, 1),
                 # ... one row per wave at a time
                 (4, 1024, 256, 1, 1, 8, 2), (4, 256, 256, 1, 1, 700, 2), (4, 64, 256, 1, 1, 5, 2),
                 (4, 1024, 256, 1, 1, 16, 2),
                 # ... walking both tiles of the row (row sums carried in LDS)
                 (4, 1024, 256, 1, 2, 64, 1), (4, 256, 256, 1, 2, 700, 1), (4, 64, 256, 1, 2, 5, 1),
                 (4, 1024, 256, 1, 2, 130, 1),
                 # throughput mode, several tiles per workgroup, ragged block counts per wave
                 (1, 1024, 128, 1, 3, 700, 0), (1, 1024, 128, 1, 3, 64, 0), (1, 1024, 128, 1, 2, 1000, 0),
                 (1, 256, 128, 1, 3, 333, 0), (1, 64, 128, 1, 3, 9, 0)]:
        _say("plan " + str(spec))
        Y = gpu_gemm(biq, K, ad, Xd, m, n, 3, mu, plan=_plan(biq, *spec)).cpu().numpy()
        assert_within_tolerance(Y, ref, alpha, X, "plan")
    # throughput mode for every plane count (4 planes: both register budgets), several tiles per
    # workgroup, inputs fetched a tile ahead (1024 threads, n a multiple of 4) and not (n = 5001)
    for q, n2 in ((1, 5000), (2, 5001), (4, 5000)):
        B, alpha, X = _rand_inputs(2000, n2, q, 1, 7002 + q)
        Bd, ad, Xd = device_inputs(B, alpha, X)
        K = gpu_pack(biq, Bd, mu)
        ref = oracle.gemm_dense(B, alpha, X)
        for spec in [(1, 1024, 128, 1, 5, 8, 0), (1, 512, 128, 1, 5, 72, 0), (1, 1024, 128, 1, 2, 520, 0),
                     (1, 1024, 128, 1, 5, 2000, 0),
                     # half tables: all three tiles in one workgroup; two of three, then one (partial sums)
                     (4, 1024, 256, 1, 3, 72, 1), (4, 1024, 256, 1, 2, 520, 1), (4, 512, 256, 1, 3, 2000, 1)]:
            for fill in ((0, 1) if spec[0] == 1 else (0,)):   # tables from pair sums / in the order of Algorithm 1
                _say("plan q=%d n=%d fill=%d " % (q, n2, fill) + str(spec))
                plan = _plan(biq, *spec)
                plan.table_fill = fill
                Y = gpu_gemm(biq, K, ad, Xd, 2000, n2, q, mu, plan=plan).cpu().numpy()
                assert_within_tolerance(Y, ref, alpha, X, "plan")
    # Algorithm 1's order on exactly representable inputs: bit for bit, like every other tiling
    from paper_2005_09904_amd.workloads import Workload, make_exact_inputs

    B, alpha, X = make_exact_inputs(Workload("exact", 600, 3000, 2, 1, 8, "uniform", seed=71))
    Bd, ad, Xd = device_inputs(B, alpha, X)
    plan = _plan(biq, 1, 1024, 128, 1, 3, 64, 0)
    plan.table_fill = 1
    Y = gpu_gemm(biq, gpu_pack(biq, Bd, mu), ad, Xd, 600, 3000, 2, mu, plan=plan).cpu().numpy()
    assert np.array_equal(Y.astype(np.float64), oracle.gemm_dense(B, alpha, X))


@pytest.mark.parametrize("q", [1, 2, 3, 4, 5])
def test_plane_counts(biq, oracle, q):
    """q = 1..4 run the specialised mu = 8 kernels, q = 5 the generic one."""
    for (m, n, b) in [(333, 1100, 1), (200, 900, 2), (150, 2100, 5)]:
        _say("planes q=%d m=%d n=%d b=%d" % (q, m, n, b))
        B, alpha, X = _rand_inputs(m, n, q, b, 9000 + q + b)
        Bd, ad, Xd = device_inputs(B, alpha, X)
        K = gpu_pack(biq, Bd, 8)
        Y = gpu_gemm(biq, K, ad, Xd, m, n, q, 8).cpu().numpy()
        assert_within_tolerance(Y, oracle.gemm_dense(B, alpha, X), alpha, X, "planes")


def test_hbm_regime_launch_sampled_rows(biq, oracle):
    """The launch bench.py puts on the roofline (cfg 2's n, q, mu, batch with m = 2^20: 512 MiB
    of keys, one workgroup per CU walking both tiles): packed keys are drawn directly as iid
    bytes, the oracle computes a sample of output rows from the signs those bytes encode."""
    import torch

    m, n, q, b, mu = 1 << 20, 2048, 2, 1, 8
    _say("hbm regime m=%d n=%d q=%d" % (m, n, q))
    rng = np.random.default_rng(31337)
    Kh = rng.integers(0, 256, size=(q, m, n // 8), dtype=np.uint8)
    alpha = rng.uniform(0.05, 1.0, size=(q, m)).astype(np.float32)
    X = rng.standard_normal((b, n), dtype=np.float32)
    rows = np.unique(np.concatenate([np.array([0, 63, 64, 4095, 4096, m - 1]),
                                     rng.integers(0, m, size=250)])).astype(np.int64)
    bits = np.unpackbits(Kh[:, rows, :], axis=2, bitorder="little")  # element j <-> bit j
    Bs = (bits.astype(np.int8) * 2 - 1)
    assert np.array_equal(oracle.pack_bitmap(Bs), Kh[:, rows, :])  # the bytes are these signs' keys
    ref = oracle.gemm_dense(Bs, alpha[:, rows], X)
    plan = biq.biq_plan_get(m, n, q, b, mu)
    assert biq.biq_kernel_name(plan.kernel) == "gemv8" and plan.chunk_splits == 1 and plan.row_mode == 0
    Y = gpu_gemm(biq, torch.from_numpy(Kh).cuda().reshape(-1), torch.from_numpy(alpha).cuda(),
                 torch.from_numpy(X).cuda(), m, n, q, mu).cpu().numpy()
    assert np.all(np.isfinite(Y))
    assert_within_tolerance(Y[:, rows], ref, alpha[:, rows], X, "hbm regime")
    # property that holds at any size: flipping every sign and every alpha's sign... is not cheap to
    # arrange here; instead check linearity in X on all rows: Y(2X) == 2 Y(X) exactly in fp32
    Y2 = gpu_gemm(biq, torch.from_numpy(Kh).cuda().reshape(-1), torch.from_numpy(alpha).cuda(),
                  torch.from_numpy(2 * X).cuda(), m, n, q, mu).cpu().numpy()
    assert np.array_equal(Y2, 2 * Y)


def test_xcd_skewed_row_split(biq, oracle):
    """Uneven row shares for even / odd XCDs (a scheduling choice) cover every row exactly once."""
    import torch

    for (m, n, q, rows, skew) in [(8 * 3 * 192, 1024, 1, 192, 64), (8 * 2 * 256 - 100, 2048, 2, 256, 128),
                                  (16 * 128 - 1, 3000, 3, 128, 64)]:
        _say("skew m=%d n=%d q=%d rows=%d skew=%d" % (m, n, q, rows, skew))
        B, alpha, X = _rand_inputs(m, n, q, 1, 9100 + m)
        Bd, ad, Xd = device_inputs(B, alpha, X)
        K = gpu_pack(biq, Bd, 8)
        tiles = -(-(-(-n // 8)) // 128)
        plan = _plan(biq, 1, 1024, 128, 1, tiles, rows)
        plan.xcd_skew = skew
        Y = gpu_gemm(biq, K, ad, Xd, m, n, q, 8, plan=plan)
        plan0 = _plan(biq, 1, 1024, 128, 1, tiles, rows)
        Y0 = gpu_gemm(biq, K, ad, Xd, m, n, q, 8, plan=plan0)
        assert torch.equal(Y, Y0)  # same arithmetic per row, whatever workgroup does it
        assert_within_tolerance(Y.cpu().numpy(), oracle.gemm_dense(B, alpha, X), alpha, X, "skew")


def test_gemm_is_deterministic(biq):
    import torch

    m, n, q, b, mu = 1024, 4096, 2, 1, 8
    B, alpha, X = _rand_inputs(m, n, q, b, 8000)
    Bd, ad, Xd = device_inputs(B, alpha, X)
    K = gpu_pack(biq, Bd, mu)
    Y0 = gpu_gemm(biq, K, ad, Xd, m, n, q, mu)
    for _ in range(3):
        assert torch.equal(gpu_gemm(biq, K, ad, Xd, m, n, q, mu), Y0)


def test_error_paths_on_device_buffers(biq):
    import torch

    m, n, q, b, mu = 64, 4096, 1, 4, 8
    K = torch.zeros(biq.biq_packed_bytes(m, n, q), dtype=torch.uint8, device="cuda")
    alpha = torch.ones((q, m), device="cuda")
    X = torch.ones((b, n), device="cuda")
    Y = torch.zeros((b, m), device="cuda")
    plan = _plan(biq, 0, 256, 16, 4, 1, 64)
    need = biq.biq_plan_workspace_bytes(biq.biq_plan_get(m, n, q, b, mu), m, b)
    lib = biq.load_library()
    import ctypes
    assert lib.biq_gemm_ex(K.data_ptr(), alpha.data_ptr(), X.data_ptr(), Y.data_ptr(), m, n, q, b, mu,
                           ctypes.byref(plan), None, 0, None) == biq.BIQ_EWORKSPACE
    assert lib.biq_gemm(K.data_ptr() + 4, alpha.data_ptr(), X.data_ptr(), Y.data_ptr(), m, n, q, b, mu,
                        None, 0, None) == biq.BIQ_EINVAL
    assert need >= 0


def _unpack_plan(biq, q, batch_tile, groups_per_split, wave_splits=1, rpw=None, terms=3):
    """Plan for the unpack-into-MFMA kernel (kernel 3): 256 threads, 32-byte key groups,
    rows_per_wg = (4 / wave_splits) waves x rpw row tiles of 32 rows; the inputs split into three
    bf16 terms (exact, the library's choice) or two scaled fp16 terms."""
    if rpw is None:
        rpw = {1: 4, 2: 2}.get(q, 1)
    plan = _plan(biq, kernel=3, threads=256, ct=32, bt=batch_tile, tps=groups_per_split,
                 rows=(4 // wave_splits) * 32 * rpw)
    plan.wave_splits = wave_splits
    plan.input_terms = terms
    return plan


UNPACK_SHAPES = [
    # m, n, q, batch, batch_tile, key groups per split, wave splits, row tiles per wave and plane
    (256, 256, 2, 64, 64, 1, 1, 2),      # one key group, full tiles
    (300, 1000, 1, 70, 64, 2, 1, 4),     # ragged rows / columns / vectors, several splits
    (129, 257, 3, 33, 64, 1, 1, 1),      # n not a multiple of 4 (scalar X reads), odd m (scalar stores)
    (1024, 2048, 2, 128, 64, 8, 1, 2),   # one split walking 8 key groups
    (512, 1536, 4, 32, 32, 3, 1, 1),     # four planes, one column tile per workgroup, two splits
    (64, 128, 1, 1, 32, 1, 1, 1),        # a single input vector, half a key group (n = 128)
    (2048, 512, 2, 100, 32, 2, 1, 1),    # 32-wide column tiles, ragged batch
    # contraction split over the waves of a workgroup
    (512, 2048, 2, 64, 64, 8, 2, 2),     # two wave groups, 4 key groups each
    (300, 1800, 2, 40, 64, 8, 2, 1),     # 8 key groups asked, 8 there (1800 -> 240 B stride): 4 + 4
    (200, 1300, 3, 33, 32, 6, 2, 1),     # 6 key groups: 3 + 3, ragged everything
    (200, 1300, 1, 65, 64, 5, 2, 2),     # 5 of 6 key groups per split: 3 + 2, then 1 + 0
    (1024, 4096, 3, 32, 32, 16, 4, 1),   # four wave groups, 4 key groups each
    (100, 2300, 2, 20, 32, 10, 4, 1),    # 10 key groups: 3 + 3 + 3 + 1
    (64, 512, 4, 96, 32, 2, 4, 1),       # fewer key groups (2) than wave groups: two of them idle
    (96, 256, 1, 32, 32, 1, 2, 4),       # one key group, second wave group idle
]


@pytest.mark.parametrize("m,n,q,b,bt,gps,ws,rpw", UNPACK_SHAPES)
def test_unpack_mfma_parity(biq, oracle, m, n, q, b, bt, gps, ws, rpw):
    _say("unpack_mfma m=%d n=%d q=%d b=%d bt=%d gps=%d ws=%d rpw=%d" % (m, n, q, b, bt, gps, ws, rpw))
    B, alpha, X = _rand_inputs(m, n, q, b, seed=4200 + m + n + q + b)
    B_dev, alpha_dev, X_dev = device_inputs(B, alpha, X)
    K = gpu_pack(biq, B_dev)
    ref = oracle.gemm_dense(B, alpha, X)
    for terms in (3, 2):
        Y = gpu_gemm(biq, K, alpha_dev, X_dev, m, n, q, 8, plan=_unpack_plan(biq, q, bt, gps, ws, rpw, terms))
        assert_within_tolerance(Y.cpu().numpy(), ref, alpha, X,
                                what="unpack_mfma %s" % ((m, n, q, b, bt, gps, ws, rpw, terms),))


def test_unpack_mfma_bit_exact_on_exact_inputs(biq, oracle):
    """Small integer inputs: every partial sum is exactly representable and every input is the sum
    of its terms (three bf16 terms always; two scaled fp16 terms for these small integers), so any
    summation order, the split and the fp32 matrix-core accumulation must reproduce Eq. 2 bit for
    bit."""
    from paper_2005_09904_amd.workloads import Workload, make_exact_inputs

    m, n, q, b = 384, 1280, 3, 96
    _say("unpack_mfma exact inputs")
    B, alpha, X = make_exact_inputs(Workload("exact", m, n, q, b, 8, "uniform", seed=77))
    B_dev, alpha_dev, X_dev = device_inputs(B, alpha, X)
    K = gpu_pack(biq, B_dev)
    ref = oracle.gemm_dense(B, alpha, X)
    for terms in (3, 2):
        for bt, gps, ws in ((64, 2, 1), (32, 5, 1), (64, 5, 2), (32, 3, 4)):
            Y = gpu_gemm(biq, K, alpha_dev, X_dev, m, n, q, 8, plan=_unpack_plan(biq, q, bt, gps, ws, terms=terms))
            assert np.array_equal(Y.cpu().numpy().astype(np.float64), ref), (terms, bt, gps, ws)


def test_unpack_mfma_exact_split_adds_no_input_error(biq, oracle):
    """Three bf16 terms by truncation hold every bit of a finite fp32 input: with inputs that carry
    all 24 significand bits the result must agree with the fp64 oracle as closely as the order of
    fp32 additions allows, and better than the two-term variant, whose input rounding shows."""
    m, n, q, b = 256, 2048, 2, 40
    _say("unpack_mfma exact split")
    B, alpha, X = _rand_inputs(m, n, q, b, seed=808)
    B_dev, alpha_dev, X_dev = device_inputs(B, alpha, X)
    K = gpu_pack(biq, B_dev)
    ref = oracle.gemm_dense(B, alpha, X)
    err = {}
    for terms in (3, 2):
        Y = gpu_gemm(biq, K, alpha_dev, X_dev, m, n, q, 8, plan=biq.biq_plan_get_mfma(m, n, q, b, 8, terms))
        _, err[terms] = assert_within_tolerance(Y.cpu().numpy(), ref, alpha, X, what="terms=%d" % terms)
    assert err[3] <= 5e-7 and err[2] <= 1e-6, err
    # a one-hot contraction shows the inputs themselves: three terms return alpha * x bit for bit
    Bh = -np.ones((1, 64, 256), dtype=np.int8)
    Xh = np.zeros((32, 256), dtype=np.float32)
    rng = np.random.default_rng(5)
    hot = rng.integers(0, 256, size=32)
    vals = rng.standard_normal(32).astype(np.float32) * np.float32(1.2345678)
    Xh[np.arange(32), hot] = vals
    ah = np.ones((1, 64), dtype=np.float32)
    B_dev, alpha_dev, X_dev = device_inputs(Bh, ah, Xh)
    K = gpu_pack(biq, B_dev)
    Y = gpu_gemm(biq, K, alpha_dev, X_dev, 64, 256, 1, 8, plan=biq.biq_plan_get_mfma(64, 256, 1, 32, 8, 3)).cpu().numpy()
    assert np.array_equal(Y, np.repeat(-vals[:, None], 64, axis=1))


def test_unpack_mfma_skips_zero_terms_without_changing_the_result(biq, oracle):
    """Exact split: terms that are zero for all of a workgroup's input vectors over a wave's part
    of the row are skipped.  Inputs that carry 11 (fp16-valued) or 8 (bf16-valued) significand
    bits take the two-term and one-term loops; one full-precision element anywhere in a wave's
    share (here: in some input vectors, in some column ranges only) brings the third term back
    for that wave alone.  Every variant must meet the bound, and agree bit for bit with the
    same call on inputs where a harmless full-precision element forces all three terms."""
    import torch

    m, n, q, b = 384, 2048, 2, 96
    _say("unpack_mfma zero-term skipping")
    B, alpha, X = _rand_inputs(m, n, q, b, seed=911)
    X16 = X.astype(np.float16).astype(np.float32)
    Xb = torch.from_numpy(X).bfloat16().float().numpy()
    Xmix = X16.copy()
    Xmix[5, 700:900] = X[5, 700:900]          # full precision in one vector, one stretch of columns
    Xmix[70:, :256] = Xb[70:, :256]
    B_dev, alpha_dev, _ = device_inputs(B, alpha, X)
    K = gpu_pack(biq, B_dev)
    for name, Xv in (("fp16-valued", X16), ("bf16-valued", Xb), ("mixed", Xmix)):
        ref = oracle.gemm_dense(B, alpha, Xv)
        for bt, gps, ws in ((64, 8, 1), (32, 3, 2), (32, 4, 4)):
            plan = _unpack_plan(biq, q, bt, gps, ws, terms=3)
            Xd = torch.from_numpy(Xv).cuda()
            Y = gpu_gemm(biq, K, alpha_dev, Xd, m, n, q, 8, plan=plan).cpu().numpy()
            assert_within_tolerance(Y, ref, alpha, Xv, what="%s %s" % (name, (bt, gps, ws)))
            # two scaled fp16 terms: the second one is zero for fp16- and bf16-valued vectors and is
            # skipped where a whole column group has none; exact on such inputs up to summation order
            Y2 = gpu_gemm(biq, K, alpha_dev, Xd, m, n, q, 8,
                          plan=_unpack_plan(biq, q, bt, gps, ws, terms=2)).cpu().numpy()
            assert_within_tolerance(Y2, ref, alpha, Xv, what="%s %s two terms" % (name, (bt, gps, ws)))
            # the same inputs plus one extra input vector of full precision in the same column
            # group: all three terms everywhere; the first b vectors must not change by a bit
            Xfull = np.concatenate([Xv, X[:1] * np.float32(1.0000001)], axis=0)
            if (b + 1 - 1) // bt == (b - 1) // bt:      # the extra vector shares the last column group only
                Yf = gpu_gemm(biq, K, alpha_dev, torch.from_numpy(Xfull).cuda(), m, n, q, 8,
                              plan=_unpack_plan(biq, q, bt, gps, ws, terms=3)).cpu().numpy()
                assert np.array_equal(Yf[:b], Y), (name, bt, gps, ws)


def test_unpack_mfma_input_scaling_covers_the_fp32_range(biq, oracle):
    """Two-term variant: every input vector is scaled by its own power of two before it is split into fp16 terms:
    vectors of very different magnitude (2^-120 .. 2^115, with subnormal elements, all zero), and vectors whose
    elements span 12 orders of magnitude, must all meet the bound, and with an error at the level
    of fp32 rounding (the split keeps 22 significand bits), not at the level of fp16."""
    m, n, q, b = 320, 1536, 2, 48
    _say("unpack_mfma input scaling")
    rng = np.random.default_rng(2024)
    B, alpha, X = _rand_inputs(m, n, q, b, seed=515)
    X = X.astype(np.float64)
    for a in range(b):
        if a % 4 == 1:       # elements over 12 orders of magnitude
            X[a] *= 10.0 ** rng.uniform(-9, 3, size=n)
        X[a] *= 2.0 ** (-120 + 5 * a)          # 2^-120 .. 2^115
    X[7] = 0.0                                   # an all-zero vector
    X[11] = rng.integers(-50, 51, size=n) * 2.0 ** -149   # subnormal fp32 elements ...
    X[11, ::7] = rng.standard_normal(len(X[11, ::7])) * 2.0 ** -118   # ... among small normal ones
    X[13, :] = 0.0
    X[13, 5] = 1.5e38                            # one element near the top of fp32 (2 planes, alpha <= 1), the rest zero
    X = X.astype(np.float32)
    B_dev, alpha_dev, X_dev = device_inputs(B, alpha, X)
    K = gpu_pack(biq, B_dev)
    ref = oracle.gemm_dense(B, alpha, X)
    for bt, gps, ws in ((64, 6, 1), (32, 3, 2)):
        Y = gpu_gemm(biq, K, alpha_dev, X_dev, m, n, q, 8,
                     plan=_unpack_plan(biq, q, bt, gps, ws, terms=2)).cpu().numpy()
        assert_within_tolerance(Y, ref, alpha, X, what="unpack_mfma scaling %s" % ((bt, gps, ws),))
        assert np.all(Y[7] == 0.0)
        err = np.sqrt(((Y - ref) ** 2).sum(axis=1)) / np.maximum(np.sqrt((ref ** 2).sum(axis=1)), 1e-300)
        assert err.max() <= 1e-6, err.max()     # 2^-22 per element at worst, far from fp16's 2^-11


def test_unpack_mfma_does_not_depend_on_mu_and_default_plan_picks_it(biq, oracle):
    """The kernel reads the packed bitmap, which is the same for every mu; for enough input
    vectors and weights it is what biq_gemm runs, while biq_plan_get_lut keeps to the tables."""
    m, n, q, b = 4096, 2048, 2, 96
    _say("unpack_mfma default plan")
    B, alpha, X = _rand_inputs(m, n, q, b, seed=99)
    B_dev, alpha_dev, X_dev = device_inputs(B, alpha, X)
    K = gpu_pack(biq, B_dev)
    ref = oracle.gemm_dense(B, alpha, X)
    first = None
    for mu in (8, 6, 4, 1):
        assert biq.biq_kernel_name(biq.biq_plan_get(m, n, q, b, mu).kernel) == "unpack_mfma"
        assert biq.biq_kernel_name(biq.biq_plan_get_lut(m, n, q, b, mu).kernel) != "unpack_mfma"
        Y = gpu_gemm(biq, K, alpha_dev, X_dev, m, n, q, mu)
        assert_within_tolerance(Y.cpu().numpy(), ref, alpha, X, what="unpack_mfma mu=%d" % mu)
        first = Y if first is None else first
        assert torch_equal(first, Y)
    # the table kernels on the same inputs, through an explicit plan
    Y = gpu_gemm(biq, K, alpha_dev, X_dev, m, n, q, 8, plan=biq.biq_plan_get_lut(m, n, q, b, 8))
    assert_within_tolerance(Y.cpu().numpy(), ref, alpha, X, what="lut plan")


def torch_equal(a, b):
    import torch

    return torch.equal(a, b)


def test_hip_graph_replay_matches_eager(biq, oracle):
    """A sequence of biq_gemm calls (GEMV with chunk split + reduce, batched table kernel,
    unpack_mfma with its input split and partial sums, with three and with two input terms)
    captured into a HIP graph: every replay,
    with eager work in between, reproduces the eager results bit for bit.  The library records
    no memset nodes and allocates nothing, so its calls can be captured."""
    import torch

    shapes = [(2048, 2048, 2, 1), (600, 1000, 3, 6), (1024, 2048, 2, 128), (1024, 2048, 2, 100)]
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        calls, outs, refs = [], [], []
        for i, (m, n, q, b) in enumerate(shapes):
            B, alpha, X = _rand_inputs(m, n, q, b, seed=31 + i)
            Bd, ad, Xd = device_inputs(B, alpha, X)
            K = gpu_pack(biq, Bd)
            Y = torch.zeros((b, m), dtype=torch.float32, device="cuda")
            ws = torch.empty(max(biq.biq_workspace_bytes(m, n, q, b, 8), 16), dtype=torch.uint8, device="cuda")
            plan = None
            if i >= 2:  # make sure the matrix-core path is in the graph whatever the planner prefers
                plan = biq.biq_plan_check(m, n, q, b, 8, _unpack_plan(biq, q, 64, 4, terms=3 if i == 2 else 2))
                ws = torch.empty(biq.biq_plan_workspace_bytes(plan, m, b), dtype=torch.uint8, device="cuda")
            calls.append(biq.PreparedGemm(K, ad, Xd, Y, m, n, q, b, 8, workspace=ws, plan=plan))
            outs.append(Y)
            refs.append((oracle.gemm_dense(B, alpha, X), alpha, X))
        for c in calls:
            c()
        torch.cuda.synchronize()
        eager = [y.clone() for y in outs]
        for y, (ref, alpha, X) in zip(eager, refs):
            assert_within_tolerance(y.cpu().numpy(), ref, alpha, X, "eager")
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            for c in calls:
                c()
        for rep in range(4):
            _say("graph replay %d" % rep)
            for y in outs:
                y.fill_(float("nan"))        # eager work between replays
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            for y, e in zip(outs, eager):
                assert torch.equal(y, e), "replay %d differs from the eager result" % rep


def test_generic_kernel_with_full_lds(biq, oracle):
    """Generic kernel, several tiles per workgroup: tables (128 KiB) plus row accumulators fill
    the 160 KiB of LDS exactly at 1024 rows x 8 input vectors; one row more is refused."""
    m, n, q, b, mu = 2100, 1600, 2, 9, 6
    B, alpha, X = _rand_inputs(m, n, q, b, 7100)
    Bd, ad, Xd = device_inputs(B, alpha, X)
    K = gpu_pack(biq, Bd, mu)
    plan = biq.biq_plan_check(m, n, q, b, mu, _plan(biq, 0, 256, 64, 8, 2, 1024))
    assert plan.lds_bytes == 160 * 1024 and plan.tiles_per_split == 2
    _say("generic kernel, LDS full")
    Y = gpu_gemm(biq, K, ad, Xd, m, n, q, mu, plan=plan).cpu().numpy()
    assert_within_tolerance(Y, oracle.gemm_dense(B, alpha, X), alpha, X, "generic full LDS")
    with pytest.raises(biq.BiqError):
        biq.biq_plan_check(m, n, q, b, mu, _plan(biq, 0, 256, 64, 8, 2, 1025))
    # a large-batch shape the planner sends to the generic kernel with two tiles per workgroup
    p = biq.biq_plan_get(8192, 2048, 5, 256, 7)
    assert biq.biq_kernel_name(p.kernel) == "query_generic" and p.lds_bytes <= 160 * 1024


def test_random_shapes_default_plans(biq, oracle):
    """Seeded random shapes through biq_gemm with the planner's own choice: every kernel family
    meets ragged m, n, batch (including the half-table and matrix-core kernels)."""
    rng = np.random.default_rng(777)
    seen = set()
    for case in range(70):
        mu = int(rng.integers(1, 11))
        q = int(rng.integers(1, 6))
        b = int(rng.choice([1, 1, 2, 3, 5, 8, 33, 70, 130]))
        n = int(rng.choice([int(rng.integers(1, 300)), int(rng.integers(300, 2200)), int(rng.integers(2200, 9000))]))
        m = int(rng.integers(1, 700))
        while m * n * q * b > 60_000_000:
            m = max(1, m // 2)
        if case % 7 == 0:                      # make sure the wide small GEMV / batched cases occur
            mu, b, n = 8, int(rng.choice([1, 4])), int(rng.integers(1030, 2048))
        if case % 10 == 6:                     # ... the full-table GEMV and batched kernels
            mu, b, n = 8, 1, int(rng.integers(100, 1000))
        if case % 10 == 8:
            mu, b, n = 8, int(rng.choice([2, 5])), int(rng.integers(64, 500))
        if case % 10 == 3:                     # ... and the matrix-core path
            m, n, q, b = int(rng.integers(2000, 3000)), int(rng.integers(1500, 2500)), 2, 130
        kname = biq.biq_kernel_name(biq.biq_plan_get(m, n, q, b, mu).kernel)
        seen.add(kname)
        _say("random case %d: m=%d n=%d q=%d b=%d mu=%d -> %s" % (case, m, n, q, b, mu, kname))
        B, alpha, X = _rand_inputs(m, n, q, b, 9900 + case)
        Bd, ad, Xd = device_inputs(B, alpha, X)
        K = gpu_pack(biq, Bd, mu)
        Y = gpu_gemm(biq, K, ad, Xd, m, n, q, mu).cpu().numpy()
        rows = None
        if m * n * q * b > 60_000_000:
            rows = np.unique(rng.integers(0, m, size=64)).astype(np.int64)
        ref = oracle.gemm_dense(B, alpha, X, rows=rows)
        if rows is None:
            assert_within_tolerance(Y, ref, alpha, X, "random case %d" % case)
        else:
            assert_within_tolerance(Y[:, rows], ref, alpha[:, rows], X, "random case %d" % case)
    assert {"query_generic", "gemv8", "gemv8_half", "gemm8x2", "gemm8x2_half", "unpack_mfma"} <= seen, seen


def test_random_matrix_core_plans(biq, oracle):
    """Seeded random shapes x random valid mappings of the matrix-core kernel (column tile, row
    tiles per wave, wave groups, key groups per split) x both input splits, with inputs of
    mixed precision so that the one-, two- and three-term loops all occur."""
    import torch

    rng = np.random.default_rng(4242)
    done = 0
    for case in range(400):
        if done == 36:
            break
        q = int(rng.integers(1, 5))
        m = int(rng.integers(1, 600))
        n = int(rng.choice([int(rng.integers(1, 260)), int(rng.integers(260, 3000)), int(rng.integers(3000, 9000))]))
        b = int(rng.choice([1, 7, 31, 32, 33, 64, 65, 100, 130]))
        while m * n * q * b > 50_000_000:
            m = max(1, m // 2)
        bt = int(rng.choice([32, 64]))
        ws = int(rng.choice([1, 2, 4]))
        r = int(rng.choice([1, 2, 4]))
        groups = -(-biq.biq_key_row_stride(n) // 32)
        gps = int(rng.integers(1, groups + 1))
        terms = int(rng.choice([3, 3, 2]))
        plan = _unpack_plan(biq, q, bt, gps, ws, r, terms)
        try:
            plan = biq.biq_plan_check(m, n, q, b, 8, plan)
        except biq.BiqError:
            continue                                   # not a valid mapping (register file, q * r > 4)
        done += 1
        _say("matrix-core case %d: m=%d n=%d q=%d b=%d bt=%d ws=%d r=%d gps=%d terms=%d" % (
            case, m, n, q, b, bt, ws, r, gps, terms))
        B, alpha, X = _rand_inputs(m, n, q, b, 5200 + case)
        kind = case % 3                               # full precision / fp16-valued / bf16-valued, one vector mixed in
        if kind == 1:
            X = X.astype(np.float16).astype(np.float32)
        elif kind == 2:
            X = torch.from_numpy(X).bfloat16().float().numpy()
            if b > 40:
                X[b - 1, n // 2:] = X[b - 1, n // 2:] * np.float32(1.0009765625)   # more bits in one vector's second half
        Bd, ad, Xd = device_inputs(B, alpha, X)
        K = gpu_pack(biq, Bd)
        Y = gpu_gemm(biq, K, ad, Xd, m, n, q, 8, plan=plan).cpu().numpy()
        assert_within_tolerance(Y, oracle.gemm_dense(B, alpha, X), alpha, X, "matrix-core case %d" % case)
    assert done == 36


@pytest.mark.parametrize("mu", [1, 2, 3, 4, 5, 6])
def test_wide_kernel_plans(biq, oracle, mu):
    """query_wide (32 lanes per row, conflict-free gathers for mu <= 6) with explicit plans:
    threads, rows per workgroup, rows narrower and wider than one tile, ragged batch, q = 5."""
    uk = {1: 128, 2: 64, 3: 32, 4: 32, 5: 32, 6: 16}[mu]
    bt = (128 * 1024) // (32 * uk * (1 << mu) * 4)
    for (m, n, q, b) in [(300, 3000, 3, 5), (77, mu * 32 * uk * 2 + 37, 2, 3), (5, 100, 5, 1)]:
        B, alpha, X = _rand_inputs(m, n, q, b, 7300 + mu + m)
        Bd, ad, Xd = device_inputs(B, alpha, X)
        K = gpu_pack(biq, Bd, mu)
        ref = oracle.gemm_dense(B, alpha, X)
        for threads, rows in [(1024, 64), (256, 33), (64, 1), (512, 300)]:
            _say("wide mu=%d m=%d n=%d q=%d b=%d threads=%d rows=%d" % (mu, m, n, q, b, threads, rows))
            plan = _plan(biq, 6, threads, 32 * uk, bt, 1, rows)
            Y = gpu_gemm(biq, K, ad, Xd, m, n, q, mu, plan=plan).cpu().numpy()
            assert_within_tolerance(Y, ref, alpha, X, "wide mu=%d" % mu)
    # exactly representable inputs: bit for bit
    from paper_2005_09904_amd.workloads import Workload, make_exact_inputs

    w = Workload("exact", 129, 5000, 2, 3, mu, "uniform", seed=600 + mu)
    B, alpha, X = make_exact_inputs(w)
    Bd, ad, Xd = device_inputs(B, alpha, X)
    K = gpu_pack(biq, Bd, mu)
    assert biq.biq_kernel_name(biq.biq_plan_get(129, 5000, 2, 3, mu).kernel) == "query_wide"
    Y = gpu_gemm(biq, K, ad, Xd, 129, 5000, 2, mu).cpu().numpy()
    assert np.array_equal(Y.astype(np.float64), oracle.gemm_dense(B, alpha, X))
