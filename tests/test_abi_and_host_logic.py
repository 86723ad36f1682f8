"""Host-side checks that need no GPU: the library loads, exports what include/biq.h declares,
its size arithmetic and planner are consistent, and argument errors are reported as codes."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def biq():
    import paper_2005_09904_amd as biq
    from paper_2005_09904_amd import build

    if build.is_stale():
        build.build_library()
    biq.load_library()
    return biq


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "biq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(biq_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol(biq):
    lib = biq.load_library()
    declared = _declared_functions()
    assert len(declared) >= 14
    for name in declared:
        assert hasattr(lib, name), "libbiq.so does not export %s" % name
    from paper_2005_09904_amd.binding import EXPORTS
    assert sorted(EXPORTS) == declared


def test_plan_struct_matches_header(biq):
    text = open(os.path.join(ROOT, "include", "biq.h")).read()
    body = re.search(r"typedef struct \{(.*?)\} biq_plan;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"int\s+([a-z_]+)(?:\[(\d+)\])?\s*;", body)
    mirror = [(n, getattr(t, "_length_", None)) for n, t in biq.BiqPlan._fields_]
    assert [(n, int(l) if l else None) for n, l in fields] == mirror


def test_size_arithmetic(biq):
    assert biq.biq_key_row_stride(1) == 16
    assert biq.biq_key_row_stride(128) == 16
    assert biq.biq_key_row_stride(129) == 32
    assert biq.biq_key_row_stride(4096) == 512
    # Table II: 512x512 with 4/3/2 planes -> q*m*n/8 bytes
    for q, nbytes in [(4, 131072), (3, 98304), (2, 65536)]:
        assert biq.biq_packed_bytes(512, 512, q) == nbytes
    assert biq.biq_num_chunks(4096, 6) == 683
    assert biq.biq_num_chunks(4096, 8) == 512
    assert biq.biq_lut_bytes(4096, 32, 8) == 16 * 1024 * 1024
    assert biq.biq_lut_bytes(512, 1, 8) == 64 * 1024
    # invalid arguments give 0, not garbage
    assert biq.biq_key_row_stride(0) == 0
    assert biq.biq_packed_bytes(0, 5, 1) == 0
    assert biq.biq_num_chunks(10, 9) == 2
    assert biq.biq_num_chunks(10, 11) == 0
    assert biq.biq_lut_bytes(10, 1, 0) == 0


def test_status_strings(biq):
    for code in (0, -1, -2, -3, -4):
        assert biq.status_str(code)
    assert biq.status_str(0) == "ok"
    assert "unknown" in biq.status_str(-99)


@pytest.mark.parametrize("mu", range(1, 11))
def test_default_plans_are_consistent(biq, mu):
    for (m, n, q, b) in [(1, 1, 1, 1), (512, 512, 1, 1), (2048, 2048, 2, 1), (4096, 1024, 3, 8),
                         (4096, 4096, 3, 32), (16384, 4096, 2, 128), (4096, 16384, 2, 128),
                         (1 << 20, 2048, 2, 1), (77, 100000, 1, 3)]:
        p = biq.biq_plan_get(m, n, q, b, mu)
        name = biq.biq_kernel_name(p.kernel)
        assert name != "unknown"
        partial = p.chunk_splits * b * m * 4 if p.chunk_splits > 1 else 0
        if name == "unpack_mfma":
            # large batch: key groups of 32 bytes per row instead of LUT tiles, prepared input
            # (three bf16 terms per element - the exact split is the library's choice -, padded to
            # whole tiles) at the start of the workspace
            assert p.threads == 256 and p.batch_tile in (32, 64)
            tiles = -(-biq.biq_key_row_stride(n) // p.chunks_per_tile)
            assert p.input_terms == 3
            pieces = 16 * (p.batch_tile // 32) * 3 * 64  # per key group: 16 MFMA steps
            xf = p.batch_tiles * p.chunk_splits * p.tiles_per_split * pieces * 16
            xf = (xf + 255) // 256 * 256
            assert xf >= 6 * b * n
            # ... and one count of non-zero terms per MFMA step and column tile
            xf += (p.batch_tiles * p.chunk_splits * p.tiles_per_split * 16 * (p.batch_tile // 32) * 4 + 255) // 256 * 256
            assert biq.biq_plan_workspace_bytes(p, m, b) == xf + partial
            assert biq.biq_workspace_bytes(m, n, q, b, mu) >= xf + partial
        else:
            tiles = -(-biq.biq_num_chunks(n, mu) // p.chunks_per_tile)
            assert p.threads % 64 == 0 and 64 <= p.threads <= 1024
            assert p.batch_tile in (1, 2, 4, 8)
            ws = biq.biq_workspace_bytes(m, n, q, b, mu)
            assert ws == biq.biq_plan_workspace_bytes(p, m, b) == partial
            lut = biq.biq_plan_get_lut(m, n, q, b, mu)
            assert biq.biq_kernel_name(lut.kernel) == name
        assert biq.biq_kernel_name(biq.biq_plan_get_lut(m, n, q, b, mu).kernel) in (
            "query_generic", "query_wide", "gemv8", "gemv8_half", "gemm8x2", "gemm8x2_half")
        assert p.chunk_splits * p.tiles_per_split >= tiles
        assert (p.chunk_splits - 1) * p.tiles_per_split < tiles
        assert p.row_blocks * p.rows_per_wg >= m > (p.row_blocks - 1) * p.rows_per_wg
        assert p.batch_tiles * p.batch_tile >= b
        assert 0 < p.lds_bytes <= 160 * 1024
        assert biq.biq_kernel_name(p.kernel) != "unknown"


def test_plans_hold_their_invariants_on_random_shapes(biq):
    """Planner invariants on a few thousand random shapes (host logic only, nothing is launched):
    every plan the library hands out passes its own check unchanged, covers all rows, chunks and
    input vectors, fits the LDS, and asks for exactly the workspace its fields imply."""
    from hypothesis import given, settings, strategies as st

    dims = st.one_of(st.integers(1, 300), st.integers(1, 20000), st.sampled_from([512, 1024, 2048, 4096, 16384, 65536]))

    @settings(max_examples=1500, deadline=None, derandomize=True)
    @given(m=dims, n=dims, q=st.integers(1, 6), b=st.one_of(st.integers(1, 40), st.sampled_from([64, 128, 256, 1000])),
           mu=st.integers(1, 10))
    def check(m, n, q, b, mu):
        for getter in (biq.biq_plan_get, biq.biq_plan_get_lut):
            p = getter(m, n, q, b, mu)
            name = biq.biq_kernel_name(p.kernel)
            assert name != "unknown"
            assert 0 < p.lds_bytes <= 160 * 1024 and p.threads % 64 == 0 and 64 <= p.threads <= 1024
            assert p.row_blocks * p.rows_per_wg >= m > (p.row_blocks - 1) * p.rows_per_wg
            assert p.batch_tiles * p.batch_tile >= b > (p.batch_tiles - 1) * p.batch_tile
            unit = biq.biq_key_row_stride(n) if name == "unpack_mfma" else biq.biq_num_chunks(n, mu)
            tiles = -(-unit // p.chunks_per_tile)
            assert p.chunk_splits * p.tiles_per_split >= tiles > (p.chunk_splits - 1) * p.tiles_per_split
            # the plan checks as it stands
            c = biq.BiqPlan()
            for k, _ in biq.BiqPlan._fields_:
                if k != "reserved":
                    setattr(c, k, getattr(p, k))
            c = biq.biq_plan_check(m, n, q, b, mu, c)
            assert c.as_dict() == p.as_dict()
            if name != "unpack_mfma":
                partial = p.chunk_splits * b * m * 4 if p.chunk_splits > 1 else 0
                assert biq.biq_plan_workspace_bytes(p, m, b) == partial
                assert p.input_terms == 0 and p.wave_splits == 0
            else:
                assert getter is biq.biq_plan_get and q <= 4 and p.input_terms == 3
            assert biq.biq_workspace_bytes(m, n, q, b, mu) >= biq.biq_plan_workspace_bytes(p, m, b)

    check()


def test_mfma_plans_for_both_input_splits(biq):
    """biq_plan_get_mfma: the matrix-core mapping on either side of the crossover, with the exact
    three-term split or, on request only, the two-term one; workspace = prepared input (2 bytes
    per term and padded element, plus one exponent per padded vector for two terms) + partials."""
    for (m, n, q, b) in [(64, 128, 1, 1), (4096, 4096, 3, 32), (16384, 4096, 2, 128), (300, 1000, 4, 70)]:
        for terms in (3, 2):
            p = biq.biq_plan_get_mfma(m, n, q, b, 8, terms)
            assert biq.biq_kernel_name(p.kernel) == "unpack_mfma" and p.input_terms == terms
            groups = -(-biq.biq_key_row_stride(n) // 32)
            assert p.chunk_splits * p.tiles_per_split >= groups
            xf = p.batch_tiles * p.chunk_splits * p.tiles_per_split * 16 * (p.batch_tile // 32) * terms * 64 * 16
            xf = (xf + 255) // 256 * 256
            if terms == 2:
                xf += (p.batch_tiles * p.batch_tile * 4 + 255) // 256 * 256
            else:
                xf += (p.batch_tiles * p.chunk_splits * p.tiles_per_split * 16 * (p.batch_tile // 32) * 4 + 255) // 256 * 256
            partial = p.chunk_splits * b * m * 4 if p.chunk_splits > 1 else 0
            assert biq.biq_plan_workspace_bytes(p, m, b) == xf + partial
            # a checked copy with the field cleared falls back to the exact split
            c = biq.BiqPlan()
            for k in ("kernel", "threads", "chunks_per_tile", "batch_tile", "tiles_per_split", "rows_per_wg",
                      "wave_splits"):
                setattr(c, k, getattr(p, k))
            assert biq.biq_plan_check(m, n, q, b, 8, c).input_terms == 3
    lib = biq.load_library()
    import ctypes
    plan = biq.BiqPlan()
    assert lib.biq_plan_get_mfma(64, 64, 1, 1, 8, 4, ctypes.byref(plan)) == biq.BIQ_EINVAL
    assert lib.biq_plan_get_mfma(64, 64, 5, 1, 8, 3, ctypes.byref(plan)) == biq.BIQ_EUNSUPPORTED
    # the field belongs to the matrix-core kernel only
    lut = biq.biq_plan_get_lut(512, 512, 1, 1, 8)
    lut.input_terms = 2
    with pytest.raises(Exception):
        biq.biq_plan_check(512, 512, 1, 1, 8, lut)


def test_argument_errors_are_reported_before_any_launch(biq):
    lib = biq.load_library()
    fake = 0x1000  # never dereferenced: every call below fails its argument checks first
    assert lib.biq_pack(None, fake, 4, 4, 1, 8, None) == biq.BIQ_EINVAL
    assert lib.biq_pack(fake, fake, 0, 4, 1, 8, None) == biq.BIQ_EINVAL
    assert lib.biq_pack(fake, fake, 4, 4, 1, 11, None) == biq.BIQ_EINVAL
    assert lib.biq_pack(fake, fake + 8, 4, 4, 1, 8, None) == biq.BIQ_EINVAL  # K not 16-byte aligned
    assert lib.biq_unpack_keys(None, fake, 4, 4, 1, 8, None) == biq.BIQ_EINVAL
    assert lib.biq_build_lut(fake, None, 4, 1, 8, None) == biq.BIQ_EINVAL
    assert lib.biq_build_lut(fake, fake, 4, 0, 8, None) == biq.BIQ_EINVAL
    assert lib.biq_gemm(None, fake, fake, fake, 4, 4, 1, 1, 8, None, 0, None) == biq.BIQ_EINVAL
    assert lib.biq_gemm(fake, fake, fake, fake, 4, 4, 1, 1, 0, None, 0, None) == biq.BIQ_EINVAL
    assert lib.biq_gemm(fake, fake, fake, fake, 4, 4, 0, 1, 8, None, 0, None) == biq.BIQ_EINVAL
    assert lib.biq_gemm(fake, fake + 2, fake, fake, 4, 4, 1, 1, 8, None, 0, None) == biq.BIQ_EINVAL
    assert lib.biq_query(fake, fake, None, fake, 4, 4, 1, 1, 8, None, 0, None) == biq.BIQ_EINVAL
    # a shape whose default plan splits the chunks needs a workspace
    m, n, q, b, mu = 2048, 2048, 2, 1, 8
    need = biq.biq_workspace_bytes(m, n, q, b, mu)
    if need:
        assert lib.biq_gemm(fake, fake, fake, fake, m, n, q, b, mu, None, 0, None) == biq.BIQ_EWORKSPACE
        assert lib.biq_gemm(fake, fake, fake, fake, m, n, q, b, mu, fake, need - 1, None) == biq.BIQ_EWORKSPACE
    bad = biq.BiqPlan()
    bad.threads, bad.chunks_per_tile, bad.batch_tile, bad.tiles_per_split, bad.rows_per_wg = 100, 16, 1, 1, 1
    assert lib.biq_gemm_ex(fake, fake, fake, fake, 4, 4, 1, 1, 8, ctypes.byref(bad), None, 0, None) == biq.BIQ_EINVAL
    bad.row_mode = 1  # latency mode exists only in the mu = 8 kernels
    bad.threads, bad.chunks_per_tile = 256, 16
    assert lib.biq_gemm_ex(fake, fake, fake, fake, 4, 4, 1, 1, 8, ctypes.byref(bad), None, 0, None) == biq.BIQ_EINVAL
    bad.row_mode = 0
    bad.threads, bad.chunks_per_tile = 256, 24  # not a power-of-two number of units
    assert lib.biq_gemm_ex(fake, fake, fake, fake, 4, 4, 1, 1, 8, ctypes.byref(bad), None, 0, None) == biq.BIQ_EINVAL
    bad.chunks_per_tile, bad.batch_tile = 256, 8  # tables would not fit LDS
    assert lib.biq_gemm_ex(fake, fake, fake, fake, 4, 4096, 1, 8, 8, ctypes.byref(bad), None, 0, None) == biq.BIQ_EINVAL
    assert lib.biq_gemm_ex(fake, fake, fake, fake, 4, 4, 1, 1, 8, None, None, 0, None) == biq.BIQ_EINVAL


def test_grouped_and_lstm_argument_errors_are_reported_before_any_launch(biq):
    lib = biq.load_library()
    fake = 0x1000  # never dereferenced: every call below fails its checks first
    assert lib.biq_gemm_grouped(None, 1, 8, None) == biq.BIQ_EINVAL
    arr = (biq.BiqProblem * 2)()
    for d, n in zip(arr, (512, 512)):
        d.K, d.alpha, d.X, d.Y, d.m, d.n, d.q, d.batch = fake, fake, fake, fake, 64, n, 1, 1
    assert lib.biq_gemm_grouped(arr, 0, 8, None) == biq.BIQ_EINVAL
    arr[1].Y = None
    assert lib.biq_gemm_grouped(arr, 2, 8, None) == biq.BIQ_EINVAL
    arr[1].Y, arr[1].n = fake, 4096           # wider than one tile of tables: needs biq_gemm
    assert lib.biq_gemm_grouped(arr, 2, 8, None) == biq.BIQ_EUNSUPPORTED
    arr[1].n, arr[1].q = 512, 5               # more planes than the specialised kernels take
    assert lib.biq_gemm_grouped(arr, 2, 8, None) == biq.BIQ_EUNSUPPORTED
    assert lib.biq_gemm_grouped(arr, 1, 6, None) == biq.BIQ_EUNSUPPORTED
    args = [fake] * 7
    assert lib.biq_lstm_cell(*args, 0, 512, 2, 1, 8, None) == biq.BIQ_EINVAL
    assert lib.biq_lstm_cell(fake, fake, None, fake, fake, fake, fake, 64, 512, 2, 1, 8, None) == biq.BIQ_EINVAL
    assert lib.biq_lstm_cell(*args, 64, 4096, 2, 1, 8, None) == biq.BIQ_EUNSUPPORTED
    assert lib.biq_lstm_cell(*args, 64, 2048, 2, 2, 8, None) == biq.BIQ_EUNSUPPORTED
    assert lib.biq_lstm_cell(*args, 64, 512, 2, 1, 7, None) == biq.BIQ_EUNSUPPORTED


def test_shapes_beyond_the_tuned_kernels_fall_back_or_are_refused(biq):
    """Rows so long that a tuned kernel's 32-bit offsets would overflow: the planner must hand out a
    finished plan of another kernel (or an error), never an unfinished one."""
    for (m, n, q, b) in [(1 << 20, 3000000, 1, 1), (100000, 2200000, 2, 1), (4096, 3000000, 1, 2)]:
        p = biq.biq_plan_get(m, n, q, b, 8)
        assert p.chunk_splits >= 1 and p.lds_bytes > 0 and p.row_blocks >= 1
        biq.biq_plan_check(m, n, q, b, 8, p)
        assert biq.biq_workspace_bytes(m, n, q, b, 8) == biq.biq_plan_workspace_bytes(p, m, b)


def test_missing_library_fails_loudly(biq, tmp_path):
    with pytest.raises(FileNotFoundError):
        biq.load_library(str(tmp_path / "libbiq_missing.so"))


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2005_09904_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "biq_oracle" not in text, f


def test_default_plans_pass_their_own_check_on_random_shapes(biq):
    """Whatever the planner returns is a plan biq_plan_check accepts unchanged, for both planners,
    over a few thousand random shapes including tiny, huge, skinny and ragged ones."""
    import numpy as np

    rng = np.random.default_rng(2005)
    fields = ("kernel", "threads", "chunks_per_tile", "batch_tile", "chunk_splits", "tiles_per_split",
              "rows_per_wg", "row_blocks", "batch_tiles", "lds_bytes", "row_mode", "xcd_skew", "wave_splits")
    for _ in range(3000):
        m = int(rng.choice([1, 2, 7, 64, 100, 511, 2048, 4097, 16384, 100000, 1 << 20]))
        n = int(rng.choice([1, 5, 64, 127, 128, 1000, 1024, 2048, 2050, 4096, 16384, 32768, 100000]))
        q = int(rng.integers(1, 7))
        b = int(rng.choice([1, 2, 3, 8, 17, 32, 33, 64, 100, 128, 500]))
        mu = int(rng.integers(1, 11))
        if m * q >= 1 << 31:
            continue
        for get in (biq.biq_plan_get, biq.biq_plan_get_lut):
            p = get(m, n, q, b, mu)
            before = {k: getattr(p, k) for k in fields}
            biq.biq_plan_check(m, n, q, b, mu, p)          # raises if the plan is rejected
            after = {k: getattr(p, k) for k in fields}
            assert before == after, (m, n, q, b, mu, before, after)
            assert p.row_blocks * p.rows_per_wg >= m and p.batch_tiles * p.batch_tile >= b
            assert 0 < p.lds_bytes <= 160 * 1024
            assert biq.biq_workspace_bytes(m, n, q, b, mu) >= biq.biq_plan_workspace_bytes(p, m, b)
