"""Parity of the HIP library against the CPU oracle, element by element, through the C
ABI.  Tolerances (fp32 1e-4, bf16-in/fp32-accumulate 2e-2) are applied to both the
normwise error max|d|/max|ref| and the componentwise error max |d_ij| / (|A|.|B|)_ij;
integer-valued inputs (every fp32 summation order exact) must match bit for bit."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle
import synth
import paper_2409_03864_amd as tsg

TOL = {tsg.F32: 1e-4, tsg.BF16_F32ACC: 2e-2}
DEV = "cuda:0"


def dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(DEV)
    return torch.from_numpy(a).to(DEV)


def run_gemm(dtype, A, B, *, trans_a=False, flags=0, C0=None, lda=None, ldb=None, ldc=None):
    K, N = B.shape
    M = A.shape[1] if trans_a else A.shape[0]
    acols = A.shape[1]
    lda, ldb, ldc = lda or acols, ldb or N, ldc or N
    Ah = np.zeros((A.shape[0], lda), A.dtype); Ah[:, :acols] = A
    Bh = np.zeros((K, ldb), B.dtype); Bh[:, :N] = B
    Ch = np.full((M, ldc), np.float32(-77.0))
    if C0 is not None:
        Ch[:, :N] = C0
    dA, dB, dC = dev(Ah), dev(Bh), dev(Ch)
    fn = tsg.gemm_transA if trans_a else tsg.gemm
    fn(dtype, M, N, K, dA, lda, dB, ldb, dC, ldc, flags)
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    if ldc > N:
        assert np.all(out[:, N:] == np.float32(-77.0)), "padding columns of C were written"
    return out[:, :N]


def check(C, A, B, dtype, *, trans_a=False, flags=0, C0=None, exact=False):
    R, S = oracle.gemm(A, B, trans_a=trans_a)
    ref = oracle.epilogue(R, flags & 3, C0)
    if C0 is not None and flags & tsg.ACCUMULATE:
        S = S + np.abs(C0)
    if exact:
        assert np.array_equal(C.astype(np.float64), ref)
    else:
        nw, cw = oracle.errors(C, ref, S)
        assert nw <= TOL[dtype] and cw <= TOL[dtype], (nw, cw)


def gate(tag, C, ref, S, tol):
    """The two gated figures (normwise, componentwise) against `tol`, and the plain element-wise
    relative error over the entries with |ref| >= 1e-3 max|ref|, which is printed, not gated."""
    nw, cw = oracle.errors(C, ref, S)
    ew = oracle.elementwise_relative(C, ref)
    print("%s: normwise %.3e componentwise %.3e element-wise (|ref| >= 1e-3 max) %.3e  [tol %.0e]" % (tag, nw, cw, ew, tol))
    assert nw <= tol and cw <= tol, (tag, nw, cw)
    return nw, cw, ew


def inputs(M, N, K, seed, dist, trans_a, dtype):
    return synth.gemm_inputs(M, N, K, seed=seed, dist=dist, trans_a=trans_a, bf16=(dtype == tsg.BF16_F32ACC))


@pytest.fixture(autouse=True)
def _clear_pins():
    yield
    for op in (tsg.OP_GEMM, tsg.OP_GEMM_TRANSA, tsg.OP_CONV2D_NHWC):
        for dt in (tsg.F32, tsg.BF16_F32ACC):
            tsg.tile_config_set(op, dt, None)
    tsg.tune_cache_clear()


# shapes spanning several tiles with ragged tails in every dimension, plus degenerate ones
SHAPES = [(1, 1, 1), (4, 4, 4), (5, 3, 2), (64, 64, 64), (65, 63, 33), (196, 256, 129), (130, 260, 72),
          (257, 129, 40), (300, 70, 2305 // 5), (32, 512, 8), (512, 32, 100)]


@pytest.mark.parametrize("dtype", [tsg.F32, tsg.BF16_F32ACC])
@pytest.mark.parametrize("trans_a", [False, True])
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_gemm_integer_inputs_bit_exact(dtype, trans_a, M, N, K):
    A, B = inputs(M, N, K, 100 + M + N + K, "ints", trans_a, dtype)
    C = run_gemm(dtype, A, B, trans_a=trans_a)
    check(C, A, B, dtype, trans_a=trans_a, exact=True)


@pytest.mark.parametrize("dtype", [tsg.F32, tsg.BF16_F32ACC])
@pytest.mark.parametrize("trans_a", [False, True])
@pytest.mark.parametrize("M,N,K", [(65, 63, 33), (196, 256, 461), (384, 256, 256), (256, 384, 512)])
def test_gemm_random_within_tolerance(dtype, trans_a, M, N, K):
    A, B = inputs(M, N, K, 7, "uniform", trans_a, dtype)
    C = run_gemm(dtype, A, B, trans_a=trans_a)
    check(C, A, B, dtype, trans_a=trans_a)


@pytest.mark.parametrize("dtype", [tsg.F32, tsg.BF16_F32ACC])
@pytest.mark.parametrize("op", [tsg.OP_GEMM, tsg.OP_GEMM_TRANSA])
def test_every_instantiated_config_bit_exact(dtype, op, workspace):
    """Each point of the search space, on a shape with remainders (edge variant) and on a
    divisible shape (no-remainder variant), pinned with TSG_STRICT so no fallback hides it."""
    trans = op == tsg.OP_GEMM_TRANSA
    for (M, N, K) in [(512, 512, 256), (300, 200, 136), (259, 131, 77)]:
        A, B = inputs(M, N, K, 11, "ints", trans, dtype)
        R = oracle.gemm(A, B, trans_a=trans, with_s=False)
        for i in range(tsg.tile_config_count(op, dtype)):
            c = tsg.tile_config_enum(op, dtype, i)
            if tsg.tile_config_check(op, dtype, M, N, K, c) != tsg.OK:
                continue
            tsg.tile_config_set(op, dtype, c)
            C = run_gemm(dtype, A, B, trans_a=trans, flags=tsg.STRICT)
            li = tsg.last_launch()
            assert li.config.as_dict() == c.as_dict() and li.alternative == 0
            assert (li.m_main, li.m_rest) == oracle.split(M, c.bm)[:2]
            assert (li.k_main, li.k_rest) == oracle.split(K, c.bk)[:2]
            assert np.array_equal(C.astype(np.float64), R), (M, N, K, c)


@pytest.mark.parametrize("dtype", [tsg.F32, tsg.BF16_F32ACC])
def test_flags_negate_is_a_sign_flip_and_accumulate_adds(dtype):
    M, N, K = 130, 97, 200
    A, B = inputs(M, N, K, 5, "uniform", False, dtype)
    C = run_gemm(dtype, A, B)
    Cn = run_gemm(dtype, A, B, flags=tsg.NEGATE)
    assert np.array_equal(Cn.view(np.uint32), C.view(np.uint32) ^ np.uint32(0x80000000))
    Z = np.zeros((M, N), np.float32)
    Ca = run_gemm(dtype, A, B, flags=tsg.ACCUMULATE, C0=Z)
    assert np.array_equal(Ca, C)                     # `+=` on a zero-initialised C
    C0 = synth.uniform_pm1(9, 2, M * N).reshape(M, N)
    for fl in (tsg.ACCUMULATE, tsg.ACCUMULATE | tsg.NEGATE):
        Cb = run_gemm(dtype, A, B, flags=fl, C0=C0)
        check(Cb, A, B, dtype, flags=fl, C0=C0)


@pytest.mark.parametrize("dtype", [tsg.F32, tsg.BF16_F32ACC])
def test_leading_dimensions_odd_rows_and_scalar_access(dtype):
    """ld larger than the row; an odd ld, so that rows start on arbitrary element
    boundaries and the 16-byte accesses are unaligned; and the scalar-access form pinned."""
    M, N, K = 70, 52, 90
    vmax = 4 if dtype == tsg.F32 else 8
    for trans in (False, True):
        op = tsg.OP_GEMM_TRANSA if trans else tsg.OP_GEMM
        A, B = inputs(M, N, K, 21, "ints", trans, dtype)
        acols = A.shape[1]
        up = lambda v: -(-v // vmax) * vmax
        C = run_gemm(dtype, A, B, trans_a=trans, lda=up(acols) + 2 * vmax, ldb=up(N) + vmax, ldc=N + 3)
        assert tsg.last_launch().config.vec == vmax
        check(C, A, B, dtype, trans_a=trans, exact=True)
        C = run_gemm(dtype, A, B, trans_a=trans, lda=up(acols) + 1, ldb=up(N) + 3, ldc=N + 5)
        li = tsg.last_launch()
        assert li.alternative == 1 and li.config.vec == vmax
        check(C, A, B, dtype, trans_a=trans, exact=True)
        c = tsg.TileConfig(bm=64, bn=64, bk=(32 if dtype == tsg.F32 else 64), wm=32, wn=32, vec=1, raster=0,
                           sched=0, split_k=1)
        tsg.tile_config_set(op, dtype, c)
        C = run_gemm(dtype, A, B, trans_a=trans, lda=acols + 1, ldb=N + 1, ldc=N + 5, flags=tsg.STRICT)
        li = tsg.last_launch()
        assert li.alternative == 0 and li.config.vec == 1
        check(C, A, B, dtype, trans_a=trans, exact=True)
        tsg.tile_config_set(op, dtype, None)


def test_strict_silenceable_failure_leaves_output_untouched():
    """A pinned config that splits k without a workspace fails silenceably under TSG_STRICT
    and touches nothing; without TSG_STRICT the chain of alternatives completes the call."""
    dt, op = tsg.F32, tsg.OP_GEMM
    tsg.workspace_set(None)
    tsg.tile_config_set(op, dt, tsg.TileConfig(bm=64, bn=64, bk=64, wm=32, wn=32, vec=4, raster=0, sched=0,
                                               split_k=2))
    M, N, K = 64, 64, 256
    A, B = inputs(M, N, K, 3, "ints", False, dt)
    dA, dB = dev(A), dev(B)
    sentinel = synth.uniform_pm1(1, 5, M * N).reshape(M, N)
    dC = dev(sentinel)
    with pytest.raises(tsg.SilenceableError):
        tsg.gemm(dt, M, N, K, dA, K, dB, N, dC, N, tsg.STRICT)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy().view(np.uint32), sentinel.view(np.uint32))
    tsg.gemm(dt, M, N, K, dA, K, dB, N, dC, N, 0)
    torch.cuda.synchronize()
    li = tsg.last_launch()
    assert li.alternative == 1 and li.config.split_k == 1
    assert np.array_equal(dC.cpu().numpy().astype(np.float64), oracle.gemm(A, B, with_s=False))


@pytest.fixture
def workspace():
    ws = torch.empty(64 << 20, dtype=torch.uint8, device=DEV)
    tsg.workspace_set(ws)
    yield ws
    torch.cuda.synchronize()
    tsg.workspace_set(None)


@pytest.mark.parametrize("dtype", [tsg.F32, tsg.BF16_F32ACC])
@pytest.mark.parametrize("trans_a", [False, True])
def test_split_k_bit_exact_and_repeatable(dtype, trans_a, workspace):
    """k loop split over 2..16 workgroups per tile: integer inputs must match the oracle bit
    for bit for every split (ragged M, N and a k remainder), twice in a row on the same
    workspace (the arrival counters reset themselves), with and without the flags."""
    op = tsg.OP_GEMM_TRANSA if trans_a else tsg.OP_GEMM
    vmax = 4 if dtype == tsg.F32 else 8
    M, N, K = 196, 130, 2305
    A, B = inputs(M, N, K, 31, "ints", trans_a, dtype)
    R = oracle.gemm(A, B, trans_a=trans_a, with_s=False)
    C0 = synth.small_ints(8, 2, M * N).reshape(M, N)
    for bm, bn, bk, wm, wn, sched in ((64, 64, 64, 32, 32, 0), (128, 128, 32, 64, 64, 4 if dtype == tsg.F32 else 0)):
        for split in (2, 4, 8, 16):
            c = tsg.TileConfig(bm=bm, bn=bn, bk=bk, wm=wm, wn=wn, vec=vmax, raster=0,
                               sched=sched, split_k=split)
            assert tsg.tile_config_check(op, dtype, M, N, K, c) == tsg.OK
            tsg.tile_config_set(op, dtype, c)
            for rep in range(2):
                C = run_gemm(dtype, A, B, trans_a=trans_a, flags=tsg.STRICT)
                li = tsg.last_launch()
                assert li.alternative == 0 and li.config.split_k == split
                assert np.array_equal(C.astype(np.float64), R), (bm, split, rep)
            fl = tsg.STRICT | tsg.NEGATE | tsg.ACCUMULATE
            C = run_gemm(dtype, A, B, trans_a=trans_a, flags=fl, C0=C0)
            assert np.array_equal(C.astype(np.float64), C0 - R), (bm, split)


def test_split_k_random_is_deterministic_and_within_tolerance(workspace):
    """Random data: the partial tiles are added in split order, so two runs agree bit for
    bit whichever workgroup arrives last, and the result stays within the fp32 tolerance."""
    dt, op = tsg.F32, tsg.OP_GEMM
    M, N, K = 196, 256, 2305
    A, B = inputs(M, N, K, 5, "uniform", False, dt)
    tsg.tile_config_set(op, dt, tsg.TileConfig(bm=64, bn=64, bk=64, wm=32, wn=32, vec=4, raster=0, sched=0,
                                               split_k=8))
    runs = [run_gemm(dt, A, B, flags=tsg.STRICT) for _ in range(4)]
    for r in runs[1:]:
        assert np.array_equal(r.view(np.uint32), runs[0].view(np.uint32))
    check(runs[0], A, B, dt)
    # 16 tiles of 64 x 64 cannot fill the chip: the library's own choice for this shape either splits k
    # (once a workspace is there) or takes the block form, 208 blocks of 16 x 16
    tsg.tile_config_set(op, dt, None)
    C = run_gemm(dt, A, B)
    cfg = tsg.last_launch().config
    assert cfg.split_k > 1 or cfg.sched == 1, cfg
    check(C, A, B, dt)


def test_split_k_batched_paper_loop_nest(workspace):
    """Case Study 4's nest (batch 6, 196 x 256 x 2305) with the k loop split: every batch
    entry has its own counters and partial tiles."""
    dt = tsg.F32
    c, a, b = synth.config_inputs(6)
    nb, M, N, K = c["B"], c["M"], c["N"], c["K"]
    tsg.tile_config_set(tsg.OP_GEMM, dt, tsg.TileConfig(bm=64, bn=64, bk=64, wm=32, wn=32, vec=4, raster=0,
                                                        sched=0, split_k=4))
    dA, dB = dev(a), dev(b)
    dC = torch.zeros((nb, M, N), dtype=torch.float32, device=DEV)
    tsg.gemm_batched(dt, False, nb, M, N, K, dA, K, M * K, dB, N, K * N, dC, N, M * N, tsg.STRICT)
    torch.cuda.synchronize()
    out = dC.cpu().numpy()
    for i in range(nb):
        R, S = oracle.gemm(a[i], b[i])
        nw, cw = oracle.errors(out[i], R, S)
        assert nw <= TOL[dt] and cw <= TOL[dt], (i, nw, cw)


def test_two_streams_split_k_concurrently_with_their_own_workspaces():
    """Each stream has a workspace of its own (tsg_workspace_set_stream), so two products that
    split k may be in flight at once.  Long k, few tiles: both launches are resident together.
    Integer data: each result must equal the oracle bit for bit, many times over."""
    dt = tsg.F32
    M, N, K = 192, 128, 8192
    cfg = tsg.TileConfig(bm=64, bn=64, bk=32, wm=32, wn=32, vec=4, raster=0, sched=4, split_k=8, split_tail=0)
    tsg.tile_config_set(tsg.OP_GEMM, dt, cfg)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    w1 = torch.empty(8 << 20, dtype=torch.uint8, device=DEV)
    w2 = torch.empty(8 << 20, dtype=torch.uint8, device=DEV)
    tsg.workspace_set_stream(s1, w1)
    tsg.workspace_set_stream(s2, w2)
    try:
        A1, B1 = synth.gemm_inputs(M, N, K, seed=41, dist="ints")
        A2, B2 = synth.gemm_inputs(M, N, K, seed=42, dist="ints")
        dA1, dB1, dA2, dB2 = dev(A1), dev(B1), dev(A2), dev(B2)
        C1 = torch.zeros((M, N), dtype=torch.float32, device=DEV)
        C2 = torch.zeros((M, N), dtype=torch.float32, device=DEV)
        R1 = oracle.gemm(A1, B1, with_s=False)
        R2 = oracle.gemm(A2, B2, with_s=False)
        torch.cuda.synchronize()
        for rep in range(20):
            tsg.gemm(dt, M, N, K, dA1, K, dB1, N, C1, N, tsg.STRICT, s1)
            assert tsg.last_launch().config.split_k == 8
            tsg.gemm(dt, M, N, K, dA2, K, dB2, N, C2, N, tsg.STRICT, s2)
        torch.cuda.synchronize()
        assert np.array_equal(C1.cpu().numpy().astype(np.float64), R1)
        assert np.array_equal(C2.cpu().numpy().astype(np.float64), R2)
        # a stream without an entry has no workspace here: the pinned split fails silenceably
        with pytest.raises(tsg.SilenceableError):
            tsg.gemm(dt, M, N, K, dA1, K, dB1, N, C1, N, tsg.STRICT)
    finally:
        torch.cuda.synchronize()
        tsg.workspace_set_stream(s1, None)
        tsg.workspace_set_stream(s2, None)


def test_gemm_and_reduce_share_one_workspace_on_one_stream(workspace):
    """The reduce counts its arrivals in a slot of its own, so a split-k product and a reduce can
    follow each other on one buffer, repeatedly, with exact results on integer data."""
    dt = tsg.F32
    M, N, K = 128, 128, 4096
    cfg = tsg.TileConfig(bm=64, bn=64, bk=32, wm=32, wn=32, vec=4, raster=0, sched=4, split_k=4, split_tail=0)
    tsg.tile_config_set(tsg.OP_GEMM, dt, cfg)
    A, B = synth.gemm_inputs(M, N, K, seed=43, dist="ints")
    x = synth.small_ints(44, 0, 1 << 22).reshape(2048, 2048)
    dA, dB, dx = dev(A), dev(B), dev(x)
    C = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    out = torch.zeros((1,), dtype=torch.float32, device=DEV)
    R = oracle.gemm(A, B, with_s=False)
    total = oracle.reduce_sum(x)[0]
    for rep in range(5):
        tsg.gemm(dt, M, N, K, dA, K, dB, N, C, N, tsg.STRICT)
        tsg.reduce_sum(dt, 2048, 2048, dx, 2048, out, tsg.STRICT)
    torch.cuda.synchronize()
    assert np.array_equal(C.cpu().numpy().astype(np.float64), R)
    assert float(out.item()) == total


@pytest.mark.parametrize("dtype", [tsg.F32, tsg.BF16_F32ACC])
@pytest.mark.parametrize("trans_a", [False, True])
def test_split_tail_only_bit_exact(dtype, trans_a, workspace):
    """Only the tiles past the last full round of 256 are split: 17 x 16 tiles of 64 x 64
    (ragged in M, a k remainder), so 256 whole tiles and 16 split ones in one launch, in the
    register-staged and the direct-to-LDS form, both rasters, twice on the same workspace;
    then the same with two batch entries.  Integer data: bit for bit against the oracle."""
    op = tsg.OP_GEMM_TRANSA if trans_a else tsg.OP_GEMM
    vmax = 4 if dtype == tsg.F32 else 8
    M, N, K = 17 * 64 - 10, 1024, 330
    A, B = inputs(M, N, K, 77, "ints", trans_a, dtype)
    R = oracle.gemm(A, B, trans_a=trans_a, with_s=False)
    C0 = synth.small_ints(8, 2, M * N).reshape(M, N)
    for sched, raster in ((0, 0), (4, 1)):
        for split in (2, 4):
            c = tsg.TileConfig(bm=64, bn=64, bk=64, wm=32, wn=32, vec=vmax, raster=raster, sched=sched,
                               split_k=split, split_tail=1)
            assert tsg.tile_config_check(op, dtype, M, N, K, c) == tsg.OK
            assert tsg.workspace_bytes(dtype, 1, M, N, c) == 65536 + 16 * split * 64 * 64 * 4
            tsg.tile_config_set(op, dtype, c)
            for rep in range(2):
                C = run_gemm(dtype, A, B, trans_a=trans_a, flags=tsg.STRICT)
                li = tsg.last_launch()
                assert li.alternative == 0 and li.config.split_k == split and li.config.split_tail == 1
                assert np.array_equal(C.astype(np.float64), R), (sched, split, rep)
            fl = tsg.STRICT | tsg.NEGATE | tsg.ACCUMULATE
            C = run_gemm(dtype, A, B, trans_a=trans_a, flags=fl, C0=C0)
            assert np.array_equal(C.astype(np.float64), C0 - R), (sched, split)
    # batched: each entry has its own 16 split tiles, counters and partials
    nb = 2
    A2 = np.stack([A, A[::-1].copy()])
    B2 = np.stack([B, B[:, ::-1].copy()])
    dA, dB = dev(A2), dev(B2)
    dC = torch.full((nb, M, N), 7.0, dtype=torch.float32, device=DEV)
    ar, ac = A.shape
    tsg.gemm_batched(dtype, trans_a, nb, M, N, K, dA, ac, ar * ac, dB, N, K * N, dC, N, M * N, tsg.STRICT)
    torch.cuda.synchronize()
    assert tsg.last_launch().config.split_tail == 1
    out = dC.cpu().numpy()
    for i in range(nb):
        assert np.array_equal(out[i].astype(np.float64), oracle.gemm(A2[i], B2[i], trans_a=trans_a, with_s=False)), i
    # a shape whose tile count is a multiple of 256 has no tail: silenceable, output untouched
    with pytest.raises(tsg.SilenceableError):
        tsg.gemm_batched(dtype, trans_a, nb, 1024, N, K, dA, ac, ar * ac, dB, N, K * N, dC, N, M * N, tsg.STRICT)


def test_default_config_with_a_tail_only_split(workspace):
    """With a workspace set the cost model's own pick for 1536^3 (576 tiles of 64 x 64, or 144
    of 128 x 128: neither a multiple of 256) may split only the tail; whatever it picks, the
    call without any pin or tuning must match the oracle bit for bit on integer data, on
    sampled rows and columns, and say what it did."""
    M = N = K = 1536
    for dtype in (tsg.F32, tsg.BF16_F32ACC):
        A, B = inputs(M, N, K, 91, "ints", False, dtype)
        want = tsg.tile_config_get(tsg.OP_GEMM, dtype, M, N, K)
        C = run_gemm(dtype, A, B)
        li = tsg.last_launch()
        assert li.alternative == 1 and li.config.as_dict() == want.as_dict()
        if dtype == tsg.F32:
            assert want.split_tail == 1 and want.split_k > 1     # the fp32 table has no tile that fills 256 CUs evenly here
        rows = [0, 63, 64, 767, 1471, 1472, 1535]
        assert np.array_equal(C[rows].astype(np.float64), oracle.gemm(np.ascontiguousarray(A[rows]), B, with_s=False))
        cols = [0, 1, 1023, 1535]
        assert np.array_equal(C[:, cols].astype(np.float64),
                              oracle.gemm(A, np.ascontiguousarray(B[:, cols]), with_s=False))


@pytest.mark.parametrize("dtype", [tsg.F32, tsg.BF16_F32ACC])
def test_remainder_variants_of_the_direct_kernels(dtype, workspace):
    """The direct-to-LDS kernels treat a remainder in three ways: rows and columns past M / N
    clamped to the last valid one, a partial last k step peeled off the ring (through the
    block of zeros when K ends on a chunk boundary, through the masked path when it cuts a
    chunk), and the general masked ring when chunks are cut along M or N.  One shape per case
    and operand layout, with and without a split of k, integer data, bit for bit."""
    v = 4 if dtype == tsg.F32 else 8
    bk = 32 if dtype == tsg.F32 else 64
    cases = [
        (3 * 64 + 5, 2 * 64 + v, 4 * bk),            # M and N remainders only
        (2 * 64, 2 * 64, 3 * bk + 2 * v),            # partial last k step, whole chunks
        (2 * 64 + 9, 64 + 2 * v, 2 * bk + v + 1),    # K cuts a chunk
        (64 + 3, 64 + v + 1, 2 * bk + 3),            # N cuts a chunk: the general variant
        (v, v, 5), (64, 64, bk - 1), (1, 2 * v, 2 * bk),
    ]
    for ta in (False, True):
        for tb in (False, True):
            op = tsg.OP_GEMM_TRANSA if ta else tsg.OP_GEMM
            for (M, N, K) in cases:
                if ta and M % v:
                    M += v - M % v                       # keep A^T's rows whole chunks except in the general case
                A = inputs(M, 1, K, 61, "ints", ta, dtype)[0]
                B = (inputs(N, 1, K, 62, "ints", False, dtype)[0] if tb
                     else inputs(1, N, K, 62, "ints", False, dtype)[1])
                R = oracle.gemm(A, B, trans_a=ta, trans_b=tb, with_s=False)
                for split in (1, 2):
                    c = tsg.TileConfig(bm=64, bn=64, bk=bk, wm=32, wn=32, vec=v, raster=0, sched=4, split_k=split)
                    if tsg.tile_config_check(op, dtype, M, N, K, c) != tsg.OK:
                        continue
                    tsg.tile_config_set(op, dtype, c)
                    dC = torch.full((M, N), -4.0, dtype=torch.float32, device=DEV)
                    tsg.gemm_trans(dtype, ta, tb, 1, M, N, K, dev(A), A.shape[1], 0, dev(B), B.shape[1], 0, dC, N, 0,
                                   tsg.STRICT)
                    torch.cuda.synchronize()
                    li = tsg.last_launch()
                    assert li.alternative == 0 and li.config.sched == 4 and li.config.split_k == split
                    assert np.array_equal(dC.cpu().numpy().astype(np.float64), R), (ta, tb, M, N, K, split)


def test_one_hot_and_identity_on_device():
    M, N, K = 150, 140, 130
    B = synth.uniform_pm1(2, 1, K * N).reshape(K, N)
    A = np.zeros((M, K), np.float32); A[101, 77] = 1
    C = run_gemm(tsg.F32, A, B)
    exp = np.zeros((M, N), np.float32); exp[101] = B[77]
    assert np.array_equal(C, exp)
    At = np.zeros((K, M), np.float32); At[77, 101] = 1
    assert np.array_equal(run_gemm(tsg.F32, At, B, trans_a=True), exp)
    Bsq = synth.uniform_pm1(2, 3, 130 * 130).reshape(130, 130)
    assert np.array_equal(run_gemm(tsg.F32, np.eye(130, dtype=np.float32), Bsq), Bsq)


@pytest.mark.parametrize("dtype", [tsg.F32, tsg.BF16_F32ACC])
def test_batched_paper_loop_nest(dtype):
    """Case Study 4, Fig. 7: batch 6, 196 x 256 x 2305 (remainders in i and k)."""
    P = synth.PAPER_BATCH_MATMUL
    Bt, M, N, K = P["B"], P["M"], P["N"], P["K"]
    bf = dtype == tsg.BF16_F32ACC
    for dist, exact in (("ints", True), ("normal", False)):
        As, Bs = [], []
        for b in range(Bt):
            a, bb = synth.gemm_inputs(M, N, K, seed=40 + b, dist=dist, bf16=bf)
            As.append(a); Bs.append(bb)
        A, B = np.stack(As), np.stack(Bs)
        dA, dB = dev(A), dev(B)
        dC = torch.zeros((Bt, M, N), dtype=torch.float32, device=DEV)
        tsg.gemm_batched(dtype, False, Bt, M, N, K, dA, K, M * K, dB, N, K * N, dC, N, M * N, tsg.ACCUMULATE)
        torch.cuda.synchronize()
        li = tsg.last_launch()
        assert li.m_main + li.m_rest == 196 and li.k_rest == K - li.k_main and li.k_rest > 0
        C = dC.cpu().numpy()
        for b in range(Bt):
            check(C[b], A[b], B[b], dtype, exact=exact)


# ------------------------------------------------------------------ convolution

def run_conv(dtype, x, w, stride, pad, flags=0, y0=None):
    N, H, W, Cin = x.shape
    KH, KW, _, Cout = w.shape
    Ho, Wo = oracle.conv_out_dim(H, KH, stride[0], pad[0]), oracle.conv_out_dim(W, KW, stride[1], pad[1])
    dx, dw = dev(x), dev(w)
    dy = dev(y0) if y0 is not None else torch.full((N, Ho, Wo, Cout), -55.0, dtype=torch.float32, device=DEV)
    tsg.conv2d_nhwc(dtype, N, H, W, Cin, Cout, KH, KW, stride[0], stride[1], pad[0], pad[1], dx, dw, dy, flags)
    torch.cuda.synchronize()
    return dy.cpu().numpy()


CONV_GEOMS = [
    # N, H, W, Cin, Cout, KH, KW, stride, pad
    (1, 3, 3, 2, 2, 3, 3, (1, 1), (1, 1)),
    (2, 9, 7, 4, 6, 3, 3, (1, 1), (1, 1)),
    (2, 12, 10, 8, 20, 3, 3, (2, 2), (1, 1)),
    (1, 14, 14, 64, 64, 3, 3, (1, 1), (1, 1)),
    (2, 11, 13, 5, 7, 3, 2, (1, 2), (2, 0)),       # Cin, Cout not multiples of 4: scalar path
    (3, 8, 8, 16, 32, 1, 1, (1, 1), (0, 0)),
    (1, 20, 20, 12, 40, 5, 5, (1, 1), (2, 2)),
    (2, 16, 16, 32, 70, 3, 3, (1, 1), (0, 0)),
]


@pytest.mark.parametrize("geom", CONV_GEOMS)
def test_conv_integer_inputs_bit_exact(geom):
    N, H, W, Cin, Cout, KH, KW, st, pd = geom
    x, w = synth.conv_inputs(N, H, W, Cin, Cout, KH, KW, seed=77, dist="ints")
    y = run_conv(tsg.F32, x, w, st, pd)
    R = oracle.conv2d_nhwc(x, w, stride=st, pad=pd, with_s=False)
    assert y.shape == R.shape
    assert np.array_equal(y.astype(np.float64), R)


@pytest.mark.parametrize("geom", CONV_GEOMS[1:5])
def test_conv_random_and_flags(geom):
    N, H, W, Cin, Cout, KH, KW, st, pd = geom
    x, w = synth.conv_inputs(N, H, W, Cin, Cout, KH, KW, seed=78)
    R, S = oracle.conv2d_nhwc(x, w, stride=st, pad=pd)
    y = run_conv(tsg.F32, x, w, st, pd)
    nw, cw = oracle.errors(y, R, S)
    assert nw <= 1e-4 and cw <= 1e-4
    yn = run_conv(tsg.F32, x, w, st, pd, flags=tsg.NEGATE)
    assert np.array_equal(yn.view(np.uint32), y.view(np.uint32) ^ np.uint32(0x80000000))
    y0 = synth.uniform_pm1(3, 9, R.size).reshape(R.shape)
    ya = run_conv(tsg.F32, x, w, st, pd, flags=tsg.ACCUMULATE, y0=y0)
    nw, cw = oracle.errors(ya, oracle.epilogue(R, oracle.ACCUMULATE, y0), S + np.abs(y0))
    assert nw <= 1e-4 and cw <= 1e-4


def test_conv_every_config_and_zero_pad_identity(workspace):
    """All instantiated configs on one geometry; and conv(x, pad 1) == conv(padded x, pad 0)
    bitwise for the same config (padding taps contribute exact zeros in any order)."""
    N, H, W, Cin, Cout = 2, 10, 9, 16, 24
    x, w = synth.conv_inputs(N, H, W, Cin, Cout, 3, 3, seed=79, dist="ints")
    R = oracle.conv2d_nhwc(x, w, pad=(1, 1), with_s=False)
    xp = np.zeros((N, H + 2, W + 2, Cin), np.float32); xp[:, 1:-1, 1:-1] = x
    op, dt = tsg.OP_CONV2D_NHWC, tsg.F32
    for i in range(tsg.tile_config_count(op, dt)):
        c = tsg.tile_config_enum(op, dt, i)
        if tsg.tile_config_check(op, dt, N * H * W, Cout, 9 * Cin, c, contig=Cin) != tsg.OK:
            # illegal here: a split beyond the number of k steps, scalar access in a direct-to-LDS form
            assert c.split_k > 1 or (c.vec == 1 and c.sched >= 4) or c.sched == 1   # (the block form takes matrices only)
            continue
        tsg.tile_config_set(op, dt, c)
        y = run_conv(dt, x, w, (1, 1), (1, 1), flags=tsg.STRICT)
        assert tsg.last_launch().config.as_dict() == c.as_dict()
        assert np.array_equal(y.astype(np.float64), R), c
        yp = run_conv(dt, xp, w, (1, 1), (0, 0), flags=tsg.STRICT)
        assert np.array_equal(yp, y)


def test_conv_all_ones_counts_valid_taps_on_device():
    x = np.ones((2, 12, 12, 64), np.float32)
    w = np.ones((3, 3, 64, 64), np.float32)
    y = run_conv(tsg.F32, x, w, (1, 1), (1, 1))
    assert np.all(y[:, 0, 0] == 256) and np.all(y[:, 0, 1:-1] == 384) and np.all(y[:, 1:-1, 1:-1] == 576)


def test_gemm_accumulated_into_window_of_zero_padded_tensor():
    """Case Study 3, add of zero pad: C_big += pad0(A.B) without forming the padded product.
    The window is addressed through C and ldc; elements outside it keep their bits."""
    M, N, K, r0, c0 = 100, 72, 130, 3, 5
    A, B = inputs(M, N, K, 41, "ints", False, tsg.F32)
    big = synth.small_ints(42, 2, (M + 7) * (N + 9)).reshape(M + 7, N + 9)
    d_big = dev(big)
    ld = N + 9
    win = d_big.data_ptr() + 4 * (r0 * ld + c0)
    tsg.gemm(tsg.F32, M, N, K, dev(A), K, dev(B), N, win, ld, tsg.ACCUMULATE)
    torch.cuda.synchronize()
    want = oracle.add_of_zero_pad(big, oracle.gemm(A, B, with_s=False), (r0, c0))
    assert np.array_equal(d_big.cpu().numpy().astype(np.float64), want)


@pytest.mark.parametrize("dtype", [tsg.F32, tsg.BF16_F32ACC])
def test_conv_into_window_of_larger_nhwc_tensor(dtype):
    """The convolution result lands in (or is added to) a spatial and channel window of a
    larger NHWC tensor; everything outside the window is untouched."""
    N, H, W, Cin, Cout = 2, 9, 11, 8, 12
    x, w = synth.conv_inputs(N, H, W, Cin, Cout, 3, 3, seed=43, dist="ints")
    if dtype == tsg.BF16_F32ACC:
        x, w = synth.f32_to_bf16_bits(x), synth.f32_to_bf16_bits(w)
    R = oracle.conv2d_nhwc(x, w, pad=(1, 1), with_s=False)
    Ho, Wo = R.shape[1], R.shape[2]
    a, b, c0, Cbig = 2, 3, 4, Cout + 7
    big = synth.small_ints(44, 2, N * (Ho + 5) * (Wo + 4) * Cbig).reshape(N, Ho + 5, Wo + 4, Cbig)
    sw, sh, sn = Cbig, (Wo + 4) * Cbig, (Ho + 5) * (Wo + 4) * Cbig
    for flags, want in ((tsg.ACCUMULATE, oracle.add_of_zero_pad(big, R, (0, a, b, c0))),
                        (tsg.ACCUMULATE | tsg.NEGATE, oracle.add_of_zero_pad(big, R, (0, a, b, c0), sign=-1))):
        d_big = dev(big)
        win = d_big.data_ptr() + 4 * (a * sh + b * sw + c0)
        tsg.conv2d_nhwc_window(dtype, N, H, W, Cin, Cout, 3, 3, 1, 1, 1, 1, dev(x), dev(w), win, sn, sh, sw, flags)
        torch.cuda.synchronize()
        assert np.array_equal(d_big.cpu().numpy().astype(np.float64), want)
    # overwrite form: the window takes the result, the rest keeps its bits
    d_big = dev(big)
    win = d_big.data_ptr() + 4 * (a * sh + b * sw + c0)
    tsg.conv2d_nhwc_window(dtype, N, H, W, Cin, Cout, 3, 3, 1, 1, 1, 1, dev(x), dev(w), win, sn, sh, sw, 0)
    torch.cuda.synchronize()
    want = big.astype(np.float64).copy()
    want[:, a:a + Ho, b:b + Wo, c0:c0 + Cout] = R
    assert np.array_equal(d_big.cpu().numpy().astype(np.float64), want)
    # overlapping pixels are a definite error
    with pytest.raises(tsg.TsgError) as e:
        tsg.conv2d_nhwc_window(dtype, N, H, W, Cin, Cout, 3, 3, 1, 1, 1, 1, dev(x), dev(w), win, sn, sh, Cout - 1, 0)
    assert e.value.status == tsg.E_INVALID


@pytest.mark.parametrize("dtype", [tsg.F32, tsg.BF16_F32ACC])
@pytest.mark.parametrize("trans_a", [False, True])
def test_transposed_right_operand_bit_exact(dtype, trans_a, workspace):
    """op(B) = B^T read in place (B stored N x K), alone and with a transposed A: integer
    inputs on ragged shapes and odd leading dimensions, the library's default config, every
    direct-to-LDS config pinned (with and without a split of k), and the flags."""
    op = tsg.OP_GEMM_TRANSA if trans_a else tsg.OP_GEMM
    for (M, N, K) in [(1, 1, 1), (5, 3, 2), (65, 63, 33), (196, 130, 461), (256, 384, 512), (130, 70, 2305)]:
        A, _ = inputs(M, N, K, 81, "ints", trans_a, dtype)
        Bt = inputs(N, 1, K, 82, "ints", False, dtype)[0]           # N x K
        R = oracle.gemm(A, Bt, trans_a=trans_a, trans_b=True, with_s=False)
        C0 = synth.small_ints(83, 2, M * N).reshape(M, N)
        acols = A.shape[1]
        for pad in (0, 1):
            lda, ldb, ldc = acols + pad, K + 3 * pad, N + pad
            Ah = np.zeros((A.shape[0], lda), A.dtype); Ah[:, :acols] = A
            Bh = np.zeros((N, ldb), Bt.dtype); Bh[:, :K] = Bt
            Ch = np.full((M, ldc), np.float32(-9.0)); Ch[:, :N] = C0
            dC = dev(Ch)
            tsg.gemm_trans(dtype, trans_a, True, 1, M, N, K, dev(Ah), lda, 0, dev(Bh), ldb, 0, dC, ldc, 0,
                           tsg.ACCUMULATE | tsg.NEGATE)
            torch.cuda.synchronize()
            out = dC.cpu().numpy()
            assert np.array_equal(out[:, :N].astype(np.float64), C0 - R), (M, N, K, pad)
            assert np.all(out[:, N:] == np.float32(-9.0))
            assert tsg.last_launch().config.sched != 0   # (the register-staged form has no transposed B)
    M, N, K = 196, 130, 461
    A, _ = inputs(M, N, K, 84, "ints", trans_a, dtype)
    Bt = inputs(N, 1, K, 85, "ints", False, dtype)[0]
    R = oracle.gemm(A, Bt, trans_a=trans_a, trans_b=True, with_s=False)
    dA, dB = dev(A), dev(Bt)
    seen = 0
    for i in range(tsg.tile_config_count(op, dtype)):
        c = tsg.tile_config_enum(op, dtype, i)
        if c.sched == 0 or c.vec == 1 or tsg.tile_config_check(op, dtype, M, N, K, c) != tsg.OK:
            continue
        tsg.tile_config_set(op, dtype, c)
        dC = torch.zeros((M, N), dtype=torch.float32, device=DEV)
        tsg.gemm_trans(dtype, trans_a, True, 1, M, N, K, dA, A.shape[1], 0, dB, K, 0, dC, N, 0, tsg.STRICT)
        torch.cuda.synchronize()
        assert tsg.last_launch().config.as_dict() == c.as_dict()
        assert np.array_equal(dC.cpu().numpy().astype(np.float64), R), c
        seen += 1
    assert seen >= 8
    # a pinned register-staged config cannot serve a transposed B: silenceable under STRICT,
    # the library's own choice otherwise
    tsg.tile_config_set(op, dtype, tsg.TileConfig(bm=64, bn=64, bk=64, wm=32, wn=32, vec=(4 if dtype == tsg.F32 else 8),
                                                  raster=0, sched=0, split_k=1))
    dC = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    with pytest.raises(tsg.SilenceableError):
        tsg.gemm_trans(dtype, trans_a, True, 1, M, N, K, dA, A.shape[1], 0, dB, K, 0, dC, N, 0, tsg.STRICT)
    tsg.gemm_trans(dtype, trans_a, True, 1, M, N, K, dA, A.shape[1], 0, dB, K, 0, dC, N, 0, 0)
    torch.cuda.synchronize()
    assert tsg.last_launch().alternative == 1
    assert np.array_equal(dC.cpu().numpy().astype(np.float64), R)


def test_transposed_right_operand_random_and_batched():
    M, N, K, nb = 300, 200, 700, 3
    for dtype in (tsg.F32, tsg.BF16_F32ACC):
        a = [inputs(M, 1, K, 90 + b, "uniform", False, dtype)[0] for b in range(nb)]
        bt = [inputs(N, 1, K, 95 + b, "uniform", False, dtype)[0] for b in range(nb)]
        dA, dB = dev(np.stack(a)), dev(np.stack(bt))
        dC = torch.zeros((nb, M, N), dtype=torch.float32, device=DEV)
        tsg.gemm_trans(dtype, False, True, nb, M, N, K, dA, K, M * K, dB, K, N * K, dC, N, M * N, 0)
        torch.cuda.synchronize()
        out = dC.cpu().numpy()
        for b in range(nb):
            R, S = oracle.gemm(a[b], bt[b], trans_b=True)
            nw, cw = oracle.errors(out[b], R, S)
            assert nw <= TOL[dtype] and cw <= TOL[dtype], (dtype, b, nw, cw)


# ------------------------------------------------------------------ the five workloads

def test_config1_gemm_256():
    c, A, B = synth.config_inputs(1)
    C = run_gemm(tsg.F32, A, B)
    R, S = oracle.gemm(A, B)
    gate("config 1", C, R, S, 1e-4)
    Ca = run_gemm(tsg.F32, A, B, flags=tsg.ACCUMULATE, C0=np.zeros((256, 256), np.float32))
    assert np.array_equal(C, Ca)


def test_config2_gemm_transA_1024():
    c, A, B = synth.config_inputs(2)
    C = run_gemm(tsg.F32, A, B, trans_a=True)
    R, S = oracle.gemm(A, B, trans_a=True)
    gate("config 2", C, R, S, 1e-4)
    # the folded transpose against the materialised one (the arithmetic order may differ
    # between operand layouts, so both are compared through the oracle bound)
    C2 = run_gemm(tsg.F32, np.ascontiguousarray(A.T), B)
    gate("config 2, A^T materialised", C2, R, S, 1e-4)


def test_config3_gemm_4096_full_oracle():
    """The headline workload, every element of C against the oracle on the workload's own data;
    all-ones; and integer-valued operands at full size, bit for bit against the oracle."""
    c, A, B = synth.config_inputs(3)
    C = run_gemm(tsg.F32, A, B)
    li = tsg.last_launch()
    assert li.edge == 0 and li.alternative == 1
    R, S = oracle.gemm(A, B)
    gate("config 3 (all 4096 x 4096 elements)", C, R, S, 1e-4)
    del R, S
    ones = np.ones((4096, 4096), np.float32)
    assert np.all(run_gemm(tsg.F32, ones, ones) == 4096.0)
    Ai, Bi = synth.gemm_inputs(4096, 4096, 4096, seed=2, dist="ints")
    Ci = run_gemm(tsg.F32, Ai, Bi)
    assert np.array_equal(Ci.astype(np.float64), oracle.gemm(Ai, Bi, with_s=False))


def test_config4_conv_resnet_layer():
    c, x, w = synth.config_inputs(4)
    y = run_conv(tsg.F32, x, w, (1, 1), (1, 1))
    li = tsg.last_launch()
    assert li.tiles_m * li.config.bm >= 25088 and li.k_main == 576
    R, S = oracle.conv2d_nhwc(x, w, pad=(1, 1))
    gate("config 4", y, R, S, 1e-4)


def test_config4_conv_tail_only_split_full_size(workspace):
    """The launch shape the tuner settles on for this layer: 392 tiles of 64 x 64, the 136 past
    the first round of 256 split four ways.  Integer data at full size, bit for bit; then the
    workload's own data within tolerance, and equal bits on a second call."""
    c, x, w = synth.config_inputs(4)
    op, dt = tsg.OP_CONV2D_NHWC, tsg.F32
    cfg = tsg.TileConfig(bm=64, bn=64, bk=32, wm=32, wn=32, vec=4, raster=1, sched=4, split_k=4, split_tail=1)
    assert tsg.tile_config_check(op, dt, 25088, 64, 576, cfg, contig=64) == tsg.OK
    assert tsg.workspace_bytes(dt, 1, 25088, 64, cfg) == 65536 + 136 * 4 * 64 * 64 * 4
    tsg.tile_config_set(op, dt, cfg)
    xi, wi = synth.conv_inputs(8, 56, 56, 64, 64, 3, 3, seed=5, dist="ints")
    yi = run_conv(dt, xi, wi, (1, 1), (1, 1), flags=tsg.STRICT)
    li = tsg.last_launch()
    assert li.alternative == 0 and li.config.split_tail == 1 and li.tiles_m == 392
    assert np.array_equal(yi.astype(np.float64), oracle.conv2d_nhwc(xi, wi, pad=(1, 1), with_s=False))
    y = run_conv(dt, x, w, (1, 1), (1, 1), flags=tsg.STRICT)
    R, S = oracle.conv2d_nhwc(x, w, pad=(1, 1))
    nw, cw = oracle.errors(y, R, S)
    assert nw <= 1e-4 and cw <= 1e-4, (nw, cw)
    y2 = run_conv(dt, x, w, (1, 1), (1, 1), flags=tsg.STRICT)
    assert np.array_equal(y2.view(np.uint32), y.view(np.uint32))


def test_bench_launch_configurations_of_the_small_workloads_full_size(workspace):
    """The tile configs the tuner settles on for the layer and for the paper's batched nest, pinned,
    at full size: 112-row tiles of 16 x 16 MFMA blocks with a k step of 64 for the layer (plain, and
    added into the interior of a larger tensor), 64 x 64 tiles with k split five ways for the batch.
    Integer data bit for bit, then the workload's own data within tolerance."""
    dt = tsg.F32
    conv_cfg = tsg.TileConfig(bm=112, bn=64, bk=64, wm=112, wn=16, vec=4, raster=0, sched=4, split_k=1, split_tail=0, mfma=1)
    assert tsg.tile_config_check(tsg.OP_CONV2D_NHWC, dt, 25088, 64, 576, conv_cfg, contig=64) == tsg.OK
    tsg.tile_config_set(tsg.OP_CONV2D_NHWC, dt, conv_cfg)
    xi, wi = synth.conv_inputs(8, 56, 56, 64, 64, 3, 3, seed=6, dist="ints")
    Ri = oracle.conv2d_nhwc(xi, wi, pad=(1, 1), with_s=False)
    yi = run_conv(dt, xi, wi, (1, 1), (1, 1), flags=tsg.STRICT)
    li = tsg.last_launch()
    assert li.alternative == 0 and li.config.mfma == 1 and li.tiles_m == 224 and li.edge == 0
    assert np.array_equal(yi.astype(np.float64), Ri)
    c, x, w = synth.config_inputs(4)
    R, S = oracle.conv2d_nhwc(x, w, pad=(1, 1))
    gate("config 4, tuned tile", run_conv(dt, x, w, (1, 1), (1, 1), flags=tsg.STRICT), R, S, 1e-4)
    # the same tile adding into a window (workload 10): integers exact everywhere, ring untouched
    ring, Ho, Co = 2, 56, 64
    big0 = synth.small_ints(14, 3, 8 * (Ho + 2 * ring) ** 2 * Co).reshape(8, Ho + 2 * ring, Ho + 2 * ring, Co)
    dbig = dev(big0)
    sw_, sh_ = Co, (Ho + 2 * ring) * Co
    sn_ = (Ho + 2 * ring) * sh_
    tsg.conv2d_nhwc_window(dt, 8, 56, 56, 64, 64, 3, 3, 1, 1, 1, 1, dev(xi), dev(wi),
                           dbig.data_ptr() + 4 * (ring * sh_ + ring * sw_), sn_, sh_, sw_, tsg.ACCUMULATE | tsg.STRICT)
    torch.cuda.synchronize()
    assert tsg.last_launch().config.as_dict() == conv_cfg.as_dict()
    assert np.array_equal(dbig.cpu().numpy().astype(np.float64), oracle.add_of_zero_pad(big0, Ri, (0, ring, ring, 0)))
    tsg.tile_config_set(tsg.OP_CONV2D_NHWC, dt, None)
    # the paper's batched nest, k split five ways
    P = synth.PAPER_BATCH_MATMUL
    Bt, M, N, K = P["B"], P["M"], P["N"], P["K"]
    gemm_cfg = tsg.TileConfig(bm=64, bn=64, bk=32, wm=32, wn=32, vec=4, raster=0, sched=4, split_k=5, split_tail=0)
    tsg.tile_config_set(tsg.OP_GEMM, dt, gemm_cfg)
    for dist, exact in (("ints", True), ("uniform", False)):
        A = np.stack([synth.gemm_inputs(M, N, K, seed=70 + b, dist=dist)[0] for b in range(Bt)])
        B = np.stack([synth.gemm_inputs(M, N, K, seed=70 + b, dist=dist)[1] for b in range(Bt)])
        dC = torch.full((Bt, M, N), 9.0, dtype=torch.float32, device=DEV)
        tsg.gemm_batched(dt, False, Bt, M, N, K, dev(A), K, M * K, dev(B), N, K * N, dC, N, M * N, tsg.STRICT)
        torch.cuda.synchronize()
        assert tsg.last_launch().config.split_k == 5
        C = dC.cpu().numpy()
        for b in range(Bt):
            check(C[b], A[b], B[b], dt, exact=exact)


def test_bench_launch_configurations_of_configs_1_2_and_8_full_size():
    """The other tile configs the tuner settles on, pinned, at the workloads' full sizes: the
    16 x 16 block form for 256^3 (either raster), 64 x 64 tiles with a k step of 64 (three stages)
    or 32 (four stages) for A^T B at 1024^3, and the 64 x 64 x 64 bf16 tile for the bf16 layer.
    Integer data bit for bit, then the workload's own data within tolerance."""
    dt = tsg.F32
    for raster in (0, 1):
        cfg = tsg.TileConfig(bm=16, bn=16, bk=64, wm=16, wn=16, vec=4, raster=raster, sched=1, split_k=1, split_tail=0, mfma=1)
        tsg.tile_config_set(tsg.OP_GEMM, dt, cfg)
        Ai, Bi = synth.gemm_inputs(256, 256, 256, seed=0, dist="ints")
        Ci = run_gemm(dt, Ai, Bi, flags=tsg.STRICT)
        assert tsg.last_launch().config.as_dict() == cfg.as_dict() and tsg.last_launch().edge == 0
        check(Ci, Ai, Bi, dt, exact=True)
        c, A, B = synth.config_inputs(1)
        R, S = oracle.gemm(A, B)
        gate("config 1, block form, raster %d" % raster, run_gemm(dt, A, B, flags=tsg.STRICT), R, S, TOL[dt])
    tsg.tile_config_set(tsg.OP_GEMM, dt, None)
    for bk, sched in ((64, 4), (32, 5)):
        cfg = tsg.TileConfig(bm=64, bn=64, bk=bk, wm=32, wn=32, vec=4, raster=1, sched=sched, split_k=1, split_tail=0)
        tsg.tile_config_set(tsg.OP_GEMM_TRANSA, dt, cfg)
        Ai, Bi = synth.gemm_inputs(1024, 1024, 1024, seed=1, dist="ints", trans_a=True)
        Ci = run_gemm(dt, Ai, Bi, trans_a=True, flags=tsg.STRICT)
        assert tsg.last_launch().config.as_dict() == cfg.as_dict()
        check(Ci, Ai, Bi, dt, trans_a=True, exact=True)
        c, A, B = synth.config_inputs(2)
        R, S = oracle.gemm(A, B, trans_a=True)
        gate("config 2, 64 x 64 x %d" % bk, run_gemm(dt, A, B, trans_a=True, flags=tsg.STRICT), R, S, TOL[dt])
    tsg.tile_config_set(tsg.OP_GEMM_TRANSA, dt, None)
    bt = tsg.BF16_F32ACC
    cfg = tsg.TileConfig(bm=64, bn=64, bk=64, wm=32, wn=32, vec=8, raster=0, sched=4, split_k=1, split_tail=0)
    tsg.tile_config_set(tsg.OP_CONV2D_NHWC, bt, cfg)
    xi, wi = synth.conv_inputs(8, 56, 56, 64, 64, 3, 3, seed=8, dist="ints")
    xb, wb = synth.f32_to_bf16_bits(xi), synth.f32_to_bf16_bits(wi)
    yi = run_conv(bt, xb, wb, (1, 1), (1, 1), flags=tsg.STRICT)
    assert tsg.last_launch().config.as_dict() == cfg.as_dict()
    assert np.array_equal(yi.astype(np.float64), oracle.conv2d_nhwc(xb, wb, pad=(1, 1), with_s=False))
    c, x, w = synth.config_inputs(8)
    R, S = oracle.conv2d_nhwc(x, w, pad=(1, 1))
    gate("config 8, tuned tile", run_conv(bt, x, w, (1, 1), (1, 1), flags=tsg.STRICT), R, S, TOL[bt])


def test_config5_bf16_gemm_8192_negated_full_oracle():
    """bf16 8192^3 with the negate fused: every element against the oracle on the workload's own
    data; integer-valued operands at full size, bit for bit (any indexing, swizzle or
    synchronisation mistake shows as such); all-ones."""
    dt = tsg.BF16_F32ACC
    c, A, B = synth.config_inputs(5)
    C = run_gemm(dt, A, B, flags=tsg.NEGATE)
    li = tsg.last_launch()
    assert li.edge == 0 and li.alternative == 1
    R, S = oracle.gemm(A, B)
    gate("config 5 (all 8192 x 8192 elements)", C, -R, S, TOL[dt])
    del C, R, S
    Ai, Bi = synth.gemm_inputs(8192, 8192, 8192, seed=4, dist="ints", bf16=True)
    Ci = run_gemm(dt, Ai, Bi, flags=tsg.NEGATE)
    ref = oracle.gemm(Ai, Bi, with_s=False)
    assert np.array_equal(Ci.astype(np.float64), -ref)
    del Ci, ref, Ai, Bi
    ones = np.full((8192, 8192), 0x3F80, np.uint16)
    assert np.all(run_gemm(dt, ones, ones, flags=tsg.NEGATE) == -8192.0)


# ------------------------------------------------------------------ search

def test_config8_bf16_conv_resnet_layer():
    """The layer of workload 4 with bfloat16 operands (rounded once on the host; the oracle
    multiplies the same rounded values in fp64)."""
    c, x, w = synth.config_inputs(8)
    assert x.dtype == np.uint16 and w.dtype == np.uint16
    y = run_conv(tsg.BF16_F32ACC, x, w, (1, 1), (1, 1))
    assert tsg.last_launch().config.vec == 8
    R, S = oracle.conv2d_nhwc(x, w, pad=(1, 1))
    gate("config 8", y, R, S, TOL[tsg.BF16_F32ACC])


def test_config9_both_operands_transposed_4096_full_oracle():
    """A stored K x M and B stored N x K at 4096^3.  Every element against the oracle's triple
    loop, which is handed a host copy of B laid out K x N (moving bytes, no arithmetic); sampled
    rows and columns against the oracle's own loop for a right operand read transposed in place;
    integer-valued operands at full size, bit for bit; all-ones."""
    c, A, Bt = synth.config_inputs(9)
    M = N = K = 4096
    dA, dB = dev(A), dev(Bt)
    dC = torch.full((M, N), -3.0, dtype=torch.float32, device=DEV)
    tsg.gemm_trans(tsg.F32, True, True, 1, M, N, K, dA, M, 0, dB, K, 0, dC, N, 0, 0)
    torch.cuda.synchronize()
    li = tsg.last_launch()
    assert li.config.sched >= 4 and li.edge == 0
    C = dC.cpu().numpy()
    R, S = oracle.gemm(A, np.ascontiguousarray(Bt.T), trans_a=True)
    gate("config 9 (all 4096 x 4096 elements)", C, R, S, 1e-4)
    rows = [0, 1, 255, 256, 2047, 4095]
    Rr, Sr = oracle.gemm(np.ascontiguousarray(A[:, rows]), Bt, trans_a=True, trans_b=True)
    gate("config 9, rows through the in-place loop", C[rows], Rr, Sr, 1e-4)
    assert np.max(np.abs(Rr - R[rows])) <= K * 2.0 ** -52 * np.max(Sr)     # the two oracle routes agree
    cols = [0, 63, 64, 4095]
    Rc, Sc = oracle.gemm(A, np.ascontiguousarray(Bt[cols]), trans_a=True, trans_b=True)
    gate("config 9, columns through the in-place loop", C[:, cols], Rc, Sc, 1e-4)
    del R, S
    Ai, Bi = synth.gemm_inputs(M, N, K, seed=8, dist="ints", trans_a=True)
    Bti = np.ascontiguousarray(Bi.T)                                      # N x K
    tsg.gemm_trans(tsg.F32, True, True, 1, M, N, K, dev(Ai), M, 0, dev(Bti), K, 0, dC, N, 0, 0)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy().astype(np.float64), oracle.gemm(Ai, Bi, trans_a=True, with_s=False))
    ones = torch.ones((K, M), dtype=torch.float32, device=DEV)
    tsg.gemm_trans(tsg.F32, True, True, 1, M, N, K, ones, M, 0, ones, K, 0, dC, N, 0, 0)
    torch.cuda.synchronize()
    assert bool((dC == float(K)).all())


def test_config10_conv_added_into_interior_full_size(workspace):
    """Workload 10: the layer's result added into the interior of a tensor with a ring of two
    pixels, the padded tensor never formed.  Against the oracle's explicit pad-then-add;
    the ring must keep its bits."""
    c, x, w = synth.config_inputs(10)
    ring = c["window_ring"]
    Nn, Ho, Co = 8, 56, 64
    big0 = synth.uniform_pm1(12, 3, Nn * (Ho + 2 * ring) ** 2 * Co).reshape(Nn, Ho + 2 * ring, Ho + 2 * ring, Co)
    dbig = dev(big0)
    sw_ = Co
    sh_ = (Ho + 2 * ring) * sw_
    sn_ = (Ho + 2 * ring) * sh_
    tsg.conv2d_nhwc_window(tsg.F32, 8, 56, 56, 64, 64, 3, 3, 1, 1, 1, 1, dev(x), dev(w),
                           dbig.data_ptr() + 4 * (ring * sh_ + ring * sw_), sn_, sh_, sw_, tsg.ACCUMULATE)
    torch.cuda.synchronize()
    out = dbig.cpu().numpy()
    R, S = oracle.conv2d_nhwc(x, w, pad=(1, 1))
    ref = oracle.add_of_zero_pad(big0, R, (0, ring, ring, 0))
    inner = (slice(None), slice(ring, ring + Ho), slice(ring, ring + Ho), slice(None))
    gate("config 10", out[inner], ref[inner], S + np.abs(big0[inner]), 1e-4)
    mask = np.ones(big0.shape, bool); mask[inner] = False
    assert np.array_equal(out[mask].view(np.uint32), big0[mask].view(np.uint32))


def test_autotune_pins_the_fastest_legal_config():
    M, N, K = 512, 384, 256
    A, B = inputs(M, N, K, 8, "ints", False, tsg.F32)
    dA, dB = dev(A), dev(B)
    dC = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    best, ms, log = tsg.autotune_gemm(tsg.F32, False, M, N, K, dA, K, dB, N, dC, N, iters=3)
    assert len(log) == tsg.tile_config_count(tsg.OP_GEMM, tsg.F32)
    timed = [r for r in log if r.ms >= 0]
    # the pinned point is the fastest up to the tie margin (an earlier point keeps a tie)
    assert timed and min(r.ms for r in timed) <= ms <= min(r.ms for r in timed) / 0.995 + 1e-6
    bests = [r.best_ms for r in log if r.best_ms >= 0]
    assert all(a >= b for a, b in zip(bests, bests[1:]))          # best-so-far curve (Fig. 11)
    # the result is remembered for this problem only: other extents still get the default
    assert tsg.tile_config_get(tsg.OP_GEMM, tsg.F32, M, N, K).as_dict() == best.as_dict()
    other = tsg.tile_config_get(tsg.OP_GEMM, tsg.F32, M + 1, N, K)
    tsg.tune_cache_clear()
    assert tsg.tile_config_get(tsg.OP_GEMM, tsg.F32, M + 1, N, K).as_dict() == other.as_dict()
    tsg.autotune_gemm(tsg.F32, False, M, N, K, dA, K, dB, N, dC, N, iters=3)
    tsg.gemm(tsg.F32, M, N, K, dA, K, dB, N, dC, N, tsg.STRICT)
    torch.cuda.synchronize()
    assert tsg.last_launch().alternative == 0
    assert np.array_equal(dC.cpu().numpy().astype(np.float64), oracle.gemm(A, B, with_s=False))


def test_search_budget_and_model_order():
    """Case Study 5: the tuner visits the points in the order of the cost model, so its first
    timed point is the config a call without tuning uses, and it stops at the budget."""
    M, N, K = 384, 320, 512
    A, B = inputs(M, N, K, 12, "ints", False, tsg.F32)
    dA, dB = dev(A), dev(B)
    dC = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    default = tsg.tile_config_get(tsg.OP_GEMM, tsg.F32, M, N, K)
    try:
        tsg.search_set(6, True)
        best, ms, log = tsg.autotune_gemm(tsg.F32, False, M, N, K, dA, K, dB, N, dC, N, iters=3)
        timed = [r for r in log if r.ms >= 0]
        assert len(timed) == 6
        first = timed[0].config.as_dict()
        want = default.as_dict()
        assert {k: first[k] for k in ("bm", "bn", "bk", "wm", "wn", "sched", "split_k", "vec")} == \
               {k: want[k] for k in ("bm", "bn", "bk", "wm", "wn", "sched", "split_k", "vec")}
        preds = [r.predicted_ms for r in log]
        assert all(a <= b for a, b in zip(preds, preds[1:]))
        assert best.as_dict() in [r.config.as_dict() for r in timed]
    finally:
        tsg.search_set(0, True)
    tsg.gemm(tsg.F32, M, N, K, dA, K, dB, N, dC, N, tsg.STRICT)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy().astype(np.float64), oracle.gemm(A, B, with_s=False))


def test_search_adaptive_order_and_pruned_points_are_told_apart(workspace):
    """Model-based order (2): the first timed point is still the cost model's pick, every
    visited point is visited once, the winner is a timed point and a tuned call is exact.  In
    the log a point that was not timed says why: -1 illegal here, -2 pruned."""
    M, N, K = 384, 320, 512
    A, B = inputs(M, N, K, 13, "ints", False, tsg.F32)
    dA, dB = dev(A), dev(B)
    dC = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    try:
        tsg.search_set(0, 1)
        best1, ms1, log1 = tsg.autotune_gemm(tsg.F32, False, M, N, K, dA, K, dB, N, dC, N, iters=3, log_cap=2048)
        assert {round(r.ms) for r in log1 if r.ms < 0} <= {-1, -2}
        # scalar access in a direct-to-LDS form is illegal; nothing is pruned while the tiles cannot fill the chip
        assert any(r.ms == -1 and r.config.vec == 1 and r.config.sched >= 4 for r in log1)
        tsg.search_set(12, 2)
        best2, ms2, log2 = tsg.autotune_gemm(tsg.F32, False, M, N, K, dA, K, dB, N, dC, N, iters=3, log_cap=2048)
        timed = [r for r in log2 if r.ms >= 0]
        assert len(timed) == 12
        first1 = next(r for r in log1 if r.ms >= 0).config.as_dict()
        assert timed[0].config.as_dict() == first1
        keys = [tuple(r.config.as_dict().values()) for r in log2]
        assert len(keys) == len(set(keys))
        assert best2.as_dict() in [r.config.as_dict() for r in timed]
        assert ms2 <= timed[0].ms
        # 4096^2 outputs in 64 x 64 tiles fill the chip sixteen times over: splits of k are pruned there
        tsg.search_set(0, 1)
        a3 = torch.zeros((4096, 64), dtype=torch.float32, device=DEV)
        b3 = torch.zeros((64, 4096), dtype=torch.float32, device=DEV)
        c3 = torch.zeros((4096, 4096), dtype=torch.float32, device=DEV)
        _, _, log3 = tsg.autotune_gemm(tsg.F32, False, 4096, 4096, 64, a3, 64, b3, 4096, c3, 4096, iters=1, log_cap=2048)
        pruned = [r for r in log3 if r.ms == -2]
        assert pruned and all(r.config.split_k > 1 and not r.config.split_tail for r in pruned)
    finally:
        tsg.search_set(0, 1)
    tsg.gemm(tsg.F32, M, N, K, dA, K, dB, N, dC, N)
    torch.cuda.synchronize()
    assert np.array_equal(dC.cpu().numpy().astype(np.float64), oracle.gemm(A, B, with_s=False))


# ------------------------------------------------------------------ full additive reduce

REDUCE_TOL = 1e-5   # of the sum of magnitudes: ~100 sequential fp32 adds per partial sum at most


@pytest.mark.parametrize("dtype", [tsg.F32, tsg.BF16_F32ACC])
@pytest.mark.parametrize("with_ws", [False, True])
def test_reduce_sum_exact_on_integers_and_views(dtype, with_ws):
    """Integer inputs (every order exact): whole tensor, ragged sizes, a strided view, the
    flags; with the workspace (many workgroups) and without (one workgroup)."""
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=DEV) if with_ws else None
    tsg.workspace_set(ws)
    try:
        for n in (1, 3, 4, 5, 255, 256 * 16 * 4 + 3, 1 << 20, (1 << 21) + 7):
            x = synth.small_ints(50, 0, n)
            h = synth.f32_to_bf16_bits(x) if dtype == tsg.BF16_F32ACC else x
            out = torch.full((1,), 5.0, dtype=torch.float32, device=DEV)
            tsg.reduce_sum(dtype, 1, n, dev(h), n, out)
            torch.cuda.synchronize()
            assert float(out.item()) == oracle.reduce_sum(h)[0], n
            tsg.reduce_sum(dtype, 1, n, dev(h), n, out, tsg.ACCUMULATE | tsg.NEGATE)
            torch.cuda.synchronize()
            assert float(out.item()) == 0.0, n
        rows, cols, ld = 37, 1001, 1024
        x = synth.small_ints(51, 0, rows * ld).reshape(rows, ld)
        h = synth.f32_to_bf16_bits(x) if dtype == tsg.BF16_F32ACC else x
        out = torch.zeros((1,), dtype=torch.float32, device=DEV)
        tsg.reduce_sum(dtype, rows, cols, dev(h), ld, out)
        torch.cuda.synchronize()
        assert float(out.item()) == oracle.reduce_sum(np.ascontiguousarray(h[:, :cols]))[0]
    finally:
        tsg.workspace_set(None)


def test_reduce_sum_random_tolerance_repeatable_and_transpose_invariant(workspace):
    x = synth.normal_scaled(52, 0, 3000 * 1111, 1.0).reshape(3000, 1111)
    ref, mag = oracle.reduce_sum(x)
    outs = []
    for view in (x, np.ascontiguousarray(x.T), x.reshape(1111, 3000)):
        out = torch.zeros((1,), dtype=torch.float32, device=DEV)
        d = dev(view)
        for _ in range(2):
            tsg.reduce_sum(tsg.F32, view.shape[0], view.shape[1], d, view.shape[1], out)
            torch.cuda.synchronize()
            outs.append(float(out.item()))
        assert abs(outs[-1] - ref) <= REDUCE_TOL * mag
        assert outs[-1] == outs[-2]                     # repeatable
    # a reshape of contiguous memory is the same run of bytes: identical bits; the transposed
    # copy holds the elements in another order and agrees within the tolerance
    assert outs[0] == outs[4]
    # without the workspace a strict call has no alternative
    tsg.workspace_set(None)
    out = torch.zeros((1,), dtype=torch.float32, device=DEV)
    with pytest.raises(tsg.SilenceableError):
        tsg.reduce_sum(tsg.F32, 3000, 1111, dev(x), 1111, out, tsg.STRICT)


def test_reduce_sum_view_of_many_short_rows(workspace):
    """2^16 rows of 24 elements inside rows of 32: the workgroups' shares span rows, so the view
    fills the chip (integers: exact; random: within the bound; both repeatable), and so does a
    view whose rows end in a short chunk."""
    rows, cols, ld = 1 << 16, 24, 32
    for dtype in (tsg.F32, tsg.BF16_F32ACC):
        xi = synth.small_ints(61, 0, rows * ld).reshape(rows, ld)
        h = synth.f32_to_bf16_bits(xi) if dtype == tsg.BF16_F32ACC else xi
        out = torch.zeros((1,), dtype=torch.float32, device=DEV)
        tsg.reduce_sum(dtype, rows, cols, dev(h), ld, out, tsg.STRICT)
        torch.cuda.synchronize()
        assert float(out.item()) == oracle.reduce_sum(np.ascontiguousarray(h[:, :cols]))[0]
    x = synth.uniform_pm1(62, 0, rows * ld).reshape(rows, ld)
    d = dev(x)
    out = torch.zeros((1,), dtype=torch.float32, device=DEV)
    got = []
    for cols in (24, 23, 5):
        ref, mag = oracle.reduce_sum(np.ascontiguousarray(x[:, :cols]))
        for _ in range(2):
            tsg.reduce_sum(tsg.F32, rows, cols, d, ld, out, tsg.STRICT)
            torch.cuda.synchronize()
            got.append(float(out.item()))
        assert abs(got[-1] - ref) <= REDUCE_TOL * mag, (cols, got[-1], ref)
        assert got[-1] == got[-2]


def test_workload11_reduce_of_a_view_full_size(workspace):
    """The benchmark's strided-view reduce at full size, in its launch configuration."""
    c, x, _ = synth.config_inputs(11)
    ref, mag = oracle.reduce_sum(np.ascontiguousarray(x[:, :c["cols"]]))
    out = torch.zeros((1,), dtype=torch.float32, device=DEV)
    d = dev(x)
    tsg.reduce_sum(tsg.F32, c["rows"], c["cols"], d, c["ld"], out)
    torch.cuda.synchronize()
    assert abs(float(out.item()) - ref) <= REDUCE_TOL * mag
    d.fill_(1.0)
    tsg.reduce_sum(tsg.F32, c["rows"], c["cols"], d, c["ld"], out)
    torch.cuda.synchronize()
    assert float(out.item()) == float(c["rows"] * c["cols"])


def test_workload7_full_reduce_one_gib(workspace):
    """The benchmark's reduce workload at full size, in its launch configuration."""
    c, x, _ = synth.config_inputs(7)
    ref, mag = oracle.reduce_sum(x)
    out = torch.zeros((1,), dtype=torch.float32, device=DEV)
    d = dev(x)
    tsg.reduce_sum(tsg.F32, c["rows"], c["cols"], d, c["cols"], out)
    torch.cuda.synchronize()
    assert abs(float(out.item()) - ref) <= REDUCE_TOL * mag
    ones = torch.ones_like(d)
    tsg.reduce_sum(tsg.F32, c["rows"], c["cols"], ones, c["cols"], out)
    torch.cuda.synchronize()
    assert float(out.item()) == float(c["rows"] * c["cols"])     # 2^28: every partial sum is exact


# ------------------------------------------------------------------ seeded sweep of shapes

@pytest.mark.parametrize("blk,bk,mfma", [(16, 64, 1), (32, 32, 0)])
@pytest.mark.parametrize("trans_a,trans_b", [(False, False), (True, False), (False, True), (True, True)])
def test_block_form_every_layout_variant_and_flag(blk, bk, mfma, trans_a, trans_b):
    """sched 1 (one MFMA block per workgroup, k dealt over its four waves): both variants
    (divisible shape: wide unmasked loads; ragged shape and vec = 1: masked scalars), the four
    operand layouts, padded leading dimensions, batches, sign and accumulate, bit-exact on
    integers and within tolerance on uniform data."""
    op = tsg.OP_GEMM_TRANSA if trans_a else tsg.OP_GEMM
    dt = tsg.F32
    for (nb, M, N, K, vec, pad) in [(1, 256, 256, 256, 4, 0), (3, 64, 96, 192, 4, 5), (2, 50, 70, 203, 4, 3),
                                    (1, 33, 17, 7, 1, 1), (1, 16, 16, 1024, 4, 0), (2, 100, 36, 129, 1, 0)]:
        cfg = tsg.TileConfig(bm=blk, bn=blk, bk=bk, wm=blk, wn=blk, vec=vec, raster=(M + N) % 2, sched=1, split_k=1, mfma=mfma)
        tsg.tile_config_set(op, dt, cfg)
        for dist, flags in (("ints", 0), ("ints", tsg.NEGATE | tsg.ACCUMULATE), ("uniform", tsg.ACCUMULATE)):
            seed = 300 + M + N + K
            n_a, n_b = nb * M * K, nb * K * N
            gen = synth.small_ints if dist == "ints" else synth.uniform_pm1
            A = gen(seed, 0, n_a).reshape((nb, K, M) if trans_a else (nb, M, K))
            B = gen(seed, 1, n_b).reshape((nb, N, K) if trans_b else (nb, K, N))
            C0 = synth.small_ints(seed, 2, nb * M * N).reshape(nb, M, N)
            lda, ldb, ldc = A.shape[2] + pad, B.shape[2] + 2 * pad, N + pad
            Ah = np.zeros((nb, A.shape[1], lda), np.float32); Ah[:, :, :A.shape[2]] = A
            Bh = np.zeros((nb, B.shape[1], ldb), np.float32); Bh[:, :, :B.shape[2]] = B
            Ch = np.full((nb, M, ldc), np.float32(-7.0)); Ch[:, :, :N] = C0
            dC = dev(Ch)
            tsg.gemm_trans(dt, trans_a, trans_b, nb, M, N, K, dev(Ah), lda, A.shape[1] * lda, dev(Bh), ldb,
                           B.shape[1] * ldb, dC, ldc, M * ldc, flags | tsg.STRICT)
            torch.cuda.synchronize()
            li = tsg.last_launch()
            assert li.alternative == 0 and li.config.sched == 1 and li.config.bm == blk
            assert li.edge == int(bool(M % blk or N % blk or K % bk or vec == 1))
            out = dC.cpu().numpy()
            assert np.all(out[:, :, N:] == np.float32(-7.0))
            for b in range(nb):
                R, S = oracle.gemm(A[b], B[b], trans_a=trans_a, trans_b=trans_b)
                sign = -1.0 if flags & tsg.NEGATE else 1.0
                want = sign * R + (C0[b] if flags & tsg.ACCUMULATE else 0.0)
                if dist == "ints":
                    assert np.array_equal(out[b, :, :N].astype(np.float64), want), (nb, M, N, K, vec, flags)
                else:
                    err = np.abs(out[b, :, :N].astype(np.float64) - want)
                    assert np.max(err / np.maximum(S, 1e-30)) <= 1e-4 and np.max(err) <= 1e-4 * np.max(np.abs(want))
    # k split over workgroups does not exist in this form: silenceable under STRICT
    ws = torch.empty(16 << 20, dtype=torch.uint8, device=DEV)
    tsg.workspace_set(ws)
    try:
        cfg = tsg.TileConfig(bm=blk, bn=blk, bk=bk, wm=blk, wn=blk, vec=4, raster=0, sched=1, split_k=2, mfma=mfma)
        assert tsg.tile_config_check(op, dt, 256, 256, 256, cfg) == tsg.E_SILENCEABLE
        tsg.tile_config_set(op, dt, cfg)
        A = synth.small_ints(1, 0, 256 * 256).reshape(256, 256)
        dC = torch.zeros((256, 256), dtype=torch.float32, device=DEV)
        with pytest.raises(tsg.SilenceableError):
            tsg.gemm_trans(dt, trans_a, trans_b, 1, 256, 256, 256, dev(A), 256, 0, dev(A), 256, 0, dC, 256, 0, tsg.STRICT)
        torch.cuda.synchronize()
        assert not dC.any()
    finally:
        torch.cuda.synchronize()
        tsg.workspace_set(None)


def test_element_offsets_beyond_32_bits():
    """Maximum sizes: leading dimensions and batch strides so large that element offsets pass 2^31
    (and byte offsets 2^33) in every operand, for each kernel form; the operands live in sparse
    views of large device buffers and the result is exact on integers."""
    dt, op = tsg.F32, tsg.OP_GEMM
    M, N, K = 300, 200, 96
    lda, ldb, ldc = (1 << 23) + 1, (1 << 25) + 3, (1 << 23) + 5     # 299 * lda, 95 * ldb, 299 * ldc > 2^31
    A, B = synth.gemm_inputs(M, N, K, seed=91, dist="ints")
    R = oracle.gemm(A, B, with_s=False)
    bufA = torch.zeros((M - 1) * lda + K, dtype=torch.float32, device=DEV)
    bufB = torch.zeros((K - 1) * ldb + N, dtype=torch.float32, device=DEV)
    bufA.as_strided((M, K), (lda, 1)).copy_(torch.from_numpy(A))
    bufB.as_strided((K, N), (ldb, 1)).copy_(torch.from_numpy(B))
    configs = [tsg.TileConfig(bm=16, bn=16, bk=64, wm=16, wn=16, vec=4, raster=0, sched=1, split_k=1, mfma=1),
               tsg.TileConfig(bm=64, bn=64, bk=32, wm=32, wn=32, vec=4, raster=0, sched=4, split_k=1),
               tsg.TileConfig(bm=64, bn=64, bk=32, wm=32, wn=32, vec=4, raster=1, sched=0, split_k=1),
               tsg.TileConfig(bm=64, bn=64, bk=32, wm=32, wn=32, vec=1, raster=0, sched=0, split_k=1)]
    for cfg in configs:
        bufC = torch.full(((M - 1) * ldc + N,), -3.0, dtype=torch.float32, device=DEV)
        tsg.tile_config_set(op, dt, cfg)
        tsg.gemm(dt, M, N, K, bufA, lda, bufB, ldb, bufC, ldc, tsg.STRICT)
        torch.cuda.synchronize()
        assert tsg.last_launch().config.as_dict() == cfg.as_dict()
        out = bufC.as_strided((M, N), (ldc, 1)).cpu().numpy()
        assert np.array_equal(out.astype(np.float64), R), cfg
        # nothing between the rows was touched (a sample of the gaps: the rows' neighbours)
        gaps = bufC.as_strided((M - 1, 8), (ldc, 1), N).cpu().numpy()
        assert np.all(gaps == np.float32(-3.0))
        del bufC
    del bufA, bufB
    # batch strides beyond 2^31 elements, direct form with k split (the workspace is per batch entry)
    tsg.tile_config_set(op, dt, None)
    nb, M, N, K = 2, 70, 96, 260
    stride = (1 << 31) + 16
    A = synth.small_ints(92, 0, nb * M * K).reshape(nb, M, K)
    B = synth.small_ints(92, 1, nb * K * N).reshape(nb, K, N)
    bufA = torch.zeros(stride + M * K, dtype=torch.float32, device=DEV)
    bufB = torch.zeros(stride + K * N, dtype=torch.float32, device=DEV)
    bufC = torch.zeros(stride + M * N, dtype=torch.float32, device=DEV)
    for b in range(nb):
        bufA[b * stride:b * stride + M * K].copy_(torch.from_numpy(A[b]).reshape(-1))
        bufB[b * stride:b * stride + K * N].copy_(torch.from_numpy(B[b]).reshape(-1))
    ws = torch.empty(16 << 20, dtype=torch.uint8, device=DEV)
    tsg.workspace_set(ws)
    try:
        for cfg in (tsg.TileConfig(bm=64, bn=64, bk=32, wm=32, wn=32, vec=4, raster=0, sched=4, split_k=3),
                    tsg.TileConfig(bm=32, bn=32, bk=32, wm=32, wn=32, vec=4, raster=0, sched=1, split_k=1)):
            bufC.zero_()
            tsg.tile_config_set(op, dt, cfg)
            tsg.gemm_batched(dt, False, nb, M, N, K, bufA, K, stride, bufB, N, stride, bufC, N, stride, tsg.STRICT)
            torch.cuda.synchronize()
            assert tsg.last_launch().config.as_dict() == cfg.as_dict()
            for b in range(nb):
                out = bufC[b * stride:b * stride + M * N].reshape(M, N).cpu().numpy()
                assert np.array_equal(out.astype(np.float64), oracle.gemm(A[b], B[b], with_s=False)), (cfg, b)
        del bufA, bufB, bufC
        # the reduce over a view whose last row starts beyond 2^31 elements
        rows, cols, ld = 300, 96, (1 << 23) + 1
        x = synth.small_ints(93, 0, rows * cols).reshape(rows, cols)
        bufX = torch.zeros((rows - 1) * ld + cols, dtype=torch.float32, device=DEV)
        bufX.as_strided((rows, cols), (ld, 1)).copy_(torch.from_numpy(x))
        out = torch.zeros(1, dtype=torch.float32, device=DEV)
        tsg.reduce_sum(dt, rows, cols, bufX, ld, out)
        torch.cuda.synchronize()
        assert float(out.item()) == float(x.astype(np.float64).sum())
        del bufX
        # a convolution written into a window whose image stride is beyond 2^31 elements
        Nb, H, W, Cin, Cout = 2, 6, 6, 8, 16
        xi, wi = synth.conv_inputs(Nb, H, W, Cin, Cout, 3, 3, seed=94, dist="ints")
        Ry = oracle.conv2d_nhwc(xi, wi, pad=(1, 1), with_s=False)
        sw_, sh_, sn_ = Cout, 1 << 20, (1 << 31) + 64
        bufY = torch.full(((Nb - 1) * sn_ + (H - 1) * sh_ + W * sw_ + 8,), 5.0, dtype=torch.float32, device=DEV)
        tsg.conv2d_nhwc_window(dt, Nb, H, W, Cin, Cout, 3, 3, 1, 1, 1, 1, dev(xi), dev(wi), bufY, sn_, sh_, sw_, 0)
        torch.cuda.synchronize()
        got = bufY.as_strided((Nb, H, W, Cout), (sn_, sh_, sw_, 1)).cpu().numpy()
        assert np.array_equal(got.astype(np.float64), Ry)
        assert bool((bufY.as_strided((Nb, H, 8), (sn_, sh_, 1), W * sw_) == 5.0).all())
    finally:
        torch.cuda.synchronize()
        tsg.workspace_set(None)


def test_measurement_aids_return_plausible_figures_and_validate_arguments():
    """tsg_launch_floor and tsg_mfma_ceiling are measurement aids, not part of the path: they must
    reject bad arguments, run, and report figures below the published peaks."""
    us = tsg.launch_floor(2000)
    assert 0.2 < us < 100.0
    with pytest.raises(tsg.TsgError):
        tsg.launch_floor(0)
    sink = torch.empty(4 << 20, dtype=torch.uint8, device=DEV)
    for dt, peak in ((tsg.F32, 157.3), (tsg.BF16_F32ACC, 2500.0)):
        for mfma in (0, 1):
            best, sustained = tsg.mfma_ceiling(dt, mfma, 1, 1, 2, sink)
            assert 0.2 * peak < sustained <= best * 1.001 and best < 1.02 * peak, (dt, mfma, best, sustained)
    with pytest.raises(tsg.TsgError):
        tsg.mfma_ceiling(tsg.F32, 2, 0, 1, 2, sink)
    with pytest.raises(tsg.TsgError):
        tsg.mfma_ceiling(tsg.F32, 0, 0, 1, 2, torch.empty(1024, dtype=torch.uint8, device=DEV))


def test_seeded_sweep_of_ragged_shapes_all_entry_points(workspace):
    """Forty shapes drawn from a seeded generator (odd extents, odd leading dimensions, tiny
    and long k), each through a random entry point, dtype, flag set and, for half of them, a
    random pinned point of the search space: integer inputs, so every result must match the
    oracle bit for bit whatever tile, form or split served the call."""
    rng = np.random.default_rng(20240903)
    for case in range(40):
        dtype = tsg.F32 if rng.integers(2) == 0 else tsg.BF16_F32ACC
        trans = bool(rng.integers(2))
        M, N = int(rng.integers(1, 300)), int(rng.integers(1, 300))
        K = int(rng.choice([1, 2, 7, 33, 64, 100, 257, 1000, 2305]))
        flags = int(rng.choice([0, tsg.NEGATE, tsg.ACCUMULATE, tsg.NEGATE | tsg.ACCUMULATE]))
        op = tsg.OP_GEMM_TRANSA if trans else tsg.OP_GEMM
        A, B = inputs(M, N, K, 1000 + case, "ints", trans, dtype)
        C0 = synth.small_ints(2000 + case, 2, M * N).reshape(M, N)
        pinned = None
        if case % 2:
            for _ in range(50):
                c = tsg.tile_config_enum(op, dtype, int(rng.integers(tsg.tile_config_count(op, dtype))))
                if tsg.tile_config_check(op, dtype, M, N, K, c) == tsg.OK:
                    pinned = c
                    tsg.tile_config_set(op, dtype, c)
                    break
        acols = A.shape[1]
        C = run_gemm(dtype, A, B, trans_a=trans, flags=flags | (tsg.STRICT if pinned is not None else 0), C0=C0,
                     lda=acols + int(rng.integers(0, 4)), ldb=N + int(rng.integers(0, 4)),
                     ldc=N + int(rng.integers(0, 4)))
        R = oracle.gemm(A, B, trans_a=trans, with_s=False)
        want = oracle.epilogue(R, flags & 3, C0) if flags & tsg.ACCUMULATE else oracle.epilogue(R, flags & 3)
        assert np.array_equal(C.astype(np.float64), want), (case, dtype, trans, M, N, K, flags, pinned)
        tsg.tile_config_set(op, dtype, None)


def test_calls_recorded_into_a_hip_graph_replay_correctly(workspace):
    """Compute calls only enqueue kernels on the given stream (no memset, no synchronisation),
    so they can be recorded into a HIP graph: a graph of a plain GEMM, a split-k GEMM (arrival
    counters reset themselves) and a reduce is replayed several times, with eager work and
    synchronisations in between, and every replay must reproduce the eager result bit for bit."""
    M, N, K = 196, 256, 2305
    A, B = inputs(M, N, K, 61, "uniform", False, tsg.F32)
    dA, dB = dev(A), dev(B)
    tsg.tile_config_set(tsg.OP_GEMM, tsg.F32, tsg.TileConfig(bm=64, bn=64, bk=64, wm=32, wn=32, vec=4, raster=0,
                                                               sched=4, split_k=4))
    eager = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    esum = torch.zeros((1,), dtype=torch.float32, device=DEV)
    tsg.gemm(tsg.F32, M, N, K, dA, K, dB, N, eager, N, tsg.STRICT)
    tsg.reduce_sum(tsg.F32, M, N, eager, N, esum)
    torch.cuda.synchronize()
    out = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    osum = torch.zeros((1,), dtype=torch.float32, device=DEV)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            tsg.gemm(tsg.F32, M, N, K, dA, K, dB, N, out, N, tsg.STRICT, side.cuda_stream)
            tsg.reduce_sum(tsg.F32, M, N, out, N, osum, 0, side.cuda_stream)
    for rep in range(4):
        out.fill_(-1.0)
        osum.fill_(-1.0)
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager) and torch.equal(osum, esum), rep
        # eager work of the program's own between replays, on the same workspace
        tmp = torch.zeros((M, N), dtype=torch.float32, device=DEV)
        tsg.gemm(tsg.F32, M, N, K, dA, K, dB, N, tmp, N, tsg.STRICT)
        torch.cuda.synchronize()
        assert torch.equal(tmp, eager)


# ------------------------------------------------------------------ seeded differential runs

def test_many_seeded_gemm_cases_random_configs(workspace):
    """1500 small products with everything drawn from a seeded generator: dtype, which operands
    are stored transposed, batch, ragged extents, flags, and (70 %) a random legal config pinned
    under TSG_STRICT, else the library's own choice.  Integer data, bit for bit."""
    import random
    rng = random.Random(20240903)
    done = 0
    while done < 1500:
        dt = rng.choice([tsg.F32, tsg.BF16_F32ACC])
        ta, tb = rng.random() < 0.4, rng.random() < 0.3
        big = rng.random() < 0.2
        M, N = rng.randint(1, 700 if big else 200), rng.randint(1, 700 if big else 200)
        K = rng.randint(1, 200 if big else 500)
        nb = rng.choice([1, 1, 1, 2, 3])
        op = tsg.OP_GEMM_TRANSA if ta else tsg.OP_GEMM
        seed = rng.randint(0, 1 << 20)
        A = synth.small_ints(seed, 0, nb * M * K).reshape((nb, K, M) if ta else (nb, M, K))
        B = synth.small_ints(seed, 1, nb * K * N).reshape((nb, N, K) if tb else (nb, K, N))
        if dt == tsg.BF16_F32ACC:
            A, B = synth.f32_to_bf16_bits(A), synth.f32_to_bf16_bits(B)
        C0 = synth.small_ints(seed, 2, nb * M * N).reshape(nb, M, N)
        flags = rng.choice([0, tsg.NEGATE, tsg.ACCUMULATE, tsg.NEGATE | tsg.ACCUMULATE])
        pin = None
        if rng.random() < 0.7:
            cnt = tsg.tile_config_count(op, dt)
            for _ in range(20):
                c = tsg.tile_config_enum(op, dt, rng.randrange(cnt))
                if tsg.tile_config_check(op, dt, M, N, K, c) == tsg.OK and not (tb and c.sched == 0):
                    pin = c
                    break
        tsg.tile_config_set(op, dt, pin)
        dA, dB, dC = dev(A), dev(B), dev(C0)
        lda, ldb = A.shape[2], B.shape[2]
        try:
            tsg.gemm_trans(dt, ta, tb, nb, M, N, K, dA, lda, A.shape[1] * lda, dB, ldb, B.shape[1] * ldb, dC, N, M * N,
                           flags | (tsg.STRICT if pin is not None else 0))
        except tsg.SilenceableError:      # a split whose workspace need exceeds the fixture's, say
            assert pin is not None
            continue
        torch.cuda.synchronize()
        out = dC.cpu().numpy()
        for b in range(nb):
            ref = oracle.epilogue(oracle.gemm(A[b], B[b], trans_a=ta, trans_b=tb, with_s=False), flags & 3, C0[b])
            assert np.array_equal(out[b].astype(np.float64), ref), (dt, ta, tb, nb, M, N, K, flags, pin, b)
        done += 1


def test_many_seeded_conv_cases_random_configs(workspace):
    """2500 small convolutions drawn from a seeded generator (geometry, strides, padding, channel
    counts on and off the access width, dtype, flags, a random legal config or the library's
    choice), each written into a window of a larger tensor with a random ring and channel
    padding.  Integer data: the whole larger tensor must match, window and surroundings."""
    import random
    rng = random.Random(3864)
    op = tsg.OP_CONV2D_NHWC
    done = 0
    while done < 2500:
        dt = rng.choice([tsg.F32, tsg.BF16_F32ACC])
        Nn, H, W = rng.randint(1, 4), rng.randint(1, 24), rng.randint(1, 24)
        Cin = rng.choice([1, 3, 4, 8, 12, 16, 24, 32, 64])
        Cout = rng.choice([1, 5, 8, 16, 64, 70, 130])
        KH, KW = rng.choice([1, 2, 3, 5]), rng.choice([1, 2, 3, 5])
        st = (rng.choice([1, 2]), rng.choice([1, 2]))
        pd = (rng.randint(0, 2), rng.randint(0, 2))
        if H + 2 * pd[0] < KH or W + 2 * pd[1] < KW:
            continue
        Ho, Wo = oracle.conv_out_dim(H, KH, st[0], pd[0]), oracle.conv_out_dim(W, KW, st[1], pd[1])
        seed = rng.randint(0, 1 << 20)
        x, w = synth.conv_inputs(Nn, H, W, Cin, Cout, KH, KW, seed=seed, dist="ints")
        if dt == tsg.BF16_F32ACC:
            x, w = synth.f32_to_bf16_bits(x), synth.f32_to_bf16_bits(w)
        flags = rng.choice([0, tsg.NEGATE, tsg.ACCUMULATE, tsg.NEGATE | tsg.ACCUMULATE])
        ring, cpad = rng.choice([0, 0, 1, 3]), rng.choice([0, 0, 4])
        pin = None
        if rng.random() < 0.7:
            cnt = tsg.tile_config_count(op, dt)
            for _ in range(20):
                c = tsg.tile_config_enum(op, dt, rng.randrange(cnt))
                if tsg.tile_config_check(op, dt, Nn * Ho * Wo, Cout, KH * KW * Cin, c, contig=Cin) == tsg.OK:
                    pin = c
                    break
        tsg.tile_config_set(op, dt, pin)
        big0 = synth.small_ints(seed, 2, Nn * (Ho + 2 * ring) * (Wo + 2 * ring) * (Cout + cpad)).reshape(
            Nn, Ho + 2 * ring, Wo + 2 * ring, Cout + cpad)
        dbig = dev(big0)
        sw_ = Cout + cpad
        sh_ = (Wo + 2 * ring) * sw_
        sn_ = (Ho + 2 * ring) * sh_
        try:
            tsg.conv2d_nhwc_window(dt, Nn, H, W, Cin, Cout, KH, KW, st[0], st[1], pd[0], pd[1], dev(x), dev(w),
                                   dbig.data_ptr() + 4 * (ring * sh_ + ring * sw_), sn_, sh_, sw_,
                                   flags | (tsg.STRICT if pin is not None else 0))
        except tsg.SilenceableError:
            assert pin is not None
            continue
        torch.cuda.synchronize()
        ref = big0.astype(np.float64).copy()
        inner = (slice(None), slice(ring, ring + Ho), slice(ring, ring + Wo), slice(0, Cout))
        ref[inner] = oracle.epilogue(oracle.conv2d_nhwc(x, w, stride=st, pad=pd, with_s=False), flags & 3, big0[inner])
        assert np.array_equal(dbig.cpu().numpy().astype(np.float64), ref), (dt, Nn, H, W, Cin, Cout, KH, KW, st, pd, flags, ring, cpad, pin)
        done += 1
