"""The allocation-free entry point (tsg_gemm_trans_static) against the entry point it is a
variant of (tsg_gemm_trans with a caller-owned workspace of the same size), through the C ABI:
the two must agree bit for bit on two calls in a row, the second with a smaller input, and both
must match the CPU oracle.  Collected last on purpose."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle
import synth
import paper_2409_03864_amd as tsg

DEV = "cuda:0"


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _both(batch, M, N, K, seed, dist, flags=0):
    """(result of the static entry point, result of tsg_gemm_trans with a workspace, launch info of each)."""
    A, B = synth.gemm_inputs(batch * M, N, K, seed=seed, dist=dist)
    A = A.reshape(batch, M, K)
    Bm = (synth.small_ints(seed, 1, batch * K * N) if dist == "ints" else synth.uniform_pm1(seed, 1, batch * K * N))
    Bm = Bm.reshape(batch, K, N)
    dA, dB = _dev(A), _dev(Bm)
    Cs = torch.full((batch, M, N), -5.0, dtype=torch.float32, device=DEV)
    Cw = torch.full((batch, M, N), -7.0, dtype=torch.float32, device=DEV)
    # the static entry point runs with NO workspace registered anywhere
    tsg.workspace_set(None)
    tsg.gemm_trans_static(tsg.F32, False, False, batch, M, N, K, dA, K, M * K, dB, N, K * N, Cs, N, M * N, flags)
    li_s = tsg.last_launch()
    torch.cuda.synchronize()
    ws = torch.empty(tsg.STATIC_SCRATCH_BYTES, dtype=torch.uint8, device=DEV)
    tsg.workspace_set(ws)
    try:
        tsg.gemm_trans(tsg.F32, False, False, batch, M, N, K, dA, K, M * K, dB, N, K * N, Cw, N, M * N, flags)
        li_w = tsg.last_launch()
        torch.cuda.synchronize()
    finally:
        tsg.workspace_set(None)
    return A, Bm, Cs.cpu().numpy(), Cw.cpu().numpy(), li_s, li_w


def test_static_scratch_entry_point_matches_the_workspace_one_twice_in_a_row():
    # first call: the paper's batched loop nest (Case Study 4), whose default config splits k;
    # second: a smaller, ragged product, for which the library's own choice does not split, so
    # a config that does is pinned (a pin applies to both entry points alike)
    split3 = tsg.TileConfig(bm=64, bn=64, bk=32, wm=32, wn=32, vec=4, raster=0, sched=4, split_k=3)
    for step, (batch, M, N, K) in enumerate(((6, 196, 256, 2305), (2, 100, 72, 1031))):
        for dist in ("ints", "uniform"):
            tsg.tile_config_set(tsg.OP_GEMM, tsg.F32, split3 if step == 1 else None)
            try:
                A, B, Cs, Cw, li_s, li_w = _both(batch, M, N, K, seed=50 + step, dist=dist)
            finally:
                tsg.tile_config_set(tsg.OP_GEMM, tsg.F32, None)
            assert li_s.config.as_dict() == li_w.config.as_dict(), (li_s.config, li_w.config)
            assert li_s.config.split_k > 1, "the scratch is only exercised when the k loop is split"
            assert np.array_equal(Cs.view(np.uint32), Cw.view(np.uint32)), (step, dist)
            for b in range(batch):
                R, S = oracle.gemm(A[b], B[b])
                if dist == "ints":
                    assert np.array_equal(Cs[b].astype(np.float64), R)
                else:
                    nw, cw = oracle.errors(Cs[b], R, S)
                    assert nw <= 1e-4 and cw <= 1e-4, (step, b, nw, cw)


def test_static_scratch_entry_point_flags_and_size_limit():
    A, B, Cs, Cw, li_s, li_w = _both(1, 130, 96, 4100, seed=60, dist="ints", flags=tsg.NEGATE)
    assert np.array_equal(Cs.view(np.uint32), Cw.view(np.uint32))
    assert np.array_equal(Cs[0].astype(np.float64), -oracle.gemm(A[0], B[0], with_s=False))
    # beyond the limit: a definite error of its own, before anything is enqueued or written
    M = N = 1088                     # 1088^2 = 1183744 > 2^20 outputs
    K = 64
    dA = torch.zeros((M, K), dtype=torch.float32, device=DEV)
    dB = torch.zeros((K, N), dtype=torch.float32, device=DEV)
    C = torch.full((M, N), 3.0, dtype=torch.float32, device=DEV)
    with pytest.raises(tsg.TsgError) as e:
        tsg.gemm_trans_static(tsg.F32, False, False, 1, M, N, K, dA, K, 0, dB, N, 0, C, N, 0, 0)
    assert e.value.status == tsg.E_TOO_LARGE and "tsg_gemm_trans" in str(e.value)
    torch.cuda.synchronize()
    assert bool((C == 3.0).all())
    # exactly at the limit it runs
    M = N = 1024
    dA = torch.ones((M, K), dtype=torch.float32, device=DEV)
    dB = torch.ones((K, N), dtype=torch.float32, device=DEV)
    C = torch.zeros((M, N), dtype=torch.float32, device=DEV)
    tsg.gemm_trans_static(tsg.F32, False, False, 1, M, N, K, dA, K, 0, dB, N, 0, C, N, 0, 0)
    torch.cuda.synchronize()
    assert bool((C == float(K)).all())
