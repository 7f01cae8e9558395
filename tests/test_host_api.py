"""Host-side behaviour of the C-ABI library (no GPU): exported symbols, the loop
split, tile-config legality, index maps and the error model."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2409_03864_amd as tsg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "tsg.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(tsg_[a-zA-Z0-9_]+)\s*\(", hdr))
    assert len(declared) >= 17
    lib = ctypes.CDLL(tsg.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert declared == set(tsg.EXPORTS)
    assert tsg.version() >= 1


def test_public_header_is_plain_c_and_links_against_the_library(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 (and as C++), and a C program that
    only uses host-side entry points must link against the built library and run without a GPU."""
    import os, shutil, subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    inc, libdir = os.path.join(root, "include"), os.path.join(root, "paper_2409_03864_amd")
    src = tmp_path / "use_tsg.c"
    src.write_text(
        '#include "tsg.h"\n#include <stdio.h>\n'
        "int main(void) {\n"
        "    int64_t main_part = 0, rest = 0, tiles = 0;\n"
        "    if (tsg_split(2042, 8, &main_part, &rest, &tiles) != TSG_OK) return 1;\n"
        '    printf("%lld %lld %lld %s\\n", (long long)main_part, (long long)rest, (long long)tiles, tsg_status_string(TSG_E_SILENCEABLE));\n'
        "    return tsg_tile_config_count(TSG_OP_GEMM, TSG_F32) > 0 ? 0 : 2;\n}\n")
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    subprocess.check_call([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-I", inc, str(src)])
    gxx = shutil.which("g++")
    if gxx:
        subprocess.check_call([gxx, "-std=c++11", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c++",
                               "-I", inc, str(src)])
    exe = tmp_path / "use_tsg"
    subprocess.check_call([gcc, "-std=c99", "-I", inc, str(src), "-o", str(exe), "-L", libdir, "-ltsg",
                           "-Wl,-rpath," + libdir])
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stderr
    assert out.stdout.split()[:3] == ["2040", "2", "255"]     # Fig. 1: 2042 = 255 * 8 + 2


def test_split_matches_paper_and_oracle(golden_dir):
    for line in open(os.path.join(golden_dir, "paper_split_examples.txt")):
        line = line.split("#")[0].split()
        if line:
            ub, d, main, rest, tiles = map(int, line)
            assert tsg.split(ub, d) == (main, rest, tiles)
    for ub in (0, 1, 31, 32, 33, 196, 2305, 4096, 25088):
        for d in (0, 1, 8, 32, 64, 128, 256):
            assert tsg.split(ub, d) == oracle.split(ub, d)
    with pytest.raises(tsg.TsgError):
        tsg.split(-1, 8)
    with pytest.raises(tsg.TsgError):
        tsg.split(8, -1)


def _direct_tile_exists(c, op, v):
    """A tile of the direct-to-LDS forms is an array of 16-byte chunks dealt over the workgroup's
    threads in whole passes: a stored row must divide a pass, and the rows must fill whole passes
    unless the operand is the k-contiguous left one (its last pass is then padded)."""
    nt = 64 * (c.bm // c.wm) * (c.bn // c.wn)
    a_kmaj = op != tsg.OP_GEMM_TRANSA
    a_cpr, a_rows = (c.bk // v, c.bm) if a_kmaj else (c.bm // v, c.bk)
    b_cpr, b_rows = c.bn // v, c.bk
    if nt % a_cpr or nt % b_cpr or b_rows % (nt // b_cpr):
        return False
    if a_rows % (nt // a_cpr) and not a_kmaj:
        return False
    return b_cpr >= 8 and (a_kmaj or a_cpr >= 8)


def test_search_space_enumeration():
    for op in (tsg.OP_GEMM, tsg.OP_GEMM_TRANSA, tsg.OP_CONV2D_NHWC):
        for dt, vmax in ((tsg.F32, 4), (tsg.BF16_F32ACC, 8)):
            n = tsg.tile_config_count(op, dt)
            assert n >= 6
            seen = set()
            for i in range(n):
                c = tsg.tile_config_enum(op, dt, i)
                blk = 16 if c.mfma else 32
                assert c.mfma in (0, 1)
                assert c.bm % c.wm == 0 and c.bn % c.wn == 0 and c.wm % blk == 0 and c.wn % blk == 0
                # the block form: one MFMA block per workgroup, fp32 only
                assert c.sched != 1 or (dt == tsg.F32 and c.bm == c.bn == c.wm == c.wn == blk)
                assert c.vec in (1, vmax) and c.raster in (0, 1) and c.sched in (0, 1, 4, 5)
                assert 1 <= c.split_k <= 16
                key = tuple(c.as_dict().values())
                assert key not in seen
                seen.add(key)
                # the direct-to-LDS forms (sched >= 4) have no scalar-access variant, some of their
                # tiles do not exist for every operand layout, and a tail-only split needs a tile
                # count that leaves a tail after rounds of 256
                assert c.split_tail in (0, 1) and (c.split_k > 1 or not c.split_tail)
                for ext in (4096, 4000 + 96 * 3):
                    tiles = -(-ext // c.bm) * -(-ext // c.bn)
                    bad = ((c.vec == 1 and c.sched >= 4) or (c.split_tail and tiles % 256 == 0) or
                           (c.sched >= 4 and not _direct_tile_exists(c, op, vmax)) or (c.sched == 0 and c.mfma == 1) or
                           (c.sched == 1 and (c.split_k > 1 or op == tsg.OP_CONV2D_NHWC)))
                    want = tsg.E_SILENCEABLE if bad else tsg.OK
                    assert tsg.tile_config_check(op, dt, ext, ext, 4096, c, contig=64) == want, (c, op, ext)
            with pytest.raises(tsg.TsgError):
                tsg.tile_config_enum(op, dt, n)
    assert tsg.tile_config_count(7, 0) == 0


def test_vect_constraint_matches_fig10_rule():
    """Fig. 10: vect is legal only when the innermost extent is divisible by the vector size.
    For the gathered operand of a convolution that extent is Cin and the library's check
    must agree with the oracle's statement of the rule; a matrix row is one contiguous run
    whose remainder is peeled, so the GEMM calls accept the wide form for every shape."""
    c = tsg.tile_config_enum(tsg.OP_GEMM, tsg.F32, 0)
    assert c.vec == 4
    for cin in (64, 3, 4, 6, 8, 30):
        legal = oracle.vect_legal(cin, 0, 4, 1)
        st = tsg.tile_config_check(tsg.OP_CONV2D_NHWC, tsg.F32, 25088, 64, 9 * cin, c, contig=cin)
        assert st == (tsg.OK if legal else tsg.E_SILENCEABLE), cin
    c8 = tsg.tile_config_enum(tsg.OP_CONV2D_NHWC, tsg.BF16_F32ACC, 0)
    assert c8.vec == 8
    for cin in (64, 8, 12, 4):
        legal = oracle.vect_legal(cin, 0, 8, 1)
        st = tsg.tile_config_check(tsg.OP_CONV2D_NHWC, tsg.BF16_F32ACC, 25088, 64, 9 * cin, c8, contig=cin)
        assert st == (tsg.OK if legal else tsg.E_SILENCEABLE), cin
    for K in (2304, 2305, 2306, 64):
        for N in (256, 255, 66):
            assert tsg.tile_config_check(tsg.OP_GEMM, tsg.F32, 196, N, K, c) == tsg.OK
            assert tsg.tile_config_check(tsg.OP_GEMM_TRANSA, tsg.F32, 197, N, K, c) == tsg.OK
    # vec = 1 has no precondition
    c.vec = 1
    assert tsg.tile_config_check(tsg.OP_CONV2D_NHWC, tsg.F32, 25088, 64, 27, c, contig=3) == tsg.OK
    # a vector size the hardware path does not have
    c.vec = 2
    assert tsg.tile_config_check(tsg.OP_GEMM, tsg.F32, 196, 256, 2304, c) == tsg.E_SILENCEABLE


def test_split_k_legality_and_workspace_size():
    """split_k tiles the k loop at the grid level: at most 16 ways, never more ways than
    there are k steps, and a call needs batch * tiles * split_k partial tiles of workspace
    after the 64 KiB of counters."""
    op, dt = tsg.OP_GEMM, tsg.F32
    c = tsg.TileConfig(bm=64, bn=64, bk=64, wm=32, wn=32, vec=4, raster=0, sched=0, split_k=4)
    assert tsg.tile_config_check(op, dt, 196, 256, 2305, c) == tsg.OK
    assert tsg.tile_config_check(op, dt, 196, 256, 200, c) == tsg.OK          # 4 steps of 64
    assert tsg.tile_config_check(op, dt, 196, 256, 192, c) == tsg.E_SILENCEABLE   # 3 steps
    c.split_k = 32
    assert tsg.tile_config_check(op, dt, 196, 256, 1 << 20, c) == tsg.E_SILENCEABLE
    c.split_k = -1
    assert tsg.tile_config_check(op, dt, 196, 256, 2305, c) == tsg.E_INVALID
    c.split_k = 4
    tiles = oracle.split(196 + 63, 64)[2] * oracle.split(256, 64)[2]
    assert tsg.workspace_bytes(dt, 6, 196, 256, c) == 65536 + 6 * tiles * 4 * 64 * 64 * 4
    c.split_k = 1
    assert tsg.workspace_bytes(dt, 6, 196, 256, c) == 0
    # tail-only split: only the tiles past the last full round of 256 take workspace
    c.split_k, c.split_tail = 4, 1
    assert tsg.tile_config_check(op, dt, 196, 256, 2305, c) == tsg.OK          # 16 tiles, all tail
    assert tsg.workspace_bytes(dt, 6, 196, 256, c) == 65536 + 6 * tiles * 4 * 64 * 64 * 4
    assert tsg.tile_config_check(op, dt, 1024, 1024, 2305, c) == tsg.E_SILENCEABLE   # 256 tiles, no tail
    assert tsg.tile_config_check(op, dt, 1024 + 64, 1024, 2305, c) == tsg.OK         # 272 tiles
    assert tsg.workspace_bytes(dt, 2, 1024 + 64, 1024, c) == 65536 + 2 * 16 * 4 * 64 * 64 * 4
    c.split_k = 1
    assert tsg.tile_config_check(op, dt, 1024 + 64, 1024, 2305, c) == tsg.E_SILENCEABLE
    c.split_k, c.split_tail = 4, 2
    assert tsg.tile_config_check(op, dt, 1024 + 64, 1024, 2305, c) == tsg.E_INVALID
    # a workspace must be a 256-byte aligned device buffer larger than the counter area
    for ws, nbytes in ((FAKE + 4, 1 << 20), (FAKE, 1024), (FAKE, 0)):
        with pytest.raises(tsg.TsgError) as e:
            tsg.workspace_set(ws, nbytes)
        assert e.value.status == tsg.E_INVALID
    tsg.workspace_set(None)


def test_tile_zero_means_default_and_oversized_tile_is_legal():
    """Sec. 3.4: tiling by 0 is a no-op (library default stands); a tile larger than the
    extent is legal (the whole loop is remainder)."""
    z = tsg.TileConfig()
    assert tsg.tile_config_check(tsg.OP_GEMM, tsg.F32, 512, 512, 512, z) == tsg.OK
    big = tsg.tile_config_enum(tsg.OP_GEMM, tsg.F32, 0)
    assert big.bm >= 128
    assert tsg.tile_config_check(tsg.OP_GEMM, tsg.F32, 5, 8, 12, big) == tsg.OK
    assert oracle.normalise_tile(5, big.bm) == 5          # the oracle's reading of the same rule
    # not instantiated -> silenceable, like a microkernel library lacking a size
    odd = tsg.TileConfig(bm=96, bn=96, bk=32, wm=32, wn=32, vec=4, raster=0, sched=0)
    assert tsg.tile_config_check(tsg.OP_GEMM, tsg.F32, 512, 512, 512, odd) == tsg.E_SILENCEABLE
    neg = tsg.TileConfig(bm=-1)
    assert tsg.tile_config_check(tsg.OP_GEMM, tsg.F32, 512, 512, 512, neg) == tsg.E_INVALID


def test_config_set_get_roundtrip_and_rollback():
    op, dt = tsg.OP_GEMM, tsg.F32
    tsg.tile_config_set(op, dt, None)
    h = tsg.tile_config_get(op, dt, 4096, 4096, 4096)
    assert h.bm * h.bn >= 128 * 128 and h.vec == 4 and h.split_k == 1
    hs = tsg.tile_config_get(op, dt, 256, 256, 256)
    assert hs.bm * hs.bn < h.bm * h.bn           # small problems get small tiles
    c = tsg.tile_config_enum(op, dt, tsg.tile_config_count(op, dt) - 1)
    tsg.tile_config_set(op, dt, c)
    g = tsg.tile_config_get(op, dt, 4096, 4096, 4096)
    assert g.as_dict() == c.as_dict()
    # a failing set leaves the registry unchanged
    with pytest.raises(tsg.SilenceableError):
        tsg.tile_config_set(op, dt, tsg.TileConfig(bm=96, bn=96, bk=32, wm=32, wn=32, vec=4))
    assert tsg.tile_config_get(op, dt, 4096, 4096, 4096).as_dict() == c.as_dict()
    # other (op, dtype) slots are independent
    assert tsg.tile_config_get(tsg.OP_GEMM_TRANSA, dt, 4096, 4096, 4096).as_dict() == h.as_dict()
    tsg.tile_config_set(op, dt, None)
    assert tsg.tile_config_get(op, dt, 4096, 4096, 4096).as_dict() == h.as_dict()


@pytest.mark.parametrize("geom", [
    (2, 4, 5, 3, 3, 2, 2, 1, 1, 1),
    (1, 7, 7, 4, 3, 3, 1, 1, 0, 0),
    (3, 9, 6, 2, 1, 1, 2, 2, 0, 0),
    (1, 5, 5, 1, 5, 5, 1, 1, 2, 2),
    (8, 56, 56, 64, 3, 3, 1, 1, 1, 1),
])
def test_conv_index_map_bit_exact(geom):
    N, H, W, Cin, KH, KW, sh, sw, ph, pw = geom
    ref = oracle.conv2d_index_map(N, H, W, Cin, KH, KW, (sh, sw), (ph, pw))
    off = np.full(ref.shape, 12345, np.int32)
    tsg.conv2d_index_map(N, H, W, Cin, KH, KW, sh, sw, ph, pw, off)
    assert off.dtype == ref.dtype and np.array_equal(off, ref)


def test_gemm_index_map_bit_exact():
    for trans in (False, True):
        ref = oracle.gemm_index_map(37, 53, 61, trans)
        off = np.zeros((37, 53), np.int64)
        tsg.gemm_index_map(trans, 37, 53, 61, off)
        assert np.array_equal(off, ref)
    with pytest.raises(tsg.TsgError):
        tsg.gemm_index_map(True, 37, 53, 30, np.zeros((37, 53), np.int64))


FAKE = 0x7F0000001000     # never dereferenced: every call below fails before a launch


def test_invalid_arguments_are_definite_errors():
    ok = dict(dtype=tsg.F32, M=8, N=8, K=8, A=FAKE, lda=8, B=FAKE, ldb=8, C=FAKE, ldc=8, flags=0, stream=0)
    bad = [dict(A=None), dict(B=None), dict(C=None), dict(M=0), dict(N=-1), dict(K=0), dict(lda=7), dict(ldb=7),
           dict(ldc=7), dict(flags=64), dict(dtype=9), dict(M=1 << 31)]
    for b in bad:
        kw = dict(ok, **b)
        with pytest.raises(tsg.TsgError) as e:
            tsg.gemm(**kw)
        assert e.value.status == tsg.E_INVALID, b
    with pytest.raises(tsg.TsgError) as e:
        tsg.gemm_transA(tsg.F32, 16, 8, 4, FAKE, 8, FAKE, 8, FAKE, 8, 0, 0)      # lda < M
    assert e.value.status == tsg.E_INVALID
    with pytest.raises(tsg.TsgError) as e:
        tsg.conv2d_nhwc(tsg.F32, 1, 2, 2, 4, 4, 3, 3, 1, 1, 0, 0, FAKE, FAKE, FAKE, 0, 0)   # kernel > image
    assert e.value.status == tsg.E_INVALID
    with pytest.raises(tsg.TsgError) as e:
        tsg.gemm_batched(tsg.F32, 0, 2, 8, 8, 8, FAKE, 8, 64, FAKE, 8, 64, FAKE, 8, 32, 0, 0)  # C overlap
    assert e.value.status == tsg.E_INVALID
    # limits of the launch grid and operand alignment are argument errors, with or without STRICT
    for flags in (0, tsg.STRICT):
        with pytest.raises(tsg.TsgError) as e:
            tsg.gemm_batched(tsg.F32, 0, 65536, 8, 8, 8, FAKE, 8, 64, FAKE, 8, 64, FAKE, 8, 64, flags, 0)
        assert e.value.status == tsg.E_INVALID
        with pytest.raises(tsg.TsgError) as e:
            tsg.gemm(tsg.F32, 1 << 20, 1 << 20, 8, FAKE, 8, FAKE, 1 << 20, FAKE, 1 << 20, flags, 0)   # 2^28 tiles
        assert e.value.status == tsg.E_INVALID
        for kw in (dict(A=FAKE + 2), dict(B=FAKE + 1), dict(C=FAKE + 2)):
            with pytest.raises(tsg.TsgError) as e:
                tsg.gemm(**dict(ok, flags=flags, **kw))
            assert e.value.status == tsg.E_INVALID, kw
        with pytest.raises(tsg.TsgError) as e:     # a transposed right operand, misaligned: definite as well
            tsg.gemm_trans(tsg.F32, 0, 1, 1, 8, 8, 8, FAKE, 8, 0, FAKE + 2, 8, 0, FAKE, 8, 0, flags, 0)
        assert e.value.status == tsg.E_INVALID
        with pytest.raises(tsg.TsgError) as e:
            tsg.gemm(tsg.BF16_F32ACC, 8, 8, 8, FAKE + 1, 8, FAKE, 8, FAKE, 8, flags, 0)
        assert e.value.status == tsg.E_INVALID
        with pytest.raises(tsg.TsgError) as e:
            tsg.conv2d_nhwc(tsg.F32, 1, 4, 4, 4, 4, 3, 3, 1, 1, 1, 1, FAKE + 2, FAKE, FAKE, flags, 0)
        assert e.value.status == tsg.E_INVALID


def test_workspace_per_stream_arguments():
    """Host side of tsg_workspace_set_stream: malformed buffers are refused, removing an entry
    that does not exist is fine."""
    for ws, nbytes in ((FAKE, 65536), (FAKE + 8, 1 << 20), (FAKE, -1), (0, 1 << 20)):
        with pytest.raises(tsg.TsgError) as e:
            tsg.workspace_set_stream(0x1234, ws, nbytes)
        assert e.value.status == tsg.E_INVALID
    tsg.workspace_set_stream(0x1234, None)


def test_strict_call_with_failed_precondition_is_silenceable_and_enqueues_nothing():
    """The pinned config splits the k loop, which needs a workspace that was never given.
    With TSG_STRICT there is no further alternative: silenceable, nothing launched (the
    pointers are fake, so a launch attempt would have been a runtime error instead)."""
    op, dt = tsg.OP_GEMM, tsg.F32
    c = tsg.TileConfig(bm=64, bn=64, bk=64, wm=32, wn=32, vec=4, raster=0, sched=0, split_k=2)
    tsg.workspace_set(None)
    tsg.tile_config_set(op, dt, c)
    try:
        with pytest.raises(tsg.SilenceableError):
            tsg.gemm(dt, 8, 8, 256, FAKE, 256, FAKE, 8, FAKE, 8, tsg.STRICT, 0)
        # more splits than k steps
        with pytest.raises(tsg.SilenceableError):
            tsg.gemm(dt, 8, 8, 8, FAKE, 8, FAKE, 8, FAKE, 8, tsg.STRICT, 0)
    finally:
        tsg.tile_config_set(op, dt, None)
    # the gathered operand: Cin = 3 cannot take 16-byte accesses
    op = tsg.OP_CONV2D_NHWC
    tsg.tile_config_set(op, dt, tsg.tile_config_enum(op, dt, 0))
    try:
        with pytest.raises(tsg.SilenceableError):
            tsg.conv2d_nhwc(dt, 1, 8, 8, 3, 8, 3, 3, 1, 1, 1, 1, FAKE, FAKE, FAKE, tsg.STRICT, 0)
    finally:
        tsg.tile_config_set(op, dt, None)


def test_reduce_sum_invalid_arguments():
    for kw in (dict(rows=0), dict(cols=0), dict(ld=3), dict(x=None), dict(out=None), dict(flags=64), dict(dtype=5)):
        a = dict(dtype=tsg.F32, rows=2, cols=4, x=FAKE, ld=4, out=FAKE, flags=0, stream=0)
        a.update(kw)
        with pytest.raises(tsg.TsgError) as e:
            tsg.reduce_sum(**a)
        assert e.value.status == tsg.E_INVALID, kw


def test_tune_cache_save_load_roundtrip(tmp_path):
    """Tuner results are kept per problem and travel through a text file: well-formed lines
    naming instantiated configs are taken, the rest is counted and skipped; a cached problem
    answers tsg_tile_config_get, any other extents still get the default; a pin wins."""
    op, dt = tsg.OP_GEMM, tsg.F32
    tsg.tune_cache_clear()
    assert tsg.tune_cache_size() == 0
    default = tsg.tile_config_get(op, dt, 1000, 900, 800).as_dict()
    f = tmp_path / "tuned.txt"
    f.write_text("# comment\n"
                 "0 0 0 1 1000 900 800 0  128 128 16 64 64 4 0 0 1 0 0  0.5\n"   # instantiated
                 "0 0 0 1 1000 900 801 0  96 96 32 32 32 4 0 0 1 0 0  0.5\n"     # not instantiated
                 "0 0 0 1 1000 900 802 0  128 128 16 64 64 3 0 0 1 0 0  0.5\n"   # no such access width
                 "0 0 0 1 1000 900 803 0  128 128 16 64 64 4 0 0 1 0 1  0.5\n"   # no such MFMA block for this tile
                 "garbage line\n"
                 "1 1 1 6 196 256 2305 0  64 64 64 32 32 8 1 4 2 1 0  0.03\n")
    assert tsg.tune_cache_load(str(f)) == (2, 4)
    assert tsg.tune_cache_size() == 2
    got = tsg.tile_config_get(op, dt, 1000, 900, 800).as_dict()
    assert (got["bm"], got["bn"], got["bk"], got["sched"], got["raster"]) == (128, 128, 16, 0, 0)
    assert tsg.tile_config_get(op, dt, 1000, 900, 801).as_dict() != got          # other extents: the default
    pin = tsg.tile_config_enum(op, dt, 5)
    tsg.tile_config_set(op, dt, pin)
    assert tsg.tile_config_get(op, dt, 1000, 900, 800).as_dict() == pin.as_dict()
    tsg.tile_config_set(op, dt, None)
    g = tmp_path / "again.txt"
    tsg.tune_cache_save(str(g))
    tsg.tune_cache_clear()
    assert tsg.tile_config_get(op, dt, 1000, 900, 800).as_dict() == default
    assert tsg.tune_cache_load(str(g)) == (2, 0)
    assert tsg.tile_config_get(op, dt, 1000, 900, 800).as_dict() == got
    tsg.tune_cache_clear()
    with pytest.raises(tsg.TsgError) as e:
        tsg.tune_cache_load(str(tmp_path / "missing.txt"))
    assert e.value.status == tsg.E_RUNTIME


def test_search_set_validates():
    for bad in ((-1, 1), (0, 3), (0, -1)):
        with pytest.raises(tsg.TsgError) as e:
            tsg._check(tsg._lib.tsg_search_set(*bad), "tsg_search_set")
        assert e.value.status == tsg.E_INVALID
    for order in (0, 1, 2):
        tsg.search_set(5, order)
    tsg.search_set(0, True)


def test_status_strings():
    assert "ok" in tsg.status_string(tsg.OK)
    assert "silenceable" in tsg.status_string(tsg.E_SILENCEABLE)
    assert "definite" in tsg.status_string(tsg.E_INVALID) and "definite" in tsg.status_string(tsg.E_RUNTIME)
    assert "definite" in tsg.status_string(tsg.E_TOO_LARGE) and "tsg_gemm_trans" in tsg.status_string(tsg.E_TOO_LARGE)


def test_bench_counts_and_traffic_lookup(monkeypatch):
    """bench.py's own arithmetic: algorithmic flops (padding taps of the convolution are not
    work), the refusal to run on more than one GPU, and the traffic table, which answers only
    for the kernel sources and the tile config its figures were measured with."""
    import subprocess
    import sys
    import bench
    import synth
    C = synth.CONFIGS
    assert bench.workload_flops(C[1]) == 2 * 256 ** 3
    assert bench.workload_flops(C[3]) == 137438953472
    assert bench.workload_flops(C[5]) == 1099511627776
    assert bench.workload_flops(C[6]) == 1387868160                      # 2 * 6 * 196 * 256 * 2305
    assert bench.workload_flops(C[4]) == 2 * 8 * 166 * 166 * 64 * 64     # 166 valid taps per axis
    assert bench.workload_flops(C[4]) == bench.workload_flops(C[8]) == bench.workload_flops(C[10])
    assert bench.workload_flops(C[7]) == 16384 * 16384
    for k, entries in bench.TRAFFIC.items():
        for e in entries:
            dtype, op = C[k]["dtype"], C[k]["op"]
            monkeypatch.setattr(bench, "kernel_hash", lambda d, o="", h=e["kernel_hash"]: h)
            assert bench.traffic_bytes(k, dtype, dict(e["tile"]), op) == (e["bytes"], e["source"])
            assert os.path.exists(os.path.join(os.path.dirname(bench.__file__), e["source"]))
            if e["tile"]:
                other = dict(e["tile"], bk=e["tile"]["bk"] * 2)
                assert bench.traffic_bytes(k, dtype, other, op)[0] in (None, *[x["bytes"] for x in entries if x is not e])
            monkeypatch.setattr(bench, "kernel_hash", lambda d, o="": "changed")
            assert bench.traffic_bytes(k, dtype, dict(e["tile"]), op) == (None, None)
    monkeypatch.undo()
    assert len(bench.kernel_hash("f32")) == 16 and bench.kernel_hash("f32") != bench.kernel_hash("bf16")
    r = subprocess.run([sys.executable, bench.__file__, "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout == ""
