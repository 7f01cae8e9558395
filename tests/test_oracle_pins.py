"""Pins for the CPU oracle: it is checked against things other than itself --
closed forms, invariants, literal brute force with exact rationals, numpy's fp64
matmul, and the values the paper prints.  None of these tests needs a GPU."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth


def _rand(shape, seed, tid=0):
    return synth.uniform_pm1(seed, tid, int(np.prod(shape))).reshape(shape)


# ------------------------------------------------------------------ GEMM special cases

def test_identity_left_and_right():
    B = _rand((7, 5), 11)
    R, S = oracle.gemm(np.eye(7, dtype=np.float32), B)
    assert np.array_equal(R, B.astype(np.float64))
    assert np.array_equal(S, np.abs(B).astype(np.float64))
    A = _rand((6, 9), 12)
    R = oracle.gemm(A, np.eye(9, dtype=np.float32), with_s=False)
    assert np.array_equal(R, A.astype(np.float64))


@pytest.mark.parametrize("M,N,K", [(3, 4, 5), (33, 17, 129), (64, 64, 8192)])
def test_all_ones_closed_form(M, N, K):
    R, S = oracle.gemm(np.ones((M, K), np.float32), np.ones((K, N), np.float32))
    assert np.all(R == K) and np.all(S == K)
    R = oracle.gemm(np.ones((K, M), np.float32), np.ones((K, N), np.float32), trans_a=True, with_s=False)
    assert np.all(R == K)


def test_one_hot_row_selects_row_of_b():
    """A single 1 at (i0,k0) copies row k0 of B into row i0 of C: catches a transposed
    or shifted index that symmetric pins cannot see."""
    M, N, K, i0, k0 = 5, 7, 6, 3, 4
    B = _rand((K, N), 3)
    A = np.zeros((M, K), np.float32)
    A[i0, k0] = 1
    R = oracle.gemm(A, B, with_s=False)
    exp = np.zeros((M, N))
    exp[i0] = B[k0]
    assert np.array_equal(R, exp)
    At = np.zeros((K, M), np.float32)
    At[k0, i0] = 1
    assert np.array_equal(oracle.gemm(At, B, trans_a=True, with_s=False), exp)


def test_brute_force_4x4x4_exact_rationals():
    """Literal triple loop with exact rationals on small-integer inputs."""
    A = synth.small_ints(5, 0, 16, -3, 3).reshape(4, 4)
    B = synth.small_ints(5, 1, 16, -3, 3).reshape(4, 4)
    R, S = oracle.gemm(A, B)
    Rt = oracle.gemm(np.ascontiguousarray(A.T), B, trans_a=True, with_s=False)
    for i in range(4):
        for j in range(4):
            acc, sacc = Fraction(0), Fraction(0)
            for k in range(4):
                acc += Fraction(int(A[i, k])) * Fraction(int(B[k, j]))
                sacc += abs(Fraction(int(A[i, k]))) * abs(Fraction(int(B[k, j])))
            assert Fraction(R[i, j]) == acc
            assert Fraction(S[i, j]) == sacc
            assert Fraction(Rt[i, j]) == acc


def test_brute_force_rectangular_nonsquare_dyadic():
    """Rectangular M != N != K with dyadic-rational entries (exact in fp64)."""
    M, N, K = 3, 5, 2
    A = (synth.small_ints(6, 0, M * K, -8, 8) / 4).astype(np.float32).reshape(M, K)
    B = (synth.small_ints(6, 1, K * N, -8, 8) / 8).astype(np.float32).reshape(K, N)
    R = oracle.gemm(A, B, with_s=False)
    for i in range(M):
        for j in range(N):
            acc = sum(Fraction(float(A[i, k])) * Fraction(float(B[k, j])) for k in range(K))
            assert Fraction(R[i, j]) == acc


@pytest.mark.parametrize("M,N,K", [(17, 9, 33), (128, 96, 257)])
def test_against_numpy_fp64_matmul(M, N, K):
    A, B = _rand((M, K), 21), _rand((K, N), 21, 1)
    R, S = oracle.gemm(A, B)
    ref = A.astype(np.float64) @ B.astype(np.float64)
    bound = K * 2.0 ** -52 * S + 1e-300
    assert np.all(np.abs(R - ref) <= bound)
    assert np.allclose(S, np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64), rtol=1e-13)
    Rt = oracle.gemm(np.ascontiguousarray(A.T), B, trans_a=True, with_s=False)
    assert np.array_equal(Rt, R)          # same sum, same order: identical bits


def test_transpose_identity_AtB_equals_BtA_transposed():
    """A^T.B = (B^T.A)^T with both stored K x (.)."""
    K, M, N = 37, 13, 21
    A, B = _rand((K, M), 31), _rand((K, N), 31, 1)
    left = oracle.gemm(A, B, trans_a=True, with_s=False)
    right = oracle.gemm(B, A, trans_a=True, with_s=False).T
    S = oracle.gemm(A, B, trans_a=True)[1]
    assert np.all(np.abs(left - right) <= K * 2.0 ** -52 * S)


def test_bf16_operands_are_their_exact_values():
    M, N, K = 9, 11, 40
    a = synth.normal_scaled(8, 0, M * K, 1.0).reshape(M, K)
    b = synth.normal_scaled(8, 1, K * N, 1.0).reshape(K, N)
    ab, bb = synth.f32_to_bf16_bits(a), synth.f32_to_bf16_bits(b)
    R16, S16 = oracle.gemm(ab, bb)
    R32, S32 = oracle.gemm(synth.bf16_bits_to_f32(ab), synth.bf16_bits_to_f32(bb))
    assert np.array_equal(R16, R32) and np.array_equal(S16, S32)


def test_bf16_rounding_known_values():
    """Round-to-nearest-even at the 8-bit significand: textbook cases."""
    x = np.array([1.0, 1.00390625, 1.01171875, 1.0078125, -1.00390625, 3.0e38, 0.0], np.float32)
    bits = synth.f32_to_bf16_bits(x)
    #  1.00390625 = 1 + 2^-8 is a tie between 1 and 1+2^-7 -> even (1.0)
    #  1.01171875 = 1 + 3*2^-8 is a tie between 1+2^-7 and 1+2^-6 -> even (1+2^-6 = 0x3f82)
    assert [int(v) for v in bits] == [0x3F80, 0x3F80, 0x3F82, 0x3F81, 0xBF80, 0x7F62, 0x0000]
    back = synth.bf16_bits_to_f32(bits)
    assert np.all(np.abs(back[:5] - x[:5]) <= np.abs(x[:5]) * 2.0 ** -8)


def test_epilogue_negate_and_accumulate():
    R = np.array([[1.5, -2.0], [0.0, 4.0]])
    C0 = np.array([[10.0, 20.0], [30.0, 40.0]], np.float32)
    assert np.array_equal(oracle.epilogue(R, 0), R)
    assert np.array_equal(oracle.epilogue(R, oracle.NEGATE), -R)
    assert np.array_equal(oracle.epilogue(R, oracle.ACCUMULATE, C0), R + C0)
    assert np.array_equal(oracle.epilogue(R, oracle.NEGATE | oracle.ACCUMULATE, C0), C0 - R)


def test_gemm_index_map():
    off = oracle.gemm_index_map(3, 4, 10, False)
    assert off[2, 3] == 23 and off[0, 0] == 0
    off = oracle.gemm_index_map(3, 4, 10, True)
    assert off[2, 3] == 32 and off[1, 0] == 1


# ------------------------------------------------------------------ convolution

def _conv_brute(x, w, stride, pad):
    N, H, W, Cin = x.shape
    KH, KW, _, Cout = w.shape
    Ho = (H + 2 * pad[0] - KH) // stride[0] + 1
    Wo = (W + 2 * pad[1] - KW) // stride[1] + 1
    out = [[[[Fraction(0) for _ in range(Cout)] for _ in range(Wo)] for _ in range(Ho)] for _ in range(N)]
    for n in range(N):
        for ho in range(Ho):
            for wo in range(Wo):
                for co in range(Cout):
                    acc = Fraction(0)
                    for kh in range(KH):
                        for kw in range(KW):
                            hi, wi = ho * stride[0] + kh - pad[0], wo * stride[1] + kw - pad[1]
                            if 0 <= hi < H and 0 <= wi < W:
                                for ci in range(Cin):
                                    acc += Fraction(float(x[n, hi, wi, ci])) * Fraction(float(w[kh, kw, ci, co]))
                    out[n][ho][wo][co] = acc
    return out


@pytest.mark.parametrize("shape,stride,pad", [
    ((1, 3, 3, 2, 2, 3, 3), (1, 1), (1, 1)),
    ((2, 5, 4, 3, 2, 3, 2), (2, 1), (1, 0)),
    ((1, 6, 7, 1, 3, 1, 3), (1, 2), (0, 2)),
])
def test_conv_brute_force_exact(shape, stride, pad):
    N, H, W, Cin, Cout, KH, KW = shape
    x, w = synth.conv_inputs(N, H, W, Cin, Cout, KH, KW, seed=9, dist="ints")
    R = oracle.conv2d_nhwc(x, w, stride=stride, pad=pad, with_s=False)
    ref = _conv_brute(x, w, stride, pad)
    assert R.shape == (N, len(ref[0]), len(ref[0][0]), Cout)
    for n in range(N):
        for ho in range(R.shape[1]):
            for wo in range(R.shape[2]):
                for co in range(Cout):
                    assert Fraction(R[n, ho, wo, co]) == ref[n][ho][wo][co]


def test_conv_all_ones_counts_valid_taps():
    """3x3, pad 1, stride 1, Cin=64: every output equals 64 * (#taps inside the image)
    = 64 * {4, 6, 9} at corner / edge / interior."""
    x = np.ones((2, 8, 9, 64), np.float32)
    w = np.ones((3, 3, 64, 5), np.float32)
    R, S = oracle.conv2d_nhwc(x, w, pad=(1, 1))
    assert R.shape == (2, 8, 9, 5)
    assert np.all(R[:, 0, 0] == 64 * 4) and np.all(R[:, -1, -1] == 64 * 4)
    assert np.all(R[:, 0, 1:-1] == 64 * 6) and np.all(R[:, 1:-1, 0] == 64 * 6)
    assert np.all(R[:, 1:-1, 1:-1] == 64 * 9)
    assert np.array_equal(R, S)


def test_conv_zero_pad_equals_explicit_padding():
    """conv(x, pad p) == conv(zero-padded x, pad 0); a wider ring of padding leaves the
    original outputs unchanged (they become the interior)."""
    x, w = synth.conv_inputs(2, 7, 6, 5, 4, 3, 3, seed=13)
    R1 = oracle.conv2d_nhwc(x, w, pad=(1, 1), with_s=False)
    xp = np.zeros((2, 9, 8, 5), np.float32)
    xp[:, 1:-1, 1:-1] = x
    R0 = oracle.conv2d_nhwc(xp, w, pad=(0, 0), with_s=False)
    assert np.array_equal(R1, R0)
    R2 = oracle.conv2d_nhwc(x, w, pad=(2, 2), with_s=False)
    assert np.array_equal(R2[:, 1:-1, 1:-1], R1)


def test_conv_one_hot_pixel_gives_flipped_filter_footprint():
    N, H, W, Cin, Cout = 1, 7, 7, 3, 2
    w = synth.conv_inputs(N, H, W, Cin, Cout, 3, 3, seed=17)[1]
    x = np.zeros((N, H, W, Cin), np.float32)
    h0, w0, c0 = 3, 4, 1
    x[0, h0, w0, c0] = 1
    R = oracle.conv2d_nhwc(x, w, pad=(1, 1), with_s=False)
    exp = np.zeros_like(R)
    for kh in range(3):
        for kw in range(3):
            # output (ho,wo) reads input (ho+kh-1, wo+kw-1): ho = h0-kh+1, wo = w0-kw+1
            exp[0, h0 - kh + 1, w0 - kw + 1] = w[kh, kw, c0]
    assert np.array_equal(R, exp)


def test_conv_1x1_is_a_gemm():
    """A 1x1 stride-1 convolution is exactly the matmul [N*H*W, Cin] x [Cin, Cout]."""
    x, w = synth.conv_inputs(2, 5, 6, 7, 3, 1, 1, seed=19)
    R = oracle.conv2d_nhwc(x, w, with_s=False)
    G = oracle.gemm(x.reshape(-1, 7), w.reshape(7, 3), with_s=False)
    assert np.array_equal(R.reshape(-1, 3), G)


def test_conv_equals_numpy_im2col_matmul():
    """Lowering check by a third route: gather with the index map, multiply with numpy."""
    N, H, W, Cin, Cout, KH, KW = 2, 6, 5, 4, 3, 3, 3
    x, w = synth.conv_inputs(N, H, W, Cin, Cout, KH, KW, seed=23)
    R, S = oracle.conv2d_nhwc(x, w, stride=(1, 1), pad=(1, 1))
    off = oracle.conv2d_index_map(N, H, W, Cin, KH, KW, (1, 1), (1, 1))
    xf = x.reshape(-1).astype(np.float64)
    M = off.shape[0]
    A = np.zeros((M, KH * KW, Cin))
    for m in range(M):
        for t in range(KH * KW):
            if off[m, t] >= 0:
                A[m, t] = xf[off[m, t]:off[m, t] + Cin]
    ref = A.reshape(M, -1) @ w.reshape(-1, Cout).astype(np.float64)
    assert np.all(np.abs(R.reshape(M, Cout) - ref) <= 1e-13 * S.reshape(M, Cout) + 1e-300)


def test_conv_index_map_literal():
    """Index map against literal loops; -1 exactly where the tap is in the padding."""
    N, H, W, Cin, KH, KW, st, pd = 2, 4, 5, 3, 3, 2, (2, 1), (1, 1)
    off = oracle.conv2d_index_map(N, H, W, Cin, KH, KW, st, pd)
    Ho, Wo = (H + 2 - KH) // 2 + 1, (W + 2 - KW) // 1 + 1
    assert off.shape == (N * Ho * Wo, KH * KW)
    for n in range(N):
        for ho in range(Ho):
            for wo in range(Wo):
                for kh in range(KH):
                    for kw in range(KW):
                        hi, wi = ho * 2 + kh - 1, wo + kw - 1
                        e = ((n * H + hi) * W + wi) * Cin if (0 <= hi < H and 0 <= wi < W) else -1
                        assert off[(n * Ho + ho) * Wo + wo, kh * KW + kw] == e


def test_conv_index_map_padding_mask_count_resnet_shape():
    """8x56x56, 3x3, pad 1: 166^2 valid taps per image out of 56^2 * 9."""
    off = oracle.conv2d_index_map(8, 56, 56, 64, 3, 3, (1, 1), (1, 1))
    assert off.shape == (25088, 9)
    assert int((off >= 0).sum()) == 8 * 166 * 166
    assert off.max() == ((7 * 56 + 55) * 56 + 55) * 64


# ------------------------------------------------------------------ paper's printed values

def _golden_lines(path):
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                yield line.split()


def test_split_matches_paper_examples(golden_dir):
    rows = list(_golden_lines(os.path.join(golden_dir, "paper_split_examples.txt")))
    assert len(rows) >= 4
    for ub, d, main, rest, tiles in rows:
        assert oracle.split(int(ub), int(d)) == (int(main), int(rest), int(tiles))


@pytest.mark.parametrize("ub,d", [(1, 1), (7, 8), (8, 8), (9, 8), (2305, 32), (196, 32), (5, 0)])
def test_split_invariants(ub, d):
    """Fig. 1(a) type annotations: main divisible by d, rest < d, sizes add up."""
    main, rest, tiles = oracle.split(ub, d)
    assert main + rest == ub
    if d > 0:
        assert main % d == 0 and 0 <= rest < d and tiles == main // d
    else:
        assert (main, rest, tiles) == (ub, 0, 1)


def test_paper_loop_nest_flops(golden_dir):
    ext = {k: int(v) for k, v in _golden_lines(os.path.join(golden_dir, "paper_loop_nest.txt"))}
    assert ext == dict(b=6, i=196, j=256, k=2305)
    P = synth.PAPER_BATCH_MATMUL
    assert (P["B"], P["M"], P["N"], P["K"]) == (ext["b"], ext["i"], ext["j"], ext["k"])
    assert 2 * ext["b"] * ext["i"] * ext["j"] * ext["k"] == 1_387_868_160


def test_tuning_constraints_fig10():
    """Tile sizes divide their dimension, 0 = untiled; vect forced to 0 when the
    innermost trip count is not a multiple of the vector size."""
    assert oracle.tile_legal(196, 0) and oracle.tile_legal(196, 49) and oracle.tile_legal(196, 196)
    assert not oracle.tile_legal(196, 32) and not oracle.tile_legal(196, 197) and not oracle.tile_legal(6, -1)
    assert oracle.tile_legal(6, 3) and oracle.tile_legal(256, 32) and not oracle.tile_legal(2305, 32)
    assert oracle.vect_legal(2305, 461, 4, 0)
    assert not oracle.vect_legal(2305, 461, 4, 1)       # 461 % 4 != 0
    assert not oracle.vect_legal(2305, 0, 4, 1)         # untiled: trip count 2305
    assert oracle.vect_legal(2304, 0, 4, 1) and oracle.vect_legal(2304, 32, 8, 1)
    assert not oracle.vect_legal(2304, 32, 8, 2)
    assert oracle.normalise_tile(196, 0) == 196 and oracle.normalise_tile(196, 500) == 196
    assert oracle.normalise_tile(196, 32) == 32


def test_error_metric_definition():
    ref = np.array([[1.0, -2.0], [0.0, 4.0]])
    S = np.array([[2.0, 2.0], [0.0, 8.0]])
    C = ref + np.array([[0.0, 0.002], [0.0, -0.004]])
    nw, cw = oracle.errors(C, ref, S)
    assert abs(nw - 0.001) < 1e-12 and abs(cw - 0.001) < 1e-12
    C[1, 0] = 1e-30
    assert oracle.errors(C, ref, S)[1] == float("inf")


def test_add_of_zero_pad_touches_only_the_interior():
    """x + pad0(y): outside the window the sum is x bit for bit, inside it is x + y; checked
    against literal loops on a small case."""
    big = _rand((5, 7), 3).astype(np.float64)
    R = _rand((2, 3), 4, tid=1).astype(np.float64)
    out = oracle.add_of_zero_pad(big, R, (1, 2))
    for i in range(5):
        for j in range(7):
            inside = 1 <= i < 3 and 2 <= j < 5
            want = big[i, j] + (R[i - 1, j - 2] if inside else 0.0)
            assert out[i, j] == want
    neg = oracle.add_of_zero_pad(big, R, (1, 2), sign=-1)
    assert np.array_equal(neg[1:3, 2:5], big[1:3, 2:5] - R)


def test_reduce_sum_pins():
    """Closed forms (all ones, 1..n), exact rational sum on a small case, and invariance
    under transpose / reshape, which is the point of the rewrite."""
    import math
    from fractions import Fraction
    assert oracle.reduce_sum(np.ones((7, 13), np.float32)) == (91.0, 91.0)
    n = 1000
    s, a = oracle.reduce_sum(np.arange(1, n + 1, dtype=np.float32))
    assert s == n * (n + 1) / 2 and a == s
    x = _rand((9, 11), 5)
    exact = sum(Fraction(float(v)) for v in x.ravel())
    s, a = oracle.reduce_sum(x)
    assert abs(Fraction(s) - exact) <= Fraction(a) * Fraction(1, 2 ** 50)
    assert s == math.fsum(float(v) for v in x.ravel()) or abs(s - math.fsum(float(v) for v in x.ravel())) < 1e-12
    st, at = oracle.reduce_sum(np.ascontiguousarray(x.T))
    sr, ar = oracle.reduce_sum(x.reshape(3, 33))
    assert abs(st - s) <= 1e-12 and abs(sr - s) <= 1e-12 and at == a == ar
    neg = x.copy(); neg[0, 0] = -abs(neg[0, 0]) - 1
    assert oracle.reduce_sum(neg)[1] > abs(oracle.reduce_sum(neg)[0])
    b = synth.f32_to_bf16_bits(x)
    sb, _ = oracle.reduce_sum(b)
    assert sb == float(np.sum(synth.bf16_bits_to_f32(b).astype(np.float64)))


def test_transposed_right_operand_pins():
    """op(B) = B^T read in place: against numpy's fp64 matmul of the explicit transpose,
    the identities A.B^T = (B.A^T)^T and A^T.B^T = (B.A)^T, a one-hot probe that tells B^T from
    B, and exact rationals on a tiny case."""
    from fractions import Fraction
    M, N, K = 13, 9, 21
    A = _rand((M, K), 71)
    Bt = _rand((N, K), 72, tid=1)
    R, S = oracle.gemm(A, Bt, trans_b=True)
    ref = A.astype(np.float64) @ Bt.astype(np.float64).T
    assert np.max(np.abs(R - ref)) <= K * 2.0 ** -52 * np.max(S)
    R2 = oracle.gemm(Bt, A, trans_b=True, with_s=False)            # B.A^T, N x M
    assert np.max(np.abs(R - R2.T)) <= K * 2.0 ** -52 * np.max(S)
    At = np.ascontiguousarray(A.T)                                   # K x M
    R3 = oracle.gemm(At, Bt, trans_a=True, trans_b=True, with_s=False)
    assert np.array_equal(R3, R)                                     # same products, same order
    R4 = oracle.gemm(Bt, At, with_s=False)                           # B.A with B = Bt (N x K), A = At (K x M)
    assert np.max(np.abs(R3 - R4.T)) <= K * 2.0 ** -52 * np.max(S)
    hot = np.zeros((4, 5), np.float32); hot[2, 3] = 1.0              # op(B)(k=3, j=2) = 1
    X = _rand((6, 5), 73)
    assert np.array_equal(oracle.gemm(X, hot, trans_b=True, with_s=False)[:, 2], X[:, 3].astype(np.float64))
    a = np.array([[1, 2], [3, 4]], np.float32); b = np.array([[5, 6], [7, 8]], np.float32)
    want = [[sum(Fraction(int(a[i, k])) * Fraction(int(b[j, k])) for k in range(2)) for j in range(2)] for i in range(2)]
    got = oracle.gemm(a, b, trans_b=True, with_s=False)
    assert all(Fraction(got[i, j]) == want[i][j] for i in range(2) for j in range(2))


def test_conv_bf16_branch_reads_the_exact_bf16_values():
    """The convolution oracle on bfloat16 bit patterns: (i) equal, bit for bit, to the fp32
    branch fed the same values widened to fp32 (R and S); (ii) one geometry with stride,
    asymmetric padding and a ragged filter against literal loops in exact rationals over the
    widened values; (iii) a value that only exists in bf16 form (0x3F81 = 1 + 2^-7) summed in
    closed form, which a branch that read the bits as integers, as halves or as fp32 words
    would miss."""
    x, w = synth.conv_inputs(2, 5, 4, 3, 2, 3, 2, seed=29)
    xb, wb = synth.f32_to_bf16_bits(x), synth.f32_to_bf16_bits(w)
    xf, wf = synth.bf16_bits_to_f32(xb), synth.bf16_bits_to_f32(wb)
    assert not np.array_equal(xf, x)          # rounding did change the inputs
    R16, S16 = oracle.conv2d_nhwc(xb, wb, stride=(2, 1), pad=(1, 0))
    R32, S32 = oracle.conv2d_nhwc(xf, wf, stride=(2, 1), pad=(1, 0))
    assert np.array_equal(R16, R32) and np.array_equal(S16, S32)
    ref = _conv_brute(xf, wf, (2, 1), (1, 0))
    N, Ho, Wo, Cout = R16.shape
    for n in range(N):
        for ho in range(Ho):
            for wo in range(Wo):
                for co in range(Cout):
                    exact = ref[n][ho][wo][co]
                    assert abs(Fraction(R16[n, ho, wo, co]) - exact) <= Fraction(S16[n, ho, wo, co]) * Fraction(1, 2 ** 48)
    xb1 = np.full((1, 4, 4, 8), 0x3F81, np.uint16)    # 1 + 2^-7
    wb1 = np.full((3, 3, 8, 2), 0x4000, np.uint16)    # 2.0
    R = oracle.conv2d_nhwc(xb1, wb1, pad=(1, 1), with_s=False)
    v = 2.0 * (1.0 + 2.0 ** -7) * 8
    assert np.all(R[0, 0, 0] == 4 * v) and np.all(R[0, 0, 1] == 6 * v) and np.all(R[0, 1, 1] == 9 * v)
    with pytest.raises(TypeError):
        oracle.conv2d_nhwc(xb, w)             # mixed element types are refused


def test_elementwise_relative_error_definition():
    """max |C-ref| / |ref| over the entries whose reference is at least `floor` of the largest."""
    ref = np.array([[100.0, -50.0], [0.05, 2.0]])
    C = ref + np.array([[0.1, 0.1], [0.04, 0.01]])
    # floor 1e-3 * 100 = 0.1: the 0.05 entry (relative error 0.8) is left out
    assert abs(oracle.elementwise_relative(C, ref) - 0.005) < 1e-15
    # with a lower floor it is the maximum
    assert abs(oracle.elementwise_relative(C, ref, floor=1e-4) - 0.8) < 1e-12
    assert oracle.elementwise_relative(ref, ref) == 0.0
    assert oracle.elementwise_relative(np.zeros((2, 2)), np.zeros((2, 2))) == 0.0
