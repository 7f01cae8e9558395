"""CPU oracle (TEST INFRASTRUCTURE ONLY) for the contraction C = +-op(A).B (+C) and
the NHWC convolution lowered to it.

Only `tests/`, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It never imports the GPU package and shares no code with it.  The heavy
loops live in `ref.c` (plain C, fp64 accumulation, OpenMP over output rows), loaded
through ctypes; this file holds the thin wrappers, the epilogue definition, the
error metrics and the paper's tuning-parameter constraints.

Cited passages: Case Study 4 (Fig. 7 loop nest, Fig. 8 split/tile/unroll), Case
Study 3 (transpose / negate / zero-pad rewrites), Case Study 5 (Fig. 10 constraints),
Fig. 1 (split worked example), Sec. 3.4 (tiling by 0 and by an oversized tile are
no-ops).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ref.c")
_LIB = os.path.join(_HERE, "libref_oracle.so")

NEGATE = 1
ACCUMULATE = 2


def build(force: bool = False) -> str:
    """Compile ref.c with gcc (no HIP, no third-party code)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _c():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        lib.ref_threads.restype = ci
        lib.ref_gemm.argtypes = [ci, ci, i64, i64, i64, vp, i64, vp, i64, vp, vp]
        lib.ref_gemm.restype = None
        lib.ref_gemm_transB.argtypes = [ci, ci, i64, i64, i64, vp, i64, vp, i64, vp, vp]
        lib.ref_gemm_transB.restype = None
        lib.ref_conv2d_nhwc.argtypes = [ci] + [i64] * 11 + [vp, vp, vp, vp]
        lib.ref_conv2d_nhwc.restype = None
        lib.ref_conv2d_index_map.argtypes = [i64] * 10 + [vp]
        lib.ref_conv2d_index_map.restype = None
        lib.ref_split.argtypes = [i64, i64, vp, vp, vp]
        lib.ref_split.restype = None
        _lib = lib
    return _lib


def threads() -> int:
    return int(_c().ref_threads())


def _operand(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.float32:
        return a, 0
    if a.dtype == np.uint16:
        return a, 1
    raise TypeError("operands are fp32 arrays or uint16 arrays of bfloat16 bit patterns")


def gemm(A, B, *, trans_a: bool = False, trans_b: bool = False, with_s: bool = True):
    """R = op(A).op(B) in fp64 and S = |op(A)|.|op(B)| (Fig. 7 with the batch index dropped).

    A is M x K row-major, or K x M when trans_a (the left operand is stored
    transposed and read in place, Case Study 3).  B is K x N, or N x K when trans_b.
    Both fp32, or both bfloat16 bit patterns (uint16) whose exact values are
    multiplied in fp64.
    """
    A, ta = _operand(A)
    B, tb = _operand(B)
    if ta != tb:
        raise TypeError("A and B must have the same element type")
    if trans_a:
        K, M = A.shape
    else:
        M, K = A.shape
    if B.shape[1 if trans_b else 0] != K:
        raise ValueError("inner dimensions differ")
    N = B.shape[0 if trans_b else 1]
    R = np.empty((M, N), dtype=np.float64)
    S = np.empty((M, N), dtype=np.float64) if with_s else None
    fn = _c().ref_gemm_transB if trans_b else _c().ref_gemm
    fn(ta, int(trans_a), M, N, K, A.ctypes.data, A.shape[1], B.ctypes.data, B.shape[1],
       R.ctypes.data, S.ctypes.data if with_s else None)
    return (R, S) if with_s else R


def conv_out_dim(L: int, Kk: int, stride: int, pad: int) -> int:
    return (L + 2 * pad - Kk) // stride + 1


def conv2d_nhwc(x, w, *, stride=(1, 1), pad=(0, 0), with_s: bool = True):
    """Direct convolution, x [N][H][W][Cin], w [KH][KW][Cin][Cout] -> [N][Ho][Wo][Cout],
    fp64 accumulation, padded taps omitted."""
    x, tx = _operand(x)
    w, tw = _operand(w)
    if tx != tw:
        raise TypeError("x and w must have the same element type")
    N, H, W, Cin = x.shape
    KH, KW, Cin2, Cout = w.shape
    if Cin != Cin2:
        raise ValueError("channel counts differ")
    Ho, Wo = conv_out_dim(H, KH, stride[0], pad[0]), conv_out_dim(W, KW, stride[1], pad[1])
    R = np.empty((N, Ho, Wo, Cout), dtype=np.float64)
    S = np.empty_like(R) if with_s else None
    _c().ref_conv2d_nhwc(tx, N, H, W, Cin, Cout, KH, KW, stride[0], stride[1], pad[0], pad[1],
                         x.ctypes.data, w.ctypes.data, R.ctypes.data,
                         S.ctypes.data if with_s else None)
    return (R, S) if with_s else R


def conv2d_index_map(N, H, W, Cin, KH, KW, stride=(1, 1), pad=(0, 0)) -> np.ndarray:
    """int32 [M][KH*KW]: offset of x[n][hi][wi][0] for output pixel m and tap t, or -1
    where the tap reads zero padding."""
    Ho, Wo = conv_out_dim(H, KH, stride[0], pad[0]), conv_out_dim(W, KW, stride[1], pad[1])
    off = np.empty((N * Ho * Wo, KH * KW), dtype=np.int32)
    _c().ref_conv2d_index_map(N, H, W, Cin, KH, KW, stride[0], stride[1], pad[0], pad[1],
                              off.ctypes.data)
    return off


def gemm_index_map(M: int, K: int, lda: int, trans_a: bool) -> np.ndarray:
    """int64 [M][K]: element offset of op(A)(i,k) inside the stored array."""
    i = np.arange(M, dtype=np.int64)[:, None]
    k = np.arange(K, dtype=np.int64)[None, :]
    return k * lda + i if trans_a else i * lda + k


def epilogue(R, flags: int = 0, C_old=None):
    """C = s.R (+ C_old), s = -1 with NEGATE; fp64.  The `+=` of Fig. 7 is ACCUMULATE."""
    out = -R if (flags & NEGATE) else R.copy()
    if flags & ACCUMULATE:
        out = out + np.asarray(C_old, dtype=np.float64)
    return out


def add_of_zero_pad(big, R, lo, sign: int = 1):
    """big + pad0(sign * R): R placed at offset `lo` (one index per axis) inside an array of
    zeros of big's shape, then added (Case Study 3: the sum with a zero-padded tensor).  The
    definition is written with the padded tensor formed explicitly, which is exactly what
    the library avoids."""
    big = np.asarray(big, dtype=np.float64)
    padded = np.zeros_like(big)
    padded[tuple(slice(o, o + n) for o, n in zip(lo, R.shape))] = sign * np.asarray(R, dtype=np.float64)
    return big + padded


def reduce_sum(x):
    """(sum, sum of magnitudes) of every element, in fp64 (Case Study 3: the full additive
    reduce, which does not depend on how the tensor is indexed).  x: fp32 array or uint16
    array of bfloat16 bits, any shape."""
    x, is_bf16 = _operand(x)
    if is_bf16:
        x = (x.astype(np.uint32) << np.uint32(16)).view(np.float32)
    v = x.astype(np.float64).ravel()
    return float(np.sum(v)), float(np.sum(np.abs(v)))


def split(ub: int, d: int):
    """(main, rest, tiles) of splitting a loop of trip count ub by divisor d (Fig. 1,
    Fig. 8): main % d == 0, rest < d, main + rest == ub."""
    m, r, t = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    _c().ref_split(ub, d, ctypes.byref(m), ctypes.byref(r), ctypes.byref(t))
    return m.value, r.value, t.value


# ---- Case Study 5 (Fig. 10): tuning parameters and their constraints --------------

def normalise_tile(dim: int, tile: int) -> int:
    """Sec. 3.4: tiling by 0 is a no-op, and so is tiling by more than the extent.
    Returns the effective tile size (dim when the loop is left untiled)."""
    if tile <= 0 or tile >= dim:
        return dim
    return tile


def tile_legal(dim: int, tile: int) -> bool:
    """Fig. 10: tile in [0, dim] and dim % tile == 0; tile 0 means 'do not tile'."""
    if tile < 0 or tile > dim:
        return False
    return tile == 0 or dim % tile == 0


def vect_legal(K: int, tile3: int, vector_size: int, vect: int) -> bool:
    """Fig. 10: vect in {0,1}; vect must be 0 when the innermost trip count
    (tile3, or K when the k loop is untiled) is not a multiple of the vector size."""
    if vect not in (0, 1):
        return False
    inner = normalise_tile(K, tile3)
    return vect == 0 or inner % vector_size == 0


# ---- error metrics used by every parity test --------------------------------------

def errors(C, ref, S):
    """Returns (normwise, componentwise): max|C-ref| / max|ref| and
    max_ij |C-ref|_ij / S_ij (S = |A|.|B|, the forward-error denominator of a dot
    product).  Entries with S == 0 must match exactly."""
    C = np.asarray(C, dtype=np.float64)
    d = np.abs(C - ref)
    mx = float(np.max(np.abs(ref))) if ref.size else 0.0
    normwise = float(d.max() / mx) if mx > 0 else float(d.max() if d.size else 0.0)
    nz = S > 0
    comp = float((d[nz] / S[nz]).max()) if nz.any() else 0.0
    if (~nz).any() and d[~nz].max() != 0:
        comp = float("inf")
    return normwise, comp


def elementwise_relative(C, ref, floor: float = 1e-3) -> float:
    """Plain element-wise relative error max |C-ref|_ij / |ref|_ij, restricted to the entries
    with |ref|_ij >= floor * max|ref| (a sum that cancels to almost nothing has no meaningful
    relative error).  Reported next to the two gated figures of `errors`; 0.0 when no entry
    qualifies."""
    C = np.asarray(C, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    mag = np.abs(ref)
    mx = float(mag.max()) if mag.size else 0.0
    keep = mag >= floor * mx
    if mx == 0.0 or not keep.any():
        return 0.0
    return float((np.abs(C - ref)[keep] / mag[keep]).max())
