"""Seeded synthetic inputs for the matmul / convolution workloads.

This module only *generates bytes*: it holds none of the arithmetic of the
contraction (no products, no sums over k, no index maps).  The same buffers are
handed to the CPU oracle and, through device copies, to the HIP library, so no
cross-implementation RNG matching is ever needed.

Generator (counter based, so any element can be produced on its own):
    key(seed, tensor_id) = mix64(seed*PHI + (tensor_id+1)*M1)
    h(seed, tensor_id, i) = mix64(key + (i+1)*PHI)      (mix64 = splitmix64's output function)
    uniform  : top 24 bits u of h  ->  (u + 0.5) / 2**23 - 1   in (-1, 1), exact in fp32
    normal   : Box-Muller in fp64 from the two 32-bit halves of h, times `scale`
               in fp64, then ONE round-to-nearest-even to fp32
    bf16     : one more round-to-nearest-even of the fp32 value to bfloat16

The five workload configurations are the shapes the contraction is measured on:
dense GEMM 256^3 and 4096^3, a transposed-left-operand GEMM 1024^3, a ResNet-like
3x3 NHWC convolution (8x56x56x64 -> 64) and a bf16 GEMM 8192^3 with a negated
result.  The paper's own loop nest (Case Study 4: batch 6, 196x256x2305) is also
available as `PAPER_BATCH_MATMUL`.
"""
from __future__ import annotations

import numpy as np

_PHI = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22


def _mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function (Steele, Lea, Flood 2014) on uint64 arrays."""
    z = z.copy()
    z ^= z >> np.uint64(30)
    z *= _M1
    z ^= z >> np.uint64(27)
    z *= _M2
    z ^= z >> np.uint64(31)
    return z


def _stream_key(seed: int, tensor_id: int) -> np.uint64:
    with np.errstate(over="ignore"):
        k = np.array([np.uint64(seed) * _PHI + np.uint64(tensor_id + 1) * _M1], dtype=np.uint64)
        return _mix64(k)[0]


def raw_bits(seed: int, tensor_id: int, n: int, start: int = 0) -> np.ndarray:
    """n 64-bit words of stream (seed, tensor_id), counters start..start+n-1."""
    key = _stream_key(seed, tensor_id)
    with np.errstate(over="ignore"):
        ctr = np.arange(start, start + n, dtype=np.uint64)
        return _mix64(key + (ctr + np.uint64(1)) * _PHI)


def uniform_pm1(seed: int, tensor_id: int, n: int) -> np.ndarray:
    """n fp32 values i.i.d. uniform on the open interval (-1, 1)."""
    out = np.empty(n, dtype=np.float32)
    for s in range(0, n, _CHUNK):
        m = min(_CHUNK, n - s)
        u = (raw_bits(seed, tensor_id, m, s) >> np.uint64(40)).astype(np.float64)
        out[s:s + m] = ((u + 0.5) / float(1 << 23) - 1.0).astype(np.float32)
    return out


def normal_scaled(seed: int, tensor_id: int, n: int, scale: float) -> np.ndarray:
    """n fp32 values: N(0,1)*scale, evaluated in fp64 and rounded once to fp32."""
    out = np.empty(n, dtype=np.float32)
    for s in range(0, n, _CHUNK):
        m = min(_CHUNK, n - s)
        h = raw_bits(seed, tensor_id, m, s)
        u1 = ((h >> np.uint64(32)).astype(np.float64) + 0.5) / 4294967296.0
        u2 = ((h & np.uint64(0xFFFFFFFF)).astype(np.float64) + 0.5) / 4294967296.0
        z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        out[s:s + m] = (z * scale).astype(np.float32)
    return out


def small_ints(seed: int, tensor_id: int, n: int, lo: int = -2, hi: int = 2) -> np.ndarray:
    """n fp32 values that are integers in [lo, hi]: every fp32 summation order of
    their products is exact while |partial sums| < 2**24."""
    span = hi - lo + 1
    out = np.empty(n, dtype=np.float32)
    for s in range(0, n, _CHUNK):
        m = min(_CHUNK, n - s)
        r = (raw_bits(seed, tensor_id, m, s) >> np.uint64(33)) % np.uint64(span)
        out[s:s + m] = r.astype(np.int64) + lo
    return out


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (round to nearest, ties to even); returns uint16 bits.
    NaN inputs are not produced by the generators above and are not handled."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return ((b + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- workloads

def gemm_inputs(M, N, K, *, seed, dist, trans_a=False, bf16=False):
    """A (M x K, or K x M when trans_a) and B (K x N), row-major, ld = row length."""
    na, nb = M * K, K * N
    if dist == "uniform":
        a, b = uniform_pm1(seed, 0, na), uniform_pm1(seed, 1, nb)
    elif dist == "normal":
        sc = 1.0 / np.sqrt(float(K))
        a, b = normal_scaled(seed, 0, na, sc), normal_scaled(seed, 1, nb, sc)
    elif dist == "ints":
        a, b = small_ints(seed, 0, na), small_ints(seed, 1, nb)
    else:
        raise ValueError(dist)
    a = a.reshape((K, M) if trans_a else (M, K))
    b = b.reshape(K, N)
    if bf16:
        a, b = f32_to_bf16_bits(a), f32_to_bf16_bits(b)
    return a, b


def conv_inputs(N, H, W, Cin, Cout, KH, KW, *, seed, dist="paper"):
    """x [N][H][W][Cin] and w [KH][KW][Cin][Cout]."""
    nx, nw = N * H * W * Cin, KH * KW * Cin * Cout
    if dist == "paper":
        x = uniform_pm1(seed, 0, nx)
        w = normal_scaled(seed, 1, nw, 1.0 / np.sqrt(float(KH * KW * Cin)))
    elif dist == "ints":
        x, w = small_ints(seed, 0, nx), small_ints(seed, 1, nw)
    else:
        raise ValueError(dist)
    return x.reshape(N, H, W, Cin), w.reshape(KH, KW, Cin, Cout)


CONFIGS = {
    1: dict(op="gemm", dtype="f32", M=256, N=256, K=256, dist="uniform", seed=0, flags=()),
    2: dict(op="gemm_transA", dtype="f32", M=1024, N=1024, K=1024, dist="uniform", seed=1, flags=()),
    3: dict(op="gemm", dtype="f32", M=4096, N=4096, K=4096, dist="normal", seed=2, flags=()),
    4: dict(op="conv2d_nhwc", dtype="f32", N=8, H=56, W=56, Cin=64, Cout=64, KH=3, KW=3,
            stride=1, pad=1, seed=3, flags=()),
    5: dict(op="gemm", dtype="bf16", M=8192, N=8192, K=8192, dist="normal", seed=4, flags=("negate",)),
    # Case Study 4 / Fig. 7 of the paper: one ResNet-50 layer's loop nest, batch loop included
    6: dict(op="gemm_batched", dtype="f32", B=6, M=196, N=256, K=2305, dist="uniform", seed=5, flags=()),
    # the full additive reduce of Case Study 3 on a tensor larger than every cache (1 GiB)
    7: dict(op="reduce_sum", dtype="f32", rows=16384, cols=16384, dist="uniform", seed=6, flags=()),
    # the rest of Case Study 3's rewrites on the contraction: the same layer in bf16; both
    # operands stored transposed; the layer's result accumulated into the interior of a tensor
    # with a ring of two more pixels (the sum with a zero-padded tensor, pad never formed)
    8: dict(op="conv2d_nhwc", dtype="bf16", N=8, H=56, W=56, Cin=64, Cout=64, KH=3, KW=3,
            stride=1, pad=1, seed=7, flags=()),
    9: dict(op="gemm_trans", dtype="f32", M=4096, N=4096, K=4096, dist="normal", seed=8, flags=()),
    10: dict(op="conv2d_nhwc", dtype="f32", N=8, H=56, W=56, Cin=64, Cout=64, KH=3, KW=3,
             stride=1, pad=1, seed=9, flags=("accumulate",), window_ring=2),
    # the same reduce on a view: 2^20 rows of 192 elements inside rows of 256 (three quarters of a
    # 1 GiB buffer are summed, a quarter is skipped)
    11: dict(op="reduce_sum", dtype="f32", rows=1 << 20, cols=192, ld=256, dist="uniform", seed=10, flags=()),
}

PAPER_BATCH_MATMUL = dict(B=6, M=196, N=256, K=2305)


def config_inputs(k: int):
    """Host arrays for workload configuration k (1-based)."""
    c = CONFIGS[k]
    if c["op"] == "reduce_sum":
        # the whole buffer is generated, rows of `ld` elements; the view is its first `cols` columns
        ld = c.get("ld", c["cols"])
        return c, uniform_pm1(c["seed"], 0, c["rows"] * ld).reshape(c["rows"], ld), None
    if c["op"] == "gemm_batched":
        # one stream per tensor: the batch index is the slowest dimension of A and of B
        a, b = gemm_inputs(c["B"] * c["M"], c["N"], c["K"], seed=c["seed"], dist=c["dist"])
        nb = c["B"] * c["K"] * c["N"]
        b = (uniform_pm1(c["seed"], 1, nb) if c["dist"] == "uniform" else small_ints(c["seed"], 1, nb))
        return c, a.reshape(c["B"], c["M"], c["K"]), b.reshape(c["B"], c["K"], c["N"])
    if c["op"] in ("gemm", "gemm_transA"):
        a, b = gemm_inputs(c["M"], c["N"], c["K"], seed=c["seed"], dist=c["dist"],
                           trans_a=(c["op"] == "gemm_transA"), bf16=(c["dtype"] == "bf16"))
        return c, a, b
    if c["op"] == "gemm_trans":
        # A stored K x M and B stored N x K: the same streams as the plain product, reshaped
        a, b = gemm_inputs(c["M"], c["N"], c["K"], seed=c["seed"], dist=c["dist"], trans_a=True)
        return c, a, np.ascontiguousarray(b.reshape(c["N"], c["K"]))
    x, w = conv_inputs(c["N"], c["H"], c["W"], c["Cin"], c["Cout"], c["KH"], c["KW"], seed=c["seed"])
    if c["dtype"] == "bf16":
        x, w = f32_to_bf16_bits(x), f32_to_bf16_bits(w)
    return c, x, w
