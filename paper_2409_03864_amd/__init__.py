"""Python binding of libtsg.so: the same names as the C ABI in include/tsg.h, argument
marshalling only.  Every step of the computation runs in the HIP kernels behind the
library; PyTorch is used by callers for device memory and streams, never for math.

The library must have been built (`python paper_2409_03864_amd/build.py`, or
`__graft_entry__.build()`); importing this package without it raises ImportError --
there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtsg.so")

OK, E_SILENCEABLE, E_INVALID, E_RUNTIME, E_TOO_LARGE = 0, 1, 2, 3, 4
STATIC_SCRATCH_BYTES = 65536 + (8 << 20)      # TSG_STATIC_SCRATCH_BYTES
STATIC_MAX_OUTPUTS = 1 << 20                  # TSG_STATIC_MAX_OUTPUTS
F32, BF16_F32ACC = 0, 1
OP_GEMM, OP_GEMM_TRANSA, OP_CONV2D_NHWC = 0, 1, 2
NEGATE, ACCUMULATE, STRICT = 1, 2, 4


class TileConfig(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("bm", "bn", "bk", "wm", "wn", "vec", "raster", "sched", "split_k",
                                                   "split_tail", "mfma")]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}

    def __repr__(self):
        return "TileConfig(%s)" % ", ".join("%s=%d" % kv for kv in self.as_dict().items())


class LaunchInfo(ctypes.Structure):
    _fields_ = ([("config", TileConfig)] +
                [(n, ctypes.c_int32) for n in ("alternative", "launches", "edge", "tiles_m", "tiles_n")] +
                [(n, ctypes.c_int64) for n in ("m_main", "m_rest", "n_main", "n_rest", "k_main", "k_rest")])


class TuneRecord(ctypes.Structure):
    _fields_ = [("config", TileConfig), ("ms", ctypes.c_float), ("best_ms", ctypes.c_float),
                ("predicted_ms", ctypes.c_float)]


class TsgError(RuntimeError):
    def __init__(self, status, what):
        super().__init__("%s: %s" % (what, status_string(status)))
        self.status = status


class SilenceableError(TsgError):
    """A precondition of the requested schedule failed; nothing was modified."""


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("libtsg.so is not built: run `python paper_2409_03864_amd/build.py` "
                          "(needs hipcc); this package has no CPU fallback")
    lib = ctypes.CDLL(LIB_PATH)
    i32, i64, u32, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32, ctypes.c_void_p
    cfgp = ctypes.POINTER(TileConfig)
    sig = {
        "tsg_gemm": [i32, i64, i64, i64, vp, i64, vp, i64, vp, i64, u32, vp],
        "tsg_gemm_transA": [i32, i64, i64, i64, vp, i64, vp, i64, vp, i64, u32, vp],
        "tsg_gemm_batched": [i32, i32, i64, i64, i64, i64, vp, i64, i64, vp, i64, i64, vp, i64, i64, u32, vp],
        "tsg_gemm_trans": [i32, i32, i32, i64, i64, i64, i64, vp, i64, i64, vp, i64, i64, vp, i64, i64, u32, vp],
        "tsg_gemm_trans_static": [i32, i32, i32, i64, i64, i64, i64, vp, i64, i64, vp, i64, i64, vp, i64, i64, u32, vp],
        "tsg_conv2d_nhwc": [i32] + [i64] * 11 + [vp, vp, vp, u32, vp],
        "tsg_conv2d_nhwc_window": [i32] + [i64] * 11 + [vp, vp, vp, i64, i64, i64, u32, vp],
        "tsg_reduce_sum": [i32, i64, i64, vp, i64, vp, u32, vp],
        "tsg_mfma_ceiling": [i32, i32, i32, i32, i32, vp, i64, ctypes.POINTER(ctypes.c_float), vp],
        "tsg_launch_floor": [i32, ctypes.POINTER(ctypes.c_float), vp],
        "tsg_split": [i64, i64, vp, vp, vp],
        "tsg_tile_config_enum": [i32, i32, i32, cfgp],
        "tsg_tile_config_check": [i32, i32, i64, i64, i64, i64, cfgp],
        "tsg_tile_config_set": [i32, i32, cfgp],
        "tsg_tile_config_get": [i32, i32, i64, i64, i64, cfgp],
        "tsg_last_launch": [ctypes.POINTER(LaunchInfo)],
        "tsg_workspace_set": [vp, i64],
        "tsg_workspace_set_stream": [vp, vp, i64],
        "tsg_search_set": [i32, i32],
        "tsg_tune_cache_clear": [],
        "tsg_tune_cache_save": [ctypes.c_char_p],
        "tsg_tune_cache_load": [ctypes.c_char_p, ctypes.POINTER(i32), ctypes.POINTER(i32)],
        "tsg_conv2d_index_map": [i64] * 10 + [vp],
        "tsg_gemm_index_map": [i32, i64, i64, i64, vp],
        "tsg_autotune_gemm": [i32, i32, i64, i64, i64, vp, i64, vp, i64, vp, i64, u32, vp, i32,
                              cfgp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(TuneRecord), i32,
                              ctypes.POINTER(i32)],
        "tsg_autotune_gemm_batched": [i32, i32, i64, i64, i64, i64, vp, i64, i64, vp, i64, i64, vp, i64, i64, u32,
                                      vp, i32, cfgp, ctypes.POINTER(ctypes.c_float),
                                      ctypes.POINTER(TuneRecord), i32, ctypes.POINTER(i32)],
        "tsg_autotune_gemm_trans": [i32, i32, i32, i64, i64, i64, i64, vp, i64, i64, vp, i64, i64, vp, i64, i64, u32,
                                    vp, i32, cfgp, ctypes.POINTER(ctypes.c_float),
                                    ctypes.POINTER(TuneRecord), i32, ctypes.POINTER(i32)],
        "tsg_autotune_conv2d_nhwc": [i32] + [i64] * 11 + [vp, vp, vp, u32, vp, i32,
                                                          cfgp, ctypes.POINTER(ctypes.c_float),
                                                          ctypes.POINTER(TuneRecord), i32, ctypes.POINTER(i32)],
    }
    for name, args in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = ctypes.c_int
    lib.tsg_tile_config_count.argtypes = [i32, i32]
    lib.tsg_tile_config_count.restype = i32
    lib.tsg_workspace_bytes.argtypes = [i32, i64, i64, i64, cfgp]
    lib.tsg_workspace_bytes.restype = i64
    lib.tsg_tune_cache_size.argtypes = []
    lib.tsg_tune_cache_size.restype = i32
    lib.tsg_status_string.argtypes = [ctypes.c_int]
    lib.tsg_status_string.restype = ctypes.c_char_p
    lib.tsg_version.argtypes = []
    lib.tsg_version.restype = i32
    return lib


_lib = _load()

EXPORTS = ("tsg_gemm", "tsg_gemm_transA", "tsg_gemm_batched", "tsg_gemm_trans", "tsg_gemm_trans_static", "tsg_autotune_gemm_trans", "tsg_conv2d_nhwc", "tsg_conv2d_nhwc_window",
           "tsg_reduce_sum", "tsg_mfma_ceiling", "tsg_launch_floor", "tsg_split",
           "tsg_tile_config_count", "tsg_tile_config_enum", "tsg_tile_config_check",
           "tsg_tile_config_set", "tsg_tile_config_get", "tsg_last_launch", "tsg_workspace_set",
           "tsg_workspace_set_stream", "tsg_workspace_bytes", "tsg_search_set", "tsg_tune_cache_size", "tsg_tune_cache_clear",
           "tsg_tune_cache_save", "tsg_tune_cache_load", "tsg_conv2d_index_map",
           "tsg_gemm_index_map", "tsg_autotune_gemm", "tsg_autotune_gemm_batched", "tsg_autotune_conv2d_nhwc",
           "tsg_status_string", "tsg_version")


def status_string(status: int) -> str:
    return _lib.tsg_status_string(int(status)).decode()


def version() -> int:
    return int(_lib.tsg_version())


def _check(status, what):
    if status == OK:
        return
    if status == E_SILENCEABLE:
        raise SilenceableError(status, what)
    raise TsgError(status, what)


def _ptr(t):
    """Device (or host, for numpy) address of a tensor / array / raw int."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    return t.ctypes.data


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


# ---- compute ------------------------------------------------------------------------

def gemm(dtype, M, N, K, A, lda, B, ldb, C, ldc, flags=0, stream=None):
    _check(_lib.tsg_gemm(dtype, M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, flags, _stream(stream)),
           "tsg_gemm")


def gemm_transA(dtype, M, N, K, A, lda, B, ldb, C, ldc, flags=0, stream=None):
    _check(_lib.tsg_gemm_transA(dtype, M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C), ldc, flags,
                                _stream(stream)), "tsg_gemm_transA")


def gemm_batched(dtype, trans_a, batch, M, N, K, A, lda, stride_a, B, ldb, stride_b, C, ldc, stride_c,
                 flags=0, stream=None):
    _check(_lib.tsg_gemm_batched(dtype, int(bool(trans_a)), batch, M, N, K, _ptr(A), lda, stride_a,
                                 _ptr(B), ldb, stride_b, _ptr(C), ldc, stride_c, flags, _stream(stream)),
           "tsg_gemm_batched")


def gemm_trans(dtype, trans_a, trans_b, batch, M, N, K, A, lda, stride_a, B, ldb, stride_b, C, ldc, stride_c,
               flags=0, stream=None):
    _check(_lib.tsg_gemm_trans(dtype, int(bool(trans_a)), int(bool(trans_b)), batch, M, N, K, _ptr(A), lda, stride_a,
                               _ptr(B), ldb, stride_b, _ptr(C), ldc, stride_c, flags, _stream(stream)),
           "tsg_gemm_trans")


def gemm_trans_static(dtype, trans_a, trans_b, batch, M, N, K, A, lda, stride_a, B, ldb, stride_b, C, ldc,
                      stride_c, flags=0, stream=None):
    _check(_lib.tsg_gemm_trans_static(dtype, int(bool(trans_a)), int(bool(trans_b)), batch, M, N, K, _ptr(A), lda,
                                      stride_a, _ptr(B), ldb, stride_b, _ptr(C), ldc, stride_c, flags,
                                      _stream(stream)), "tsg_gemm_trans_static")


def conv2d_nhwc(dtype, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w, pad_h, pad_w, x, w, y,
                flags=0, stream=None):
    _check(_lib.tsg_conv2d_nhwc(dtype, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w, pad_h, pad_w,
                                _ptr(x), _ptr(w), _ptr(y), flags, _stream(stream)), "tsg_conv2d_nhwc")


def conv2d_nhwc_window(dtype, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w, pad_h, pad_w, x, w, y,
                       y_stride_n, y_stride_h, y_stride_w, flags=0, stream=None):
    _check(_lib.tsg_conv2d_nhwc_window(dtype, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w, pad_h, pad_w,
                                       _ptr(x), _ptr(w), _ptr(y), y_stride_n, y_stride_h, y_stride_w, flags,
                                       _stream(stream)), "tsg_conv2d_nhwc_window")


def reduce_sum(dtype, rows, cols, x, ld, out, flags=0, stream=None):
    _check(_lib.tsg_reduce_sum(dtype, rows, cols, _ptr(x), ld, _ptr(out), flags, _stream(stream)), "tsg_reduce_sum")


def mfma_ceiling(dtype, mfma, random_operands, waves_per_simd, launches, sink, stream=None):
    """(fastest, sustained) TFLOP/s of the register-only MFMA loop; `sink` is a device tensor of >= 2 MiB."""
    out = (ctypes.c_float * 2)()
    _check(_lib.tsg_mfma_ceiling(dtype, mfma, int(bool(random_operands)), waves_per_simd, launches, _ptr(sink),
                                 sink.numel() * sink.element_size(), out, _stream(stream)), "tsg_mfma_ceiling")
    return float(out[0]), float(out[1])


def launch_floor(launches=20000, stream=None):
    """Microseconds per launch of an empty kernel, back to back on one stream."""
    out = ctypes.c_float()
    _check(_lib.tsg_launch_floor(launches, ctypes.byref(out), _stream(stream)), "tsg_launch_floor")
    return float(out.value)


# ---- schedule parameters (host only) -----------------------------------------------

def split(ub, d):
    m, r, t = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    _check(_lib.tsg_split(ub, d, ctypes.addressof(m), ctypes.addressof(r), ctypes.addressof(t)), "tsg_split")
    return m.value, r.value, t.value


def tile_config_count(op, dtype) -> int:
    return int(_lib.tsg_tile_config_count(op, dtype))


def tile_config_enum(op, dtype, idx) -> TileConfig:
    c = TileConfig()
    _check(_lib.tsg_tile_config_enum(op, dtype, idx, ctypes.byref(c)), "tsg_tile_config_enum")
    return c


def tile_config_check(op, dtype, M, N, K, cfg, contig=0) -> int:
    """Returns the status code (OK / E_SILENCEABLE / E_INVALID) without raising."""
    return int(_lib.tsg_tile_config_check(op, dtype, M, N, K, contig, ctypes.byref(cfg)))


def tile_config_set(op, dtype, cfg):
    _check(_lib.tsg_tile_config_set(op, dtype, ctypes.byref(cfg) if cfg is not None else None),
           "tsg_tile_config_set")


def tile_config_get(op, dtype, M, N, K) -> TileConfig:
    c = TileConfig()
    _check(_lib.tsg_tile_config_get(op, dtype, M, N, K, ctypes.byref(c)), "tsg_tile_config_get")
    return c


def workspace_set(ws, nbytes=None):
    """Hand the library a device buffer for split_k > 1 (a tensor, or a raw address plus
    nbytes); None clears it.  The caller keeps the buffer alive."""
    if ws is None:
        _check(_lib.tsg_workspace_set(None, 0), "tsg_workspace_set")
        return
    if nbytes is None:
        nbytes = ws.numel() * ws.element_size()
    _check(_lib.tsg_workspace_set(_ptr(ws), nbytes), "tsg_workspace_set")


def workspace_set_stream(stream, ws, nbytes=None):
    """The same for the calls made on one stream (a torch stream or a raw handle; None = the
    current stream): ws None removes the stream's entry."""
    if ws is None:
        _check(_lib.tsg_workspace_set_stream(_stream(stream), None, 0), "tsg_workspace_set_stream")
        return
    if nbytes is None:
        nbytes = ws.numel() * ws.element_size()
    _check(_lib.tsg_workspace_set_stream(_stream(stream), _ptr(ws), nbytes), "tsg_workspace_set_stream")


def workspace_bytes(dtype, batch, M, N, cfg) -> int:
    return int(_lib.tsg_workspace_bytes(dtype, batch, M, N, ctypes.byref(cfg)))


def last_launch() -> LaunchInfo:
    li = LaunchInfo()
    _check(_lib.tsg_last_launch(ctypes.byref(li)), "tsg_last_launch")
    return li


# ---- index maps (host arrays) ---------------------------------------------------------

def conv2d_index_map(N, H, W, Cin, KH, KW, stride_h, stride_w, pad_h, pad_w, off):
    _check(_lib.tsg_conv2d_index_map(N, H, W, Cin, KH, KW, stride_h, stride_w, pad_h, pad_w, _ptr(off)),
           "tsg_conv2d_index_map")


def gemm_index_map(trans_a, M, K, lda, off):
    _check(_lib.tsg_gemm_index_map(int(bool(trans_a)), M, K, lda, _ptr(off)), "tsg_gemm_index_map")


# ---- search ---------------------------------------------------------------------------

def search_set(max_evals=0, model_order=1):
    """model_order: 0 enumeration order, 1 (or True) cost-model order, 2 model corrected by the timed points."""
    _check(_lib.tsg_search_set(max_evals, int(model_order)), "tsg_search_set")


def tune_cache_size() -> int:
    return int(_lib.tsg_tune_cache_size())


def tune_cache_clear():
    _check(_lib.tsg_tune_cache_clear(), "tsg_tune_cache_clear")


def tune_cache_save(path):
    _check(_lib.tsg_tune_cache_save(os.fsencode(path)), "tsg_tune_cache_save")


def tune_cache_load(path):
    """Returns (entries loaded, lines rejected)."""
    ok, bad = ctypes.c_int32(), ctypes.c_int32()
    _check(_lib.tsg_tune_cache_load(os.fsencode(path), ctypes.byref(ok), ctypes.byref(bad)), "tsg_tune_cache_load")
    return ok.value, bad.value


def _tune_out(cap):
    return TileConfig(), ctypes.c_float(), (TuneRecord * cap)(), ctypes.c_int32()


def autotune_gemm(dtype, trans_a, M, N, K, A, lda, B, ldb, C, ldc, flags=0, stream=None, iters=5,
                  log_cap=512):
    best, ms, log, n = _tune_out(log_cap)
    _check(_lib.tsg_autotune_gemm(dtype, int(bool(trans_a)), M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(C),
                                  ldc, flags, _stream(stream), iters, ctypes.byref(best), ctypes.byref(ms),
                                  log, log_cap, ctypes.byref(n)), "tsg_autotune_gemm")
    return best, float(ms.value), [log[i] for i in range(n.value)]


def autotune_gemm_batched(dtype, trans_a, batch, M, N, K, A, lda, stride_a, B, ldb, stride_b, C, ldc, stride_c,
                          flags=0, stream=None, iters=5, log_cap=512):
    best, ms, log, n = _tune_out(log_cap)
    _check(_lib.tsg_autotune_gemm_batched(dtype, int(bool(trans_a)), batch, M, N, K, _ptr(A), lda, stride_a,
                                          _ptr(B), ldb, stride_b, _ptr(C), ldc, stride_c, flags, _stream(stream),
                                          iters, ctypes.byref(best), ctypes.byref(ms), log, log_cap,
                                          ctypes.byref(n)), "tsg_autotune_gemm_batched")
    return best, float(ms.value), [log[i] for i in range(n.value)]


def autotune_gemm_trans(dtype, trans_a, trans_b, batch, M, N, K, A, lda, stride_a, B, ldb, stride_b, C, ldc,
                        stride_c, flags=0, stream=None, iters=5, log_cap=512):
    best, ms, log, n = _tune_out(log_cap)
    _check(_lib.tsg_autotune_gemm_trans(dtype, int(bool(trans_a)), int(bool(trans_b)), batch, M, N, K, _ptr(A), lda,
                                        stride_a, _ptr(B), ldb, stride_b, _ptr(C), ldc, stride_c, flags,
                                        _stream(stream), iters, ctypes.byref(best), ctypes.byref(ms), log, log_cap,
                                        ctypes.byref(n)), "tsg_autotune_gemm_trans")
    return best, float(ms.value), [log[i] for i in range(n.value)]


def autotune_conv2d_nhwc(dtype, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w, pad_h, pad_w, x, w, y,
                         flags=0, stream=None, iters=5, log_cap=512):
    best, ms, log, n = _tune_out(log_cap)
    _check(_lib.tsg_autotune_conv2d_nhwc(dtype, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w, pad_h,
                                         pad_w, _ptr(x), _ptr(w), _ptr(y), flags, _stream(stream), iters,
                                         ctypes.byref(best), ctypes.byref(ms), log, log_cap,
                                         ctypes.byref(n)), "tsg_autotune_conv2d_nhwc")
    return best, float(ms.value), [log[i] for i in range(n.value)]
