/*
 * tsg -- tile-scheduled dense contraction for AMD CDNA4 (gfx950), C ABI.
 *
 * The library computes the loop nest that the paper's schedules optimise
 * (Case Study 4, Fig. 7):
 *
 *        C[i][j] (+)= sum_k op(A)[i][k] * op(B)[k][j]
 *
 * with the rewrites of Case Study 3 folded into addressing instead of being
 * materialised: a transposed operand is read in place (tsg_gemm_transA,
 * tsg_gemm_trans), a negate is applied in the store epilogue (TSG_NEGATE), elements
 * produced by zero padding are never formed, read or added (tsg_conv2d_nhwc, an
 * implicit GEMM over M = N*Ho*Wo, N = Cout, K = KH*KW*Cin with k ordered (kh, kw,
 * ci); tsg_conv2d_nhwc_window adds a result into the interior of a padded tensor),
 * and the full additive reduce reads its operand as it lies in memory
 * (tsg_reduce_sum).
 * The knobs of the schedule -- tile sizes per loop, the vectorise flag and their
 * legality constraints (Case Study 5, Fig. 9 and Fig. 10), the split of a loop
 * into a divisible main part and a remainder (Fig. 1, Fig. 8) -- are data:
 * tsg_tile_config and tsg_split.
 *
 * Conventions for every entry point
 *  - All matrices are row-major.  Leading dimensions are in ELEMENTS.
 *  - Pointers named A, B, C, x, w, y are DEVICE pointers owned by the caller; the
 *    library never allocates, frees or retains them.  C / y must not overlap the
 *    inputs.  Pointers named `out`, `off`, `log` ... are HOST pointers.
 *  - Compute calls only enqueue work on `stream` (a hipStream_t passed as void*,
 *    NULL = the default stream) and return; they never synchronise.
 *  - Error model (Sec. 3, silenceable vs. definite errors; Case Study 4,
 *    `alternatives`): TSG_E_SILENCEABLE means a precondition of the requested
 *    schedule failed; NOTHING was enqueued and no output byte was touched, so the
 *    caller may try another alternative.  TSG_E_INVALID and TSG_E_RUNTIME are
 *    definite.  Without TSG_STRICT a compute call walks its own chain of
 *    alternatives (the config pinned by the caller, else the tuner's result for
 *    this very problem -> the library's default for the shape -> that tile with
 *    scalar accesses) and only fails definitely: the last alternative has no
 *    precondition beyond valid arguments.  With TSG_STRICT the call takes the first
 *    alternative only -- the pinned config; with no pin, the tuner's remembered
 *    result for this problem; with neither, the library's default -- and returns
 *    TSG_E_SILENCEABLE if its preconditions fail.
 *  - Operands are fetched in 16-byte accesses from any element-aligned address.  An access
 *    that starts inside a row may run past the row's end (by less than 16 bytes) into the following
 *    row of the same operand (ld >= row length keeps that inside the operand); the last
 *    row of an operand is never read past its end, and nothing outside
 *    [base, base + (rows - 1) * ld + row length) is touched.
 *  - Extents must fit in int32 (each of M, N, K, and every tensor's element count
 *    for convolution), batch <= 65535 and ceil(M/64) * ceil(N/64) <= 2^26; operand
 *    pointers must be aligned to their element type.  Anything else is TSG_E_INVALID.
 *  - The config registry, the tuner's results and the workspace table are guarded
 *    by a mutex; compute calls are re-entrant.  Calls that share one workspace
 *    buffer must be ordered on one stream; calls on different streams may split k
 *    at the same time if each stream has a buffer of its own
 *    (tsg_workspace_set_stream).
 */
#ifndef TSG_H
#define TSG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TSG_OK = 0,
    TSG_E_SILENCEABLE = 1, /* precondition failed, nothing modified (Sec. 3) */
    TSG_E_INVALID = 2,     /* definite: null pointer, bad extent / ld / enum */
    TSG_E_RUNTIME = 3,     /* definite: HIP launch or runtime failure */
    TSG_E_TOO_LARGE = 4    /* definite: beyond the size limit of tsg_gemm_trans_static */
} tsg_status;

typedef enum {
    TSG_F32 = 0,        /* fp32 operands, fp32 MFMA accumulate */
    TSG_BF16_F32ACC = 1 /* bfloat16 operands (bit patterns), fp32 accumulate; C is fp32 */
} tsg_dtype;

typedef enum { TSG_OP_GEMM = 0, TSG_OP_GEMM_TRANSA = 1, TSG_OP_CONV2D_NHWC = 2 } tsg_op;

/* flags of the compute calls */
enum {
    TSG_NEGATE = 1u,     /* C = -(op(A).B): the negate sunk into the epilogue (Case Study 3) */
    TSG_ACCUMULATE = 2u, /* C += ... : the `+=` of Fig. 7; without it C is overwritten */
    TSG_STRICT = 4u      /* first alternative only (pin, else tuned result, else default) or fail silenceably */
};

/*
 * The tuning parameters of Fig. 9 / Fig. 10 as they exist on this hardware.
 *   bm, bn, bk : workgroup tile of the i, j and k loops (tile1..tile3 of Fig. 10; the
 *                batch loop is not tiled).  0 = "library default for this loop" (tiling
 *                by 0 is a no-op, Sec. 3.4).  A tile larger than the extent is legal:
 *                the whole loop becomes remainder.
 *   wm, wn     : per-wavefront sub-tile (multiples of the MFMA block, see mfma).
 *   vec        : elements per global access along the contiguous dimension, the
 *                paper's `vect`: 1, or 4 (fp32) / 8 (bf16) = 16-byte accesses.  Fig. 10
 *                allows vect only when the innermost extent is divisible by the vector
 *                size.  Here the k tile always is, a loop's remainder is peeled into
 *                masked scalar code (Fig. 8), and a matrix row is one contiguous run
 *                whatever its leading dimension, so for the GEMM calls the wide form is
 *                always legal; for the convolution the gathered operand is contiguous
 *                only along Cin, and vec must divide Cin.
 *   raster     : 0 = tiles in row-major order, 1 = XCD-aware grouped order.
 *   sched      : kernel form: 0 = operand tiles staged through registers into two padded LDS
 *                stages, instruction order left to the compiler (serves every access width);
 *                4 / 5 = operand tiles loaded from global memory straight into a ring of
 *                3 / 4 LDS stages (two / three k steps in flight), wide accesses only;
 *                1 = one MFMA block of C per workgroup (bm = bn = wm = wn = 16 or 32), the k
 *                loop dealt over its four wavefronts and operands loaded straight into
 *                registers: for products too small to give every compute unit a tile (the
 *                inner fixed-size matmul of Fig. 8 taken as the whole tile); fp32 matrices
 *                only, split_k must be 1.
 *                -1 = library default.  Only (tile, sched) pairs that are instantiated are
 *                legal.
 *   split_k    : number of workgroups that share one tile of C, each taking a contiguous
 *                range of k steps (tiling the k loop at the grid level when i x j tiles
 *                alone cannot fill the chip).  1 = none; 0 = library default.  Values
 *                above 1 need a workspace (tsg_workspace_set) and at most 16; the partial
 *                tiles are added in split order, so the result does not depend on timing.
 *   split_tail : 0 = split_k applies to every tile.  1 = only the tiles left over after
 *                the last full round of one tile per compute unit (256) are split, the
 *                earlier ones stay whole, all in one launch: the peeled remainder of the
 *                tile loop itself (Fig. 8 applied at the grid level), for tile counts just
 *                above a multiple of 256.  Needs split_k > 1 and a tile count (per batch
 *                entry) that is not a multiple of 256, else silenceable.
 *   mfma       : the MFMA block the wavefront tiles are built from, i.e. the fixed-size inner
 *                matmul of Fig. 8: 0 = 32 x 32 outputs per instruction (32x32x2 fp32,
 *                32x32x16 bf16), 1 = 16 x 16 (16x16x4 fp32, 16x16x32 bf16), which lets wm and wn
 *                move in steps of 16 for extents that a 32-row block would pad (112-row tiles
 *                for 56-pixel image rows).  Part of a tile's identity, like sched.
 */
typedef struct {
    int32_t bm, bn, bk;
    int32_t wm, wn;
    int32_t vec;
    int32_t raster;
    int32_t sched;
    int32_t split_k;
    int32_t split_tail;
    int32_t mfma;
} tsg_tile_config;

/* What the most recent compute call on the calling thread enqueued. */
typedef struct {
    tsg_tile_config config; /* config actually used */
    int32_t alternative;    /* 0 = caller's config, 1 = heuristic, 2 = scalar-access fallback */
    int32_t launches;       /* kernels enqueued */
    int32_t edge;           /* 1 if a remainder (masked) path was compiled into the launch */
    int32_t tiles_m, tiles_n;
    int64_t m_main, m_rest, n_main, n_rest, k_main, k_rest; /* the split (Fig. 8) */
} tsg_launch_info;

/* One evaluation of the tuner (Case Study 5, Fig. 11: runtime per evaluated point). */
typedef struct {
    tsg_tile_config config;
    float ms;        /* mean time of one call (best of three batches); not timed: -1 = illegal
                        here, -2 = pruned (a split of k where the unsplit tiles already fill the
                        chip twice over) */
    float best_ms;   /* best so far, including this evaluation */
    float predicted_ms; /* the cost model's estimate for this point (at 2.4 GHz) */
} tsg_tune_record;

/* ---- compute (device pointers, asynchronous) ---------------------------------- */

/* C[M x N] = +-(A[M x K] . B[K x N]) (+ C).  Fig. 7 without the batch loop.
 * lda >= K, ldb >= N, ldc >= N.  A, B: float (TSG_F32) or uint16 bfloat16 bits. */
tsg_status tsg_gemm(tsg_dtype dtype, int64_t M, int64_t N, int64_t K,
                    const void *A, int64_t lda, const void *B, int64_t ldb,
                    float *C, int64_t ldc, uint32_t flags, void *stream);

/* Same with the left operand stored transposed: A is K x M row-major (lda >= M) and
 * op(A) = A^T is read in place (Case Study 3, transpose folded into the matmul). */
tsg_status tsg_gemm_transA(tsg_dtype dtype, int64_t M, int64_t N, int64_t K,
                           const void *A, int64_t lda, const void *B, int64_t ldb,
                           float *C, int64_t ldc, uint32_t flags, void *stream);

/* Batched form of Fig. 7: `batch` independent products, operand b at base + b*stride
 * (strides in elements; stride 0 broadcasts an input). */
tsg_status tsg_gemm_batched(tsg_dtype dtype, int32_t trans_a, int64_t batch,
                            int64_t M, int64_t N, int64_t K,
                            const void *A, int64_t lda, int64_t stride_a,
                            const void *B, int64_t ldb, int64_t stride_b,
                            float *C, int64_t ldc, int64_t stride_c,
                            uint32_t flags, void *stream);

/* The general form: either operand, or both, stored transposed and read in place (Case
 * Study 3: transposes folded into a matmul that takes transposed operands).  trans_a: A is
 * K x M (lda >= M); trans_b: B is N x K (ldb >= K).  Batched like tsg_gemm_batched.  A
 * transposed B is served by the direct-to-LDS kernel forms (sched 4, 5) and the block form (sched 1): a pinned config
 * of another form is a silenceable failure and the library's default for the shape is used. */
tsg_status tsg_gemm_trans(tsg_dtype dtype, int32_t trans_a, int32_t trans_b, int64_t batch,
                          int64_t M, int64_t N, int64_t K,
                          const void *A, int64_t lda, int64_t stride_a,
                          const void *B, int64_t ldb, int64_t stride_b,
                          float *C, int64_t ldc, int64_t stride_c,
                          uint32_t flags, void *stream);

/* tsg_gemm_trans for callers that cannot allocate device memory and so have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same results (bit for bit, for the same tile config) as
 * tsg_gemm_trans with a workspace of TSG_STATIC_SCRATCH_BYTES bytes; the scratch for the
 * split of the k loop is a device array of that size inside the library's code object (each
 * GPU the library runs on holds one copy until the process ends).  The call allocates and
 * frees nothing and only enqueues kernels on `stream`; its first use on a device also enqueues
 * a kernel that zeroes the arrival counters.  Limit: batch * M * N, with M and N rounded up to
 * multiples of 64, at most TSG_STATIC_MAX_OUTPUTS (a two-way split of every tile then fits):
 * beyond it TSG_E_TOO_LARGE, nothing enqueued -- such outputs have tiles enough to fill the
 * chip and do not need the split, so tsg_gemm_trans serves them without a workspace.  All
 * calls on one GPU share that GPU's array: two of them in flight at once (different streams,
 * or replays of two graphs) race, exactly like two calls sharing one caller-owned workspace.
 * A pinned or tuned config that needs more scratch than the array holds is a silenceable
 * failure and the chain of alternatives goes on, as in tsg_gemm_trans. */
#define TSG_STATIC_SCRATCH_BYTES (65536 + (8 << 20))
#define TSG_STATIC_MAX_OUTPUTS (1 << 20)
tsg_status tsg_gemm_trans_static(tsg_dtype dtype, int32_t trans_a, int32_t trans_b, int64_t batch,
                                 int64_t M, int64_t N, int64_t K,
                                 const void *A, int64_t lda, int64_t stride_a,
                                 const void *B, int64_t ldb, int64_t stride_b,
                                 float *C, int64_t ldc, int64_t stride_c,
                                 uint32_t flags, void *stream);

/* y[N][Ho][Wo][Cout] = +-conv(x[N][H][W][Cin], w[KH][KW][Cin][Cout]) (+ y), zero
 * padding (pad_h, pad_w) never materialised; Ho = (H + 2*pad_h - KH)/stride_h + 1. */
tsg_status tsg_conv2d_nhwc(tsg_dtype dtype, int64_t N, int64_t H, int64_t W, int64_t Cin,
                           int64_t Cout, int64_t KH, int64_t KW,
                           int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                           const void *x, const void *w, float *y,
                           uint32_t flags, void *stream);

/* The same convolution with its result placed in a window of a larger NHWC tensor: output
 * pixel (n, ho, wo), channel co goes to y[n*y_stride_n + ho*y_stride_h + wo*y_stride_w + co]
 * (strides in elements, y = address of pixel (0, 0, 0)).  With TSG_ACCUMULATE this adds the
 * result to the interior of a zero-padded tensor without forming the padded result (Case
 * Study 3, the add-of-zero-pad rewrite); elements outside the window are never touched.
 * The same for a GEMM needs no extra call: pass C = &C_big[r0][c0] and ldc = pitch of C_big.
 * TSG_E_INVALID if the strides let two pixels of the window overlap. */
tsg_status tsg_conv2d_nhwc_window(tsg_dtype dtype, int64_t N, int64_t H, int64_t W, int64_t Cin,
                                  int64_t Cout, int64_t KH, int64_t KW,
                                  int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                                  const void *x, const void *w, float *y,
                                  int64_t y_stride_n, int64_t y_stride_h, int64_t y_stride_w,
                                  uint32_t flags, void *stream);

/* Full additive reduce: out[0] = +-(sum over r < rows, c < cols of x[r*ld + c]) (+ out[0]),
 * x fp32 or bfloat16 bits, accumulated in fp32 in a fixed order (results are repeatable).
 * Case Study 3: a full additive reduce may ignore a reshape or transpose of its operand, so
 * a tensor is passed as it lies in memory, whatever view the program had of it (ld >= cols;
 * ld == cols means one contiguous run).  x, out: DEVICE pointers.  One workgroup per 16 K
 * elements, up to 768; more than one needs the workspace (tsg_workspace_set) for the
 * workgroup sums: without it the call runs as one workgroup, or fails silenceably under
 * TSG_STRICT. */
tsg_status tsg_reduce_sum(tsg_dtype dtype, int64_t rows, int64_t cols, const void *x, int64_t ld,
                          float *out, uint32_t flags, void *stream);

/* ---- schedule parameters (host only; no GPU needed) --------------------------- */

/* Loop split of Fig. 1 / Fig. 8: main = largest multiple of d <= ub, rest = ub - main
 * (< d), tiles = main / d.  d == 0 leaves the loop whole (main = ub, one tile).
 * TSG_E_INVALID for ub < 0, d < 0 or null outputs. */
tsg_status tsg_split(int64_t ub, int64_t d, int64_t *main_part, int64_t *rest, int64_t *tiles);

/* Size of the instantiated search space and its idx-th point. */
int32_t tsg_tile_config_count(tsg_op op, tsg_dtype dtype);
tsg_status tsg_tile_config_enum(tsg_op op, tsg_dtype dtype, int32_t idx, tsg_tile_config *out);

/* Legality of a config for a problem with natural leading dimensions and aligned
 * pointers.  For convolution pass the implicit extents and Cin as `contig`
 * (the contiguous run of the gathered operand); for GEMM contig is ignored.
 * TSG_E_SILENCEABLE if the tile is not instantiated, `vec` violates Fig. 10's
 * divisibility rule, split_k exceeds 16 or the number of k steps, or split_tail is set with
 * split_k = 1 or a tile count that leaves no tail; TSG_E_INVALID for
 * malformed arguments. */
tsg_status tsg_tile_config_check(tsg_op op, tsg_dtype dtype, int64_t M, int64_t N, int64_t K,
                                 int64_t contig, const tsg_tile_config *cfg);

/* Pin the config used by later calls of (op, dtype), whatever their extents; NULL clears the pin.
 * Zero fields are filled from the default.  Validates instantiation first:
 * on TSG_E_SILENCEABLE the registry is unchanged. */
tsg_status tsg_tile_config_set(tsg_op op, tsg_dtype dtype, const tsg_tile_config *cfg);

/* The config a call with these extents would try first right now. */
tsg_status tsg_tile_config_get(tsg_op op, tsg_dtype dtype, int64_t M, int64_t N, int64_t K,
                               tsg_tile_config *out);

/* Workspace for split_k > 1: `ws` is a DEVICE buffer of `bytes` bytes, 256-byte aligned,
 * owned by the caller, who keeps it alive and unused by anything else until it is replaced
 * or cleared with (NULL, 0).  The library keeps arrival counters in its first 64 KiB (this
 * call zeroes them, synchronously; the kernels leave them at zero; the last one is the full
 * reduce's, so a GEMM and a reduce may follow each other on one buffer) and partial tiles
 * after that.  Compute calls that use
 * the workspace must be ordered on one stream: two of them in flight at once race.
 * Without a workspace (or with one that is too small for a config) split_k > 1 is a
 * silenceable failure and the chain of alternatives continues with split_k = 1. */
tsg_status tsg_workspace_set(void *ws, int64_t bytes);

/* The same for the calls made on one stream only: a compute call on `stream` (the handle it
 * is given, NULL = the default stream) uses this buffer in place of the process-wide one, so
 * calls on different streams, each with its own buffer, may split k concurrently.  (NULL, 0)
 * removes the stream's entry.  Same requirements and return codes as tsg_workspace_set. */
tsg_status tsg_workspace_set_stream(void *stream, void *ws, int64_t bytes);

/* Bytes of workspace a call with this batch, M, N and config needs (0 when split_k is 1);
 * -1 for malformed arguments or a tile that is not instantiated. */
int64_t tsg_workspace_bytes(tsg_dtype dtype, int64_t batch, int64_t M, int64_t N,
                            const tsg_tile_config *cfg);

/* Details of the last compute call made by the calling thread. */
tsg_status tsg_last_launch(tsg_launch_info *out);

/* ---- index maps (host only, integer, compared bit-exactly) -------------------- */

/* off[m*KH*KW + kh*KW + kw] = element offset of x[n][hi][wi][0] for output pixel
 * m = (n*Ho + ho)*Wo + wo, hi = ho*stride_h + kh - pad_h, wi likewise; -1 where the
 * tap falls in the zero padding.  `off` is a HOST array of N*Ho*Wo*KH*KW int32.
 * This is the map the lowering is DEFINED by, evaluated on the host; the kernels' own
 * gather is not exported (it runs on the device) and is held to this map through results:
 * on integer-valued data a wrong offset or mask changes C, which must match bit for bit. */
tsg_status tsg_conv2d_index_map(int64_t N, int64_t H, int64_t W, int64_t Cin,
                                int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w,
                                int64_t pad_h, int64_t pad_w, int32_t *off);

/* off[i*K + k] = element offset of op(A)(i,k): i*lda + k, or k*lda + i if trans_a. */
tsg_status tsg_gemm_index_map(int32_t trans_a, int64_t M, int64_t K, int64_t lda, int64_t *off);

/* ---- search (Case Study 5) ----------------------------------------------------- */

/* Budget and order of the tuner calls that follow.  max_evals: stop after that many timed
 * points (0 = all).  model_order: 0 = visit the points in enumeration order; 1 = in the order
 * of the library's cost model, so that the first timed point is the library's default for the
 * shape and a small budget covers the likely winners; 2 = model-based search: the cost model is
 * a prior, every timed point corrects it (the ratio measured / predicted, per kernel and
 * overall), and the next point timed is the one with the smallest corrected prediction, so a
 * kernel family the prior flatters drops back after its first measurement (Case Study 5 couples
 * the parameters to a model-based tuner; this is the same loop with a hand-made surrogate).
 * Default (0, 1). */
tsg_status tsg_search_set(int32_t max_evals, int32_t model_order);

/* Time every legal instantiated config on the caller's buffers (three batches of `iters`
 * back-to-back calls each, after one warm-up) and remember the fastest for THIS problem (op,
 * dtype, transposition, batch, extents): later calls with the same problem use it like a
 * pinned config, unless tsg_tile_config_set has pinned another.  This
 * call SYNCHRONISES the stream and overwrites C / y.  `log` (host, may be NULL)
 * receives up to log_cap records in evaluation order; *n_log the number written. */
tsg_status tsg_autotune_gemm(tsg_dtype dtype, int32_t trans_a, int64_t M, int64_t N, int64_t K,
                             const void *A, int64_t lda, const void *B, int64_t ldb,
                             float *C, int64_t ldc, uint32_t flags, void *stream, int32_t iters,
                             tsg_tile_config *best, float *best_ms,
                             tsg_tune_record *log, int32_t log_cap, int32_t *n_log);

/* The same search on a batched call (the config that is fastest for the whole batch). */
tsg_status tsg_autotune_gemm_batched(tsg_dtype dtype, int32_t trans_a, int64_t batch,
                                     int64_t M, int64_t N, int64_t K,
                                     const void *A, int64_t lda, int64_t stride_a,
                                     const void *B, int64_t ldb, int64_t stride_b,
                                     float *C, int64_t ldc, int64_t stride_c,
                                     uint32_t flags, void *stream, int32_t iters,
                                     tsg_tile_config *best, float *best_ms,
                                     tsg_tune_record *log, int32_t log_cap, int32_t *n_log);

/* The same search for the general form (tsg_gemm_trans). */
tsg_status tsg_autotune_gemm_trans(tsg_dtype dtype, int32_t trans_a, int32_t trans_b, int64_t batch,
                                   int64_t M, int64_t N, int64_t K,
                                   const void *A, int64_t lda, int64_t stride_a,
                                   const void *B, int64_t ldb, int64_t stride_b,
                                   float *C, int64_t ldc, int64_t stride_c,
                                   uint32_t flags, void *stream, int32_t iters,
                                   tsg_tile_config *best, float *best_ms,
                                   tsg_tune_record *log, int32_t log_cap, int32_t *n_log);

tsg_status tsg_autotune_conv2d_nhwc(tsg_dtype dtype, int64_t N, int64_t H, int64_t W, int64_t Cin,
                                    int64_t Cout, int64_t KH, int64_t KW,
                                    int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w,
                                    const void *x, const void *w, float *y,
                                    uint32_t flags, void *stream, int32_t iters,
                                    tsg_tile_config *best, float *best_ms,
                                    tsg_tune_record *log, int32_t log_cap, int32_t *n_log);

/* The tuner's results (host only).  save writes one text line per tuned problem; load adds
 * the lines of such a file to the cache (entries whose config is not instantiated in this
 * build, or malformed lines, are counted in *rejected and skipped; both counters may be
 * NULL).  TSG_E_RUNTIME if the file cannot be opened or written. */
int32_t    tsg_tune_cache_size(void);
tsg_status tsg_tune_cache_clear(void);
tsg_status tsg_tune_cache_save(const char *path);
tsg_status tsg_tune_cache_load(const char *path, int32_t *loaded, int32_t *rejected);

/* Measurement aid for the roofline figures: the rate the matrix pipes sustain with every
 * operand in registers (no LDS, no memory, no barrier), one or two wavefronts per SIMD on every
 * compute unit, for the MFMA block shape `mfma` (0 = 32 x 32, 1 = 16 x 16) of the dtype, with
 * constant operands or (random_operands = 1) operands distributed like the workloads' entries.
 * Runs `launches` (2..1000) kernels of about 10 ms on `stream` and SYNCHRONISES; tflops[0] =
 * fastest launch, tflops[1] = mean over the second half of the launches (the sustained rate),
 * both HOST floats.  `sink` is a DEVICE buffer of at least 2 MiB that receives throw-away
 * results. */
tsg_status tsg_mfma_ceiling(tsg_dtype dtype, int32_t mfma, int32_t random_operands, int32_t waves_per_simd,
                            int32_t launches, float *sink, int64_t sink_bytes, float *tflops, void *stream);

/* Measurement aid for the small shapes: the time per launch, in microseconds (HOST float), of
 * `launches` (1..1000000) back-to-back launches of a kernel that does nothing, between two
 * events on `stream`: the cost that every compute call of this library pays before its first
 * instruction.  SYNCHRONISES. */
tsg_status tsg_launch_floor(int32_t launches, float *us_per_launch, void *stream);

const char *tsg_status_string(tsg_status s);
int32_t tsg_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TSG_H */
