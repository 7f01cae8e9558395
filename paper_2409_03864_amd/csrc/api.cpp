// C-ABI layer: argument validation, the loop split, the tile-config registry with its
// legality rules, the chain of alternatives, launch planning and the tuner.
// Host code, plus the static scratch of the allocation-free entry point; the kernels live in
// gemm_kernel.h (instantiated by gemm_f32_*.hip and gemm_bf16_*.hip) and reduce.hip.
#include <algorithm>
#include <array>
#include <cmath>
#include <cstdio>
#include <map>
#include <cstring>
#include <mutex>
#include <vector>

#include "../../include/tsg.h"
#include "tsg_internal.h"

namespace {

using tsg::KArgs;
using tsg::KernelEntry;

constexpr int kNumOps = 3, kNumDtypes = 2;
constexpr int kCUs = 256;

struct Problem {
    tsg_op op;
    tsg_dtype dtype;
    int64_t batch = 1;
    int64_t M, N, K;
    const void* A;
    const void* B;
    float* C;
    int64_t lda, ldb, ldc;
    int64_t stride_a = 0, stride_b = 0, stride_c = 0;
    bool trans_b = false;   // B stored N x K (direct-to-LDS kernel forms only)
    uint32_t flags;
    // convolution geometry
    int64_t H = 0, W = 0, Cin = 0, Ho = 0, Wo = 0, KH = 0, KW = 0, sh = 1, sw = 1, ph = 0, pw = 0;
    // output window strides (elements); y_window = 0: y is a plain [N*Ho*Wo][Cout] matrix
    int y_window = 0;
    int64_t y_sn = 0, y_sh = 0, y_sw = 0;
    // scratch for split k, resolved when the call enters the library: the buffer registered for
    // the call's stream, else the process-wide one (none: split k is not available)
    void* ws = nullptr;
    int64_t ws_bytes = 0;
};

std::mutex g_mu;
bool g_pinned[kNumOps][kNumDtypes];
tsg_tile_config g_pin[kNumOps][kNumDtypes];

// Results of the tuner, per problem: (op, dtype, B transposed, batch, M, N, K, contiguous run
// of the gathered operand) -> (config, time).  A call whose problem has an entry uses it
// like a pinned config; tsg_tune_cache_save / _load carry the entries across processes.
using TuneKey = std::array<int64_t, 8>;
struct TuneVal { tsg_tile_config cfg; float ms; };
std::map<TuneKey, TuneVal> g_tuned;

// Caller-owned workspace for split k: arrival counters first, partial tiles after them.  The
// last counter belongs to the full reduce, the others to the (batch x tile) slots of a GEMM.
constexpr int64_t kMaxSlots = tsg::kWorkspaceReduceSlot;
constexpr int64_t kCounterBytes = tsg::kWorkspaceCounterBytes;
static_assert(kCounterBytes == (kMaxSlots + 1) * 4, "one counter per slot, and the reduce's");
constexpr int kMaxSplit = 16;
constexpr int64_t kMaxBatch = 65535;                       // the batch index is the grid's y dimension
constexpr int64_t kMaxTiles = (int64_t)1 << 26;            // 64 x 64 tiles of C (x 16 splits fits the grid's x)
void* g_ws = nullptr;
int64_t g_ws_bytes = 0;
// workspaces registered for one stream each (tsg_workspace_set_stream): calls on different
// streams then split k at the same time without sharing scratch
struct StreamWs { void* ws; int64_t bytes; };
std::map<void*, StreamWs> g_stream_ws;
thread_local tsg_launch_info t_last;

void resolve_workspace(void* stream, void** ws, int64_t* bytes) {
    std::lock_guard<std::mutex> g(g_mu);
    const auto it = g_stream_ws.find(stream);
    if (it != g_stream_ws.end()) { *ws = it->second.ws; *bytes = it->second.bytes; return; }
    *ws = g_ws;
    *bytes = g_ws ? g_ws_bytes : 0;
}

// ---- scratch of the allocation-free entry point (tsg_gemm_trans_static) -------------------
// Device memory that belongs to the library's code object: arrival counters first, partial
// tiles after them, laid out like a caller's workspace.  Every GPU holds its own copy at its
// own address; in host code the array's name only stands for the symbol, so the address is
// looked up once per device and that pointer is what kernels are given.
constexpr int64_t kStaticScratchBytes = TSG_STATIC_SCRATCH_BYTES;
static_assert(kStaticScratchBytes > kCounterBytes && kStaticScratchBytes % 256 == 0, "scratch layout");
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];     // device address of `scratch` on device d, null until first used there
std::mutex g_scratch_mu;

__global__ void clear_words_kernel(int* w, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) w[i] = 0;
}

// The current device's copy of `scratch`.  The first call on a device looks the address up and
// enqueues a kernel on `s` that zeroes the counters (a kernel, not a memset: the call may be
// recorded into a graph); after that the kernels themselves leave every counter at zero.
tsg_status static_scratch(hipStream_t s, void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TSG_E_RUNTIME;
    std::lock_guard<std::mutex> g(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return TSG_E_RUNTIME;
        const int words = (int)(kCounterBytes / 4);
        hipLaunchKernelGGL(clear_words_kernel, dim3((words + 255) / 256), dim3(256), 0, s, (int*)ptr, words);
        if (hipGetLastError() != hipSuccess) return TSG_E_RUNTIME;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return TSG_OK;
}

const KernelEntry* kernels(tsg_dtype dt, int* n) {
    return dt == TSG_F32 ? tsg::f32_kernels(n) : tsg::bf16_kernels(n);
}

int elem_size(tsg_dtype dt) { return dt == TSG_F32 ? 4 : 2; }
int vec_max(tsg_dtype dt) { return 16 / elem_size(dt); }

bool valid_op(int op) { return op >= 0 && op < kNumOps; }
bool valid_dtype(int dt) { return dt >= 0 && dt < kNumDtypes; }

const KernelEntry* find_entry(tsg_dtype dt, const tsg_tile_config& c) {
    int n = 0;
    const KernelEntry* t = kernels(dt, &n);
    for (int i = 0; i < n; ++i)
        if (t[i].bm == c.bm && t[i].bn == c.bn && t[i].bk == c.bk && t[i].wm == c.wm && t[i].wn == c.wn &&
            t[i].sched == c.sched && t[i].mfma == c.mfma)
            return &t[i];
    return nullptr;
}

tsg_tile_config config_of(const KernelEntry& e, int vec, int raster, int split_k = 1, int split_tail = 0) {
    tsg_tile_config c;
    c.bm = e.bm; c.bn = e.bn; c.bk = e.bk; c.wm = e.wm; c.wn = e.wn;
    c.vec = vec; c.raster = raster; c.sched = e.sched; c.split_k = split_k; c.split_tail = split_tail;
    c.mfma = e.mfma;
    return c;
}

// Tiles that a split applies to: all of them, or (split_tail) those beyond the last full
// round of one tile per CU -- the tail that would otherwise leave most of the chip idle.
int64_t split_tiles(int64_t tiles, int split_k, int split_tail) {
    if (split_k <= 1) return 0;
    return split_tail ? tiles % kCUs : tiles;
}

int64_t ws_bytes_needed(const KernelEntry& e, int64_t batch, int64_t M, int64_t N, int split_k, int split_tail = 0) {
    const int64_t tiles = ((M + e.bm - 1) / e.bm) * ((N + e.bn - 1) / e.bn);
    const int64_t st = split_tiles(tiles, split_k, split_tail);
    if (st == 0) return 0;
    return kCounterBytes + batch * st * split_k * (int64_t)e.bm * e.bn * 4;
}

// Cost model of one launch, in cycles of a CU.  A workgroup step costs its MFMA cycles on
// the SIMDs it shares with the other resident workgroups, but never less than the part of
// the global-memory latency that its prefetch depth leaves exposed; the kernel costs
// (rounds of workgroups) x (steps x step cost + pipeline fill) plus the split-k reduction.
// It ranks the search space: the heuristic default is its minimum, and the tuner visits
// the points in its order (tsg_autotune_*), so a small budget of evaluations already
// covers the likely winners.  Constants are fitted to the tuner's own measurements on six
// shapes (256^3, 1024^3 transposed, 4096^3, the 3x3 convolution, bf16 8192^3, and the batched
// 196 x 256 x 2305); on those the model's pick is within 12 % of the measured optimum.
constexpr double kModelLaunch = 7682.0;      // launch, first loads and epilogue of a kernel

// `ntiles` tiles of C (all batch entries together), each split `split` ways; no launch cost
double model_core(tsg_dtype dt, const KernelEntry& e, double ntiles, int split, int64_t K) {
    const double kLatency = 2324.0;     // cycles from issuing a tile's loads to LDS-ready
    const double kLds = 160.0 * 1024;
    if (e.sched == 1) {
        // One block per workgroup, one wave per SIMD: a wave takes every fourth k group, sixteen
        // groups per workgroup in flight together.  A batch of sixteen groups costs one exposed
        // latency (operands that small sit in L2: about 1000 cycles) when a CU holds a single
        // workgroup; with several they overlap, and the CU is bound by its MFMA time or, sooner, by
        // the operand bytes it draws from L2: nothing is shared between blocks, 32 KiB per batch
        // at 14 (32 x 32 blocks) to 18.5 (16 x 16) bytes per cycle and CU.  Fitted on 128^3 .. 2048^3,
        // 64 x 64 x 4096, 256 x 256 x 2048: within 15 % of the measured time on those.
        const int64_t kg = e.bk / 4, groups = (K + kg - 1) / kg;
        const double batches = (double)((groups + 15) / 16);
        const double batch_mfma = 4.0 * 4.0 * (e.mfma ? 32.0 : 64.0);   // four groups of four MFMAs per wave
        const double batch_bytes = 16.0 * kg * e.bm * 4.0 * 2.0;
        const double per_cu = (double)(int64_t)((ntiles + kCUs - 1) / kCUs);
        return batches * std::max(per_cu * std::max(batch_mfma * 1.2, batch_bytes / (e.mfma ? 18.5 : 14.0)),
                                  1000.0 + batch_mfma);
    }
    const int64_t nk_all = (K + e.bk - 1) / e.bk;
    const double tiles = ntiles * split;
    const double wg_wps = e.threads / 256.0;                        // waves per SIMD of one workgroup
    const double wps_cap = (double)(int)(512.0 / (e.wm * e.wn / 64.0 + 64.0));   // register-file limit
    const double resident = std::max(1.0, std::min((double)(int)(kLds / e.lds_bytes),
                                                   (double)(int)(wps_cap / wg_wps)));
    const double rounds = (double)(int64_t)((tiles + kCUs * resident - 1) / (kCUs * resident));
    const double conc = std::min(resident, (double)(int64_t)((tiles + kCUs - 1) / kCUs));
    const double steps = (double)((nk_all + split - 1) / split);
    // cycles one wave spends in MFMA per step: a SIMD retires 64 fp32 or 1024 bf16 flop per cycle
    const double wave_mfma = (double)e.wm * e.wn * e.bk * (dt == TSG_F32 ? 1.0 / 32.0 : 1.0 / 512.0);
    const double wg_mfma = wave_mfma * wg_wps;
    // fewer waves per SIMD hide less of the barrier and LDS latency; small wave tiles
    // re-read LDS more often per MFMA; the finely pipelined forms pay a little for their order
    double ineff = (1.0 + 0.16 / (conc * wg_wps)) * (1.0 + 17.7 / (e.wm + e.wn));
    if (e.sched >= 4) ineff *= 0.95;   // the LDS rings keep the barrier and the loads off the MFMA chain
    // k steps in flight ahead of the one being multiplied: register staging 1, the LDS rings 2 / 3
    const double depth = e.sched == 5 ? 3.0 : e.sched == 4 ? 2.0 : 1.0;
    // how much of a step's MFMA time is added to its exposed latency rather than overlapped
    // (the LDS rings issue their loads behind the MFMAs of the step itself)
    const double serial = e.sched >= 4 ? 0.3 : 0.91;
    const double step_cost = std::max(conc * wg_mfma * ineff, kLatency / depth + serial * wg_mfma);
    // split k: every partial tile goes through to memory and back (about 48 bytes per cycle)
    const double reduce = split > 1 ? 2.0 * e.bm * e.bn * 4.0 / 48.5 * split + 3814.0 : 0.0;
    return rounds * (steps * step_cost + reduce);
}

// Per-kernel calibration of the model for fp32: the geometric mean of measured / predicted time of
// each tile shape and form over the tuner's logs of eleven shapes (640^3, 896^3, 1280^3 plain and
// transposed, 1792^3, 2560^3, 512 x 4096 x 1024, 4096 x 512 x 2048, 1024 x 1024 x 4096,
// 3072 x 3072 x 768, four times 512^3), shrunk towards 1.  None of the shapes the search report
// is taken on is among them.  Tiles without an entry (and bf16) keep the uncalibrated prediction.
struct Calib { int bm, bn, bk, wm, wn, sched, mfma; double factor; };
constexpr Calib kCalibF32[] = {
    {16, 16, 64, 16, 16, 1, 1, 0.997},
    {32, 32, 32, 32, 32, 1, 0, 1.073},
    {64, 64, 32, 32, 32, 0, 0, 0.852},
    {64, 64, 32, 32, 32, 4, 0, 0.878},
    {64, 64, 32, 32, 32, 5, 0, 0.884},
    {64, 64, 32, 64, 16, 4, 1, 0.963},
    {64, 64, 64, 32, 32, 0, 0, 0.900},
    {64, 64, 64, 32, 32, 4, 0, 0.894},
    {64, 64, 64, 32, 32, 5, 0, 0.922},
    {112, 64, 32, 112, 16, 4, 1, 1.016},
    {112, 64, 32, 112, 16, 5, 1, 1.012},
    {112, 64, 64, 112, 16, 4, 1, 0.992},
    {128, 64, 32, 64, 32, 0, 0, 0.871},
    {128, 64, 32, 64, 32, 4, 0, 0.902},
    {128, 128, 16, 64, 64, 0, 0, 0.914},
    {128, 128, 16, 64, 64, 4, 0, 0.994},
    {128, 128, 32, 64, 64, 4, 0, 0.884},
    {256, 128, 16, 64, 64, 0, 0, 0.923},
    {256, 128, 16, 64, 64, 4, 0, 0.983},
    {256, 128, 16, 64, 64, 5, 0, 0.905},
    {256, 256, 16, 128, 64, 0, 0, 0.932},
    {256, 256, 16, 128, 64, 4, 0, 0.932},
};

double calibration(tsg_dtype dt, const KernelEntry& e) {
    if (dt != TSG_F32) return 1.0;
    for (const Calib& c : kCalibF32)
        if (c.bm == e.bm && c.bn == e.bn && c.bk == e.bk && c.wm == e.wm && c.wn == e.wn && c.sched == e.sched &&
            c.mfma == e.mfma)
            return c.factor;
    return 1.0;
}

double model_cycles_raw(tsg_dtype dt, const KernelEntry& e, int split, int split_tail, int64_t batch, int64_t M,
                        int64_t N, int64_t K);

double model_cycles(tsg_dtype dt, const KernelEntry& e, int split, int split_tail, int64_t batch, int64_t M,
                    int64_t N, int64_t K) {
    // (the fixed cost of a launch is the same for every kernel: only the rest is scaled)
    return calibration(dt, e) * (model_cycles_raw(dt, e, split, split_tail, batch, M, N, K) - kModelLaunch) + kModelLaunch;
}

double model_cycles_raw(tsg_dtype dt, const KernelEntry& e, int split, int split_tail, int64_t batch, int64_t M,
                        int64_t N, int64_t K) {
    const int64_t tiles = ((M + e.bm - 1) / e.bm) * ((N + e.bn - 1) / e.bn);
    if (split > 1 && split_tail) {
        // full rounds of one tile per CU unsplit, then the tail split so that it fills the chip
        const int64_t rem = tiles % kCUs, full = tiles - rem;
        if (rem == 0) return model_core(dt, e, (double)(tiles * batch), 1, K) + kModelLaunch;
        return (full ? model_core(dt, e, (double)(full * batch), 1, K) : 0.0) +
               model_core(dt, e, (double)(rem * batch), split, K) + kModelLaunch;
    }
    return model_core(dt, e, (double)(tiles * batch), split, K) + kModelLaunch;
}

bool split_allowed(const KernelEntry& e, int split, int split_tail, int64_t batch, int64_t M, int64_t N, int64_t K,
                   int64_t ws_bytes) {
    if (split == 1) return !split_tail;
    if (e.sched == 1) return false;   // the block form splits k inside the workgroup only
    const int64_t nk_all = (K + e.bk - 1) / e.bk;
    const int64_t n_split = split_tiles(((M + e.bm - 1) / e.bm) * ((N + e.bn - 1) / e.bn), split, split_tail);
    return n_split > 0 && split * 2 <= nk_all && ws_bytes_needed(e, batch, M, N, split, split_tail) <= ws_bytes &&
           batch * n_split <= kMaxSlots;
}

// The default config of a shape: the model's minimum over instantiated tiles and splits.
tsg_tile_config heuristic(tsg_dtype dt, int64_t batch, int64_t M, int64_t N, int64_t K, int64_t ws_bytes,
                          int amode = tsg::A_ROW) {
    int n = 0;
    const KernelEntry* t = kernels(dt, &n);
    double best = 0;
    int best_i = 0, best_split = 1, best_tail = 0;
    bool first = true;
    for (int i = 0; i < n; ++i)
        for (int tail = 0; tail < 2; ++tail)
            for (int split = 1; split <= kMaxSplit; ++split) {
                if (!(t[i].modes >> amode & 1)) break;   // the tile does not exist for this operand layout
                if (!split_allowed(t[i], split, tail, batch, M, N, K, ws_bytes)) {
                    if (split == 1) continue;   // tail = 1 starts at split 2
                    break;
                }
                const double est = model_cycles(dt, t[i], split, tail, batch, M, N, K);
                if (first || est < best * 0.999) { best = est; best_i = i; best_split = split; best_tail = tail; first = false; }
            }
    // fp32: the XCD-aware raster takes the same time and fetches fewer bytes once there is a tile for
    // every CU; below that the row-major order does as well and decodes with one division instead of
    // four.  bf16: the row-major order measured 1-6 % faster at every size tried
    const int64_t n_tiles = batch * ((M + t[best_i].bm - 1) / t[best_i].bm) * ((N + t[best_i].bn - 1) / t[best_i].bn);
    return config_of(t[best_i], vec_max(dt), dt == TSG_F32 && n_tiles >= kCUs ? 1 : 0, best_split, best_tail);
}

// Fill zero fields from `def` (Sec. 3.4: a tile size of 0 changes nothing, so the library default stands).
tsg_tile_config fill_defaults(tsg_tile_config c, const tsg_tile_config& def) {
    const bool tile_given = c.bm > 0 || c.bn > 0 || c.bk > 0 || c.wm > 0 || c.wn > 0;
    if (c.bm <= 0) c.bm = def.bm;
    if (c.bn <= 0) c.bn = def.bn;
    if (c.bk <= 0) c.bk = def.bk;
    if (!tile_given) { c.wm = def.wm; c.wn = def.wn; c.sched = def.sched; c.mfma = def.mfma; }
    if (c.wm <= 0) c.wm = std::min(c.bm, 64);
    if (c.wn <= 0) c.wn = std::min(c.bn, 64);
    if (c.vec <= 0) c.vec = def.vec;
    if (c.raster < 0) c.raster = def.raster;
    if (c.sched < 0) c.sched = def.sched;
    if (c.mfma < 0) c.mfma = 0;
    if (c.split_k <= 0) { c.split_k = tile_given ? 1 : def.split_k; c.split_tail = tile_given ? 0 : def.split_tail; }
    return c;
}

// Fig. 10's rule for `vect` on this hardware.  The k tile is a multiple of the vector size
// by construction and the remainder of a loop is peeled into masked scalar code, so a wide
// access only has to stay inside one contiguous run of its operand.  Rows of a matrix are
// such runs whatever their leading dimension (the hardware fetches a 16-byte chunk from any
// element-aligned address); the gathered operand of a convolution is contiguous only along
// Cin, so there the innermost extent Cin must be divisible by the vector size.
bool vec_legal(const Problem& p, int vec) {
    if (vec == 1) return true;
    if (vec != vec_max(p.dtype)) return false;
    if (p.op == TSG_OP_CONV2D_NHWC) return p.Cin % vec == 0;
    return true;
}

TuneKey tune_key(const Problem& p) {
    return TuneKey{(int64_t)p.op, (int64_t)p.dtype, p.trans_b ? 1 : 0, p.batch, p.M, p.N, p.K,
                   p.op == TSG_OP_CONV2D_NHWC ? p.Cin : 0};
}

int amode_of(const Problem& p) {
    return p.op == TSG_OP_GEMM ? (p.trans_b ? tsg::A_ROW_BT : tsg::A_ROW)
           : p.op == TSG_OP_GEMM_TRANSA ? (p.trans_b ? tsg::A_COL_BT : tsg::A_COL) : tsg::A_CONV;
}

struct Plan {
    const KernelEntry* entry;
    tsg_tile_config cfg;
    int variant;
    KArgs args;
    tsg_launch_info info;
};

// One alternative: SILENCEABLE if its preconditions fail (nothing is touched).
tsg_status make_plan(const Problem& p, const tsg_tile_config& cfg, int alternative, Plan* out) {
    const KernelEntry* e = find_entry(p.dtype, cfg);
    if (!e) return TSG_E_SILENCEABLE;
    if (!vec_legal(p, cfg.vec)) return TSG_E_SILENCEABLE;
    if (e->sched >= 4 && cfg.vec == 1) return TSG_E_SILENCEABLE;   // direct-to-LDS forms move 16-byte chunks
    if (e->sched == 1 && cfg.split_k > 1) return TSG_E_SILENCEABLE;   // the block form splits k inside the workgroup only
    if (!(e->modes >> amode_of(p) & 1)) return TSG_E_SILENCEABLE;   // the tile does not exist for this operand layout
    if (cfg.raster != 0 && cfg.raster != 1) return TSG_E_SILENCEABLE;
    if (cfg.split_k < 1 || cfg.split_k > kMaxSplit) return TSG_E_SILENCEABLE;
    if ((cfg.split_tail != 0 && cfg.split_tail != 1) || (cfg.split_tail && cfg.split_k == 1)) return TSG_E_SILENCEABLE;

    int64_t m_main, m_rest, n_main, n_rest, k_main, k_rest, t;
    tsg_split(p.M, e->bm, &m_main, &m_rest, &t);
    tsg_split(p.N, e->bn, &n_main, &n_rest, &t);
    tsg_split(p.K, e->bk, &k_main, &k_rest, &t);
    const int64_t tiles_m = (p.M + e->bm - 1) / e->bm, tiles_n = (p.N + e->bn - 1) / e->bn;
    void* ws = nullptr;
    const int64_t n_split = split_tiles(tiles_m * tiles_n, cfg.split_k, cfg.split_tail);
    if (cfg.split_k > 1) {
        // every split needs at least one k step, a tail to split if only the tail is split, and
        // the partial tiles need the workspace
        if (cfg.split_k > (p.K + e->bk - 1) / e->bk) return TSG_E_SILENCEABLE;
        if (n_split == 0) return TSG_E_SILENCEABLE;
        if (p.batch * n_split > kMaxSlots) return TSG_E_SILENCEABLE;
        if (!p.ws || ws_bytes_needed(*e, p.batch, p.M, p.N, cfg.split_k, cfg.split_tail) > p.ws_bytes)
            return TSG_E_SILENCEABLE;
        ws = p.ws;
    }

    const bool edge = m_rest || n_rest || k_rest;
    out->entry = e;
    out->cfg = cfg;
    // remainder variant 3 (clamped rows, peeled last k step) serves every shape whose extents
    // along the operands' contiguous dimensions hold at least one whole access; narrower ones
    // (N < 4 with a row-major B, M < 4 with a transposed A) take the general variant 1
    const int64_t v = vec_max(p.dtype);
    const bool cut = (!p.trans_b && p.N < v) || (p.op == TSG_OP_GEMM_TRANSA && p.M < v);
    out->variant = cfg.vec == 1 ? 2 : (edge ? (cut ? 1 : 3) : 0);

    KArgs& a = out->args;
    std::memset(&a, 0, sizeof a);
    a.A = p.A; a.B = p.B; a.C = p.C;
    a.lda = p.lda; a.ldb = p.ldb; a.ldc = p.ldc;
    a.stride_a = p.stride_a; a.stride_b = p.stride_b; a.stride_c = p.stride_c;
    a.M = (int)p.M; a.N = (int)p.N; a.K = (int)p.K;
    a.tiles_m = (int)tiles_m; a.tiles_n = (int)tiles_n;
    a.m_main = (int)m_main; a.n_main = (int)n_main; a.k_full = (int)(k_main / e->bk);
    a.flags = p.flags & (TSG_NEGATE | TSG_ACCUMULATE);
    a.raster = cfg.raster;
    a.split_k = cfg.split_k;
    a.split_first = (int)(tiles_m * tiles_n - n_split);
    a.counters = (int*)ws;
    a.ws = ws ? (float*)((char*)ws + kCounterBytes) : nullptr;
    a.H = (int)p.H; a.W = (int)p.W; a.Cin = (int)p.Cin; a.Ho = (int)p.Ho; a.Wo = (int)p.Wo;
    a.KW = (int)p.KW; a.sh = (int)p.sh; a.sw = (int)p.sw; a.ph = (int)p.ph; a.pw = (int)p.pw;
    a.y_window = p.y_window; a.y_sn = p.y_sn; a.y_sh = p.y_sh; a.y_sw = p.y_sw;

    tsg_launch_info& li = out->info;
    li.config = cfg;
    li.alternative = alternative;
    li.launches = 1;
    li.edge = out->variant != 0;
    li.tiles_m = (int)tiles_m; li.tiles_n = (int)tiles_n;
    li.m_main = m_main; li.m_rest = m_rest; li.n_main = n_main; li.n_rest = n_rest;
    li.k_main = k_main; li.k_rest = k_rest;
    return TSG_OK;
}

tsg_status enqueue(const Problem& p, const Plan& pl, hipStream_t s) {
    const int amode = amode_of(p);
    int n = 0;
    const int tile = (int)(pl.entry - kernels(p.dtype, &n));
    const hipError_t e = pl.entry->launch(tile, amode, pl.variant, pl.args, (int)p.batch, s);
    if (e != hipSuccess) return TSG_E_RUNTIME;
    t_last = pl.info;
    return TSG_OK;
}

// The cost model's pick walks the whole table times the splits, which is worth remembering in
// a loop that calls the same problem again and again: the last few problems of each thread.
tsg_tile_config heuristic_cached(tsg_dtype dt, int64_t batch, int64_t M, int64_t N, int64_t K, int64_t ws_bytes,
                                 int amode) {
    struct Memo { int64_t key[7]; tsg_tile_config cfg; bool used; };
    thread_local Memo memo[8] = {};
    thread_local int next = 0;
    const int64_t key[7] = {(int64_t)dt, batch, M, N, K, ws_bytes, (int64_t)amode};
    for (const Memo& m : memo)
        if (m.used && std::memcmp(m.key, key, sizeof key) == 0) return m.cfg;
    Memo& m = memo[next];
    next = (next + 1) % 8;
    std::memcpy(m.key, key, sizeof key);
    m.cfg = heuristic(dt, batch, M, N, K, ws_bytes, amode);
    m.used = true;
    return m.cfg;
}

// The chain of alternatives (Case Study 4: try, and on a silenceable failure fall through
// to the next region): the caller's pinned config, else the tuner's result for this problem
// -> the cost model's default -> that tile with scalar accesses, which has no precondition
// beyond a valid problem.
tsg_status run(const Problem& p, hipStream_t s) {
    bool pinned;
    tsg_tile_config pin;
    const int64_t ws_bytes = p.ws ? p.ws_bytes : 0;
    {
        std::lock_guard<std::mutex> g(g_mu);
        pinned = g_pinned[p.op][p.dtype];
        pin = g_pin[p.op][p.dtype];
        if (!pinned) {   // no config pinned by the caller: the tuner's result for this very problem, if any
            const auto it = g_tuned.find(tune_key(p));
            if (it != g_tuned.end()) { pinned = true; pin = it->second.cfg; }
        }
    }
    Plan pl;
    if (pinned) {
        if (make_plan(p, pin, 0, &pl) == TSG_OK) return enqueue(p, pl, s);
        if (p.flags & TSG_STRICT) return TSG_E_SILENCEABLE;
    }
    const tsg_tile_config heur = heuristic_cached(p.dtype, p.batch, p.M, p.N, p.K, ws_bytes, amode_of(p));
    if (make_plan(p, heur, 1, &pl) == TSG_OK) return enqueue(p, pl, s);
    if (p.flags & TSG_STRICT) return TSG_E_SILENCEABLE;
    // (a valid problem always passes the default's preconditions when B is stored transposed:
    // those forms have no scalar variant to fall back to)
    if (p.trans_b) return TSG_E_INVALID;
    // last alternative: scalar accesses, which have no precondition.  The direct-to-LDS forms
    // have no scalar variant, so the same tile is taken in a register-staged form (or, if
    // that one is not instantiated, the smallest tile of the table).
    tsg_tile_config scalar = heur;
    scalar.vec = 1;
    scalar.split_k = 1;
    scalar.split_tail = 0;
    if (scalar.sched >= 4) {
        scalar.sched = 0;
        if (!find_entry(p.dtype, scalar)) {
            int n = 0;
            const KernelEntry* t = kernels(p.dtype, &n);
            int pick = -1;
            for (int i = 0; i < n; ++i)
                if (t[i].sched == 0 && (pick < 0 || t[i].bm * t[i].bn < t[pick].bm * t[pick].bn)) pick = i;
            if (pick < 0) return TSG_E_INVALID;
            scalar = config_of(t[pick], 1, heur.raster, 1);
        }
    }
    if (make_plan(p, scalar, 2, &pl) == TSG_OK) return enqueue(p, pl, s);
    return TSG_E_INVALID;   // unreachable for arguments that passed validation: the scalar form has no precondition
}

bool fits_i32(int64_t v) { return v >= 0 && v <= 0x7fffffff; }

tsg_status check_gemm(int dtype, int64_t batch, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                      const void* B, int64_t ldb, const float* C, int64_t ldc, bool trans_a, uint32_t flags,
                      bool trans_b = false) {
    if (!valid_dtype(dtype)) return TSG_E_INVALID;
    if (!A || !B || !C) return TSG_E_INVALID;
    if (M <= 0 || N <= 0 || K <= 0 || batch <= 0) return TSG_E_INVALID;
    if (!fits_i32(M) || !fits_i32(N) || !fits_i32(K)) return TSG_E_INVALID;
    if (batch > kMaxBatch || ((M + 63) / 64) * ((N + 63) / 64) > kMaxTiles) return TSG_E_INVALID;
    const uintptr_t es = dtype == TSG_F32 ? 4 : 2;
    if (reinterpret_cast<uintptr_t>(A) % es || reinterpret_cast<uintptr_t>(B) % es ||
        reinterpret_cast<uintptr_t>(C) % 4)
        return TSG_E_INVALID;   // operands are arrays of their element type
    if (lda < (trans_a ? M : K) || ldb < (trans_b ? K : N) || ldc < N) return TSG_E_INVALID;
    if (flags & ~(uint32_t)(TSG_NEGATE | TSG_ACCUMULATE | TSG_STRICT)) return TSG_E_INVALID;
    return TSG_OK;
}

tsg_status conv_problem(int dtype, int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t KH,
                        int64_t KW, int64_t sh, int64_t sw, int64_t ph, int64_t pw, const void* x, const void* w,
                        float* y, uint32_t flags, Problem* p) {
    if (!valid_dtype(dtype) || !x || !w || !y) return TSG_E_INVALID;
    if (N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || Cout <= 0 || KH <= 0 || KW <= 0) return TSG_E_INVALID;
    if (sh <= 0 || sw <= 0 || ph < 0 || pw < 0) return TSG_E_INVALID;
    if (H + 2 * ph < KH || W + 2 * pw < KW) return TSG_E_INVALID;
    if (flags & ~(uint32_t)(TSG_NEGATE | TSG_ACCUMULATE | TSG_STRICT)) return TSG_E_INVALID;
    const int64_t Ho = (H + 2 * ph - KH) / sh + 1, Wo = (W + 2 * pw - KW) / sw + 1;
    const int64_t lim = 0x7fffffff;
    if (N > lim / H || N * H > lim / W || N * H * W > lim / Cin) return TSG_E_INVALID;
    if (N > lim / Ho || N * Ho > lim / Wo || N * Ho * Wo > lim / Cout) return TSG_E_INVALID;
    if (KH > lim / KW || KH * KW > lim / Cin || KH * KW * Cin > lim / Cout) return TSG_E_INVALID;
    if (ph > (1 << 20) || pw > (1 << 20) || sh > (1 << 20) || sw > (1 << 20)) return TSG_E_INVALID;
    if (((N * Ho * Wo + 63) / 64) * ((Cout + 63) / 64) > kMaxTiles) return TSG_E_INVALID;
    const uintptr_t es = dtype == TSG_F32 ? 4 : 2;
    if (reinterpret_cast<uintptr_t>(x) % es || reinterpret_cast<uintptr_t>(w) % es ||
        reinterpret_cast<uintptr_t>(y) % 4)
        return TSG_E_INVALID;
    p->op = TSG_OP_CONV2D_NHWC;
    p->dtype = (tsg_dtype)dtype;
    p->M = N * Ho * Wo; p->N = Cout; p->K = KH * KW * Cin;
    p->A = x; p->B = w; p->C = y;
    p->lda = 0; p->ldb = Cout; p->ldc = Cout;
    p->flags = flags;
    p->H = H; p->W = W; p->Cin = Cin; p->Ho = Ho; p->Wo = Wo; p->KH = KH; p->KW = KW;
    p->sh = sh; p->sw = sw; p->ph = ph; p->pw = pw;
    return TSG_OK;
}

// Enumerated search space: every instantiated tile x {wide access with either raster order,
// scalar access, wide access with the k loop split 2, 3, 4, 5, 6, 8, 10, 12 or 16 ways, or
// with only the tail tiles split 2, 4 or 8 ways}.
constexpr int kSplits[] = {2, 3, 4, 5, 6, 8, 10, 12, 16};
constexpr int kNumSplits = (int)(sizeof(kSplits) / sizeof(kSplits[0]));
constexpr int kPointsPerTile = 3 + kNumSplits + 3;
int space_size(tsg_dtype dt) {
    int n = 0;
    kernels(dt, &n);
    return kPointsPerTile * n;
}

tsg_tile_config space_point(tsg_dtype dt, int idx) {
    int n = 0;
    const KernelEntry* t = kernels(dt, &n);
    const KernelEntry& e = t[idx / kPointsPerTile];
    const int k = idx % kPointsPerTile;
    if (k == 0) return config_of(e, vec_max(dt), 1);
    if (k == 1) return config_of(e, vec_max(dt), 0);
    if (k == 2) return config_of(e, 1, 1);
    if (k < 3 + kNumSplits) return config_of(e, vec_max(dt), 0, kSplits[k - 3]);
    return config_of(e, vec_max(dt), 1, 2 << (k - 3 - kNumSplits), 1);   // tail only, split 2, 4, 8
}

// Search state (Case Study 5): evaluation budget and visiting order of later tuner calls.
int g_search_max_evals = 0;      // 0 = every legal point
int g_search_model_order = 1;    // 0 = enumeration order, 1 = cost-model order, 2 = cost model corrected by the timed points

tsg_status autotune(Problem p, hipStream_t s, int iters, tsg_tile_config* best, float* best_ms,
                    tsg_tune_record* log, int32_t log_cap, int32_t* n_log) {
    if (iters <= 0 || iters > 256) return TSG_E_INVALID;
    if (log_cap < 0 || (log_cap > 0 && !log)) return TSG_E_INVALID;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return TSG_E_RUNTIME;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return TSG_E_RUNTIME; }
    p.flags &= ~(uint32_t)TSG_STRICT;
    int max_evals, model_order;
    {
        std::lock_guard<std::mutex> g(g_mu);
        max_evals = g_search_max_evals;
        model_order = g_search_model_order;
    }

    // candidates with the model's prediction (ms at 2.4 GHz); scalar access is priced at four
    // times the wide form, and the raster orders tie (the XCD-aware one is listed first)
    struct Cand { tsg_tile_config c; double pred; int idx; };
    const int n = space_size(p.dtype);
    std::vector<Cand> cand;
    cand.reserve(n);
    for (int i = 0; i < n; ++i) {
        const tsg_tile_config c = space_point(p.dtype, i);
        const KernelEntry* e = find_entry(p.dtype, c);
        double pred = model_cycles(p.dtype, *e, c.split_k, c.split_tail, p.batch, p.M, p.N, p.K) / 2.4e6;
        if (c.vec == 1) pred *= 4.0;
        cand.push_back(Cand{c, pred, i});
    }
    if (model_order)
        std::stable_sort(cand.begin(), cand.end(), [](const Cand& a, const Cand& b) { return a.pred < b.pred; });

    // Adaptive order (model_order 2): the cost model is a prior that every timed point corrects.
    // The ratio measured / predicted is kept per kernel (tile shape and form: its splits, raster
    // orders and access widths share it) and overall, as sums of logarithms; a candidate's
    // prediction is scaled by its kernel's mean ratio shrunk towards the overall one (a kernel
    // without a timed point yet takes the overall ratio), and the next point timed is the
    // candidate with the smallest corrected prediction.  A kernel family the prior flatters
    // falls back after its first timed point instead of filling the head of the list.
    struct Resid { double sum = 0.0; int n = 0; };
    std::map<const KernelEntry*, Resid> resid;
    Resid overall;
    std::vector<char> done(n, 0);
    auto corrected = [&](const Cand& cd) {
        const auto it = resid.find(find_entry(p.dtype, cd.c));
        const double g = overall.n ? overall.sum / overall.n : 0.0;
        const double m = it == resid.end() ? g : (it->second.sum + g) / (it->second.n + 1);
        return cd.pred * std::exp(m);
    };

    float bms = -1.f;
    tsg_tile_config bcfg{};
    int written = 0, evals = 0;
    tsg_status st = TSG_OK;
    for (int visit = 0; visit < n && st == TSG_OK; ++visit) {
        if (max_evals > 0 && evals >= max_evals) break;
        int i = visit;
        if (model_order == 2) {
            i = -1;
            double best_pred = 0.0;
            for (int j = 0; j < n; ++j) {
                if (done[j]) continue;
                const double cp = corrected(cand[j]);
                if (i < 0 || cp < best_pred) { i = j; best_pred = cp; }
            }
        }
        done[i] = 1;
        const tsg_tile_config c = cand[i].c;
        Plan pl;
        // splitting k only pays while the unsplit tiles cannot fill the chip twice over: other
        // split points are pruned, and logged as such (-2), apart from the illegal ones (-1)
        const bool worth = c.split_k == 1 || c.split_tail ||
                           p.batch * ((p.M + c.bm - 1) / c.bm) * ((p.N + c.bn - 1) / c.bn) < 2 * kCUs;
        float med = worth ? -1.f : -2.f;
        if (worth && make_plan(p, c, 0, &pl) == TSG_OK) {
            st = enqueue(p, pl, s);   // warm-up
            // the first point also brings the clocks up from idle: untimed batches until 30 ms
            // of device time have passed, so that its time compares with the later points'
            if (evals == 0) {
                float spent = 0.f;
                for (int round = 0; round < 64 && spent < 30.f && st == TSG_OK; ++round) {
                    if (hipEventRecord(e0, s) != hipSuccess) { st = TSG_E_RUNTIME; break; }
                    for (int it = 0; it < iters && st == TSG_OK; ++it) st = enqueue(p, pl, s);
                    float t = 0.f;
                    if (st != TSG_OK) break;
                    if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                        hipEventElapsedTime(&t, e0, e1) != hipSuccess) { st = TSG_E_RUNTIME; break; }
                    spent += t;
                }
            }
            // best of three batches of `iters` back-to-back calls, mean time per call
            for (int round = 0; round < 3 && st == TSG_OK; ++round) {
                if (hipEventRecord(e0, s) != hipSuccess) { st = TSG_E_RUNTIME; break; }
                for (int it = 0; it < iters && st == TSG_OK; ++it) st = enqueue(p, pl, s);
                if (st != TSG_OK) break;
                float t = 0.f;
                if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                    hipEventElapsedTime(&t, e0, e1) != hipSuccess) { st = TSG_E_RUNTIME; break; }
                t /= (float)iters;
                if (med < 0 || t < med) med = t;
            }
            if (st != TSG_OK) break;
            ++evals;
            // a later point must win by more than timing noise: among ties the earlier point stays
            if (bms < 0 || med < bms * 0.995f) { bms = med; bcfg = c; }
            // what this point teaches about its kernel and about the model as a whole (scalar
            // access is priced by a flat factor, not by the model: it teaches nothing)
            if (c.vec != 1 && cand[i].pred > 0) {
                const double lr = std::log((double)med / cand[i].pred);
                Resid& r = resid[find_entry(p.dtype, c)];
                r.sum += lr; ++r.n;
                overall.sum += lr; ++overall.n;
            }
        }
        if (written < log_cap) {
            log[written].config = c;
            log[written].ms = med;
            log[written].best_ms = bms;
            log[written].predicted_ms = (float)cand[i].pred;
            ++written;
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (n_log) *n_log = written;
    if (st != TSG_OK) return st;
    if (bms < 0) return TSG_E_SILENCEABLE;
    if (best) *best = bcfg;
    if (best_ms) *best_ms = bms;
    std::lock_guard<std::mutex> g(g_mu);
    g_tuned[tune_key(p)] = TuneVal{bcfg, bms};
    return TSG_OK;
}

}  // namespace

bool tsg::workspace_get(void* stream, void** ws, long long* bytes) {
    int64_t b = 0;
    resolve_workspace(stream, ws, &b);
    *bytes = b;
    return *ws != nullptr;
}

extern "C" {

const char* tsg_status_string(tsg_status s) {
    switch (s) {
        case TSG_OK: return "ok";
        case TSG_E_SILENCEABLE: return "silenceable: precondition of the requested schedule failed, nothing modified";
        case TSG_E_INVALID: return "definite: invalid argument";
        case TSG_E_RUNTIME: return "definite: HIP runtime failure";
        case TSG_E_TOO_LARGE:
            return "definite: the output exceeds what the allocation-free entry point serves "
                   "(batch * M * N, padded to 64 x 64 tiles, above TSG_STATIC_MAX_OUTPUTS); use tsg_gemm_trans";
    }
    return "unknown status";
}

int32_t tsg_version(void) { return 1; }

tsg_status tsg_split(int64_t ub, int64_t d, int64_t* main_part, int64_t* rest, int64_t* tiles) {
    if (ub < 0 || d < 0 || !main_part || !rest || !tiles) return TSG_E_INVALID;
    const int64_t t = d == 0 ? 1 : ub / d;
    *tiles = t;
    *main_part = d == 0 ? ub : t * d;
    *rest = ub - *main_part;
    return TSG_OK;
}

tsg_status tsg_gemm_trans(tsg_dtype dtype, int32_t trans_a, int32_t trans_b, int64_t batch, int64_t M, int64_t N,
                          int64_t K, const void* A, int64_t lda, int64_t stride_a, const void* B, int64_t ldb,
                          int64_t stride_b, float* C, int64_t ldc, int64_t stride_c, uint32_t flags, void* stream) {
    const tsg_status v = check_gemm(dtype, batch, M, N, K, A, lda, B, ldb, C, ldc, trans_a != 0, flags, trans_b != 0);
    if (v != TSG_OK) return v;
    if (stride_a < 0 || stride_b < 0 || stride_c < 0) return TSG_E_INVALID;
    if (batch > 1 && stride_c < (M - 1) * ldc + N) return TSG_E_INVALID;   // outputs must not overlap
    Problem p;
    p.op = trans_a ? TSG_OP_GEMM_TRANSA : TSG_OP_GEMM;
    p.dtype = dtype;
    p.batch = batch;
    p.M = M; p.N = N; p.K = K;
    p.A = A; p.B = B; p.C = C;
    p.lda = lda; p.ldb = ldb; p.ldc = ldc;
    p.stride_a = stride_a; p.stride_b = stride_b; p.stride_c = stride_c;
    p.trans_b = trans_b != 0;
    p.flags = flags;
    resolve_workspace(stream, &p.ws, &p.ws_bytes);
    return run(p, (hipStream_t)stream);
}

tsg_status tsg_gemm_trans_static(tsg_dtype dtype, int32_t trans_a, int32_t trans_b, int64_t batch, int64_t M,
                                 int64_t N, int64_t K, const void* A, int64_t lda, int64_t stride_a, const void* B,
                                 int64_t ldb, int64_t stride_b, float* C, int64_t ldc, int64_t stride_c,
                                 uint32_t flags, void* stream) {
    const tsg_status v = check_gemm(dtype, batch, M, N, K, A, lda, B, ldb, C, ldc, trans_a != 0, flags, trans_b != 0);
    if (v != TSG_OK) return v;
    if (stride_a < 0 || stride_b < 0 || stride_c < 0) return TSG_E_INVALID;
    if (batch > 1 && stride_c < (M - 1) * ldc + N) return TSG_E_INVALID;
    // served: outputs small enough that their tiles cannot fill the chip without a split of k,
    // sized so that a two-way split of every 64 x 64 tile fits the scratch
    if (batch * (((M + 63) / 64) * 64) * (((N + 63) / 64) * 64) > TSG_STATIC_MAX_OUTPUTS) return TSG_E_TOO_LARGE;
    Problem p;
    p.op = trans_a ? TSG_OP_GEMM_TRANSA : TSG_OP_GEMM;
    p.dtype = dtype;
    p.batch = batch;
    p.M = M; p.N = N; p.K = K;
    p.A = A; p.B = B; p.C = C;
    p.lda = lda; p.ldb = ldb; p.ldc = ldc;
    p.stride_a = stride_a; p.stride_b = stride_b; p.stride_c = stride_c;
    p.trans_b = trans_b != 0;
    p.flags = flags;
    const tsg_status ss = static_scratch((hipStream_t)stream, &p.ws);
    if (ss != TSG_OK) return ss;
    p.ws_bytes = kStaticScratchBytes;
    return run(p, (hipStream_t)stream);
}

tsg_status tsg_gemm_batched(tsg_dtype dtype, int32_t trans_a, int64_t batch, int64_t M, int64_t N, int64_t K,
                            const void* A, int64_t lda, int64_t stride_a, const void* B, int64_t ldb,
                            int64_t stride_b, float* C, int64_t ldc, int64_t stride_c, uint32_t flags,
                            void* stream) {
    return tsg_gemm_trans(dtype, trans_a, 0, batch, M, N, K, A, lda, stride_a, B, ldb, stride_b, C, ldc, stride_c,
                          flags, stream);
}

tsg_status tsg_gemm(tsg_dtype dtype, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B,
                    int64_t ldb, float* C, int64_t ldc, uint32_t flags, void* stream) {
    return tsg_gemm_batched(dtype, 0, 1, M, N, K, A, lda, 0, B, ldb, 0, C, ldc, 0, flags, stream);
}

tsg_status tsg_gemm_transA(tsg_dtype dtype, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                           const void* B, int64_t ldb, float* C, int64_t ldc, uint32_t flags, void* stream) {
    return tsg_gemm_batched(dtype, 1, 1, M, N, K, A, lda, 0, B, ldb, 0, C, ldc, 0, flags, stream);
}

tsg_status tsg_conv2d_nhwc(tsg_dtype dtype, int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                           int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w, int64_t pad_h,
                           int64_t pad_w, const void* x, const void* w, float* y, uint32_t flags, void* stream) {
    Problem p;
    const tsg_status v = conv_problem(dtype, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w, pad_h, pad_w, x, w, y,
                                      flags, &p);
    if (v != TSG_OK) return v;
    resolve_workspace(stream, &p.ws, &p.ws_bytes);
    return run(p, (hipStream_t)stream);
}

tsg_status tsg_conv2d_nhwc_window(tsg_dtype dtype, int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                  int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w, int64_t pad_h,
                                  int64_t pad_w, const void* x, const void* w, float* y, int64_t y_stride_n,
                                  int64_t y_stride_h, int64_t y_stride_w, uint32_t flags, void* stream) {
    Problem p;
    const tsg_status v = conv_problem(dtype, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w, pad_h, pad_w, x, w, y,
                                      flags, &p);
    if (v != TSG_OK) return v;
    // pixels of the window must not overlap: each stride covers the extent below it
    if (y_stride_w < Cout || y_stride_h < (p.Wo - 1) * y_stride_w + Cout ||
        y_stride_n < (p.Ho - 1) * y_stride_h + (p.Wo - 1) * y_stride_w + Cout)
        return TSG_E_INVALID;
    if (y_stride_n > (int64_t)0x7fffffff * 64) return TSG_E_INVALID;
    p.y_window = 1;
    p.y_sn = y_stride_n; p.y_sh = y_stride_h; p.y_sw = y_stride_w;
    resolve_workspace(stream, &p.ws, &p.ws_bytes);
    return run(p, (hipStream_t)stream);
}

int32_t tsg_tile_config_count(tsg_op op, tsg_dtype dtype) {
    if (!valid_op(op) || !valid_dtype(dtype)) return 0;
    return space_size(dtype);
}

tsg_status tsg_tile_config_enum(tsg_op op, tsg_dtype dtype, int32_t idx, tsg_tile_config* out) {
    if (!valid_op(op) || !valid_dtype(dtype) || !out) return TSG_E_INVALID;
    if (idx < 0 || idx >= space_size(dtype)) return TSG_E_INVALID;
    *out = space_point(dtype, idx);
    return TSG_OK;
}

tsg_status tsg_tile_config_check(tsg_op op, tsg_dtype dtype, int64_t M, int64_t N, int64_t K, int64_t contig,
                                 const tsg_tile_config* cfg) {
    if (!valid_op(op) || !valid_dtype(dtype) || !cfg) return TSG_E_INVALID;
    if (M <= 0 || N <= 0 || K <= 0) return TSG_E_INVALID;
    if (cfg->bm < 0 || cfg->bn < 0 || cfg->bk < 0 || cfg->wm < 0 || cfg->wn < 0 || cfg->vec < 0 || cfg->split_k < 0 ||
        (cfg->split_tail != 0 && cfg->split_tail != 1))
        return TSG_E_INVALID;
    if (op == TSG_OP_CONV2D_NHWC && contig <= 0) return TSG_E_INVALID;
    const int amode = op == TSG_OP_GEMM ? tsg::A_ROW : op == TSG_OP_GEMM_TRANSA ? tsg::A_COL : tsg::A_CONV;
    const tsg_tile_config c = fill_defaults(*cfg, heuristic(dtype, 1, M, N, K, 0, amode));
    const KernelEntry* e = find_entry(dtype, c);
    if (!e || !(e->modes >> amode & 1)) return TSG_E_SILENCEABLE;
    if (c.raster != 0 && c.raster != 1) return TSG_E_SILENCEABLE;
    if (c.split_k < 1 || c.split_k > kMaxSplit || c.split_k > (K + e->bk - 1) / e->bk) return TSG_E_SILENCEABLE;
    if (c.split_tail && c.split_k == 1) return TSG_E_SILENCEABLE;
    if (e->sched == 1 && c.split_k > 1) return TSG_E_SILENCEABLE;   // the block form splits k inside the workgroup only
    if (c.split_k > 1 && split_tiles(((M + e->bm - 1) / e->bm) * ((N + e->bn - 1) / e->bn), c.split_k, c.split_tail) == 0)
        return TSG_E_SILENCEABLE;   // no tail to split
    if (c.vec == 1) return e->sched >= 4 ? TSG_E_SILENCEABLE : TSG_OK;
    if (c.vec != vec_max(dtype)) return TSG_E_SILENCEABLE;
    // the innermost contiguous extent of the gathered operand is Cin; matrix rows are
    // contiguous runs of any length and their remainder is peeled (see vec_legal)
    if (op == TSG_OP_CONV2D_NHWC && contig % c.vec) return TSG_E_SILENCEABLE;
    return TSG_OK;
}

tsg_status tsg_tile_config_set(tsg_op op, tsg_dtype dtype, const tsg_tile_config* cfg) {
    if (!valid_op(op) || !valid_dtype(dtype)) return TSG_E_INVALID;
    std::lock_guard<std::mutex> g(g_mu);
    if (!cfg) { g_pinned[op][dtype] = false; return TSG_OK; }
    if (cfg->bm < 0 || cfg->bn < 0 || cfg->bk < 0 || cfg->wm < 0 || cfg->wn < 0 || cfg->vec < 0 || cfg->split_k < 0 ||
        (cfg->split_tail != 0 && cfg->split_tail != 1))
        return TSG_E_INVALID;
    int n = 0;
    const KernelEntry* t = kernels(dtype, &n);
    const tsg_tile_config c = fill_defaults(*cfg, config_of(t[0], vec_max(dtype), 1));
    if (!find_entry(dtype, c)) return TSG_E_SILENCEABLE;
    if (c.split_k > kMaxSplit || (c.split_tail && c.split_k == 1)) return TSG_E_SILENCEABLE;
    if (c.vec != 1 && c.vec != vec_max(dtype)) return TSG_E_SILENCEABLE;
    if (c.raster != 0 && c.raster != 1) return TSG_E_SILENCEABLE;
    g_pin[op][dtype] = c;
    g_pinned[op][dtype] = true;
    return TSG_OK;
}

tsg_status tsg_tile_config_get(tsg_op op, tsg_dtype dtype, int64_t M, int64_t N, int64_t K, tsg_tile_config* out) {
    if (!valid_op(op) || !valid_dtype(dtype) || !out) return TSG_E_INVALID;
    if (M <= 0 || N <= 0 || K <= 0) return TSG_E_INVALID;
    std::lock_guard<std::mutex> g(g_mu);
    if (g_pinned[op][dtype]) { *out = g_pin[op][dtype]; return TSG_OK; }
    // the tuner's result for an unbatched problem of these extents (any contiguous run), else the default
    for (const auto& kv : g_tuned) {
        const TuneKey& k = kv.first;
        if (k[0] == op && k[1] == dtype && k[2] == 0 && k[3] == 1 && k[4] == M && k[5] == N && k[6] == K) {
            *out = kv.second.cfg;
            return TSG_OK;
        }
    }
    *out = heuristic(dtype, 1, M, N, K, g_ws ? g_ws_bytes : 0,
                     op == TSG_OP_GEMM ? tsg::A_ROW : op == TSG_OP_GEMM_TRANSA ? tsg::A_COL : tsg::A_CONV);
    return TSG_OK;
}

tsg_status tsg_workspace_set(void* ws, int64_t bytes) {
    if ((ws == nullptr) != (bytes == 0) || bytes < 0) return TSG_E_INVALID;
    if (ws && (bytes <= kCounterBytes || (reinterpret_cast<uintptr_t>(ws) & 255u))) return TSG_E_INVALID;
    if (ws && hipMemset(ws, 0, kCounterBytes) != hipSuccess) return TSG_E_RUNTIME;   // counters start at zero
    std::lock_guard<std::mutex> g(g_mu);
    g_ws = ws;
    g_ws_bytes = bytes;
    return TSG_OK;
}

tsg_status tsg_workspace_set_stream(void* stream, void* ws, int64_t bytes) {
    if ((ws == nullptr) != (bytes == 0) || bytes < 0) return TSG_E_INVALID;
    if (ws && (bytes <= kCounterBytes || (reinterpret_cast<uintptr_t>(ws) & 255u))) return TSG_E_INVALID;
    if (ws && hipMemset(ws, 0, kCounterBytes) != hipSuccess) return TSG_E_RUNTIME;   // counters start at zero
    std::lock_guard<std::mutex> g(g_mu);
    if (ws) g_stream_ws[stream] = StreamWs{ws, bytes};
    else g_stream_ws.erase(stream);
    return TSG_OK;
}

int64_t tsg_workspace_bytes(tsg_dtype dtype, int64_t batch, int64_t M, int64_t N, const tsg_tile_config* cfg) {
    if (!valid_dtype(dtype) || !cfg || batch <= 0 || M <= 0 || N <= 0) return -1;
    const KernelEntry* e = find_entry(dtype, *cfg);
    if (!e || cfg->split_k < 1 || cfg->split_k > kMaxSplit) return -1;
    return ws_bytes_needed(*e, batch, M, N, cfg->split_k, cfg->split_tail);
}

tsg_status tsg_search_set(int32_t max_evals, int32_t model_order) {
    if (max_evals < 0 || model_order < 0 || model_order > 2) return TSG_E_INVALID;
    std::lock_guard<std::mutex> g(g_mu);
    g_search_max_evals = max_evals;
    g_search_model_order = model_order;
    return TSG_OK;
}

int32_t tsg_tune_cache_size(void) {
    std::lock_guard<std::mutex> g(g_mu);
    return (int32_t)g_tuned.size();
}

tsg_status tsg_tune_cache_clear(void) {
    std::lock_guard<std::mutex> g(g_mu);
    g_tuned.clear();
    return TSG_OK;
}

tsg_status tsg_tune_cache_save(const char* path) {
    if (!path) return TSG_E_INVALID;
    std::FILE* f = std::fopen(path, "w");
    if (!f) return TSG_E_RUNTIME;
    std::lock_guard<std::mutex> g(g_mu);
    std::fprintf(f, "# tsg tuner results: op dtype trans_b batch M N K contig  bm bn bk wm wn vec raster sched split_k split_tail mfma  ms\n");
    for (const auto& kv : g_tuned) {
        const TuneKey& k = kv.first;
        const tsg_tile_config& c = kv.second.cfg;
        std::fprintf(f, "%lld %lld %lld %lld %lld %lld %lld %lld  %d %d %d %d %d %d %d %d %d %d %d  %.6f\n", (long long)k[0],
                     (long long)k[1], (long long)k[2], (long long)k[3], (long long)k[4], (long long)k[5],
                     (long long)k[6], (long long)k[7], c.bm, c.bn, c.bk, c.wm, c.wn, c.vec, c.raster, c.sched,
                     c.split_k, c.split_tail, c.mfma, kv.second.ms);
    }
    return std::fclose(f) == 0 ? TSG_OK : TSG_E_RUNTIME;
}

tsg_status tsg_tune_cache_load(const char* path, int32_t* loaded, int32_t* rejected) {
    if (!path) return TSG_E_INVALID;
    std::FILE* f = std::fopen(path, "r");
    if (!f) return TSG_E_RUNTIME;
    int ok = 0, bad = 0;
    char line[512];
    while (std::fgets(line, sizeof line, f)) {
        if (line[0] == '#' || line[0] == '\n') continue;
        long long k[8];
        tsg_tile_config c;
        float ms = 0.f;
        const int n = std::sscanf(line, "%lld %lld %lld %lld %lld %lld %lld %lld %d %d %d %d %d %d %d %d %d %d %d %f", &k[0],
                                  &k[1], &k[2], &k[3], &k[4], &k[5], &k[6], &k[7], &c.bm, &c.bn, &c.bk, &c.wm, &c.wn,
                                  &c.vec, &c.raster, &c.sched, &c.split_k, &c.split_tail, &c.mfma, &ms);
        // an entry is taken only if it names an instantiated, well-formed config of a valid problem
        const bool good = n == 20 && valid_op((int)k[0]) && valid_dtype((int)k[1]) && (k[2] == 0 || k[2] == 1) &&
                          k[3] >= 1 && k[4] >= 1 && k[5] >= 1 && k[6] >= 1 && find_entry((tsg_dtype)k[1], c) &&
                          (c.vec == 1 || c.vec == vec_max((tsg_dtype)k[1])) && (c.raster == 0 || c.raster == 1) &&
                          c.split_k >= 1 && c.split_k <= kMaxSplit &&
                          (c.split_tail == 0 || (c.split_tail == 1 && c.split_k > 1));
        if (!good) { ++bad; continue; }
        std::lock_guard<std::mutex> g(g_mu);
        g_tuned[TuneKey{k[0], k[1], k[2], k[3], k[4], k[5], k[6], k[7]}] = TuneVal{c, ms};
        ++ok;
    }
    std::fclose(f);
    if (loaded) *loaded = ok;
    if (rejected) *rejected = bad;
    return TSG_OK;
}

tsg_status tsg_last_launch(tsg_launch_info* out) {
    if (!out) return TSG_E_INVALID;
    *out = t_last;
    return TSG_OK;
}

tsg_status tsg_conv2d_index_map(int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t KH, int64_t KW,
                                int64_t stride_h, int64_t stride_w, int64_t pad_h, int64_t pad_w, int32_t* off) {
    if (!off || N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || KH <= 0 || KW <= 0) return TSG_E_INVALID;
    if (stride_h <= 0 || stride_w <= 0 || pad_h < 0 || pad_w < 0) return TSG_E_INVALID;
    if (H + 2 * pad_h < KH || W + 2 * pad_w < KW) return TSG_E_INVALID;
    const int64_t lim = 0x7fffffff;
    if (N > lim / H || N * H > lim / W || N * H * W > lim / Cin) return TSG_E_INVALID;
    const int64_t Ho = (H + 2 * pad_h - KH) / stride_h + 1, Wo = (W + 2 * pad_w - KW) / stride_w + 1;
    const int64_t taps = KH * KW, M = N * Ho * Wo;
    // Same decode as the kernel's gather: m -> (n, ho, wo), tap -> (kh, kw).
    for (int64_t m = 0; m < M; ++m) {
        const int64_t wo = m % Wo, t = m / Wo, ho = t % Ho, n = t / Ho;
        const int64_t hi0 = ho * stride_h - pad_h, wi0 = wo * stride_w - pad_w;
        for (int64_t tap = 0; tap < taps; ++tap) {
            const int64_t kh = tap / KW, kw = tap - kh * KW;
            const int64_t hi = hi0 + kh, wi = wi0 + kw;
            const bool inside = hi >= 0 && hi < H && wi >= 0 && wi < W;
            off[m * taps + tap] = inside ? (int32_t)(((n * H + hi) * W + wi) * Cin) : -1;
        }
    }
    return TSG_OK;
}

tsg_status tsg_gemm_index_map(int32_t trans_a, int64_t M, int64_t K, int64_t lda, int64_t* off) {
    if (!off || M <= 0 || K <= 0 || lda < (trans_a ? M : K)) return TSG_E_INVALID;
    for (int64_t i = 0; i < M; ++i)
        for (int64_t k = 0; k < K; ++k) off[i * K + k] = trans_a ? k * lda + i : i * lda + k;
    return TSG_OK;
}

tsg_status tsg_autotune_gemm_trans(tsg_dtype dtype, int32_t trans_a, int32_t trans_b, int64_t batch, int64_t M,
                                   int64_t N, int64_t K, const void* A, int64_t lda, int64_t stride_a, const void* B,
                                     int64_t ldb, int64_t stride_b, float* C, int64_t ldc, int64_t stride_c,
                                     uint32_t flags, void* stream, int32_t iters, tsg_tile_config* best,
                                     float* best_ms, tsg_tune_record* log, int32_t log_cap, int32_t* n_log) {
    const tsg_status v = check_gemm(dtype, batch, M, N, K, A, lda, B, ldb, C, ldc, trans_a != 0, flags, trans_b != 0);
    if (v != TSG_OK) return v;
    if (stride_a < 0 || stride_b < 0 || stride_c < 0) return TSG_E_INVALID;
    if (batch > 1 && stride_c < (M - 1) * ldc + N) return TSG_E_INVALID;
    Problem p;
    p.trans_b = trans_b != 0;
    p.op = trans_a ? TSG_OP_GEMM_TRANSA : TSG_OP_GEMM;
    p.dtype = dtype;
    p.batch = batch;
    p.M = M; p.N = N; p.K = K;
    p.A = A; p.B = B; p.C = C;
    p.lda = lda; p.ldb = ldb; p.ldc = ldc;
    p.stride_a = stride_a; p.stride_b = stride_b; p.stride_c = stride_c;
    p.flags = flags;
    resolve_workspace(stream, &p.ws, &p.ws_bytes);
    return autotune(p, (hipStream_t)stream, iters, best, best_ms, log, log_cap, n_log);
}

tsg_status tsg_autotune_gemm(tsg_dtype dtype, int32_t trans_a, int64_t M, int64_t N, int64_t K, const void* A,
                             int64_t lda, const void* B, int64_t ldb, float* C, int64_t ldc, uint32_t flags,
                             void* stream, int32_t iters, tsg_tile_config* best, float* best_ms,
                             tsg_tune_record* log, int32_t log_cap, int32_t* n_log) {
    return tsg_autotune_gemm_trans(dtype, trans_a, 0, 1, M, N, K, A, lda, 0, B, ldb, 0, C, ldc, 0, flags, stream,
                                   iters, best, best_ms, log, log_cap, n_log);
}

tsg_status tsg_autotune_gemm_batched(tsg_dtype dtype, int32_t trans_a, int64_t batch, int64_t M, int64_t N,
                                     int64_t K, const void* A, int64_t lda, int64_t stride_a, const void* B,
                                     int64_t ldb, int64_t stride_b, float* C, int64_t ldc, int64_t stride_c,
                                     uint32_t flags, void* stream, int32_t iters, tsg_tile_config* best,
                                     float* best_ms, tsg_tune_record* log, int32_t log_cap, int32_t* n_log) {
    return tsg_autotune_gemm_trans(dtype, trans_a, 0, batch, M, N, K, A, lda, stride_a, B, ldb, stride_b, C, ldc,
                                   stride_c, flags, stream, iters, best, best_ms, log, log_cap, n_log);
}

tsg_status tsg_autotune_conv2d_nhwc(tsg_dtype dtype, int64_t N, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                                    int64_t KH, int64_t KW, int64_t stride_h, int64_t stride_w, int64_t pad_h,
                                    int64_t pad_w, const void* x, const void* w, float* y, uint32_t flags,
                                    void* stream, int32_t iters, tsg_tile_config* best, float* best_ms,
                                    tsg_tune_record* log, int32_t log_cap, int32_t* n_log) {
    Problem p;
    const tsg_status v = conv_problem(dtype, N, H, W, Cin, Cout, KH, KW, stride_h, stride_w, pad_h, pad_w, x, w, y,
                                      flags, &p);
    if (v != TSG_OK) return v;
    resolve_workspace(stream, &p.ws, &p.ws_bytes);
    return autotune(p, (hipStream_t)stream, iters, best, best_ms, log, log_cap, n_log);
}

}  // extern "C"
