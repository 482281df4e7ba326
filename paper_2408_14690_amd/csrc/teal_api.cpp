// C ABI of the library (include/teal.h): argument checks on the host, choice
// of the launch shape, then the kernel launches.  Nothing here allocates or
// synchronises; the only state kept is the per-device address of the
// library's own scratch array (teal_sparse_gemv_bf16_static).
#include "teal.h"
#include "teal_probe.h"

#include <atomic>
#include <cmath>

#include "teal_internal.h"

namespace {

using teal::GemvShape;

constexpr size_t kAlignWorkspace = 256;
constexpr int kComputeUnits = 256;

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

bool threshold_ok(float t) { return std::isfinite(t) && t >= 0.0f; }
bool norm_eps_ok(float eps) { return std::isfinite(eps) && eps >= 0.0f; }

int max_splits_for(int m)
{
    const int forced = (m + teal::kMaxSlice - 1) / teal::kMaxSlice;   // LDS list capacity
    return forced > teal::kMaxSplits ? forced : teal::kMaxSplits;
}

// Launch shape for one GEMV, from sweeps on MI355X.  A call costs a fixed latency
// chain (load x, compact, first weight rows), the row stream, and with split-K
// (Section 4.4) the publish / ticket / second-pass chain, which grows with the
// number of splits.  Measured times are flat over a wide range of shapes as long
// as (a) there is about one block of 8 wavefronts per compute unit and never a
// nearly empty second round, (b) the split-K depth is about 8, at most 16, and
// (c) a block's row segment is 256 B .. 1 KiB and starts on a 128-byte boundary
// (or neighbouring blocks would each fetch the cache line they share).
GemvShape auto_shape(int m, int n, int elems_per_lane, int min_lanes, int max_lanes,
                     int ks_multiple, int max_slice = teal::kMaxSlice)
{
    const int tc_min = min_lanes * elems_per_lane, tc_max = max_lanes * elems_per_lane;
    const int unit = 8 * elems_per_lane;                       // 128 bytes of a row
    int tc = (n + 31) / 32;                                    // 32 tiles x 8 splits = 256 blocks
    tc = (tc + unit - 1) / unit * unit;
    if (tc < tc_min) tc = tc_min;
    if (tc > tc_max) tc = tc_max;
    const int tiles = (n + tc - 1) / tc;
    int splits = 8;
    if (tiles * splits > kComputeUnits) splits = kComputeUnits / tiles;
    if (tiles * splits < 200) {
        splits = kComputeUnits / tiles;
        if (splits > 16) splits = 16;
    }
    const int most = (m + 127) / 128;                          // at least 128 channels per block
    if (splits > most) splits = most;
    const int least = (m + max_slice - 1) / max_slice;         // LDS list capacity
    if (splits < least) splits = least;
    if (splits < 1) splits = 1;
    int ks = (m + splits - 1) / splits;
    ks = (ks + ks_multiple - 1) / ks_multiple * ks_multiple;
    GemvShape sh;
    sh.splits = (m + ks - 1) / ks;
    sh.tile_cols = tc;
    int lanes = min_lanes;
    while (lanes * elems_per_lane < tc) lanes *= 2;
    sh.lanes_per_row = lanes;
    sh.waves = 8;
    sh.unroll = 4;
    return sh;
}

// Launch shape for several matrices in one launch.  The tiles of the matrices lie side by
// side and a tile never spans two matrices, so the tile count is the sum of the per-matrix
// counts, and a width that divides the matrices unevenly leaves ragged tiles.  Every
// candidate (tile width in steps of 128 bytes of a row, 1..16 splits) that fits one block
// per compute unit is scored by how evenly it spreads the work: total work over 256 times
// the largest block's work, with a small penalty per split beyond 8 (longer combine chain)
// and a slight preference for wider row segments.  For one matrix this reproduces the
// choices of auto_shape above.
GemvShape auto_shape_multi(int m, const int *n, int count, int elems_per_lane, int min_lanes,
                           int max_lanes, int ks_multiple, int max_slice = teal::kMaxSlice)
{
    long long n_total = 0;
    for (int k = 0; k < count; ++k) n_total += n[k];
    const int tc_min = min_lanes * elems_per_lane, tc_max = max_lanes * elems_per_lane;
    const int unit = 8 * elems_per_lane;
    double best = -1.0;
    int best_tc = tc_min, best_splits = 1;
    for (int tc = tc_min; tc <= tc_max; tc += unit) {
        long long tiles = 0;
        for (int k = 0; k < count; ++k) tiles += (n[k] + tc - 1) / tc;
        for (int splits = 1; splits <= 16; ++splits) {
            if (splits > 1 && splits > (m + 127) / 128) break;
            int ks = (m + splits - 1) / splits;
            ks = (ks + ks_multiple - 1) / ks_multiple * ks_multiple;
            if (ks > max_slice) continue;
            const int s = (m + ks - 1) / ks;
            if (tiles * s > kComputeUnits) continue;
            double score = (double)n_total * m / ((double)kComputeUnits * tc * ks);
            for (int e = 8; e < s; ++e) score *= 0.97;
            score *= 1.0 + 0.00002 * tc;
            if (score > best) {
                best = score;
                best_tc = tc;
                best_splits = s;
            }
        }
    }
    if (best < 0.0)                    // more tiles than compute units at every width
        return auto_shape(m, (int)n_total, elems_per_lane, min_lanes, max_lanes, ks_multiple,
                          max_slice);
    GemvShape sh;
    sh.splits = best_splits;
    sh.tile_cols = best_tc;
    int lanes = min_lanes;
    while (lanes * elems_per_lane < best_tc) lanes *= 2;
    sh.lanes_per_row = lanes;
    sh.waves = 8;
    sh.unroll = 4;
    return sh;
}

// A grouped call on matrices with padded rows.  When every matrix's rows lie an odd multiple
// of 256 bytes apart, a 256-byte tile meets all four 256-byte quarters of a KiB over its
// rows, so tiles of that width finish together whatever the split count; then, if the group
// has about one such tile per compute unit and a block can take the whole input dimension,
// split-K is not needed at all: a tile is finished by the block that streamed it, with no
// partial rows, ticket or second pass (measured 22.1 -> 20.3 us for the Llama-3-8B gate + up
// pair at 50 %, 18.5 -> 17.1 us for the Llama-2-7B pair, 13.1 -> 11.9 us for one 14336-wide
// matrix in tiles of 128 bytes).  Otherwise the shape of the packed call.
bool pitches_rotate(const int *row_pitch, int count, int bits)
{
    if (!row_pitch) return false;
    for (int k = 0; k < count; ++k) {
        const long long bytes = (long long)row_pitch[k] * bits / 8;
        if (bytes % 512 != 256) return false;
    }
    return true;
}

// Row pitches of a grouped call: NULL (packed rows), or per matrix at least the row, a
// multiple of `multiple` elements (rows stay 16-byte aligned), a row within 2^30 bytes.
bool pitches_ok(const int *row_pitch, const int *n, int count, int multiple, int bits)
{
    if (!row_pitch) return true;
    for (int k = 0; k < count; ++k)
        if (row_pitch[k] < n[k] || row_pitch[k] % multiple != 0 ||
            (long long)row_pitch[k] * bits / 8 > (1LL << 30))
            return false;
    return true;
}

GemvShape auto_shape_multi_pitch(int m, const int *n, const int *row_pitch, int count, int bits,
                                 int elems_per_lane, int min_lanes, int max_lanes,
                                 int ks_multiple)
{
    if (pitches_rotate(row_pitch, count, bits) && m <= teal::kMaxLongSlice) {
        // tiles of 256 bytes of a row, else of 512 (the 70B-sized gate + up pair), else of 128
        // (one cache line: a single 14336-wide matrix; with slices above kMaxSlice measured
        // slower than split-K: the 70B-sized q + k + v group 18.6 against 18.0 us)
        const int widths[3] = {256, 512, 128};
        for (int wi = 0; wi < 3; ++wi) {
            const int bytes = widths[wi];
            if (bytes == 128 && m > teal::kMaxSlice) continue;
            const int narrow = bytes * 8 / bits;
            long long tiles = 0;
            for (int k = 0; k < count; ++k) tiles += (n[k] + narrow - 1) / narrow;
            if (tiles >= 160 && tiles <= 384 && narrow / elems_per_lane >= 8 &&
                narrow / elems_per_lane <= max_lanes) {
                GemvShape sh;
                sh.lanes_per_row = narrow / elems_per_lane;
                sh.tile_cols = narrow;
                sh.splits = 1;
                sh.waves = 8;
                sh.unroll = 4;
                return sh;
            }
        }
    }
    int n_total = 0;
    for (int k = 0; k < count; ++k) n_total += n[k];
    return count > 1 ? auto_shape_multi(m, n, count, elems_per_lane, min_lanes, max_lanes, ks_multiple)
                     : auto_shape(m, n_total, elems_per_lane, min_lanes, max_lanes, ks_multiple);
}

// Partial rows a batched call may need: one per (split, batch row).
int batch_split_rows(int m)
{
    const int forced = (m + teal::kMaxSliceBatch - 1) / teal::kMaxSliceBatch;
    return forced > 16 ? forced : 16;
}

int batch_accumulators(int batch) { return batch <= 2 ? 2 : batch <= 4 ? 4 : 8; }

struct GemvArgs {
    const void *W;
    const void *x;
    float t;
    float *y;
    int m, n;
    void *workspace;
    size_t workspace_bytes;
};

teal_status check_gemv(const GemvArgs &a, int n_multiple)
{
    if (!a.W || !a.x || !a.y || !a.workspace) return TEAL_ERR_NULL;
    if (a.m < 1 || a.m > teal::kMaxDim || a.n < n_multiple || a.n > teal::kMaxDim ||
        a.n % n_multiple != 0)
        return TEAL_ERR_SHAPE;
    if (!aligned(a.W, 16) || !aligned(a.x, 2) || !aligned(a.y, 4) ||
        !aligned(a.workspace, kAlignWorkspace))
        return TEAL_ERR_ALIGN;
    if (!threshold_ok(a.t)) return TEAL_ERR_THRESHOLD;
    if (a.workspace_bytes < teal_workspace_bytes(a.m, a.n)) return TEAL_ERR_WORKSPACE;
    return TEAL_OK;
}

// The head of the workspace holds one arrival counter per output tile.  The shapes the
// library picks itself have tiles of at least kMinTile columns, which always fit; a
// caller-chosen tile width may not.
bool tiles_fit_counters(int n, const GemvShape &sh)
{
    const int tc = sh.tile_cols > 0 ? sh.tile_cols : sh.lanes_per_row * 8;
    const long long tiles = ((long long)n + tc - 1) / tc;
    return tiles <= (long long)(teal::kCounterBytes / sizeof(int));
}

teal_status from_hip(hipError_t e) { return e == hipSuccess ? TEAL_OK : TEAL_ERR_HIP; }

// Workspace layout: [arrival counters, kCounterBytes][survivor report, report_bytes(m)]
// [partial rows, splits x n fp32].  The report holds one total per matrix of the call and,
// per matrix, one count per split; its size allows for the most splits any call with this
// m can run with.
size_t report_bytes(int m)
{
    const int forced = (m + teal::kMaxSliceBatch - 1) / teal::kMaxSliceBatch;
    const size_t rows = forced > teal::kMaxSplits ? forced : teal::kMaxSplits;
    const size_t bytes = (teal::kReportHeaderInts + teal::kMaxMatrices * rows) * sizeof(int);
    return (bytes + kAlignWorkspace - 1) / kAlignWorkspace * kAlignWorkspace;
}
int *ws_counters(void *workspace) { return static_cast<int *>(workspace); }
float *ws_partials(void *workspace, int m)
{
    return reinterpret_cast<float *>(static_cast<unsigned char *>(workspace) +
                                     teal::kCounterBytes + report_bytes(m));
}

// ---- the library's own scratch, for teal_sparse_gemv_bf16_static ----
//
// One array per GPU the library runs on, held until the process ends, laid out like a
// caller's workspace for the largest call the entry point takes: [arrival counters]
// [survivor report][kStaticRows partial rows of kStaticMaxDim floats].  Zero at load; every
// call leaves the counters at zero again (the block that finishes a tile last resets the
// tile's counter), and the report and the partial rows are written before they are read, so
// the contents a call finds from the call before it never reach a result.
constexpr int kStaticMaxDim = 65536;           // largest m and n of a static-scratch call
constexpr int kStaticRows = 16;                // most splits the library picks for m <= kStaticMaxDim
constexpr size_t kStaticReportBytes =
    ((teal::kReportHeaderInts + (size_t)teal::kMaxMatrices * teal::kMaxSplits) * sizeof(int) +
     kAlignWorkspace - 1) / kAlignWorkspace * kAlignWorkspace;
constexpr size_t kStaticScratchBytes =
    teal::kCounterBytes + kStaticReportBytes + (size_t)kStaticRows * kStaticMaxDim * sizeof(float);

// `used`: no kernel of this file names the array, and it must still be emitted and registered
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device.  In host code the array's name is only a
// handle for this lookup; the address is what kernels and copies must be given.  Looked up on
// a device's first call (that device current), then kept; concurrent first calls look it up
// twice and store the same value.
hipError_t static_scratch(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return hipSuccess;
}

}  // namespace

extern "C" {

const char *teal_status_string(teal_status s)
{
    switch (s) {
    case TEAL_OK: return "ok";
    case TEAL_ERR_NULL: return "a required pointer is NULL";
    case TEAL_ERR_SHAPE: return "dimension out of range or not a multiple of the vector width";
    case TEAL_ERR_ALIGN: return "pointer not aligned as required";
    case TEAL_ERR_THRESHOLD: return "threshold must be finite and non-negative";
    case TEAL_ERR_WORKSPACE: return "workspace too small";
    case TEAL_ERR_UNSUPPORTED: return "unsupported group size or launch shape";
    case TEAL_ERR_HIP: return "HIP runtime error at launch";
    case TEAL_ERR_STATIC_LIMIT: return "m or n beyond what the library's static scratch holds";
    }
    return "unknown status";
}

int teal_version(void) { return 415; }

size_t teal_survivors_offset(void) { return teal::kCounterBytes; }

size_t teal_workspace_bytes(int m, int n)
{
    if (m < 1 || m > teal::kMaxDim || n < 1 || n > teal::kMaxDim) return 0;
    const size_t rows = (size_t)max_splits_for(m);
    const size_t bytes = teal::kCounterBytes + report_bytes(m) + rows * (size_t)n * sizeof(float);
    return (bytes + kAlignWorkspace - 1) / kAlignWorkspace * kAlignWorkspace;
}

teal_status teal_sparsify(const void *x_f16, int m, float t, uint8_t *mask, int32_t *idx,
                          int32_t *count, void *stream)
{
    if (m < 0) return TEAL_ERR_SHAPE;
    if (!x_f16 && m > 0) return TEAL_ERR_NULL;
    if (!aligned(x_f16, 2) || !aligned(idx, 4) || !aligned(count, 4)) return TEAL_ERR_ALIGN;
    if (!threshold_ok(t)) return TEAL_ERR_THRESHOLD;
    if (!mask && !idx && !count) return TEAL_OK;
    return from_hip(teal::launch_sparsify(x_f16, m, t, mask, idx, count,
                                          static_cast<hipStream_t>(stream)));
}

teal_status teal_sparse_gemv_bf16_ex(const void *Wt_bf16, const void *x_f16, float t, float *y,
                                     int m, int n, void *workspace, size_t workspace_bytes,
                                     void *stream, int lanes_per_row, int tile_cols, int splits,
                                     int waves, int unroll)
{
    const GemvArgs a{Wt_bf16, x_f16, t, y, m, n, workspace, workspace_bytes};
    const teal_status st = check_gemv(a, 8);
    if (st != TEAL_OK) return st;
    GemvShape sh = auto_shape(m, n, 8, 16, 64, 64);
    if (lanes_per_row) {
        sh.lanes_per_row = lanes_per_row;
        if (!tile_cols && sh.tile_cols > lanes_per_row * 8) sh.tile_cols = lanes_per_row * 8;
    }
    if (splits) sh.splits = splits;
    if (tile_cols) sh.tile_cols = tile_cols;
    if (waves) sh.waves = waves;
    if (unroll) sh.unroll = unroll;
    if (!teal::gemv_shape_supported(sh)) return TEAL_ERR_UNSUPPORTED;
    if (sh.splits > max_splits_for(m)) return TEAL_ERR_UNSUPPORTED;           // partial rows
    if (!tiles_fit_counters(n, sh)) return TEAL_ERR_UNSUPPORTED;
    return from_hip(teal::launch_gemv_bf16(Wt_bf16, x_f16, t, y, m, n, ws_partials(workspace, m),
                                           ws_counters(workspace), sh,
                                           static_cast<hipStream_t>(stream)));
}

teal_status teal_gemv_plan(int weight_bits, int m, int n, int *lanes_per_row, int *tile_cols,
                           int *splits, int *waves, int *unroll)
{
    if (m < 1 || m > teal::kMaxDim || n < 1 || n > teal::kMaxDim) return TEAL_ERR_SHAPE;
    GemvShape sh;
    if (weight_bits == 16) sh = auto_shape(m, n, 8, 16, 64, 64);
    else if (weight_bits == 8) sh = auto_shape(m, n, 16, 8, 64, 64);
    else if (weight_bits == 4) sh = auto_shape(m, n, 32, 16, 32, 128);
    else return TEAL_ERR_UNSUPPORTED;
    if (lanes_per_row) *lanes_per_row = sh.lanes_per_row;
    if (tile_cols) *tile_cols = sh.tile_cols;
    if (splits) *splits = sh.splits;
    if (waves) *waves = sh.waves;
    if (unroll) *unroll = sh.unroll;
    return TEAL_OK;
}

teal_status teal_gemv_plan_multi(int weight_bits, int m, const int *n, int count,
                                 int *lanes_per_row, int *tile_cols, int *splits, int *waves,
                                 int *unroll)
{
    if (!n) return TEAL_ERR_NULL;
    if (count < 1 || count > teal::kMaxMatrices) return TEAL_ERR_UNSUPPORTED;
    long long n_total = 0;
    for (int k = 0; k < count; ++k) {
        if (n[k] < 1 || n[k] > teal::kMaxDim) return TEAL_ERR_SHAPE;
        n_total += n[k];
    }
    if (m < 1 || m > teal::kMaxDim || n_total > teal::kMaxDim) return TEAL_ERR_SHAPE;
    if (count == 1)
        return teal_gemv_plan(weight_bits, m, n[0], lanes_per_row, tile_cols, splits, waves, unroll);
    GemvShape sh;
    if (weight_bits == 16) sh = auto_shape_multi(m, n, count, 8, 16, 64, 64);
    else if (weight_bits == 8) sh = auto_shape_multi(m, n, count, 16, 8, 64, 64);
    else if (weight_bits == 4) sh = auto_shape_multi(m, n, count, 32, 16, 32, 128);
    else return TEAL_ERR_UNSUPPORTED;
    if (lanes_per_row) *lanes_per_row = sh.lanes_per_row;
    if (tile_cols) *tile_cols = sh.tile_cols;
    if (splits) *splits = sh.splits;
    if (waves) *waves = sh.waves;
    if (unroll) *unroll = sh.unroll;
    return TEAL_OK;
}

teal_status teal_gemv_plan_multi_pitch(int weight_bits, int m, const int *n, const int *row_pitch,
                                       int count, int *lanes_per_row, int *tile_cols, int *splits,
                                       int *waves, int *unroll)
{
    if (!n || !row_pitch) return TEAL_ERR_NULL;
    if (count < 1 || count > teal::kMaxMatrices) return TEAL_ERR_UNSUPPORTED;
    if (weight_bits != 16 && weight_bits != 8) return TEAL_ERR_UNSUPPORTED;
    const int mult = weight_bits == 16 ? 8 : 16;
    long long n_total = 0;
    for (int k = 0; k < count; ++k) {
        if (n[k] < mult || n[k] > teal::kMaxDim || n[k] % mult != 0) return TEAL_ERR_SHAPE;
        n_total += n[k];
    }
    if (m < 1 || m > teal::kMaxDim || n_total > teal::kMaxDim) return TEAL_ERR_SHAPE;
    if (!pitches_ok(row_pitch, n, count, mult, weight_bits)) return TEAL_ERR_SHAPE;
    const GemvShape sh = weight_bits == 16
                             ? auto_shape_multi_pitch(m, n, row_pitch, count, 16, 8, 16, 64, 64)
                             : auto_shape_multi_pitch(m, n, row_pitch, count, 8, 16, 8, 64, 64);
    if (lanes_per_row) *lanes_per_row = sh.lanes_per_row;
    if (tile_cols) *tile_cols = sh.tile_cols;
    if (splits) *splits = sh.splits;
    if (waves) *waves = sh.waves;
    if (unroll) *unroll = sh.unroll;
    return TEAL_OK;
}

teal_status teal_sparse_gemv_bf16(const void *Wt_bf16, const void *x_f16, float t, float *y,
                                  int m, int n, void *workspace, size_t workspace_bytes,
                                  void *stream)
{
    return teal_sparse_gemv_bf16_ex(Wt_bf16, x_f16, t, y, m, n, workspace, workspace_bytes,
                                    stream, 0, 0, 0, 0, 0);
}

size_t teal_static_scratch_limit(void) { return (size_t)kStaticMaxDim; }

teal_status teal_static_scratch_init(void)
{
    void *base = nullptr;
    return from_hip(static_scratch(&base));
}

teal_status teal_sparse_gemv_bf16_static(const void *Wt_bf16, const void *x_f16, float t, float *y,
                                         int m, int n, void *stream)
{
    // the checks of teal_sparse_gemv_bf16, in its order, without those of a workspace
    if (!Wt_bf16 || !x_f16 || !y) return TEAL_ERR_NULL;
    if (m < 1 || m > teal::kMaxDim || n < 8 || n > teal::kMaxDim || n % 8 != 0)
        return TEAL_ERR_SHAPE;
    if (m > kStaticMaxDim || n > kStaticMaxDim) return TEAL_ERR_STATIC_LIMIT;
    if (!aligned(Wt_bf16, 16) || !aligned(x_f16, 2) || !aligned(y, 4)) return TEAL_ERR_ALIGN;
    if (!threshold_ok(t)) return TEAL_ERR_THRESHOLD;
    const GemvShape sh = auto_shape(m, n, 8, 16, 64, 64);      // as teal_sparse_gemv_bf16 picks
    if (sh.splits > kStaticRows) return TEAL_ERR_STATIC_LIMIT;  // cannot happen within the limit
    void *base = nullptr;
    if (static_scratch(&base) != hipSuccess) return TEAL_ERR_HIP;
    float *partial = reinterpret_cast<float *>(static_cast<unsigned char *>(base) +
                                               teal::kCounterBytes + kStaticReportBytes);
    return from_hip(teal::launch_gemv_bf16(Wt_bf16, x_f16, t, y, m, n, partial,
                                           static_cast<int *>(base), sh,
                                           static_cast<hipStream_t>(stream)));
}

teal_status teal_sparse_gemv_bf16_batch_multi(int count, const void *const *Wt_bf16,
                                              const float *t, float *const *Y, const int *n,
                                              const void *X_f16, int batch, int m,
                                              void *workspace, size_t workspace_bytes,
                                              void *stream)
{
    if (count < 1 || count > teal::kMaxMatrices) return TEAL_ERR_UNSUPPORTED;
    if (!Wt_bf16 || !t || !Y || !n || !X_f16 || !workspace) return TEAL_ERR_NULL;
    if (batch < 1 || batch > teal::kMaxBatch) return TEAL_ERR_SHAPE;
    long long n_total = 0;
    for (int k = 0; k < count; ++k) {
        if (!Wt_bf16[k] || !Y[k]) return TEAL_ERR_NULL;
        if (n[k] < 8 || n[k] > teal::kMaxDim || n[k] % 8 != 0) return TEAL_ERR_SHAPE;
        n_total += n[k];
    }
    if (m < 1 || m > teal::kMaxDim || n_total > teal::kMaxDim) return TEAL_ERR_SHAPE;
    for (int k = 0; k < count; ++k)
        if (!aligned(Wt_bf16[k], 16) || !aligned(Y[k], 4)) return TEAL_ERR_ALIGN;
    if (!aligned(X_f16, 2) || !aligned(workspace, kAlignWorkspace)) return TEAL_ERR_ALIGN;
    for (int k = 0; k < count; ++k)
        if (!threshold_ok(t[k])) return TEAL_ERR_THRESHOLD;
    if (workspace_bytes < teal_workspace_bytes_batch(m, (int)n_total, batch))
        return TEAL_ERR_WORKSPACE;
    const int max_lanes = batch_accumulators(batch) >= 4 ? 16 : 64;
    const GemvShape sh =
        count > 1 ? auto_shape_multi(m, n, count, 8, 16, max_lanes, 64, teal::kMaxSliceBatch)
                  : auto_shape(m, (int)n_total, 8, 16, max_lanes, 64, teal::kMaxSliceBatch);
    if (!teal::gemv_batch_shape_supported(batch, sh)) return TEAL_ERR_UNSUPPORTED;
    return from_hip(teal::launch_gemv_bf16_batch_multi(count, Wt_bf16, t, Y, n, X_f16, batch, m,
                                                       ws_partials(workspace, m),
                                                       ws_counters(workspace), sh,
                                                       static_cast<hipStream_t>(stream)));
}

teal_status teal_swiglu_f16(const float *gate, const float *up, void *h_f16, int m, void *stream)
{
    if (m < 0 || m > teal::kMaxDim) return TEAL_ERR_SHAPE;
    if ((!gate || !up || !h_f16) && m > 0) return TEAL_ERR_NULL;
    if (!aligned(gate, 4) || !aligned(up, 4) || !aligned(h_f16, 2)) return TEAL_ERR_ALIGN;
    return from_hip(teal::launch_swiglu_f16(gate, up, h_f16, m, static_cast<hipStream_t>(stream)));
}

teal_status teal_sparse_gemv_bf16_swiglu(const void *Wt_bf16, const float *gate, const float *up,
                                         float t, float *y, int m, int n, void *workspace,
                                         size_t workspace_bytes, void *stream)
{
    if (!up) return TEAL_ERR_NULL;
    const GemvArgs a{Wt_bf16, gate, t, y, m, n, workspace, workspace_bytes};
    const teal_status st = check_gemv(a, 8);
    if (st != TEAL_OK) return st;
    if (!aligned(gate, 4) || !aligned(up, 4)) return TEAL_ERR_ALIGN;
    const GemvShape sh = auto_shape(m, n, 8, 16, 64, 64);
    return from_hip(teal::launch_gemv_bf16_swiglu(Wt_bf16, gate, up, t, y, m, n,
                                                  ws_partials(workspace, m), ws_counters(workspace),
                                                  sh, static_cast<hipStream_t>(stream)));
}

static teal_status gemv_bf16_multi(int count, const void *const *Wt_bf16, const int *row_pitch,
                                   const float *t, float *const *y, const int *n,
                                   const void *x_f16, int m, void *workspace,
                                   size_t workspace_bytes, void *stream)
{
    if (count < 1 || count > teal::kMaxMatrices) return TEAL_ERR_UNSUPPORTED;
    if (!Wt_bf16 || !t || !y || !n || !x_f16 || !workspace) return TEAL_ERR_NULL;
    long long n_total = 0;
    for (int k = 0; k < count; ++k) {
        if (!Wt_bf16[k] || !y[k]) return TEAL_ERR_NULL;
        if (n[k] < 8 || n[k] > teal::kMaxDim || n[k] % 8 != 0) return TEAL_ERR_SHAPE;
        n_total += n[k];
    }
    if (m < 1 || m > teal::kMaxDim || n_total > teal::kMaxDim) return TEAL_ERR_SHAPE;
    if (!pitches_ok(row_pitch, n, count, 8, 16)) return TEAL_ERR_SHAPE;
    for (int k = 0; k < count; ++k)
        if (!aligned(Wt_bf16[k], 16) || !aligned(y[k], 4)) return TEAL_ERR_ALIGN;
    if (!aligned(x_f16, 2) || !aligned(workspace, kAlignWorkspace)) return TEAL_ERR_ALIGN;
    for (int k = 0; k < count; ++k)
        if (!threshold_ok(t[k])) return TEAL_ERR_THRESHOLD;
    if (workspace_bytes < teal_workspace_bytes(m, (int)n_total)) return TEAL_ERR_WORKSPACE;
    // Shape as for one matrix with all the output columns; a tile never spans two matrices.
    const GemvShape sh = auto_shape_multi_pitch(m, n, row_pitch, count, 16, 8, 16, 64, 64);
    return from_hip(teal::launch_gemv_bf16_multi(count, Wt_bf16, row_pitch, t, y, n, x_f16, m,
                                                 ws_partials(workspace, m), ws_counters(workspace),
                                                 sh, static_cast<hipStream_t>(stream)));
}

teal_status teal_sparse_gemv_bf16_multi(int count, const void *const *Wt_bf16, const float *t,
                                        float *const *y, const int *n, const void *x_f16, int m,
                                        void *workspace, size_t workspace_bytes, void *stream)
{
    return gemv_bf16_multi(count, Wt_bf16, nullptr, t, y, n, x_f16, m, workspace, workspace_bytes,
                           stream);
}

teal_status teal_sparse_gemv_bf16_multi_pitch(int count, const void *const *Wt_bf16,
                                              const int *row_pitch, const float *t,
                                              float *const *y, const int *n, const void *x_f16,
                                              int m, void *workspace, size_t workspace_bytes,
                                              void *stream)
{
    if (!row_pitch) return TEAL_ERR_NULL;
    return gemv_bf16_multi(count, Wt_bf16, row_pitch, t, y, n, x_f16, m, workspace,
                           workspace_bytes, stream);
}

// Region of group g in a stack call's workspace: the groups' regions follow each other,
// each laid out and sized as the workspace of that group's own grouped call.
static bool stack_group_dims(int count, const int *n, int m, int n_multiple, long long &n_total)
{
    if (count < 1 || count > teal::kMaxMatrices) return false;
    n_total = 0;
    for (int k = 0; k < count; ++k) {
        if (n[k] < n_multiple || n[k] > teal::kMaxDim || n[k] % n_multiple != 0) return false;
        n_total += n[k];
    }
    return m >= 1 && m <= teal::kMaxDim && n_total <= teal::kMaxDim;
}

size_t teal_workspace_bytes_stack(int groups, const int *counts, const int *n, const int *m)
{
    if (groups < 1 || groups > teal::kMaxStackGroups || !counts || !n || !m) return 0;
    size_t bytes = 0;
    for (int g = 0, first = 0; g < groups; first += counts[g], ++g) {
        long long n_total;
        if (counts[g] < 1 || counts[g] > teal::kMaxMatrices) return 0;
        if (!stack_group_dims(counts[g], n + first, m[g], 8, n_total)) return 0;
        bytes += teal_workspace_bytes(m[g], (int)n_total);
    }
    return bytes;
}

// The three stack entry points: the checks of the format's grouped call for every group,
// the groups' workspace regions, the launch shape of each group's own grouped call (same
// sums, bit for bit).  weight_bits 16: scale_f16 unused.
static teal_status stack_call(int weight_bits, int groups, const int *counts,
                              const void *const *W, const void *const *scale_f16, int group,
                              const float *t, float *const *y, const int *n,
                              const void *const *x_f16, const int *m, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    const bool quantised = weight_bits != 16;
    const int n_multiple = weight_bits == 16 ? 8 : weight_bits == 8 ? 16 : 32;
    if (groups < 1 || groups > teal::kMaxStackGroups) return TEAL_ERR_UNSUPPORTED;
    if (!counts || !W || (quantised && !scale_f16) || !t || !y || !n || !x_f16 || !m || !workspace)
        return TEAL_ERR_NULL;
    for (int g = 0; g < groups; ++g)
        if (counts[g] < 1 || counts[g] > teal::kMaxMatrices) return TEAL_ERR_UNSUPPORTED;
    if (!aligned(workspace, kAlignWorkspace)) return TEAL_ERR_ALIGN;
    teal::StackGroupDesc d[teal::kMaxStackGroups];
    size_t offset = 0;
    for (int g = 0, first = 0; g < groups; first += counts[g], ++g) {
        const int count = counts[g];
        if (!x_f16[g]) return TEAL_ERR_NULL;
        for (int k = 0; k < count; ++k)
            if (!W[first + k] || !y[first + k] || (quantised && !scale_f16[first + k]))
                return TEAL_ERR_NULL;
        long long n_total;
        if (!stack_group_dims(count, n + first, m[g], n_multiple, n_total)) return TEAL_ERR_SHAPE;
        for (int k = 0; k < count; ++k) {
            if (!aligned(W[first + k], 16) || !aligned(y[first + k], 4)) return TEAL_ERR_ALIGN;
            if (quantised && !aligned(scale_f16[first + k], weight_bits == 4 ? 16 : 2))
                return TEAL_ERR_ALIGN;
        }
        if (!aligned(x_f16[g], 2)) return TEAL_ERR_ALIGN;
        for (int k = 0; k < count; ++k)
            if (!threshold_ok(t[first + k])) return TEAL_ERR_THRESHOLD;
        if (weight_bits == 4 && (group != 128 || m[g] % 128 != 0)) return TEAL_ERR_UNSUPPORTED;
        unsigned char *region = static_cast<unsigned char *>(workspace) + offset;
        offset += teal_workspace_bytes(m[g], (int)n_total);
        if (offset > workspace_bytes) return TEAL_ERR_WORKSPACE;
        GemvShape sh;
        if (weight_bits == 16)
            sh = count > 1 ? auto_shape_multi(m[g], n + first, count, 8, 16, 64, 64)
                           : auto_shape(m[g], (int)n_total, 8, 16, 64, 64);
        else if (weight_bits == 8)
            sh = count > 1 ? auto_shape_multi(m[g], n + first, count, 16, 8, 64, 64)
                           : auto_shape(m[g], (int)n_total, 16, 8, 64, 64);
        else
            sh = count > 1 ? auto_shape_multi(m[g], n + first, count, 32, 16, 32, 128)
                           : auto_shape(m[g], (int)n_total, 32, 16, 32, 128);
        d[g] = teal::StackGroupDesc{count, W + first, quantised ? scale_f16 + first : nullptr,
                                    t + first, y + first, n + first, x_f16[g], m[g],
                                    ws_partials(region, m[g]), ws_counters(region), sh};
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (weight_bits == 16) return from_hip(teal::launch_gemv_bf16_stack(groups, d, st));
    if (weight_bits == 8) return from_hip(teal::launch_gemv_w8_stack(groups, d, st));
    return from_hip(teal::launch_gemv_w4_stack(groups, d, st));
}

teal_status teal_sparse_gemv_bf16_stack(int groups, const int *counts,
                                        const void *const *Wt_bf16, const float *t,
                                        float *const *y, const int *n, const void *const *x_f16,
                                        const int *m, void *workspace, size_t workspace_bytes,
                                        void *stream)
{
    return stack_call(16, groups, counts, Wt_bf16, nullptr, 0, t, y, n, x_f16, m, workspace,
                      workspace_bytes, stream);
}

teal_status teal_sparse_gemv_w8_stack(int groups, const int *counts, const int8_t *const *Wq,
                                      const void *const *scale_f16, const float *t,
                                      float *const *y, const int *n, const void *const *x_f16,
                                      const int *m, void *workspace, size_t workspace_bytes,
                                      void *stream)
{
    return stack_call(8, groups, counts, reinterpret_cast<const void *const *>(Wq), scale_f16, 0,
                      t, y, n, x_f16, m, workspace, workspace_bytes, stream);
}

teal_status teal_sparse_gemv_w4_stack(int groups, const int *counts, const uint8_t *const *Wq,
                                      const void *const *scale_f16, int group, const float *t,
                                      float *const *y, const int *n, const void *const *x_f16,
                                      const int *m, void *workspace, size_t workspace_bytes,
                                      void *stream)
{
    return stack_call(4, groups, counts, reinterpret_cast<const void *const *>(Wq), scale_f16,
                      group, t, y, n, x_f16, m, workspace, workspace_bytes, stream);
}

teal_status teal_rmsnorm_f16(const float *h, const float *gamma, float eps, void *x_f16, int m,
                             void *stream)
{
    if (m < 8 || m > teal::kMaxNormInput || m % 8 != 0) return TEAL_ERR_SHAPE;
    if (!h || !gamma || !x_f16) return TEAL_ERR_NULL;
    if (!aligned(h, 16) || !aligned(gamma, 4) || !aligned(x_f16, 2)) return TEAL_ERR_ALIGN;
    if (!norm_eps_ok(eps)) return TEAL_ERR_THRESHOLD;
    return from_hip(teal::launch_rmsnorm_f16(h, gamma, eps, x_f16, m,
                                             static_cast<hipStream_t>(stream)));
}

static teal_status gemv_bf16_rmsnorm_multi(int count, const void *const *Wt_bf16,
                                           const int *row_pitch, const float *t, float *const *y,
                                           const int *n, const float *h, const float *gamma,
                                           float eps, int m, void *workspace,
                                           size_t workspace_bytes, void *stream)
{
    if (count < 1 || count > teal::kMaxMatrices) return TEAL_ERR_UNSUPPORTED;
    if (!Wt_bf16 || !t || !y || !n || !h || !gamma || !workspace) return TEAL_ERR_NULL;
    long long n_total = 0;
    for (int k = 0; k < count; ++k) {
        if (!Wt_bf16[k] || !y[k]) return TEAL_ERR_NULL;
        if (n[k] < 8 || n[k] > teal::kMaxDim || n[k] % 8 != 0) return TEAL_ERR_SHAPE;
        n_total += n[k];
    }
    if (m < 8 || m > teal::kMaxNormInput || m % 8 != 0 || n_total > teal::kMaxDim)
        return TEAL_ERR_SHAPE;
    if (!pitches_ok(row_pitch, n, count, 8, 16)) return TEAL_ERR_SHAPE;
    for (int k = 0; k < count; ++k)
        if (!aligned(Wt_bf16[k], 16) || !aligned(y[k], 4)) return TEAL_ERR_ALIGN;
    if (!aligned(h, 16) || !aligned(gamma, 4) || !aligned(workspace, kAlignWorkspace))
        return TEAL_ERR_ALIGN;
    for (int k = 0; k < count; ++k)
        if (!threshold_ok(t[k])) return TEAL_ERR_THRESHOLD;
    if (!norm_eps_ok(eps)) return TEAL_ERR_THRESHOLD;
    if (workspace_bytes < teal_workspace_bytes(m, (int)n_total)) return TEAL_ERR_WORKSPACE;
    // The launch shape of teal_sparse_gemv_bf16_multi (_pitch): same sums, bit for bit.  This
    // kernel has no instance with 8 lanes per row: there the shape of the packed call.
    GemvShape sh = auto_shape_multi_pitch(m, n, row_pitch, count, 16, 8, 16, 64, 64);
    if (sh.lanes_per_row < 16)
        sh = auto_shape_multi_pitch(m, n, nullptr, count, 16, 8, 16, 64, 64);
    return from_hip(teal::launch_gemv_bf16_rmsnorm_multi(
        count, Wt_bf16, row_pitch, t, y, n, h, gamma, eps, m, ws_partials(workspace, m),
        ws_counters(workspace), sh, static_cast<hipStream_t>(stream)));
}

teal_status teal_sparse_gemv_bf16_rmsnorm_multi(int count, const void *const *Wt_bf16,
                                                const float *t, float *const *y, const int *n,
                                                const float *h, const float *gamma, float eps,
                                                int m, void *workspace, size_t workspace_bytes,
                                                void *stream)
{
    return gemv_bf16_rmsnorm_multi(count, Wt_bf16, nullptr, t, y, n, h, gamma, eps, m, workspace,
                                   workspace_bytes, stream);
}

teal_status teal_sparse_gemv_bf16_rmsnorm_multi_pitch(int count, const void *const *Wt_bf16,
                                                      const int *row_pitch, const float *t,
                                                      float *const *y, const int *n,
                                                      const float *h, const float *gamma,
                                                      float eps, int m, void *workspace,
                                                      size_t workspace_bytes, void *stream)
{
    if (!row_pitch) return TEAL_ERR_NULL;
    return gemv_bf16_rmsnorm_multi(count, Wt_bf16, row_pitch, t, y, n, h, gamma, eps, m,
                                   workspace, workspace_bytes, stream);
}

size_t teal_workspace_bytes_batch(int m, int n, int batch)
{
    if (m < 1 || m > teal::kMaxDim || n < 1 || n > teal::kMaxDim || batch < 1 ||
        batch > teal::kMaxBatch)
        return 0;
    const size_t rows = (size_t)batch_split_rows(m) * (size_t)batch;
    const size_t bytes = teal::kCounterBytes + report_bytes(m) + rows * (size_t)n * sizeof(float);
    return (bytes + kAlignWorkspace - 1) / kAlignWorkspace * kAlignWorkspace;
}

teal_status teal_sparsify_batch(const void *X_f16, int batch, int m, float t, uint8_t *mask,
                                int32_t *idx, int32_t *count, void *stream)
{
    if (m < 0 || batch < 1 || batch > teal::kMaxBatch) return TEAL_ERR_SHAPE;
    if (!X_f16 && m > 0) return TEAL_ERR_NULL;
    if (!aligned(X_f16, 2) || !aligned(idx, 4) || !aligned(count, 4)) return TEAL_ERR_ALIGN;
    if (!threshold_ok(t)) return TEAL_ERR_THRESHOLD;
    if (!mask && !idx && !count) return TEAL_OK;
    return from_hip(teal::launch_sparsify_batch(X_f16, batch, m, t, mask, idx, count,
                                                static_cast<hipStream_t>(stream)));
}

teal_status teal_sparse_gemv_bf16_batch_ex(const void *Wt_bf16, const void *X_f16, int batch,
                                           float t, float *Y, int m, int n, void *workspace,
                                           size_t workspace_bytes, void *stream,
                                           int lanes_per_row, int tile_cols, int splits)
{
    if (!Wt_bf16 || !X_f16 || !Y || !workspace) return TEAL_ERR_NULL;
    if (batch < 1 || batch > teal::kMaxBatch || m < 1 || m > teal::kMaxDim || n < 8 ||
        n > teal::kMaxDim || n % 8 != 0)
        return TEAL_ERR_SHAPE;
    if (!aligned(Wt_bf16, 16) || !aligned(X_f16, 2) || !aligned(Y, 4) ||
        !aligned(workspace, kAlignWorkspace))
        return TEAL_ERR_ALIGN;
    if (!threshold_ok(t)) return TEAL_ERR_THRESHOLD;
    if (workspace_bytes < teal_workspace_bytes_batch(m, n, batch)) return TEAL_ERR_WORKSPACE;
    // With several accumulator sets per lane, sweeps favour narrow tiles (128 columns) and
    // correspondingly fewer splits over the wide tiles of the single-vector kernel.
    const int max_lanes = batch_accumulators(batch) >= 4 ? 16 : 64;
    GemvShape sh = auto_shape(m, n, 8, 16, max_lanes, 64, teal::kMaxSliceBatch);
    if (lanes_per_row) {
        sh.lanes_per_row = lanes_per_row;
        if (!tile_cols && sh.tile_cols > lanes_per_row * 8) sh.tile_cols = lanes_per_row * 8;
    }
    if (splits) sh.splits = splits;
    if (tile_cols) sh.tile_cols = tile_cols;
    if (!teal::gemv_batch_shape_supported(batch, sh)) return TEAL_ERR_UNSUPPORTED;
    if (!tiles_fit_counters(n, sh)) return TEAL_ERR_UNSUPPORTED;
    const int ks = ((m + sh.splits - 1) / sh.splits + 63) / 64 * 64;
    if (ks > teal::kMaxSliceBatch) return TEAL_ERR_UNSUPPORTED;
    if ((m + ks - 1) / ks > batch_split_rows(m)) return TEAL_ERR_UNSUPPORTED;   // partial rows
    return from_hip(teal::launch_gemv_bf16_batch(Wt_bf16, X_f16, batch, t, Y, m, n,
                                                 ws_partials(workspace, m), ws_counters(workspace),
                                                 sh, static_cast<hipStream_t>(stream)));
}

teal_status teal_sparse_gemv_bf16_batch(const void *Wt_bf16, const void *X_f16, int batch, float t,
                                        float *Y, int m, int n, void *workspace,
                                        size_t workspace_bytes, void *stream)
{
    return teal_sparse_gemv_bf16_batch_ex(Wt_bf16, X_f16, batch, t, Y, m, n, workspace,
                                          workspace_bytes, stream, 0, 0, 0);
}

teal_status teal_sparse_gemv_w8(const int8_t *Wq, const void *scale_f16, const void *x_f16,
                                float t, float *y, int m, int n, void *workspace,
                                size_t workspace_bytes, void *stream)
{
    const GemvArgs a{Wq, x_f16, t, y, m, n, workspace, workspace_bytes};
    if (!scale_f16) return TEAL_ERR_NULL;
    const teal_status st = check_gemv(a, 16);
    if (st != TEAL_OK) return st;
    if (!aligned(scale_f16, 2)) return TEAL_ERR_ALIGN;
    const GemvShape sh = auto_shape(m, n, 16, 8, 64, 64);
    return from_hip(teal::launch_gemv_w8(Wq, scale_f16, x_f16, t, y, m, n, ws_partials(workspace, m),
                                         ws_counters(workspace), sh,
                                         static_cast<hipStream_t>(stream)));
}

teal_status teal_sparse_gemv_w8_swiglu(const int8_t *Wq, const void *scale_f16, const float *gate,
                                       const float *up, float t, float *y, int m, int n,
                                       void *workspace, size_t workspace_bytes, void *stream)
{
    if (!up || !scale_f16) return TEAL_ERR_NULL;
    const GemvArgs a{Wq, gate, t, y, m, n, workspace, workspace_bytes};
    const teal_status st = check_gemv(a, 16);
    if (st != TEAL_OK) return st;
    if (!aligned(gate, 4) || !aligned(up, 4) || !aligned(scale_f16, 2)) return TEAL_ERR_ALIGN;
    // The launch shape of teal_sparse_gemv_w8: same sums, bit for bit.
    const GemvShape sh = auto_shape(m, n, 16, 8, 64, 64);
    return from_hip(teal::launch_gemv_w8_swiglu(Wq, scale_f16, gate, up, t, y, m, n,
                                                ws_partials(workspace, m), ws_counters(workspace),
                                                sh, static_cast<hipStream_t>(stream)));
}

teal_status teal_sparse_gemv_w8_rmsnorm_multi(int count, const int8_t *const *Wq,
                                              const void *const *scale_f16, const float *t,
                                              float *const *y, const int *n, const float *h,
                                              const float *gamma, float eps, int m,
                                              void *workspace, size_t workspace_bytes,
                                              void *stream)
{
    if (count < 1 || count > teal::kMaxMatrices) return TEAL_ERR_UNSUPPORTED;
    if (!Wq || !scale_f16 || !t || !y || !n || !h || !gamma || !workspace) return TEAL_ERR_NULL;
    long long n_total = 0;
    for (int k = 0; k < count; ++k) {
        if (!Wq[k] || !scale_f16[k] || !y[k]) return TEAL_ERR_NULL;
        if (n[k] < 16 || n[k] > teal::kMaxDim || n[k] % 16 != 0) return TEAL_ERR_SHAPE;
        n_total += n[k];
    }
    if (m < 8 || m > teal::kMaxNormInput || m % 8 != 0 || n_total > teal::kMaxDim)
        return TEAL_ERR_SHAPE;
    for (int k = 0; k < count; ++k)
        if (!aligned(Wq[k], 16) || !aligned(scale_f16[k], 2) || !aligned(y[k], 4))
            return TEAL_ERR_ALIGN;
    if (!aligned(h, 16) || !aligned(gamma, 4) || !aligned(workspace, kAlignWorkspace))
        return TEAL_ERR_ALIGN;
    for (int k = 0; k < count; ++k)
        if (!threshold_ok(t[k])) return TEAL_ERR_THRESHOLD;
    if (!norm_eps_ok(eps)) return TEAL_ERR_THRESHOLD;
    if (workspace_bytes < teal_workspace_bytes(m, (int)n_total)) return TEAL_ERR_WORKSPACE;
    // The launch shape of teal_sparse_gemv_w8_multi: same sums, bit for bit.
    const GemvShape sh = count > 1 ? auto_shape_multi(m, n, count, 16, 8, 64, 64)
                                   : auto_shape(m, (int)n_total, 16, 8, 64, 64);
    return from_hip(teal::launch_gemv_w8_rmsnorm_multi(
        count, Wq, nullptr, scale_f16, t, y, n, h, gamma, eps, m, ws_partials(workspace, m),
        ws_counters(workspace), sh, static_cast<hipStream_t>(stream)));
}

static teal_status gemv_w8_multi(int count, const int8_t *const *Wq, const int *row_pitch,
                                 const void *const *scale_f16, const float *t, float *const *y,
                                 const int *n, const void *x_f16, int m, void *workspace,
                                 size_t workspace_bytes, void *stream)
{
    if (count < 1 || count > teal::kMaxMatrices) return TEAL_ERR_UNSUPPORTED;
    if (!Wq || !scale_f16 || !t || !y || !n || !x_f16 || !workspace) return TEAL_ERR_NULL;
    long long n_total = 0;
    for (int k = 0; k < count; ++k) {
        if (!Wq[k] || !scale_f16[k] || !y[k]) return TEAL_ERR_NULL;
        if (n[k] < 16 || n[k] > teal::kMaxDim || n[k] % 16 != 0) return TEAL_ERR_SHAPE;
        n_total += n[k];
    }
    if (m < 1 || m > teal::kMaxDim || n_total > teal::kMaxDim) return TEAL_ERR_SHAPE;
    if (!pitches_ok(row_pitch, n, count, 16, 8)) return TEAL_ERR_SHAPE;
    for (int k = 0; k < count; ++k)
        if (!aligned(Wq[k], 16) || !aligned(scale_f16[k], 2) || !aligned(y[k], 4))
            return TEAL_ERR_ALIGN;
    if (!aligned(x_f16, 2) || !aligned(workspace, kAlignWorkspace)) return TEAL_ERR_ALIGN;
    for (int k = 0; k < count; ++k)
        if (!threshold_ok(t[k])) return TEAL_ERR_THRESHOLD;
    if (workspace_bytes < teal_workspace_bytes(m, (int)n_total)) return TEAL_ERR_WORKSPACE;
    const GemvShape sh = auto_shape_multi_pitch(m, n, row_pitch, count, 8, 16, 8, 64, 64);
    return from_hip(teal::launch_gemv_w8_multi(count, Wq, row_pitch, scale_f16, t, y, n, x_f16, m,
                                               ws_partials(workspace, m), ws_counters(workspace), sh,
                                               static_cast<hipStream_t>(stream)));
}

teal_status teal_sparse_gemv_w8_multi(int count, const int8_t *const *Wq,
                                      const void *const *scale_f16, const float *t,
                                      float *const *y, const int *n, const void *x_f16, int m,
                                      void *workspace, size_t workspace_bytes, void *stream)
{
    return gemv_w8_multi(count, Wq, nullptr, scale_f16, t, y, n, x_f16, m, workspace,
                         workspace_bytes, stream);
}

teal_status teal_sparse_gemv_w8_multi_pitch(int count, const int8_t *const *Wq,
                                            const int *row_pitch, const void *const *scale_f16,
                                            const float *t, float *const *y, const int *n,
                                            const void *x_f16, int m, void *workspace,
                                            size_t workspace_bytes, void *stream)
{
    if (!row_pitch) return TEAL_ERR_NULL;
    return gemv_w8_multi(count, Wq, row_pitch, scale_f16, t, y, n, x_f16, m, workspace,
                         workspace_bytes, stream);
}

teal_status teal_sparse_gemv_w4(const uint8_t *Wq, const void *scale_f16, int group,
                                const void *x_f16, float t, float *y, int m, int n,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    const GemvArgs a{Wq, x_f16, t, y, m, n, workspace, workspace_bytes};
    if (!scale_f16) return TEAL_ERR_NULL;
    const teal_status st = check_gemv(a, 32);
    if (st != TEAL_OK) return st;
    if (!aligned(scale_f16, 16)) return TEAL_ERR_ALIGN;
    if (group != 128 || m % 128 != 0) return TEAL_ERR_UNSUPPORTED;
    const GemvShape sh = auto_shape(m, n, 32, 16, 32, 128);
    return from_hip(teal::launch_gemv_w4(Wq, scale_f16, x_f16, t, y, m, n, ws_partials(workspace, m),
                                         ws_counters(workspace), sh,
                                         static_cast<hipStream_t>(stream)));
}

teal_status teal_sparse_gemv_w4_swiglu(const uint8_t *Wq, const void *scale_f16, int group,
                                       const float *gate, const float *up, float t, float *y,
                                       int m, int n, void *workspace, size_t workspace_bytes,
                                       void *stream)
{
    if (!up || !scale_f16) return TEAL_ERR_NULL;
    const GemvArgs a{Wq, gate, t, y, m, n, workspace, workspace_bytes};
    const teal_status st = check_gemv(a, 32);
    if (st != TEAL_OK) return st;
    if (!aligned(gate, 4) || !aligned(up, 4) || !aligned(scale_f16, 16)) return TEAL_ERR_ALIGN;
    if (group != 128 || m % 128 != 0) return TEAL_ERR_UNSUPPORTED;
    // The launch shape of teal_sparse_gemv_w4: same sums, bit for bit.
    const GemvShape sh = auto_shape(m, n, 32, 16, 32, 128);
    return from_hip(teal::launch_gemv_w4_swiglu(Wq, scale_f16, gate, up, t, y, m, n,
                                                ws_partials(workspace, m), ws_counters(workspace),
                                                sh, static_cast<hipStream_t>(stream)));
}

teal_status teal_sparse_gemv_w4_rmsnorm_multi(int count, const uint8_t *const *Wq,
                                              const void *const *scale_f16, int group,
                                              const float *t, float *const *y, const int *n,
                                              const float *h, const float *gamma, float eps,
                                              int m, void *workspace, size_t workspace_bytes,
                                              void *stream)
{
    if (count < 1 || count > teal::kMaxMatrices) return TEAL_ERR_UNSUPPORTED;
    if (!Wq || !scale_f16 || !t || !y || !n || !h || !gamma || !workspace) return TEAL_ERR_NULL;
    long long n_total = 0;
    for (int k = 0; k < count; ++k) {
        if (!Wq[k] || !scale_f16[k] || !y[k]) return TEAL_ERR_NULL;
        if (n[k] < 32 || n[k] > teal::kMaxDim || n[k] % 32 != 0) return TEAL_ERR_SHAPE;
        n_total += n[k];
    }
    if (m < 8 || m > teal::kMaxNormInput || m % 8 != 0 || n_total > teal::kMaxDim)
        return TEAL_ERR_SHAPE;
    for (int k = 0; k < count; ++k)
        if (!aligned(Wq[k], 16) || !aligned(scale_f16[k], 16) || !aligned(y[k], 4))
            return TEAL_ERR_ALIGN;
    if (!aligned(h, 16) || !aligned(gamma, 4) || !aligned(workspace, kAlignWorkspace))
        return TEAL_ERR_ALIGN;
    for (int k = 0; k < count; ++k)
        if (!threshold_ok(t[k])) return TEAL_ERR_THRESHOLD;
    if (!norm_eps_ok(eps)) return TEAL_ERR_THRESHOLD;
    if (group != 128 || m % 128 != 0) return TEAL_ERR_UNSUPPORTED;
    if (workspace_bytes < teal_workspace_bytes(m, (int)n_total)) return TEAL_ERR_WORKSPACE;
    // The launch shape of teal_sparse_gemv_w4_multi: same sums, bit for bit.
    const GemvShape sh = count > 1 ? auto_shape_multi(m, n, count, 32, 16, 32, 128)
                                   : auto_shape(m, (int)n_total, 32, 16, 32, 128);
    return from_hip(teal::launch_gemv_w4_rmsnorm_multi(
        count, Wq, scale_f16, t, y, n, h, gamma, eps, m, ws_partials(workspace, m),
        ws_counters(workspace), sh, static_cast<hipStream_t>(stream)));
}

teal_status teal_sparse_gemv_w4_multi(int count, const uint8_t *const *Wq,
                                      const void *const *scale_f16, int group, const float *t,
                                      float *const *y, const int *n, const void *x_f16, int m,
                                      void *workspace, size_t workspace_bytes, void *stream)
{
    if (count < 1 || count > teal::kMaxMatrices) return TEAL_ERR_UNSUPPORTED;
    if (!Wq || !scale_f16 || !t || !y || !n || !x_f16 || !workspace) return TEAL_ERR_NULL;
    long long n_total = 0;
    for (int k = 0; k < count; ++k) {
        if (!Wq[k] || !scale_f16[k] || !y[k]) return TEAL_ERR_NULL;
        if (n[k] < 32 || n[k] > teal::kMaxDim || n[k] % 32 != 0) return TEAL_ERR_SHAPE;
        n_total += n[k];
    }
    if (m < 1 || m > teal::kMaxDim || n_total > teal::kMaxDim) return TEAL_ERR_SHAPE;
    for (int k = 0; k < count; ++k)
        if (!aligned(Wq[k], 16) || !aligned(scale_f16[k], 16) || !aligned(y[k], 4))
            return TEAL_ERR_ALIGN;
    if (!aligned(x_f16, 2) || !aligned(workspace, kAlignWorkspace)) return TEAL_ERR_ALIGN;
    for (int k = 0; k < count; ++k)
        if (!threshold_ok(t[k])) return TEAL_ERR_THRESHOLD;
    if (group != 128 || m % 128 != 0) return TEAL_ERR_UNSUPPORTED;
    if (workspace_bytes < teal_workspace_bytes(m, (int)n_total)) return TEAL_ERR_WORKSPACE;
    const GemvShape sh = count > 1 ? auto_shape_multi(m, n, count, 32, 16, 32, 128)
                                   : auto_shape(m, (int)n_total, 32, 16, 32, 128);
    return from_hip(teal::launch_gemv_w4_multi(count, Wq, scale_f16, t, y, n, x_f16, m,
                                               ws_partials(workspace, m), ws_counters(workspace), sh,
                                               static_cast<hipStream_t>(stream)));
}

teal_status teal_stream_read_probe(const void *buf, size_t bytes, int blocks, uint32_t match,
                                   uint32_t *sink, void *stream)
{
    if (!buf || !sink) return TEAL_ERR_NULL;
    if (bytes < 16 || bytes % 16 != 0 || blocks < 1 || blocks > 65536) return TEAL_ERR_SHAPE;
    if (!aligned(buf, 16) || !aligned(sink, 4)) return TEAL_ERR_ALIGN;
    return from_hip(teal::launch_stream_read(buf, bytes, blocks, match, sink,
                                             static_cast<hipStream_t>(stream)));
}

teal_status teal_abs_histogram(const void *x_f16, size_t count, uint64_t *hist, void *stream)
{
    if (!hist || (!x_f16 && count > 0)) return TEAL_ERR_NULL;
    if (!aligned(x_f16, 2) || !aligned(hist, 8)) return TEAL_ERR_ALIGN;
    if (count > ((size_t)1 << 38)) return TEAL_ERR_SHAPE;   // 512 GiB of fp16: beyond any one device
    return from_hip(teal::launch_abs_histogram(x_f16, count,
                                               reinterpret_cast<unsigned long long *>(hist),
                                               static_cast<hipStream_t>(stream)));
}

teal_status teal_histogram_thresholds(const uint64_t *hist, const double *p, int np, float *t,
                                      void *stream)
{
    if (!hist || !p || !t) return TEAL_ERR_NULL;
    if (np < 1 || np > 16) return TEAL_ERR_SHAPE;
    if (!aligned(hist, 8) || !aligned(t, 4)) return TEAL_ERR_ALIGN;
    for (int l = 0; l < np; ++l)
        if (!(p[l] >= 0.0 && p[l] <= 1.0)) return TEAL_ERR_THRESHOLD;
    return from_hip(teal::launch_histogram_thresholds(
        reinterpret_cast<const unsigned long long *>(hist), p, np, t,
        static_cast<hipStream_t>(stream)));
}

teal_status teal_pack_bf16(const void *W_rowmajor, void *Wt, int m, int n, void *stream)
{
    if (!W_rowmajor || !Wt) return TEAL_ERR_NULL;
    if (m < 1 || n < 1 || m > teal::kMaxDim || n > teal::kMaxDim ||
        (long long)m * (long long)n > (1LL << 40))
        return TEAL_ERR_SHAPE;
    if (!aligned(W_rowmajor, 2) || !aligned(Wt, 2)) return TEAL_ERR_ALIGN;
    return from_hip(
        teal::launch_pack_bf16(W_rowmajor, Wt, m, n, n, static_cast<hipStream_t>(stream)));
}

teal_status teal_pack_bf16_pitch(const void *W_rowmajor, void *Wt, int m, int n, int row_pitch,
                                 void *stream)
{
    if (!W_rowmajor || !Wt) return TEAL_ERR_NULL;
    if (m < 1 || n < 1 || m > teal::kMaxDim || n > teal::kMaxDim || row_pitch < n ||
        row_pitch > (1 << 29) || (long long)m * (long long)row_pitch > (1LL << 40))
        return TEAL_ERR_SHAPE;
    if (!aligned(W_rowmajor, 2) || !aligned(Wt, 2)) return TEAL_ERR_ALIGN;
    return from_hip(teal::launch_pack_bf16(W_rowmajor, Wt, m, n, row_pitch,
                                           static_cast<hipStream_t>(stream)));
}

}  // extern "C"

// ---- the MLP of a block in one launch ----

namespace {

using teal::kMlpControlBytes;
constexpr int kMlpDefaultSpinLimit = 1 << 20;      // about a second of polling

struct MlpFormat {
    int bits, elems_per_lane, min_lanes, max_lanes, ks_multiple, n_multiple;
};
bool mlp_format(int weight_bits, MlpFormat &f)
{
    if (weight_bits == 16) f = MlpFormat{16, 8, 16, 64, 64, 8};
    else if (weight_bits == 8) f = MlpFormat{8, 16, 8, 64, 64, 16};
    else if (weight_bits == 4) f = MlpFormat{4, 32, 16, 32, 128, 32};
    else return false;
    return true;
}

bool mlp_dims_ok(const MlpFormat &fm, int m, int f, int d)
{
    return m >= 1 && m <= teal::kMaxDim && f >= fm.n_multiple && 2LL * f <= teal::kMaxDim &&
           f % fm.n_multiple == 0 && d >= fm.n_multiple && d <= teal::kMaxDim &&
           d % fm.n_multiple == 0;
}

GemvShape to_shape(int lanes, int tile_cols, int splits)
{
    GemvShape sh;
    sh.lanes_per_row = lanes;
    sh.tile_cols = tile_cols;
    sh.splits = splits;
    sh.waves = 8;
    sh.unroll = 4;
    return sh;
}

// The library's choice.  W_down: the launch shape of its own call.  Gate / up: no split-K with
// tiles of 256 bytes of a row when that alone gives about one block per compute unit (the
// tile is then finished by the block that streamed it, and its consumers are told without the
// publish / ticket / second-pass chain in between: measured 1.3-1.6 us per call on
// Llama-2-7B- and Llama-3-8B-sized layers); else the launch shape of the grouped gate + up
// call.
// On rows that rotate over the address quarters (gu_row_pitch an odd multiple of 256 bytes;
// bf16 and int8) the rule of the grouped call on padded rows applies to gate / up: narrow
// tiles without split-K also for slices of up to 8192 channels and in tiles of 512 or 128
// bytes (int8 at Llama-3-8B sizes: 26.8 -> 23.7 us; bf16 at 70B sizes: 113.5 -> 109.5 us).
void mlp_default_shape(const MlpFormat &fm, int m, int f, int d, int gu_row_pitch,
                       teal_mlp_shape *out)
{
    const int n2[2] = {f, f};
    const int pitch2[2] = {gu_row_pitch, gu_row_pitch};
    GemvShape gu =
        auto_shape_multi(m, n2, 2, fm.elems_per_lane, fm.min_lanes, fm.max_lanes, fm.ks_multiple);
    const int narrow = 256 * 8 / fm.bits;                     // columns in 256 bytes of a row
    const long long narrow_blocks = 2LL * ((f + narrow - 1) / narrow);
    GemvShape rotating = gu;
    if (fm.bits != 4 && gu_row_pitch > 0 && pitches_rotate(pitch2, 2, fm.bits))
        rotating = auto_shape_multi_pitch(m, n2, pitch2, 2, fm.bits, fm.elems_per_lane,
                                          fm.min_lanes, fm.max_lanes, fm.ks_multiple);
    if (rotating.splits == 1 && rotating.lanes_per_row >= fm.min_lanes)   // this kernel's instances
        gu = rotating;
    else if (m <= teal::kMaxSlice && narrow_blocks >= 160 && narrow_blocks <= 384 &&
             narrow / fm.elems_per_lane >= fm.min_lanes)
        gu = to_shape(narrow / fm.elems_per_lane, narrow, 1);
    const GemvShape dn = auto_shape(f, d, fm.elems_per_lane, fm.min_lanes, fm.max_lanes, fm.ks_multiple);
    out->gu_lanes_per_row = gu.lanes_per_row;
    out->gu_tile_cols = gu.tile_cols;
    out->gu_splits = gu.splits;
    out->gu_phase_tiles = 0;
    out->down_lanes_per_row = dn.lanes_per_row;
    out->down_tile_cols = dn.tile_cols;
    out->down_splits = dn.splits;
    out->extra_lds_bytes = 0;
    out->spin_limit = kMlpDefaultSpinLimit;
}

bool mlp_launch_of(const MlpFormat &fm, const teal_mlp_shape &sh, int m, int f, int d,
                   teal::MlpLaunch &L, teal::MlpGrid &grid)
{
    if (sh.gu_phase_tiles < 0 || sh.extra_lds_bytes < 0 || sh.extra_lds_bytes > 48 * 1024 ||
        sh.spin_limit < 0)
        return false;
    // Row pitches: 0 (rows packed) or at least the row, rows 16-byte aligned, and a row's
    // bytes within what the kernels address with 32 bits; int4 rows are always packed.
    const auto pitch_ok = [&](int pitch, int n) {
        if (pitch == 0) return true;
        return fm.bits != 4 && pitch >= n && pitch % fm.n_multiple == 0 &&
               (long long)pitch * fm.bits / 8 <= (1LL << 30);
    };
    if (!pitch_ok(sh.gu_row_pitch, f) || !pitch_ok(sh.down_row_pitch, d)) return false;
    L.gu = to_shape(sh.gu_lanes_per_row, sh.gu_tile_cols, sh.gu_splits);
    L.down = to_shape(sh.down_lanes_per_row, sh.down_tile_cols, sh.down_splits);
    L.phase_tiles = sh.gu_phase_tiles;
    L.extra_lds = sh.extra_lds_bytes;
    L.spin_limit = (unsigned)sh.spin_limit;
    const auto lanes_ok = [&](int l) {
        return l >= fm.min_lanes && l <= fm.max_lanes && (l & (l - 1)) == 0;
    };
    if (!lanes_ok(L.gu.lanes_per_row) || !lanes_ok(L.down.lanes_per_row)) return false;
    if (!teal::mlp_grid_of(fm.bits, L, m, f, d, grid)) return false;
    // partial rows and arrival counters of the two regions
    if (grid.splits_gu > max_splits_for(m) || grid.splits_d > max_splits_for(f)) return false;
    if (2LL * grid.tiles_gu > (long long)(teal::kCounterBytes / sizeof(int)) ||
        grid.tiles_d > (long long)(teal::kCounterBytes / sizeof(int)))
        return false;
    return true;
}

struct MlpCall {
    const void *W_gate, *W_up, *W_down;
    const void *scale_gate, *scale_up, *scale_down;
    const void *x_f16;
    float t_gate, t_up, t_down;
    float *gate, *up, *y;
    int m, f, d;
    void *workspace;
    size_t workspace_bytes;
    void *stream;
};

teal_status mlp_call(int weight_bits, const MlpCall &c, int group, const teal_mlp_shape *shape)
{
    MlpFormat fm;
    if (!mlp_format(weight_bits, fm)) return TEAL_ERR_UNSUPPORTED;
    const bool quantised = weight_bits != 16;
    if (!c.W_gate || !c.W_up || !c.W_down || !c.x_f16 || !c.gate || !c.up || !c.y || !c.workspace)
        return TEAL_ERR_NULL;
    if (quantised && (!c.scale_gate || !c.scale_up || !c.scale_down)) return TEAL_ERR_NULL;
    if (!mlp_dims_ok(fm, c.m, c.f, c.d)) return TEAL_ERR_SHAPE;
    if (!aligned(c.W_gate, 16) || !aligned(c.W_up, 16) || !aligned(c.W_down, 16) ||
        !aligned(c.x_f16, 2) || !aligned(c.gate, 4) || !aligned(c.up, 4) || !aligned(c.y, 4) ||
        !aligned(c.workspace, kAlignWorkspace))
        return TEAL_ERR_ALIGN;
    const size_t scale_align = weight_bits == 4 ? 16 : 2;
    if (quantised && (!aligned(c.scale_gate, scale_align) || !aligned(c.scale_up, scale_align) ||
                      !aligned(c.scale_down, scale_align)))
        return TEAL_ERR_ALIGN;
    if (!threshold_ok(c.t_gate) || !threshold_ok(c.t_up) || !threshold_ok(c.t_down))
        return TEAL_ERR_THRESHOLD;
    if (weight_bits == 4 && (group != 128 || c.m % 128 != 0 || c.f % 128 != 0))
        return TEAL_ERR_UNSUPPORTED;
    if (c.workspace_bytes < teal_workspace_bytes_mlp(c.m, c.f, c.d)) return TEAL_ERR_WORKSPACE;
    teal_mlp_shape chosen;
    if (!shape) {
        mlp_default_shape(fm, c.m, c.f, c.d, 0, &chosen);
        chosen.gu_row_pitch = 0;
        chosen.down_row_pitch = 0;
        shape = &chosen;
    }
    teal::MlpLaunch L;
    teal::MlpGrid grid;
    if (!mlp_launch_of(fm, *shape, c.m, c.f, c.d, L, grid)) return TEAL_ERR_UNSUPPORTED;
    unsigned char *region_gu = static_cast<unsigned char *>(c.workspace);
    unsigned char *region_d = region_gu + teal_workspace_bytes(c.m, 2 * c.f);
    unsigned char *control = region_d + teal_workspace_bytes(c.f, c.d);
    const teal::MlpHostArgs h{c.W_gate, c.W_up, c.W_down, c.scale_gate, c.scale_up, c.scale_down,
                              c.x_f16, c.t_gate, c.t_up, c.t_down, c.gate, c.up, c.y, c.m, c.f,
                              c.d, shape->gu_row_pitch, shape->down_row_pitch,
                              ws_partials(region_gu, c.m), ws_counters(region_gu),
                              ws_partials(region_d, c.f), ws_counters(region_d),
                              reinterpret_cast<int *>(control)};
    hipStream_t st = static_cast<hipStream_t>(c.stream);
    if (weight_bits == 16) return from_hip(teal::launch_mlp_bf16(h, L, st));
    if (weight_bits == 8) return from_hip(teal::launch_mlp_w8(h, L, st));
    return from_hip(teal::launch_mlp_w4(h, L, st));
}

}  // namespace

extern "C" {

size_t teal_workspace_bytes_mlp(int m, int f, int d)
{
    if (f < 1 || f > teal::kMaxDim / 2) return 0;
    const size_t gu = teal_workspace_bytes(m, 2 * f), dn = teal_workspace_bytes(f, d);
    if (gu == 0 || dn == 0) return 0;
    return gu + dn + kMlpControlBytes;
}

size_t teal_mlp_down_region_offset(int m, int f)
{
    if (f < 1 || f > teal::kMaxDim / 2) return 0;
    return teal_workspace_bytes(m, 2 * f);
}

size_t teal_mlp_status_offset(int m, int f, int d)
{
    const size_t total = teal_workspace_bytes_mlp(m, f, d);
    if (total == 0) return 0;
    return total - kMlpControlBytes;
}

teal_status teal_mlp_plan(int weight_bits, int m, int f, int d, teal_mlp_shape *shape)
{
    MlpFormat fm;
    if (!shape) return TEAL_ERR_NULL;
    if (!mlp_format(weight_bits, fm)) return TEAL_ERR_UNSUPPORTED;
    if (!mlp_dims_ok(fm, m, f, d)) return TEAL_ERR_SHAPE;
    // the row pitches are the caller's (read here, left as they are): 0 = packed rows
    const auto pitch_ok = [&](int pitch, int n) {
        return pitch == 0 || (fm.bits != 4 && pitch >= n && pitch % fm.n_multiple == 0 &&
                              (long long)pitch * fm.bits / 8 <= (1LL << 30));
    };
    if (!pitch_ok(shape->gu_row_pitch, f) || !pitch_ok(shape->down_row_pitch, d))
        return TEAL_ERR_UNSUPPORTED;
    mlp_default_shape(fm, m, f, d, shape->gu_row_pitch, shape);
    return TEAL_OK;
}

teal_status teal_mlp_block_info(int weight_bits, int m, int f, int d, const teal_mlp_shape *shape,
                                int block, int *info)
{
    MlpFormat fm;
    if (!shape || !info) return TEAL_ERR_NULL;
    if (!mlp_format(weight_bits, fm)) return TEAL_ERR_UNSUPPORTED;
    if (!mlp_dims_ok(fm, m, f, d)) return TEAL_ERR_SHAPE;
    teal::MlpLaunch L;
    teal::MlpGrid g;
    if (!mlp_launch_of(fm, *shape, m, f, d, L, g)) return TEAL_ERR_UNSUPPORTED;
    const int blocks = teal::mlp_blocks(g);
    info[0] = blocks;
    if (block < 0 || block >= blocks) {
        for (int k = 1; k < 8; ++k) info[k] = -1;
        return TEAL_OK;
    }
    const teal::MlpBlock b = teal::mlp_block(g, block);
    info[1] = b.kind;
    info[2] = b.tile;
    info[3] = b.split;
    if (b.kind == teal::kMlpDown) {
        const int k0 = b.split * g.ks_d;
        info[4] = k0;
        info[5] = k0 + g.ks_d < f ? k0 + g.ks_d : f;
        info[6] = b.split;
        info[7] = teal::mlp_expected(g, b.split);
    } else {
        const int c0 = b.tile * g.tile_cols_gu;
        info[4] = c0;
        info[5] = c0 + g.tile_cols_gu < f ? c0 + g.tile_cols_gu : f;
        teal::mlp_signal_range(g, b.tile, info[6], info[7]);
    }
    return TEAL_OK;
}

teal_status teal_sparse_mlp_bf16(const void *Wt_gate, const void *Wt_up, const void *Wt_down,
                                 const void *x_f16, float t_gate, float t_up, float t_down,
                                 float *gate, float *up, float *y, int m, int f, int d,
                                 void *workspace, size_t workspace_bytes, void *stream,
                                 const teal_mlp_shape *shape)
{
    const MlpCall c{Wt_gate, Wt_up, Wt_down, nullptr, nullptr, nullptr, x_f16, t_gate, t_up,
                    t_down, gate, up, y, m, f, d, workspace, workspace_bytes, stream};
    return mlp_call(16, c, 0, shape);
}

teal_status teal_sparse_mlp_w8(const int8_t *Wq_gate, const int8_t *Wq_up,
                                  const int8_t *Wq_down, const void *scale_gate,
                                  const void *scale_up, const void *scale_down, const void *x_f16,
                                  float t_gate, float t_up, float t_down, float *gate, float *up,
                                  float *y, int m, int f, int d, void *workspace,
                                  size_t workspace_bytes, void *stream, const teal_mlp_shape *shape)
{
    const MlpCall c{Wq_gate, Wq_up, Wq_down, scale_gate, scale_up, scale_down, x_f16, t_gate,
                    t_up, t_down, gate, up, y, m, f, d, workspace, workspace_bytes, stream};
    return mlp_call(8, c, 0, shape);
}

teal_status teal_sparse_mlp_w4(const uint8_t *Wq_gate, const uint8_t *Wq_up,
                                  const uint8_t *Wq_down, const void *scale_gate,
                                  const void *scale_up, const void *scale_down, int group,
                                  const void *x_f16, float t_gate, float t_up, float t_down,
                                  float *gate, float *up, float *y, int m, int f, int d,
                                  void *workspace, size_t workspace_bytes, void *stream,
                                  const teal_mlp_shape *shape)
{
    const MlpCall c{Wq_gate, Wq_up, Wq_down, scale_gate, scale_up, scale_down, x_f16, t_gate,
                    t_up, t_down, gate, up, y, m, f, d, workspace, workspace_bytes, stream};
    return mlp_call(4, c, group, shape);
}

}  // extern "C"
