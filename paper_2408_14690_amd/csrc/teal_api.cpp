// C ABI of the library (include/teal.h): argument checks on the host, choice
// of the launch shape, then the kernel launches.  Nothing here allocates,
// synchronises or keeps state.
#include "teal.h"

#include <cmath>

#include "teal_internal.h"

namespace {

using teal::GemvShape;

constexpr size_t kAlignWorkspace = 256;
constexpr int kComputeUnits = 256;

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

bool threshold_ok(float t) { return std::isfinite(t) && t >= 0.0f; }

int max_splits_for(int m)
{
    const int forced = (m + teal::kMaxSlice - 1) / teal::kMaxSlice;   // LDS list capacity
    return forced > teal::kMaxSplits ? forced : teal::kMaxSplits;
}

// Launch shape for one GEMV.  Measured on MI355X, the time of a call is a fixed
// latency chain (load x, compact, first weight rows; then publish partial rows,
// ticket, second pass) plus the row stream at HBM speed, and is flat over a wide
// range of shapes as long as (a) every compute unit has one block of 8
// wavefronts, (b) the split-K depth (Section 4.4) stays small, so that the
// partial rows and the second pass are cheap, and (c) a row segment per block is
// 256 B .. 1 KiB.  So: aim at tiles * splits == number of compute units, prefer
// about 8 splits, and size the output tile to fit.
GemvShape auto_shape(int m, int n, int elems_per_lane, int min_lanes, int max_lanes,
                     int ks_multiple)
{
    static const int preferred_splits[] = {8, 7, 6, 5, 4, 12, 14, 16, 10, 3, 2, 24, 32, 1, 48, 64, 128};
    const int tc_min = min_lanes * elems_per_lane, tc_max = max_lanes * elems_per_lane;
    GemvShape best{};
    double best_cost = 1e30;
    int rank = 0;
    for (int asked : preferred_splits) {
        ++rank;
        int ks = (m + asked - 1) / asked;
        ks = (ks + ks_multiple - 1) / ks_multiple * ks_multiple;
        if (ks > teal::kMaxSlice) continue;
        if (asked > 1 && ks < 128) continue;                // too few channels per block
        const int splits = (m + ks - 1) / ks;               // after rounding the slice up
        const int tiles_wanted = (kComputeUnits + splits / 2) / splits;
        int tc = (n + tiles_wanted - 1) / tiles_wanted;
        tc = (tc + elems_per_lane - 1) / elems_per_lane * elems_per_lane;
        if (tc < tc_min) tc = tc_min;
        if (tc > tc_max) tc = tc_max;
        const int tiles = (n + tc - 1) / tc;
        const double blocks = (double)tiles * splits;
        double cost = (blocks > kComputeUnits ? (blocks - kComputeUnits) * 2.0 : kComputeUnits - blocks)
                      / kComputeUnits + 0.01 * rank;
        if (cost < best_cost) {
            best_cost = cost;
            best.splits = splits;
            best.tile_cols = tc;
        }
    }
    if (best_cost == 1e30) {     // very long input: as few splits as the LDS list allows
        best.splits = (m + teal::kMaxSlice - 1) / teal::kMaxSlice;
        best.tile_cols = tc_max;
    }
    int lanes = min_lanes;
    while (lanes * elems_per_lane < best.tile_cols) lanes *= 2;
    best.lanes_per_row = lanes;
    best.waves = 8;
    best.unroll = 4;
    return best;
}

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

teal_status from_hip(hipError_t e) { return e == hipSuccess ? TEAL_OK : TEAL_ERR_HIP; }

// Workspace layout: [arrival counters, kCounterBytes][partial rows, splits x n fp32].
int *ws_counters(void *workspace) { return static_cast<int *>(workspace); }
float *ws_partials(void *workspace)
{
    return reinterpret_cast<float *>(static_cast<unsigned char *>(workspace) + teal::kCounterBytes);
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
    }
    return "unknown status";
}

int teal_version(void) { return 100; }

size_t teal_workspace_bytes(int m, int n)
{
    if (m < 1 || m > teal::kMaxDim || n < 1 || n > teal::kMaxDim) return 0;
    const size_t rows = (size_t)max_splits_for(m);
    const size_t bytes = teal::kCounterBytes + rows * (size_t)n * sizeof(float);
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
    return from_hip(teal::launch_gemv_bf16(Wt_bf16, x_f16, t, y, m, n, ws_partials(workspace),
                                           ws_counters(workspace), sh,
                                           static_cast<hipStream_t>(stream)));
}

teal_status teal_gemv_plan(int weight_bits, int m, int n, int *lanes_per_row, int *tile_cols,
                           int *splits, int *waves, int *unroll)
{
    if (m < 1 || m > teal::kMaxDim || n < 1 || n > teal::kMaxDim) return TEAL_ERR_SHAPE;
    GemvShape sh;
    if (weight_bits == 16) sh = auto_shape(m, n, 8, 16, 64, 64);
    else if (weight_bits == 8) sh = auto_shape(m, n, 16, 16, 64, 64);
    else if (weight_bits == 4) sh = auto_shape(m, n, 32, 16, 32, 128);
    else return TEAL_ERR_UNSUPPORTED;
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

teal_status teal_sparse_gemv_w8(const int8_t *Wq, const void *scale_f16, const void *x_f16,
                                float t, float *y, int m, int n, void *workspace,
                                size_t workspace_bytes, void *stream)
{
    const GemvArgs a{Wq, x_f16, t, y, m, n, workspace, workspace_bytes};
    if (!scale_f16) return TEAL_ERR_NULL;
    const teal_status st = check_gemv(a, 16);
    if (st != TEAL_OK) return st;
    if (!aligned(scale_f16, 2)) return TEAL_ERR_ALIGN;
    const GemvShape sh = auto_shape(m, n, 16, 16, 64, 64);
    return from_hip(teal::launch_gemv_w8(Wq, scale_f16, x_f16, t, y, m, n, ws_partials(workspace),
                                         ws_counters(workspace), sh,
                                         static_cast<hipStream_t>(stream)));
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
    return from_hip(teal::launch_gemv_w4(Wq, scale_f16, x_f16, t, y, m, n, ws_partials(workspace),
                                         ws_counters(workspace), sh,
                                         static_cast<hipStream_t>(stream)));
}

teal_status teal_pack_bf16(const void *W_rowmajor, void *Wt, int m, int n, void *stream)
{
    if (!W_rowmajor || !Wt) return TEAL_ERR_NULL;
    if (m < 1 || n < 1 || m > teal::kMaxDim || n > teal::kMaxDim ||
        (long long)m * (long long)n > (1LL << 40))
        return TEAL_ERR_SHAPE;
    if (!aligned(W_rowmajor, 2) || !aligned(Wt, 2)) return TEAL_ERR_ALIGN;
    return from_hip(teal::launch_pack_bf16(W_rowmajor, Wt, m, n, static_cast<hipStream_t>(stream)));
}

}  // extern "C"
