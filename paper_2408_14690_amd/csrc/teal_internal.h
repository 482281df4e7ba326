// Internal interface between the C-ABI layer (teal_api.cpp: argument checks,
// launch-shape choice) and the gfx950 kernels (*.hip).  Not installed.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "mlp_schedule.h"

namespace teal {

constexpr int kMaxSplits = 128;     // most split-K blocks a caller may ask for (longer inputs force more)
constexpr int kMaxSlice = 4096;     // most input channels one block compacts (LDS list capacity)
constexpr int kMaxLongSlice = 8192; // the same for the launches that run without split-K on
                                    // padded rows (the list then takes 64 KiB of LDS)
constexpr int kMaxDim = 1 << 24;    // largest m or n accepted
constexpr int kMaxMatrices = 4;     // matrices per fused launch
constexpr int kMinTile = 64;        // narrowest output tile of any kernel variant
constexpr int kMaxNormInput = 16384; // longest hidden state the fused normalisation takes
constexpr int kMaxBatch = 8;        // rows of a small batch (Section 5.4.4)
constexpr int kMaxSliceBatch = 2048;  // most input channels one block compacts for a batch
// Head of the workspace: one arrival counter per output tile (zero between calls).
constexpr size_t kCounterBytes = (size_t)(kMaxDim / kMinTile) * sizeof(int);
// The survivor report follows the counters: kReportHeaderInts ints that start with one
// total per matrix of the call, then kMaxMatrices rows of per-split counts.
constexpr int kReportHeaderInts = 64;

// How one sparse GEMV is laid over the chip.
struct GemvShape {
    int lanes_per_row;   // 64, 32, 16 or 8 lanes read one weight row per load (16 bytes each)
    int splits;          // blocks along the input dimension
    int tile_cols;       // output columns per block; 0 = lanes_per_row * elements per lane
    int waves;           // wavefronts per block (4, 8 or 16)
    int unroll;          // row loads per batch, two batches in flight per wavefront (4 or 8; 4 with 16 waves)
};

bool gemv_shape_supported(const GemvShape &s);

// Each returns the HIP status of its launches; all are asynchronous on `stream`.
hipError_t launch_sparsify(const void *x_f16, int m, float t, uint8_t *mask,
                           int32_t *idx, int32_t *count, hipStream_t stream);

hipError_t launch_gemv_bf16(const void *Wt, const void *x_f16, float t, float *y,
                            int m, int n, float *partial, int *counters,
                            const GemvShape &shape, hipStream_t stream);

hipError_t launch_gemv_bf16_swiglu(const void *Wt, const float *gate, const float *up, float t,
                                   float *y, int m, int n, float *partial, int *counters,
                                   const GemvShape &shape, hipStream_t stream);

// The grouped bf16 launch with its shared input formed from the hidden state h before the
// normalisation layer and the layer's weights gamma.  8 <= m <= 16384, m % 8 == 0; shapes
// with 8 wavefronts, 4 loads per batch and 16, 32 or 64 lanes per row.
hipError_t launch_gemv_bf16_rmsnorm_multi(int count, const void *const *Wt, const int *row_pitch,
                                          const float *t, float *const *y, const int *n,
                                          const float *h, const float *gamma, float eps, int m,
                                          float *partial, int *counters, const GemvShape &sh,
                                          hipStream_t stream);
hipError_t launch_rmsnorm_f16(const float *h, const float *gamma, float eps, void *x_f16, int m,
                              hipStream_t stream);
hipError_t launch_swiglu_f16(const float *gate, const float *up, void *h_f16, int m,
                             hipStream_t stream);

hipError_t launch_gemv_bf16_multi(int count, const void *const *Wt, const int *row_pitch,
                                  const float *t, float *const *y, const int *n,
                                  const void *x_f16, int m, float *partial, int *counters,
                                  const GemvShape &sh, hipStream_t stream);

// Up to kMaxStackGroups grouped calls of one weight format that do not depend on each other,
// in one launch.  Shapes with 8 wavefronts, 4 loads per batch and the format's lanes per row.
constexpr int kMaxStackGroups = 16;
struct StackGroupDesc {
    int count;                 // matrices of the group, 1..kMaxMatrices
    const void *const *Wt;
    const void *const *scale;  // quantised formats; NULL for bf16
    const float *t;
    float *const *y;
    const int *n;
    const void *x_f16;
    int m;
    float *partial;            // the group's own partial rows and counters
    int *counters;
    GemvShape shape;
};
hipError_t launch_gemv_bf16_stack(int groups, const StackGroupDesc *g, hipStream_t stream);
hipError_t launch_gemv_w8_stack(int groups, const StackGroupDesc *g, hipStream_t stream);
hipError_t launch_gemv_w4_stack(int groups, const StackGroupDesc *g, hipStream_t stream);

// Small batch (Section 5.4.4).  The slice of a block, ceil(m / splits) rounded up to 64,
// must not exceed kMaxSliceBatch.
bool gemv_batch_shape_supported(int batch, const GemvShape &s);

hipError_t launch_gemv_bf16_batch(const void *Wt, const void *X_f16, int batch, float t, float *Y,
                                  int m, int n, float *partial, int *counters,
                                  const GemvShape &shape, hipStream_t stream);

hipError_t launch_gemv_bf16_batch_multi(int count, const void *const *Wt, const float *t,
                                        float *const *Y, const int *n, const void *X_f16,
                                        int batch, int m, float *partial, int *counters,
                                        const GemvShape &shape, hipStream_t stream);

hipError_t launch_sparsify_batch(const void *X_f16, int batch, int m, float t, uint8_t *mask,
                                 int32_t *idx, int32_t *count, hipStream_t stream);

hipError_t launch_gemv_w8(const int8_t *Wq, const void *scale_f16, const void *x_f16,
                          float t, float *y, int m, int n, float *partial, int *counters,
                          const GemvShape &shape, hipStream_t stream);

hipError_t launch_gemv_w8_multi(int count, const int8_t *const *Wq, const int *row_pitch,
                                const void *const *scale_f16, const float *t, float *const *y,
                                const int *n, const void *x_f16, int m, float *partial,
                                int *counters, const GemvShape &sh, hipStream_t stream);

hipError_t launch_gemv_w8_swiglu(const int8_t *Wq, const void *scale_f16, const float *gate,
                                 const float *up, float t, float *y, int m, int n, float *partial,
                                 int *counters, const GemvShape &shape, hipStream_t stream);

hipError_t launch_gemv_w8_rmsnorm_multi(int count, const int8_t *const *Wq, const int *row_pitch,
                                        const void *const *scale_f16, const float *t,
                                        float *const *y, const int *n, const float *h,
                                        const float *gamma, float eps, int m, float *partial,
                                        int *counters, const GemvShape &sh, hipStream_t stream);

hipError_t launch_gemv_w4(const uint8_t *Wq, const void *scale_f16, const void *x_f16,
                          float t, float *y, int m, int n, float *partial, int *counters,
                          const GemvShape &shape, hipStream_t stream);

hipError_t launch_gemv_w4_swiglu(const uint8_t *Wq, const void *scale_f16, const float *gate,
                                 const float *up, float t, float *y, int m, int n, float *partial,
                                 int *counters, const GemvShape &shape, hipStream_t stream);

hipError_t launch_gemv_w4_rmsnorm_multi(int count, const uint8_t *const *Wq,
                                        const void *const *scale_f16, const float *t,
                                        float *const *y, const int *n, const float *h,
                                        const float *gamma, float eps, int m, float *partial,
                                        int *counters, const GemvShape &shape, hipStream_t stream);

hipError_t launch_gemv_w4_multi(int count, const uint8_t *const *Wq, const void *const *scale_f16,
                                const float *t, float *const *y, const int *n, const void *x_f16,
                                int m, float *partial, int *counters, const GemvShape &shape,
                                hipStream_t stream);

// The MLP of a block in one launch (Appendix A.3): gate and up from x, then W_down on
// SiLU(gate) . up, the blocks of W_down waiting for the gate / up tiles they read.
struct MlpLaunch {
    GemvShape gu, down;          // 8 wavefronts, 4 loads per batch
    int phase_tiles;             // gate / up tiles per phase of the grid order; 0 = one phase
    int extra_lds;               // dynamic LDS requested beyond need (fewer blocks per unit)
    unsigned spin_limit;         // polls before a waiting block gives up
};
struct MlpHostArgs {
    const void *W_gate, *W_up, *W_down;
    const void *scale_gate, *scale_up, *scale_down;   // quantised formats, else NULL
    const void *x_f16;
    float t_gate, t_up, t_down;
    float *gate, *up, *y;
    int m, f, d;                 // model width in, MLP width, model width out
    int gu_pitch, down_pitch;    // elements between rows of W_gate / W_up and of W_down; 0 = f, d
    float *partial_gu;
    int *counters_gu;            // head of the gate / up region of the workspace
    float *partial_d;
    int *counters_d;             // head of the W_down region
    int *control;                // kMlpControlBytes: status word, one readiness counter per W_down block
};
constexpr int kMlpMaxConsumers = 4096;       // most thread blocks of the W_down product
constexpr size_t kMlpControlBytes = 128 * (size_t)(1 + kMlpMaxConsumers);
// The grid of such a launch for a weight format (16, 8 or 4 bits); false if the shapes do
// not give a launchable grid.
bool mlp_grid_of(int weight_bits, const MlpLaunch &L, int m, int f, int d, MlpGrid &grid);
hipError_t launch_mlp_bf16(const MlpHostArgs &h, const MlpLaunch &L, hipStream_t stream);
hipError_t launch_mlp_w8(const MlpHostArgs &h, const MlpLaunch &L, hipStream_t stream);
hipError_t launch_mlp_w4(const MlpHostArgs &h, const MlpLaunch &L, hipStream_t stream);

hipError_t launch_abs_histogram(const void *x_f16, size_t count, unsigned long long *hist,
                                hipStream_t stream);

hipError_t launch_histogram_thresholds(const unsigned long long *hist, const double *p, int np,
                                       float *t_out, hipStream_t stream);

hipError_t launch_stream_read(const void *buf, size_t bytes, int blocks, uint32_t match,
                              uint32_t *sink, hipStream_t stream);

hipError_t launch_pack_bf16(const void *W_rowmajor, void *Wt, int m, int n, int pitch,
                            hipStream_t stream);

}  // namespace teal
