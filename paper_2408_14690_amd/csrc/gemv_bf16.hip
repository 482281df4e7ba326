// y = s_t(x) W^T for bf16 weights stored input-channel-major (Sections 3, 4.2, 4.4).
#include "gemv_common.h"
#include "gemv_dispatch.h"
#include "gemv_mlp.h"

namespace teal {

struct FmtBF16 {
    static constexpr int kElemsPerLane = 8;   // 16 bytes = 8 bf16
    static constexpr int kBitsPerElem = 16;
    struct Args {
        const void *W;
        int ld = 0;             // elements from one row of W to the next; 0 = n
    };
    // bf16 -> fp32 is a 16-bit shift; bf16 * fp16 is exact in fp32 (8 + 11 significand bits).
    static __device__ __forceinline__ void fma(float (&acc)[8], u32x4 v, float xv)
    {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            acc[2 * q] = fmaf(xv, __uint_as_float(v[q] << 16), acc[2 * q]);
            acc[2 * q + 1] = fmaf(xv, __uint_as_float(v[q] & 0xffff0000u), acc[2 * q + 1]);
        }
    }
    struct ColumnScale {};
    static __device__ __forceinline__ ColumnScale column_scale(const Args &, int) { return {}; }
    static __device__ __forceinline__ float finish(float sum, ColumnScale) { return sum; }
};

bool gemv_shape_supported(const GemvShape &s)
{
    const bool lpr = s.lanes_per_row == 64 || s.lanes_per_row == 32 || s.lanes_per_row == 16 ||
                     s.lanes_per_row == 8;
    const bool wv = s.waves == 4 || s.waves == 8 || s.waves == 16;
    const bool un = s.unroll == 4 || (s.unroll == 8 && s.waves != 16);
    const bool tc = s.tile_cols >= 0 && s.tile_cols % 8 == 0 && s.tile_cols <= s.lanes_per_row * 8;
    return lpr && wv && un && tc && s.splits >= 1;
}

hipError_t launch_gemv_bf16(const void *Wt, const void *x_f16, float t, float *y, int m, int n,
                            float *partial, int *counters, const GemvShape &sh,
                            hipStream_t stream)
{
    const GemvGeometry g = gemv_geometry(m, n, sh, FmtBF16::kElemsPerLane, 64, kMaxLongSlice);
    FmtBF16::Args a{Wt};
    const __half *x = static_cast<const __half *>(x_f16);
#define TEAL_LAUNCH(F, LPR, WAVES, U)                                                          \
    do {                                                                                       \
        if (!allow_large_lds(sparse_gemv_kernel<F, LPR, WAVES, U>, g.lds))                     \
            return hipErrorInvalidValue;                                                       \
        hipLaunchKernelGGL((sparse_gemv_kernel<F, LPR, WAVES, U>), dim3(g.tiles * g.splits),   \
                           dim3(WAVES * 64), g.lds, stream, a, x, t, partial, counters, y, m,  \
                           n, g.ks, g.tiles, g.tile_cols, g.splits);                           \
    } while (0)
    TEAL_DISPATCH(TEAL_LAUNCH, FmtBF16, sh);
#undef TEAL_LAUNCH
    return hipGetLastError();
}

hipError_t launch_gemv_bf16_swiglu(const void *Wt, const float *gate, const float *up, float t,
                                   float *y, int m, int n, float *partial, int *counters,
                                   const GemvShape &sh, hipStream_t stream)
{
    const GemvGeometry g = gemv_geometry(m, n, sh, FmtBF16::kElemsPerLane, 64);
    FmtBF16::Args a{Wt};
#define TEAL_LAUNCH(F, LPR, WAVES, U)                                                          \
    hipLaunchKernelGGL((sparse_gemv_swiglu_kernel<F, LPR, WAVES, U>), dim3(g.tiles * g.splits), \
                       dim3(WAVES * 64), g.lds, stream, a, gate, up, t, partial, counters, y,  \
                       m, n, g.ks, g.tiles, g.tile_cols, g.splits)
    TEAL_DISPATCH(TEAL_LAUNCH, FmtBF16, sh);
#undef TEAL_LAUNCH
    return hipGetLastError();
}

hipError_t launch_gemv_bf16_multi(int count, const void *const *Wt, const int *row_pitch,
                                  const float *t, float *const *y, const int *n,
                                  const void *x_f16, int m, float *partial, int *counters,
                                  const GemvShape &sh, hipStream_t stream)
{
    int n_max = 0;
    for (int k = 0; k < count; ++k) n_max = n[k] > n_max ? n[k] : n_max;
    // slice length, split count and LDS size do not depend on n
    const GemvGeometry g =
        gemv_geometry(m, n_max, sh, FmtBF16::kElemsPerLane, 64, kMaxLongSlice);
    MultiArgs<FmtBF16> ma{};
    ma.count = count;
    ma.tile_begin[0] = 0;
    for (int k = 0; k < count; ++k) {
        ma.a[k].W = Wt[k];
        ma.a[k].ld = row_pitch ? row_pitch[k] : 0;
        ma.y[k] = y[k];
        ma.t[k] = t[k];
        ma.n[k] = n[k];
        ma.tile_begin[k + 1] = ma.tile_begin[k] + (n[k] + g.tile_cols - 1) / g.tile_cols;
    }
    const int tiles = ma.tile_begin[count];
    const __half *x = static_cast<const __half *>(x_f16);
#define TEAL_LAUNCH(F, LPR, WAVES, U)                                                          \
    do {                                                                                       \
        if (!allow_large_lds(sparse_gemv_multi_kernel<F, LPR, WAVES, U>, g.lds))               \
            return hipErrorInvalidValue;                                                       \
        hipLaunchKernelGGL((sparse_gemv_multi_kernel<F, LPR, WAVES, U>),                       \
                           dim3(tiles * g.splits), dim3(WAVES * 64), g.lds, stream, ma, x,     \
                           partial, counters, m, g.ks, g.tile_cols, g.splits);                 \
    } while (0)
    TEAL_DISPATCH(TEAL_LAUNCH, FmtBF16, sh);
#undef TEAL_LAUNCH
    return hipGetLastError();
}

hipError_t launch_gemv_bf16_stack(int groups, const StackGroupDesc *d, hipStream_t stream)
{
    StackArgs<FmtBF16> sa{};
    size_t lds;
    const hipError_t e = fill_stack_args<FmtBF16>(
        sa, lds, groups, d, 64, 16, 64,
        [](FmtBF16::Args &a, const StackGroupDesc &g, int k) { a.W = g.Wt[k]; });
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((sparse_gemv_stack_kernel<FmtBF16, 8, 4, false>),
                       dim3(sa.block_begin[groups]), dim3(8 * 64), lds, stream, sa);
    return hipGetLastError();
}

hipError_t launch_gemv_bf16_rmsnorm_multi(int count, const void *const *Wt, const int *row_pitch,
                                          const float *t, float *const *y, const int *n,
                                          const float *h,
                                          const float *gamma, float eps, int m, float *partial,
                                          int *counters, const GemvShape &sh, hipStream_t stream)
{
    if (m < 8 || m > kMaxNormDim || m % 8 != 0 || sh.waves != kNormWaves || sh.unroll != 4 ||
        !gemv_shape_supported(sh) || sh.lanes_per_row < 16)
        return hipErrorInvalidValue;
    int n_max = 0;
    for (int k = 0; k < count; ++k) n_max = n[k] > n_max ? n[k] : n_max;
    const GemvGeometry g =
        gemv_geometry(m, n_max, sh, FmtBF16::kElemsPerLane, 64, kMaxLongSlice);
    MultiArgs<FmtBF16> ma{};
    ma.count = count;
    ma.tile_begin[0] = 0;
    for (int k = 0; k < count; ++k) {
        ma.a[k].W = Wt[k];
        ma.a[k].ld = row_pitch ? row_pitch[k] : 0;
        ma.y[k] = y[k];
        ma.t[k] = t[k];
        ma.n[k] = n[k];
        ma.tile_begin[k + 1] = ma.tile_begin[k] + (n[k] + g.tile_cols - 1) / g.tile_cols;
    }
    const int tiles = ma.tile_begin[count];
#define TEAL_LAUNCH_N(LPR)                                                                     \
    do {                                                                                       \
        if (!allow_large_lds(sparse_gemv_rmsnorm_multi_kernel<FmtBF16, LPR, 4>, g.lds))        \
            return hipErrorInvalidValue;                                                       \
        hipLaunchKernelGGL((sparse_gemv_rmsnorm_multi_kernel<FmtBF16, LPR, 4>),                \
                           dim3(tiles * g.splits), dim3(kNormWaves * 64), g.lds, stream, ma,   \
                           h, gamma, eps, partial, counters, m, g.ks, g.tile_cols, g.splits);  \
    } while (0)
    if (sh.lanes_per_row == 64) TEAL_LAUNCH_N(64);
    else if (sh.lanes_per_row == 32) TEAL_LAUNCH_N(32);
    else TEAL_LAUNCH_N(16);
#undef TEAL_LAUNCH_N
    return hipGetLastError();
}

bool mlp_grid_of(int weight_bits, const MlpLaunch &L, int m, int f, int d, MlpGrid &grid)
{
    GemvGeometry ggu, gd;
    const int epl = weight_bits == 16 ? 8 : weight_bits == 8 ? 16 : 32;
    if (weight_bits != 16 && weight_bits != 8 && weight_bits != 4) return false;
    if (!mlp_shape_ok(L.gu, epl) || !mlp_shape_ok(L.down, epl)) return false;
    return mlp_grid(grid, ggu, gd, L, m, f, d, epl, weight_bits == 4 ? 128 : 64,
                    weight_bits == 4 ? kMaxSlice : kMaxLongSlice);
}

hipError_t launch_mlp_bf16(const MlpHostArgs &h, const MlpLaunch &L, hipStream_t stream)
{
    if (!mlp_shape_ok(L.gu, 8) || !mlp_shape_ok(L.down, 8)) return hipErrorInvalidValue;
    MlpArgs<FmtBF16> A{};
    size_t lds;
    if (!fill_mlp_args<FmtBF16>(A, lds, h, L, 64,
                                [](FmtBF16::Args &a, const void *W, const void *, int pitch) {
                                    a.W = W;
                                    a.ld = pitch;
                                }))
        return hipErrorInvalidValue;
    return launch_mlp_kernel<GemvBody<FmtBF16>, false>(A, L.gu.lanes_per_row,
                                                       L.down.lanes_per_row, lds, stream);
}

}  // namespace teal

#ifdef TEAL_TRACE_BLOCKS
// The trace build's read-out (see trace_mark in gemv_common.h): copies the marks of this
// file's kernels to HOST memory after synchronising the device, and clears them.
extern "C" int teal_trace_read(unsigned long long *host, size_t count)
{
    const size_t all = (size_t)teal::kTraceBlocks * teal::kTraceMarks;
    if (!host || count > all) return 1;
    if (hipDeviceSynchronize() != hipSuccess) return 2;
    if (hipMemcpyFromSymbol(host, HIP_SYMBOL(teal::teal_trace),
                            count * sizeof(unsigned long long)) != hipSuccess)
        return 3;
    static unsigned long long zeros[4096];
    for (size_t at = 0; at < all; at += 4096)
        if (hipMemcpyToSymbol(HIP_SYMBOL(teal::teal_trace), zeros, sizeof(zeros),
                              at * sizeof(unsigned long long)) != hipSuccess)
            return 4;
    return 0;
}
#endif
