// y = s_t(x) W^T for bf16 weights stored input-channel-major (Sections 3, 4.2, 4.4).
#include "gemv_common.h"
#include "gemv_dispatch.h"

namespace teal {

struct FmtBF16 {
    static constexpr int kElemsPerLane = 8;   // 16 bytes = 8 bf16
    static constexpr int kBitsPerElem = 16;
    struct Args {
        const void *W;
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
    static __device__ __forceinline__ float finish(float sum, const Args &, int) { return sum; }
};

bool gemv_shape_supported(const GemvShape &s)
{
    const bool lpr = s.lanes_per_row == 64 || s.lanes_per_row == 32 || s.lanes_per_row == 16 ||
                     s.lanes_per_row == 8;
    const bool wv = s.waves == 4 || s.waves == 8 || s.waves == 16;
    const bool un = s.unroll == 4 || (s.unroll == 8 && s.waves != 16);
    const bool tc = s.tile_cols >= 0 && s.tile_cols % 8 == 0 && s.tile_cols <= s.lanes_per_row * 8;
    return lpr && wv && un && tc && s.splits >= 1 && s.splits <= kMaxSplits;
}

hipError_t launch_gemv_bf16(const void *Wt, const void *x_f16, float t, float *y, int m, int n,
                            float *partial, int *counters, const GemvShape &sh,
                            hipStream_t stream)
{
    const GemvGeometry g = gemv_geometry(m, n, sh, FmtBF16::kElemsPerLane, 64);
    FmtBF16::Args a{Wt};
    const __half *x = static_cast<const __half *>(x_f16);
#define TEAL_LAUNCH(F, LPR, WAVES, U)                                                          \
    hipLaunchKernelGGL((sparse_gemv_kernel<F, LPR, WAVES, U>), dim3(g.tiles * g.splits), \
                       dim3(WAVES * 64), g.lds, stream, a, x, t, partial, counters, y, m, n,   \
                       g.ks, g.tiles, g.tile_cols, g.splits)
    TEAL_DISPATCH(TEAL_LAUNCH, FmtBF16, sh);
#undef TEAL_LAUNCH
    return hipGetLastError();
}

}  // namespace teal
