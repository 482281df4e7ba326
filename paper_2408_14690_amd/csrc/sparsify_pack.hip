// teal_sparsify (Definition 1 as a stand-alone mask / index list) and the
// one-time weight layout step (canonical W[n][m] -> input-channel-major Wt[m][n]).
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "gemv_common.h"
#include "teal_internal.h"

namespace teal {

namespace {

constexpr int kSparsifyWaves = 16;

// One block walks x in chunks of 1024 channels.  Per chunk: each wavefront
// ballots its 64 keep-bits and counts them (popcount); the per-wavefront
// counts go through LDS, where every wavefront reads the prefix below itself;
// a survivor's slot is running base + wavefront prefix + set bits below its lane,
// which keeps the index list ascending.
__global__ __launch_bounds__(kSparsifyWaves * 64) void sparsify_kernel(
    const __half *__restrict__ x, int m, float t, uint8_t *__restrict__ mask,
    int32_t *__restrict__ idx, int32_t *__restrict__ count)
{
    __shared__ int wave_cnt[2][kSparsifyWaves];
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    int base = 0;
    int buf = 0;
    for (int c0 = 0; c0 < m; c0 += kSparsifyWaves * 64, buf ^= 1) {
        const int i = c0 + (int)threadIdx.x;
        bool keep = false;
        if (i < m) {
            keep = fabsf(__half2float(x[i])) > t;
            if (mask) mask[i] = keep ? 1 : 0;
        }
        const unsigned long long b = __ballot(keep);
        if (lane == 0) wave_cnt[buf][w] = __popcll(b);
        __syncthreads();
        int below = 0, total = 0;
#pragma unroll
        for (int ww = 0; ww < kSparsifyWaves; ++ww) {
            const int c = wave_cnt[buf][ww];
            below += ww < w ? c : 0;
            total += c;
        }
        if (keep && idx) {
            const int in_wave = (int)__builtin_amdgcn_mbcnt_hi(
                (unsigned)(b >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)b, 0u));
            idx[base + below + in_wave] = i;
        }
        base += total;
        // wave_cnt is double-buffered: the next chunk writes the other half, and the
        // barrier of that chunk orders it against this chunk's reads.
    }
    if (threadIdx.x == 0 && count) *count = base;
}

// h[i] = fp16(SiLU(gate[i]) * up[i]): the producer of W_down's input on its own
// (Appendix A.3), in the arithmetic the fused kernel uses.
__global__ __launch_bounds__(256) void swiglu_f16_kernel(const float *__restrict__ gate,
                                                         const float *__restrict__ up,
                                                         __half *__restrict__ h, int m)
{
    const int i = (int)(blockIdx.x * 256 + threadIdx.x);
    if (i < m) h[i] = __float2half_rn(swiglu_value(gate[i], up[i]));
}

// x[i] = fp16(gamma[i] * h[i] * r): the normalisation that produces the input of
// W_q/W_k/W_v and W_gate/W_up on its own, in the arithmetic the fused kernel uses.
// Every block computes the scale from all of h and writes its 512 entries.
__global__ __launch_bounds__(kNormWaves * 64) void rmsnorm_f16_kernel(
    const float *__restrict__ h, const float *__restrict__ gamma, float eps,
    __half *__restrict__ x, int m)
{
    __shared__ double wave_sums[kMaxNormChunks * kNormWaves];
    const float r = rms_scale(h, m, eps, wave_sums);
    const int i = (int)(blockIdx.x * (kNormWaves * 64) + threadIdx.x);
    if (i < m) x[i] = __float2half_rn(rmsnorm_value(h[i], gamma[i], r));
}

constexpr int kPackTile = 64;

// 64 x 64 tile transpose through LDS: reads run along m (contiguous in W),
// writes run along n (contiguous in Wt).
__global__ __launch_bounds__(256) void pack_bf16_kernel(const uint16_t *__restrict__ W,
                                                        uint16_t *__restrict__ Wt, int m, int n,
                                                        int tiles_m)
{
    __shared__ uint16_t tile[kPackTile][kPackTile + 2];
    const int i0 = (int)(blockIdx.x % tiles_m) * kPackTile;   // input-channel origin
    const int j0 = (int)(blockIdx.x / tiles_m) * kPackTile;   // output-channel origin
    const int c = threadIdx.x & 63;
    const int r0 = threadIdx.x >> 6;
    for (int r = r0; r < kPackTile; r += 4) {
        const int j = j0 + r, i = i0 + c;
        if (j < n && i < m) tile[r][c] = W[(size_t)j * m + i];
    }
    __syncthreads();
    for (int r = r0; r < kPackTile; r += 4) {
        const int i = i0 + r, j = j0 + c;
        if (i < m && j < n) Wt[(size_t)i * n + j] = tile[c][r];
    }
}

}  // namespace

hipError_t launch_sparsify(const void *x_f16, int m, float t, uint8_t *mask, int32_t *idx,
                           int32_t *count, hipStream_t stream)
{
    hipLaunchKernelGGL(sparsify_kernel, dim3(1), dim3(kSparsifyWaves * 64), 0, stream,
                       static_cast<const __half *>(x_f16), m, t, mask, idx, count);
    return hipGetLastError();
}

hipError_t launch_swiglu_f16(const float *gate, const float *up, void *h_f16, int m,
                             hipStream_t stream)
{
    if (m == 0) return hipSuccess;
    hipLaunchKernelGGL(swiglu_f16_kernel, dim3((unsigned)((m + 255) / 256)), dim3(256), 0, stream,
                       gate, up, static_cast<__half *>(h_f16), m);
    return hipGetLastError();
}

hipError_t launch_rmsnorm_f16(const float *h, const float *gamma, float eps, void *x_f16, int m,
                              hipStream_t stream)
{
    if (m < 8 || m > kMaxNormDim || m % 8 != 0) return hipErrorInvalidValue;
    const int threads = kNormWaves * 64;
    hipLaunchKernelGGL(rmsnorm_f16_kernel, dim3((unsigned)((m + threads - 1) / threads)),
                       dim3(threads), 0, stream, h, gamma, eps, static_cast<__half *>(x_f16), m);
    return hipGetLastError();
}

hipError_t launch_pack_bf16(const void *W_rowmajor, void *Wt, int m, int n, hipStream_t stream)
{
    const int tiles_m = (m + kPackTile - 1) / kPackTile;
    const int tiles_n = (n + kPackTile - 1) / kPackTile;
    hipLaunchKernelGGL(pack_bf16_kernel, dim3((unsigned)tiles_m * (unsigned)tiles_n), dim3(256), 0,
                       stream, static_cast<const uint16_t *>(W_rowmajor),
                       static_cast<uint16_t *>(Wt), m, n, tiles_m);
    return hipGetLastError();
}

}  // namespace teal
