// teal_sparsify (Definition 1 as a stand-alone mask / index list) and the
// one-time weight layout step (canonical W[n][m] -> input-channel-major Wt[m][n]).
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "gemv_common.h"
#include "teal_internal.h"

namespace teal {

namespace {

constexpr int kSparsifyWaves = 16;
constexpr int kSparsifyChunk = kSparsifyWaves * 64;   // channels one pass of the block covers

// One block walks x in groups of G chunks of 1024 channels; the loads of a group are
// issued together, and G is chosen so that a vector of decode size (up to 32768 channels)
// is one group: the kernel then costs one memory round trip, and no load waits behind
// the stores of an earlier group.  Per chunk each wavefront ballots
// its 64 keep-bits and counts them (popcount); the counts of the group go through LDS,
// where every wavefront reads the prefix below itself; a survivor's slot is running base
// + prefix of the chunks and wavefronts before it + set bits below its lane, which keeps
// the index list ascending.
template <int kSparsifyGroup>
__global__ __launch_bounds__(kSparsifyChunk) void sparsify_kernel(
    const __half *__restrict__ x, int m, float t, uint8_t *__restrict__ mask,
    int32_t *__restrict__ idx, int32_t *__restrict__ count)
{
    __shared__ int wave_cnt[2][kSparsifyGroup][kSparsifyWaves];
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    int base = 0;
    int buf = 0;
    for (int c0 = 0; c0 < m; c0 += kSparsifyGroup * kSparsifyChunk, buf ^= 1) {
        __half raw[kSparsifyGroup];
#pragma unroll
        for (int j = 0; j < kSparsifyGroup; ++j)      // unconditional, from a clamped position
            raw[j] = x[min(c0 + j * kSparsifyChunk + (int)threadIdx.x, m - 1)];
        unsigned long long bal[kSparsifyGroup];
#pragma unroll
        for (int j = 0; j < kSparsifyGroup; ++j) {
            const int i = c0 + j * kSparsifyChunk + (int)threadIdx.x;
            const bool keep = i < m && fabsf(__half2float(raw[j])) > t;
            if (i < m && mask) mask[i] = keep ? 1 : 0;
            bal[j] = __ballot(keep);
            if (lane == 0) wave_cnt[buf][j][w] = __popcll(bal[j]);
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < kSparsifyGroup; ++j) {
            if (c0 + j * kSparsifyChunk < m) {        // block-uniform
                int below = 0, total = 0;
#pragma unroll
                for (int ww = 0; ww < kSparsifyWaves; ++ww) {
                    const int c = wave_cnt[buf][j][ww];
                    below += ww < w ? c : 0;
                    total += c;
                }
                if (idx && ((bal[j] >> lane) & 1ull))
                    idx[base + below + lanes_below(bal[j])] =
                        c0 + j * kSparsifyChunk + (int)threadIdx.x;
                base += total;
            }
        }
        // wave_cnt is double-buffered: the next group writes the other half, and the
        // barrier of that group orders it against this group's reads.
    }
    if (threadIdx.x == 0 && count) *count = base;
}

// The same result with eight channels per thread (one 16-byte load), for x on a 16-byte
// boundary: a pass of the block covers 8192 channels, P passes are in flight together, and
// the per-channel work of the kernel above (LDS prefix, one store per channel) is shared by
// eight channels.  A thread counts its survivors, the block scans the 1024 counts (lanes by
// data-parallel shifts, wavefronts through LDS), and the thread writes its survivors'
// positions to consecutive slots.  The last m % 8 channels are read one by one by the
// thread that owns them.
constexpr int kVecChannels = 8;
constexpr int kVecPass = kSparsifyChunk * kVecChannels;

template <int P>
__global__ __launch_bounds__(kSparsifyChunk) void sparsify_vec_kernel(
    const __half *__restrict__ x, int m, float t, uint8_t *__restrict__ mask, bool mask_aligned,
    int32_t *__restrict__ idx, int32_t *__restrict__ count)
{
    __shared__ int wave_tot[2][P][kSparsifyWaves];
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int m_vec = m & ~(kVecChannels - 1);          // >= 8: the launcher sees to it
    int base = 0;
    int buf = 0;
    for (int c0 = 0; c0 < m; c0 += P * kVecPass, buf ^= 1) {
        uint4 raw[P];
#pragma unroll
        for (int p = 0; p < P; ++p) {                   // unconditional, from a clamped position
            const int i0 = c0 + (p * kSparsifyChunk + (int)threadIdx.x) * kVecChannels;
            raw[p] = *reinterpret_cast<const uint4 *>(x + min(i0, m_vec - kVecChannels));
        }
        unsigned bits[P];
        int cnt[P], incl[P];
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int i0 = c0 + (p * kSparsifyChunk + (int)threadIdx.x) * kVecChannels;
            const unsigned wd[4] = {raw[p].x, raw[p].y, raw[p].z, raw[p].w};
            unsigned b = 0;
            if (i0 < m_vec) {
#pragma unroll
                for (int e = 0; e < kVecChannels; ++e) {
                    const unsigned short h = (unsigned short)(wd[e >> 1] >> (16 * (e & 1)));
                    const float v = __half2float(__ushort_as_half(h));
                    b |= (fabsf(v) > t ? 1u : 0u) << e;
                }
            } else if (i0 < m) {                        // the ragged end: at most 7 channels
                for (int e = 0; i0 + e < m; ++e)
                    b |= (fabsf(__half2float(x[i0 + e])) > t ? 1u : 0u) << e;
            }
            bits[p] = b;
            cnt[p] = __popc(b);
            incl[p] = wave_inclusive_scan(cnt[p]);
            if (lane == 63) wave_tot[buf][p][w] = incl[p];
            if (mask && i0 < m) {
                if (mask_aligned && i0 + kVecChannels <= m) {
                    // byte e = bit e: spread the 8 bits over 8 bytes
                    const unsigned lo = b & 0xFu, hi = (b >> 4) & 0xFu;
                    uint2 mv;
                    mv.x = (lo & 1u) | ((lo & 2u) << 7) | ((lo & 4u) << 14) | ((lo & 8u) << 21);
                    mv.y = (hi & 1u) | ((hi & 2u) << 7) | ((hi & 4u) << 14) | ((hi & 8u) << 21);
                    *reinterpret_cast<uint2 *>(mask + i0) = mv;
                } else {
                    for (int e = 0; e < kVecChannels && i0 + e < m; ++e)
                        mask[i0 + e] = (uint8_t)((b >> e) & 1u);
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int p = 0; p < P; ++p) {
            if (c0 + p * kVecPass < m) {                // block-uniform
                int below = 0, total = 0;
#pragma unroll
                for (int ww = 0; ww < kSparsifyWaves; ++ww) {
                    const int c = wave_tot[buf][p][ww];
                    below += ww < w ? c : 0;
                    total += c;
                }
                if (idx) {
                    const int i0 = c0 + (p * kSparsifyChunk + (int)threadIdx.x) * kVecChannels;
                    int o = base + below + incl[p] - cnt[p];
#pragma unroll
                    for (int e = 0; e < kVecChannels; ++e)
                        if ((bits[p] >> e) & 1u) idx[o++] = i0 + e;
                }
                base += total;
            }
        }
        // wave_tot is double-buffered like wave_cnt above.
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
                                                        int pitch, int tiles_m)
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
        if (i < m && j < n) Wt[(size_t)i * pitch + j] = tile[c][r];
    }
}

}  // namespace

hipError_t launch_sparsify(const void *x_f16, int m, float t, uint8_t *mask, int32_t *idx,
                           int32_t *count, hipStream_t stream)
{
    const __half *x = static_cast<const __half *>(x_f16);
    if (m >= kVecChannels && (reinterpret_cast<uintptr_t>(x_f16) & 15) == 0) {
        const bool mask_aligned = (reinterpret_cast<uintptr_t>(mask) & 7) == 0;
        const int passes = (m + kVecPass - 1) / kVecPass;
#define TEAL_LAUNCH_V(P)                                                                        \
    hipLaunchKernelGGL(sparsify_vec_kernel<P>, dim3(1), dim3(kSparsifyChunk), 0, stream, x, m,  \
                       t, mask, mask_aligned, idx, count)
        if (passes <= 1) TEAL_LAUNCH_V(1);
        else if (passes <= 2) TEAL_LAUNCH_V(2);
        else TEAL_LAUNCH_V(4);
#undef TEAL_LAUNCH_V
        return hipGetLastError();
    }
    const int chunks = (m + kSparsifyChunk - 1) / kSparsifyChunk;
#define TEAL_LAUNCH_S(G)                                                                        \
    hipLaunchKernelGGL(sparsify_kernel<G>, dim3(1), dim3(kSparsifyChunk), 0, stream, x, m, t,   \
                       mask, idx, count)
    if (chunks <= 4) TEAL_LAUNCH_S(4);
    else if (chunks <= 8) TEAL_LAUNCH_S(8);
    else if (chunks <= 16) TEAL_LAUNCH_S(16);
    else TEAL_LAUNCH_S(32);
#undef TEAL_LAUNCH_S
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

hipError_t launch_pack_bf16(const void *W_rowmajor, void *Wt, int m, int n, int pitch,
                            hipStream_t stream)
{
    const int tiles_m = (m + kPackTile - 1) / kPackTile;
    const int tiles_n = (n + kPackTile - 1) / kPackTile;
    hipLaunchKernelGGL(pack_bf16_kernel, dim3((unsigned)tiles_m * (unsigned)tiles_n), dim3(256), 0,
                       stream, static_cast<const uint16_t *>(W_rowmajor),
                       static_cast<uint16_t *>(Wt), m, n, pitch, tiles_m);
    return hipGetLastError();
}

// Measurement aid: a plain streaming read of `vecs` 16-byte vectors with the loads the
// row stream uses (non-temporal, 8 in flight per thread), no arithmetic beyond an XOR fold
// that keeps the loads alive.  What this reaches is the rate a kernel that only reads can
// reach on the part, for the size of one launch: the practical ceiling under the 8 TB/s
// peak.  A thread writes one word, and only if its fold equals a value the caller chose.
typedef uint32_t probe_u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(512) void stream_read_kernel(const probe_u32x4 *__restrict__ p,
                                                          size_t vecs, uint32_t match,
                                                          uint32_t *sink)
{
    constexpr int L = 8;
    const size_t threads = (size_t)gridDim.x * blockDim.x;
    size_t v = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    probe_u32x4 acc = {0u, 0u, 0u, 0u};
    for (; v + (L - 1) * threads < vecs; v += L * threads) {
        probe_u32x4 d[L];
#pragma unroll
        for (int u = 0; u < L; ++u) d[u] = __builtin_nontemporal_load(p + v + u * threads);
#pragma unroll
        for (int u = 0; u < L; ++u) acc ^= d[u];
    }
    for (; v < vecs; v += threads) acc ^= __builtin_nontemporal_load(p + v);
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == match) sink[blockIdx.x] = match;
}

hipError_t launch_stream_read(const void *buf, size_t bytes, int blocks, uint32_t match,
                              uint32_t *sink, hipStream_t stream)
{
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)blocks), dim3(512), 0, stream,
                       static_cast<const probe_u32x4 *>(buf), bytes / 16, match, sink);
    return hipGetLastError();
}

}  // namespace teal
