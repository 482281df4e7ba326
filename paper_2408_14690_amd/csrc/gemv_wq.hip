// y = s_t(x) W^T for weight-quantised W (Section 5.3 names the formats; a kernel
// that is both sparse and quantised is what that section leaves open).
//   int8: W[j][i] = q[i][j] * scale[j]            (channel-wise)
//   int4: W[j][i] = nibble(i, j) * scale[i/128][j] (groups of 128 input channels)
// Dequantisation happens in registers; only surviving rows are read.
#include "gemv_common.h"
#include "gemv_dispatch.h"

namespace teal {

struct FmtW8 {
    static constexpr int kElemsPerLane = 16;   // 16 bytes = 16 int8
    static constexpr int kBitsPerElem = 8;
    struct Args {
        const void *W;
        const __half *scale;
    };
    static __device__ __forceinline__ void fma(float (&acc)[16], u32x4 v, float xv)
    {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int wq = (int)(v[q] << (24 - 8 * b)) >> 24;   // sign-extend byte b
                acc[4 * q + b] = fmaf(xv, (float)wq, acc[4 * q + b]);
            }
        }
    }
    // The per-output-channel scale factors out of the sum over input channels.
    static __device__ __forceinline__ float finish(float sum, const Args &a, int col)
    {
        return sum * __half2float(a.scale[col]);
    }
};

struct FmtW4 {
    static constexpr int kElemsPerLane = 32;   // 16 bytes = 32 nibbles
    static constexpr int kBitsPerElem = 4;
    struct Args {
        const void *W;
        const __half *scale;
    };
    // Converting a nibble to fp32 the plain way costs two instructions per element.
    // Instead: q + 8 (the nibble with its top bit flipped) is placed in the top four
    // mantissa bits of an fp16 1.0, two nibbles per 32-bit operation, which gives
    // v = 1 + (q + 8) / 16 in [1, 2), i.e. q = 16 (v - 1.5).  The FMA then reads the
    // fp16 halves directly, and the affine map is undone once per group from
    // sum x*v and sum x (both exact products, fp32 sums).
    static constexpr float kAffineScale = 16.f;    // q = kAffineScale * (v - kAffineOffset)
    static constexpr float kAffineOffset = 1.5f;
    static __device__ __forceinline__ void fma(float (&acc)[32], u32x4 v, float xv)
    {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t d = v[q] ^ 0x88888888u;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                // nibble k -> bits 6..9, nibble k + 4 -> bits 22..25
                const uint32_t sh = k == 0 ? d << 6 : k == 1 ? d << 2 : k == 2 ? d >> 2 : d >> 6;
                const uint32_t pair = (sh & 0x03C003C0u) | 0x3C003C00u;
                const __half2 h = *reinterpret_cast<const __half2 *>(&pair);
                acc[8 * q + k] = fmaf(__low2float(h), xv, acc[8 * q + k]);
                acc[8 * q + k + 4] = fmaf(__high2float(h), xv, acc[8 * q + k + 4]);
            }
        }
    }
    static __device__ __forceinline__ float finish(float sum, const Args &, int) { return sum; }
};

constexpr int kGroup = 128;

// One 128-channel group's worth of work of one wavefront: its share of the
// group's surviving rows (at most 128 / WAVES of them, LOADS wavefront loads)
// and the group's scales for this lane's 32 columns.
template <int LOADS>
struct GroupBatch {
    u32x4 v[LOADS];
    float xv[LOADS];
    uint4 sc[4];      // 32 fp16 scales
    int mine;         // rows in this batch (wavefront-uniform)
};

// int4: the compacted list is ascending, so each 128-channel group is a run
// of it, delimited by the segment prefixes (two 64-channel segments per group).
// Per group the block's wavefronts split the run, accumulate sum_i x_i q[i][j]
// unscaled, then fold it into the running sums with that group's scales.
// Groups are software-pipelined: the rows and scales of the next group are in
// flight while the current one is multiplied out.
template <int LPR, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void sparse_gemv_w4_kernel(
    FmtW4::Args a, const __half *__restrict__ x, float t, float *partial, int *counters, float *y,
    int m, int n, int ks, int tiles, int tile_cols, int splits)
{
    using F = FmtW4;
    constexpr int EPL = F::kElemsPerLane;
    constexpr int R = 64 / LPR;
    constexpr int LOADS = (kGroup / WAVES + R - 1) / R;   // covers a group in which every row survives
    extern __shared__ __align__(16) unsigned char smem[];
    int2 *list = reinterpret_cast<int2 *>(smem);
    float *red = reinterpret_cast<float *>(smem + (size_t)ks * sizeof(int2));
    __shared__ int seg_cnt[kMaxSegs];

    const int tile = blockIdx.x % tiles;
    const int s = blockIdx.x / tiles;
    const int k0 = s * ks;                       // multiple of 128
    const int k1 = min(m, k0 + ks);
    int seg_excl;
    const int cnt = compact_slice<WAVES>(x, t, k0, k1, list, seg_cnt, seg_excl);

    const int lane = threadIdx.x & 63;
    const int g = lane / LPR;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col0 = tile * tile_cols;
    const int col = lane_column<EPL>(col0, tile_cols, n, lane % LPR);
    const unsigned row_bytes = (unsigned)(n / 2);
    const unsigned char *lane_base = static_cast<const unsigned char *>(a.W) + col / 2;
    const __half *scale_base = a.scale + (size_t)(k0 / kGroup) * n + col;

    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;

    auto issue = [&](GroupBatch<LOADS> &b, int gi) {
        // two 64-channel segments per group; the prefix of segment j sits in lane j
        const int g0 = __builtin_amdgcn_readlane(seg_excl, 2 * gi);
        const int g1 = 2 * gi + 2 < 64 ? __builtin_amdgcn_readlane(seg_excl, 2 * gi + 2) : cnt;
        int start, mine;
        wave_share(g1 - g0, w, WAVES, start, mine);
        b.mine = mine;
        if (mine <= 0) return;                    // wavefront-uniform
        const int last = mine - 1;
#pragma unroll
        for (int u = 0; u < LOADS; ++u) {
            const int e = u * R + g;
            const int2 ent = list[g0 + start + min(e, last)];
            b.xv[u] = e <= last ? __int_as_float(ent.y) : 0.f;
            b.v[u] = load_stream16(lane_base + (size_t)(unsigned)ent.x * row_bytes);
        }
        const uint4 *sp = reinterpret_cast<const uint4 *>(scale_base + (size_t)gi * n);
#pragma unroll
        for (int q = 0; q < 4; ++q) b.sc[q] = sp[q];
    };
    auto consume = [&](const GroupBatch<LOADS> &b) {
        if (b.mine <= 0) return;
        float gacc[EPL];
#pragma unroll
        for (int e = 0; e < EPL; ++e) gacc[e] = 0.f;
        float xsum = 0.f;                         // sum of x over this lane's rows of the group
#pragma unroll
        for (int u = 0; u < LOADS; ++u) {
            if (u * R < b.mine) {                 // wavefront-uniform
                F::fma(gacc, b.v[u], b.xv[u]);
                xsum += b.xv[u];
            }
        }
        // sum x*q = 16 (sum x*v - 1.5 sum x); then times the group's scale
        const float corr = -F::kAffineScale * F::kAffineOffset * xsum;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const unsigned sw[4] = {b.sc[q].x, b.sc[q].y, b.sc[q].z, b.sc[q].w};
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                const __half2 sh = *reinterpret_cast<const __half2 *>(&sw[h]);
                const float q0 = fmaf(gacc[8 * q + 2 * h], F::kAffineScale, corr);
                const float q1 = fmaf(gacc[8 * q + 2 * h + 1], F::kAffineScale, corr);
                acc[8 * q + 2 * h] = fmaf(__low2float(sh), q0, acc[8 * q + 2 * h]);
                acc[8 * q + 2 * h + 1] = fmaf(__high2float(sh), q1, acc[8 * q + 2 * h + 1]);
            }
        }
    };

    const int ngroups = (k1 - k0) / kGroup;       // >= 1
    GroupBatch<LOADS> b0, b1;
    issue(b0, 0);
    int gi = 0;
    for (; gi + 2 < ngroups; gi += 2) {
        issue(b1, gi + 1);
        consume(b0);
        issue(b0, gi + 2);
        consume(b1);
    }
    if (gi + 1 < ngroups) {
        issue(b1, gi + 1);
        consume(b0);
        consume(b1);
    } else {
        consume(b0);
    }
    fold_row_groups<LPR>(acc);
    block_finish<F, LPR, WAVES>(acc, red, partial, counters, y, tile, col0, tile_cols, s, splits, n,
                                a);
}

hipError_t launch_gemv_w8(const int8_t *Wq, const void *scale_f16, const void *x_f16, float t,
                          float *y, int m, int n, float *partial, int *counters,
                          const GemvShape &sh, hipStream_t stream)
{
    const GemvGeometry g = gemv_geometry(m, n, sh, FmtW8::kElemsPerLane, 64);
    FmtW8::Args a{Wq, static_cast<const __half *>(scale_f16)};
    const __half *x = static_cast<const __half *>(x_f16);
#define TEAL_LAUNCH(F, LPR, WAVES, U)                                                          \
    hipLaunchKernelGGL((sparse_gemv_kernel<F, LPR, WAVES, U>), dim3(g.tiles * g.splits), \
                       dim3(WAVES * 64), g.lds, stream, a, x, t, partial, counters, y, m, n,   \
                       g.ks, g.tiles, g.tile_cols, g.splits)
    TEAL_DISPATCH(TEAL_LAUNCH, FmtW8, sh);
#undef TEAL_LAUNCH
    return hipGetLastError();
}

hipError_t launch_gemv_w8_multi(int count, const int8_t *const *Wq, const void *const *scale_f16,
                                const float *t, float *const *y, const int *n, const void *x_f16,
                                int m, float *partial, int *counters, const GemvShape &sh,
                                hipStream_t stream)
{
    int n_max = 0;
    for (int k = 0; k < count; ++k) n_max = n[k] > n_max ? n[k] : n_max;
    // slice length, split count and LDS size do not depend on n
    const GemvGeometry g = gemv_geometry(m, n_max, sh, FmtW8::kElemsPerLane, 64);
    MultiArgs<FmtW8> ma{};
    ma.count = count;
    ma.tile_begin[0] = 0;
    for (int k = 0; k < count; ++k) {
        ma.a[k].W = Wq[k];
        ma.a[k].scale = static_cast<const __half *>(scale_f16[k]);
        ma.y[k] = y[k];
        ma.t[k] = t[k];
        ma.n[k] = n[k];
        ma.tile_begin[k + 1] = ma.tile_begin[k] + (n[k] + g.tile_cols - 1) / g.tile_cols;
    }
    const int tiles = ma.tile_begin[count];
    const __half *x = static_cast<const __half *>(x_f16);
#define TEAL_LAUNCH(F, LPR, WAVES, U)                                                          \
    hipLaunchKernelGGL((sparse_gemv_multi_kernel<F, LPR, WAVES, U>), dim3(tiles * g.splits),   \
                       dim3(WAVES * 64), g.lds, stream, ma, x, partial, counters, m, g.ks,     \
                       g.tile_cols, g.splits)
    TEAL_DISPATCH(TEAL_LAUNCH, FmtW8, sh);
#undef TEAL_LAUNCH
    return hipGetLastError();
}

hipError_t launch_gemv_w4(const uint8_t *Wq, const void *scale_f16, const void *x_f16, float t,
                          float *y, int m, int n, float *partial, int *counters,
                          const GemvShape &sh, hipStream_t stream)
{
    GemvShape w4 = sh;
    w4.waves = 8;                                 // the int4 kernel is built for 8 wavefronts
    const GemvGeometry g = gemv_geometry(m, n, w4, FmtW4::kElemsPerLane, kGroup);
    FmtW4::Args a{Wq, static_cast<const __half *>(scale_f16)};
    const __half *x = static_cast<const __half *>(x_f16);
#define TEAL_LAUNCH_W4(LPR, WAVES)                                                             \
    hipLaunchKernelGGL((sparse_gemv_w4_kernel<LPR, WAVES>), dim3(g.tiles * g.splits),           \
                       dim3(WAVES * 64), g.lds, stream, a, x, t, partial, counters, y, m, n,   \
                       g.ks, g.tiles, g.tile_cols, g.splits)
    // A lane covers 32 columns: 16 lanes per row (tiles up to 512 columns) or 32 lanes
    // per row (up to 1024 columns).
    if (sh.lanes_per_row == 32) TEAL_LAUNCH_W4(32, 8);
    else TEAL_LAUNCH_W4(16, 8);
#undef TEAL_LAUNCH_W4
    return hipGetLastError();
}

}  // namespace teal