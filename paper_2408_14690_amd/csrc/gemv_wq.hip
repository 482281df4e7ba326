// y = s_t(x) W^T for weight-quantised W (Section 5.3 names the formats; a kernel
// that is both sparse and quantised is what that section leaves open).
//   int8: W[j][i] = q[i][j] * scale[j]            (channel-wise)
//   int4: W[j][i] = nibble(i, j) * scale[i/128][j] (groups of 128 input channels)
// Dequantisation happens in registers; only surviving rows are read.
#include "gemv_common.h"
#include "gemv_dispatch.h"
#include "gemv_mlp.h"

namespace teal {

struct FmtW8 {
    static constexpr int kElemsPerLane = 16;   // 16 bytes = 16 int8
    static constexpr int kBitsPerElem = 8;
    struct Args {
        const void *W;
        const __half *scale;
        int ld = 0;             // elements from one row of W to the next; 0 = n
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
    typedef __half ColumnScale;
    static __device__ __forceinline__ ColumnScale column_scale(const Args &a, int col)
    {
        return a.scale[col];
    }
    static __device__ __forceinline__ float finish(float sum, ColumnScale sc)
    {
        return sum * __half2float(sc);
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
    // Instead: q + 8 (the nibble with its top bit flipped) is left where it lies and read
    // as an fp16 subnormal: a nibble in bits 0..3 of a 16-bit half is the value
    // (q + 8) 2^-24, in bits 4..7 it is (q + 8) 2^-20 (no implicit one, so no offset
    // that would cost accumulator precision).  One AND isolates two nibbles (one per
    // half), one shift by 8 serves the upper two nibbles of each half, and the FMA reads
    // the fp16 halves directly: 14 vector instructions per 8 weights.  The scaling by
    // 2^24 / 2^20 and the offset 8 are undone once per group from sum x*v and sum x
    // (exact products, fp32 sums).  Relies on fp16 subnormals being honoured by the
    // mixed-precision FMA (they are in the default floating-point mode).  (Pairing two
    // rows per fp16 dot-product instruction saves another 1 % of the step time, but that
    // instruction's sum is less accurate: 5e-5 relative on a dense 14336-channel input.)
    static constexpr float kScaleEven = 16777216.f;   // 2^24: columns 0, 2 of each group of 4
    static constexpr float kScaleOdd = 1048576.f;     // 2^20: columns 1, 3
    static constexpr float kOffset = 8.f;             // q = scale * v - kOffset
    static __device__ __forceinline__ void fma(float (&acc)[32], u32x4 v, float xv)
    {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t d = v[q] ^ 0x88888888u;
            const uint32_t d8 = d >> 8;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                // nibble k in the low half, nibble k + 4 in the high half
                const uint32_t pair = (k < 2 ? d : d8) & ((k & 1) ? 0x00F000F0u : 0x000F000Fu);
                const __half2 h = *reinterpret_cast<const __half2 *>(&pair);
                acc[8 * q + k] = fmaf(__low2float(h), xv, acc[8 * q + k]);
                acc[8 * q + k + 4] = fmaf(__high2float(h), xv, acc[8 * q + k + 4]);
            }
        }
    }
    struct ColumnScale {};
    static __device__ __forceinline__ ColumnScale column_scale(const Args &, int) { return {}; }
    static __device__ __forceinline__ float finish(float sum, ColumnScale) { return sum; }
};

constexpr int kGroup = 128;
constexpr int kW4Waves = 8;
constexpr int kW4Unroll = 4;

// One batch of row loads of the int4 kernel: up to U wavefront loads, all from
// one 128-channel group, and, if the batch is the wavefront's last of that
// group, the group's scales for this lane's 32 columns.
template <int U>
struct W4Batch {
    u32x4 v[U];
    float xv[U];
    uint4 sc[4];      // 32 fp16 scales (loaded only when ends_run)
    int rows;         // live rows in this batch (wavefront-uniform); 0 = the share is exhausted
    bool ends_run;    // wavefront-uniform
};

// Work of one block for int4 weights with group scales: output tile `tile`
// (tile_cols columns) x K-slice `s` (ks channels, a multiple of 128).
//
// The wavefronts take equal contiguous shares of the compacted list, as for
// the other formats.  The list is ascending, so each 128-channel group is a
// run of it, delimited by the segment prefixes (two 64-channel segments per
// group), and a wavefront's share crosses few group boundaries.  Within a group
// a wavefront accumulates sum_i x_i v[i][j] unscaled (v = the offset nibble
// read as a tiny fp16, see FmtW4); at the end of its rows of that group it undoes the
// affine map and folds the sums into the running sums with the group's scales:
// once per (wavefront, group it touches), not once per row.  Batches never
// straddle a group, and two batches are in flight per wavefront across group
// boundaries.
// Returns (block-uniform) whether this block wrote the tile's outputs.
template <int LPR, int WAVES, int U, class XS>
__device__ __forceinline__ bool w4_block(const FmtW4::Args &a, const XS &x,
                                         float t, float *partial, int *counters, float *y, int m,
                                         int n, int ks, int tile, int s, int tile_cols, int splits,
                                         const SurvivorReport &report)
{
    using F = FmtW4;
    constexpr int EPL = F::kElemsPerLane;
    constexpr int R = 64 / LPR;
    extern __shared__ __align__(16) unsigned char smem[];
    int2 *list = reinterpret_cast<int2 *>(smem);
    float *red = reinterpret_cast<float *>(smem + (size_t)ks * sizeof(int2));
    __shared__ int seg_cnt[kMaxSegs];

    const int k0 = s * ks;                       // multiple of 128
    const int k1 = min(m, k0 + ks);
    int seg_excl;
    int cnt;
    if constexpr (XS::kPlainHalf) {
        if (k1 - k0 <= 8 * 64)         // block-uniform: short slices need no barrier
            cnt = compact_slice_private<8, WAVES>(x.x, t, k0, k1, list, seg_excl);
        else
            cnt = compact_slice<WAVES>(x, t, k0, k1, list, seg_cnt, seg_excl);
    } else {
        cnt = compact_slice<WAVES>(x, t, k0, k1, list, seg_cnt, seg_excl);
    }

    trace_mark(2);
    const int lane = threadIdx.x & 63;
    const int g = lane / LPR;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col0 = tile * tile_cols;
    const int col = lane_column<EPL>(col0, tile_cols, n, lane % LPR);
    const unsigned row_bytes = (unsigned)(n / 2);
    const unsigned char *lane_base = static_cast<const unsigned char *>(a.W) + col / 2;
    const __half *scale_base = a.scale + (size_t)(k0 / kGroup) * n + col;

    float acc[EPL], gacc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = gacc[e] = 0.f;
    float xsum = 0.f;                             // sum of x over this lane's rows of the current run

    int start, mine;
    wave_share(cnt, w, WAVES, start, mine);
    // Walk state (all wavefront-uniform): next list position, end of the share, current
    // group of the slice and the end of this wavefront's rows in it.
    // list offset at which group j of the slice begins: the prefix of segment 2j (lanes past
    // the last segment hold the total)
    auto group_begin = [&](int j) {
        return 2 * j < 64 ? __builtin_amdgcn_readlane(seg_excl, 2 * j) : cnt;
    };
    int cur = start;
    const int end = start + mine;
    int gi = 0, gend = min(end, group_begin(1));

    // Every call issues exactly U row loads and the four scale loads of the batch's group,
    // whether or not rows are left: the compiler then knows how many loads are outstanding at
    // every wait and waits for a batch's own loads only.  (With a conditional scale load and an
    // early return for an exhausted share it waited for older loads between the loads of a
    // batch, and little more than one batch was ever in flight.)  A batch past the end of the
    // share re-reads the share's last row with zero multipliers.
    auto issue = [&](W4Batch<U> &b) {
        const bool live = cur < end;                  // wavefront-uniform
        if (live) {
            while (cur >= gend) {                     // next group with rows in this share
                ++gi;
                gend = min(end, group_begin(gi + 1));
            }
        }
        const int nb = live ? min(U * R, gend - cur) : 0;
        const int last = live ? cur + nb - 1 : end - 1;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = cur + u * R + g;
            const int2 ent = list[min(e, last)];
            b.xv[u] = (live && e <= last) ? __int_as_float(ent.y) : 0.f;
            b.v[u] = load_stream16(lane_base + (size_t)(unsigned)ent.x * row_bytes);
        }
        b.rows = nb;
        b.ends_run = live && cur + nb == gend;
        const uint4 *sp = reinterpret_cast<const uint4 *>(scale_base + (size_t)gi * n);
#pragma unroll
        for (int q = 0; q < 4; ++q) b.sc[q] = sp[q];
        cur += nb;
    };
    auto consume = [&](const W4Batch<U> &b) {
#pragma unroll
        for (int u = 0; u < U; ++u) {             // slots past the end of a run multiply by zero
            F::fma(gacc, b.v[u], b.xv[u]);
            xsum += b.xv[u];
        }
        if (!b.ends_run) return;
        // sum x*q = scale * sum x*v - 8 sum x; then times the group's scale
        const float corr = -F::kOffset * xsum;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const unsigned sw[4] = {b.sc[q].x, b.sc[q].y, b.sc[q].z, b.sc[q].w};
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                const __half2 sh = *reinterpret_cast<const __half2 *>(&sw[h]);
                const float q0 = fmaf(gacc[8 * q + 2 * h], F::kScaleEven, corr);
                const float q1 = fmaf(gacc[8 * q + 2 * h + 1], F::kScaleOdd, corr);
                acc[8 * q + 2 * h] = fmaf(__low2float(sh), q0, acc[8 * q + 2 * h]);
                acc[8 * q + 2 * h + 1] = fmaf(__high2float(sh), q1, acc[8 * q + 2 * h + 1]);
                gacc[8 * q + 2 * h] = 0.f;
                gacc[8 * q + 2 * h + 1] = 0.f;
            }
        }
        xsum = 0.f;
    };

    // Two batches in flight.  The fences keep the compiler from sinking a batch's loads into
    // the consumption of the batch before it.  (A third batch in flight was measured slower:
    // the row stream of this format is held back by its vector instructions, about 2.2 per
    // weight with the addressing, issued by two wavefronts per SIMD -- the older of the two
    // finishes its share 4-5 us before the younger -- not by the loads in flight.)
    if (mine > 0) {                               // wavefront-uniform
        W4Batch<U> b0, b1;
        issue(b0);
        while (b0.rows > 0) {
            issue(b1);
            __builtin_amdgcn_sched_barrier(0);
            consume(b0);
            __builtin_amdgcn_sched_barrier(0);
            if (b1.rows <= 0) break;
            issue(b0);
            __builtin_amdgcn_sched_barrier(0);
            consume(b1);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    trace_mark(3);
    trace_mark_thread(1, (WAVES - 1) * 64);
    store_wave_sums<LPR>(acc, red + (threadIdx.x >> 6) * combine_row<EPL, LPR>);
    return block_finish<F, LPR, WAVES>(red, partial, counters, y, tile, col0, tile_cols, s, splits,
                                       n, a, cnt, report);
}

template <int LPR, int WAVES, int U>
__global__ __launch_bounds__(WAVES * 64) void sparse_gemv_w4_kernel(
    FmtW4::Args a, const __half *__restrict__ x, float t, float *partial, int *counters, float *y,
    int m, int n, int ks, int tiles, int tile_cols, int splits)
{
    trace_mark(0);
    w4_block<LPR, WAVES, U>(a, HalfSource{x}, t, partial, counters, y, m, n, ks,
                            blockIdx.x % tiles, blockIdx.x / tiles, tile_cols, splits,
                            survivor_report(counters, 0, splits));
    trace_mark(6);
}

// The int4 product with its input formed in the kernel from the two products that precede
// W_down (Appendix A.3), as sparse_gemv_swiglu_kernel does for the other formats.
template <int LPR, int WAVES, int U>
__global__ __launch_bounds__(WAVES * 64) void sparse_gemv_w4_swiglu_kernel(
    FmtW4::Args a, const float *__restrict__ gate, const float *__restrict__ up, float t,
    float *partial, int *counters, float *y, int m, int n, int ks, int tiles, int tile_cols,
    int splits)
{
    w4_block<LPR, WAVES, U>(a, SwigluSource{gate, up}, t, partial, counters, y, m, n, ks,
                            blockIdx.x % tiles, blockIdx.x / tiles, tile_cols, splits,
                            survivor_report(counters, 0, splits));
}

// Several int4 matrices that read the same hidden state in one launch; the block finds its
// matrix from its tile index as in sparse_gemv_multi_kernel.
template <int LPR, int WAVES, int U, class XS>
__device__ __forceinline__ void w4_multi_block(const MultiArgs<FmtW4> &ma, const XS &x,
                                               float *partial, int *counters, int m, int ks,
                                               int tile_cols, int splits, int block)
{
    const int tiles = ma.tile_begin[ma.count];
    const int gtile = block % tiles;
    const int s = block / tiles;
    int k = 0;
    size_t partial_off = 0;
#pragma unroll
    for (int j = 1; j < kMaxMulti; ++j) {
        if (j < ma.count && gtile >= ma.tile_begin[j]) {
            partial_off += (size_t)splits * ma.n[j - 1];
            k = j;
        }
    }
    w4_block<LPR, WAVES, U>(ma.a[k], x, ma.t[k], partial + partial_off,
                            counters + ma.tile_begin[k], ma.y[k], m, ma.n[k], ks,
                            gtile - ma.tile_begin[k], s, tile_cols, splits,
                            survivor_report(counters, k, splits));
}

template <int LPR, int WAVES, int U>
__global__ __launch_bounds__(WAVES * 64) void sparse_gemv_w4_multi_kernel(
    MultiArgs<FmtW4> ma, const __half *__restrict__ x, float *partial, int *counters, int m,
    int ks, int tile_cols, int splits)
{
    w4_multi_block<LPR, WAVES, U>(ma, HalfSource{x}, partial, counters, m, ks, tile_cols, splits,
                                  (int)blockIdx.x);
}

// The grouped int4 launch with its shared input formed from the hidden state before the
// normalisation layer, as sparse_gemv_rmsnorm_multi_kernel does for the other formats.
template <int LPR, int U>
__global__ __launch_bounds__(kNormWaves * 64) void sparse_gemv_w4_rmsnorm_multi_kernel(
    MultiArgs<FmtW4> ma, const float *__restrict__ h, const float *__restrict__ gamma, float eps,
    float *partial, int *counters, int m, int ks, int tile_cols, int splits)
{
    __shared__ double wave_sums[kMaxNormChunks * kNormWaves];
    w4_multi_block<LPR, kNormWaves, U>(ma, RmsnormSource{h, gamma, m, eps, wave_sums}, partial,
                                       counters, m, ks, tile_cols, splits, (int)blockIdx.x);
}

// Independent int4 groups in one launch (see sparse_gemv_stack_kernel).
template <int WAVES, int U>
__global__ __launch_bounds__(WAVES * 64) void sparse_gemv_w4_stack_kernel(StackArgs<FmtW4> sa)
{
    int block;
    const StackGroup<FmtW4> &sg = sa.g[stack_group_of_block(sa, block)];
    if (sg.lanes_per_row == 32)
        w4_multi_block<32, WAVES, U>(sg.ma, HalfSource{sg.x}, sg.partial, sg.counters, sg.m, sg.ks,
                                     sg.tile_cols, sg.splits, block);
    else
        w4_multi_block<16, WAVES, U>(sg.ma, HalfSource{sg.x}, sg.partial, sg.counters, sg.m, sg.ks,
                                     sg.tile_cols, sg.splits, block);
}

hipError_t launch_gemv_w8_stack(int groups, const StackGroupDesc *d, hipStream_t stream)
{
    StackArgs<FmtW8> sa{};
    size_t lds;
    const hipError_t e = fill_stack_args<FmtW8>(
        sa, lds, groups, d, 64, 8, 64, [](FmtW8::Args &a, const StackGroupDesc &g, int k) {
            a.W = g.Wt[k];
            a.scale = static_cast<const __half *>(g.scale[k]);
        });
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((sparse_gemv_stack_kernel<FmtW8, 8, 4, true>), dim3(sa.block_begin[groups]),
                       dim3(8 * 64), lds, stream, sa);
    return hipGetLastError();
}

hipError_t launch_gemv_w4_stack(int groups, const StackGroupDesc *d, hipStream_t stream)
{
    StackArgs<FmtW4> sa{};
    size_t lds;
    const hipError_t e = fill_stack_args<FmtW4>(
        sa, lds, groups, d, kGroup, 16, 32, [](FmtW4::Args &a, const StackGroupDesc &g, int k) {
            a.W = g.Wt[k];
            a.scale = static_cast<const __half *>(g.scale[k]);
        });
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((sparse_gemv_w4_stack_kernel<kW4Waves, kW4Unroll>),
                       dim3(sa.block_begin[groups]), dim3(kW4Waves * 64), lds, stream, sa);
    return hipGetLastError();
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

hipError_t launch_gemv_w8_multi(int count, const int8_t *const *Wq, const int *row_pitch,
                                const void *const *scale_f16, const float *t, float *const *y,
                                const int *n, const void *x_f16, int m, float *partial,
                                int *counters, const GemvShape &sh, hipStream_t stream)
{
    int n_max = 0;
    for (int k = 0; k < count; ++k) n_max = n[k] > n_max ? n[k] : n_max;
    // slice length, split count and LDS size do not depend on n
    const GemvGeometry g = gemv_geometry(m, n_max, sh, FmtW8::kElemsPerLane, 64, kMaxLongSlice);
    MultiArgs<FmtW8> ma{};
    ma.count = count;
    ma.tile_begin[0] = 0;
    for (int k = 0; k < count; ++k) {
        ma.a[k].W = Wq[k];
        ma.a[k].ld = row_pitch ? row_pitch[k] : 0;
        ma.a[k].scale = static_cast<const __half *>(scale_f16[k]);
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
    TEAL_DISPATCH(TEAL_LAUNCH, FmtW8, sh);
#undef TEAL_LAUNCH
    return hipGetLastError();
}

static bool w8_lanes_supported(const GemvShape &s)
{
    const int l = s.lanes_per_row;
    return (l == 8 || l == 16 || l == 32 || l == 64) && s.splits >= 1 && s.tile_cols >= 0 &&
           s.tile_cols % FmtW8::kElemsPerLane == 0 && s.tile_cols <= l * FmtW8::kElemsPerLane;
}

// The int8 kernels with their input formed in the kernel (the activation sources of the bf16
// kernels: Appendix A.3's MLP intermediate, the normalised hidden state).  Shapes with 8
// wavefronts and 4 loads per batch, which is what the launch-shape rule produces.
hipError_t launch_gemv_w8_swiglu(const int8_t *Wq, const void *scale_f16, const float *gate,
                                 const float *up, float t, float *y, int m, int n, float *partial,
                                 int *counters, const GemvShape &sh, hipStream_t stream)
{
    if (sh.waves != 8 || sh.unroll != 4 || !w8_lanes_supported(sh)) return hipErrorInvalidValue;
    const GemvGeometry g = gemv_geometry(m, n, sh, FmtW8::kElemsPerLane, 64);
    FmtW8::Args a{Wq, static_cast<const __half *>(scale_f16)};
#define TEAL_LAUNCH_S(LPR)                                                                     \
    hipLaunchKernelGGL((sparse_gemv_swiglu_kernel<FmtW8, LPR, 8, 4>), dim3(g.tiles * g.splits), \
                       dim3(8 * 64), g.lds, stream, a, gate, up, t, partial, counters, y, m, n, \
                       g.ks, g.tiles, g.tile_cols, g.splits)
    if (sh.lanes_per_row == 64) TEAL_LAUNCH_S(64);
    else if (sh.lanes_per_row == 32) TEAL_LAUNCH_S(32);
    else if (sh.lanes_per_row == 16) TEAL_LAUNCH_S(16);
    else TEAL_LAUNCH_S(8);
#undef TEAL_LAUNCH_S
    return hipGetLastError();
}

hipError_t launch_gemv_w8_rmsnorm_multi(int count, const int8_t *const *Wq, const int *row_pitch,
                                        const void *const *scale_f16, const float *t,
                                        float *const *y, const int *n, const float *h,
                                        const float *gamma, float eps, int m, float *partial,
                                        int *counters, const GemvShape &sh, hipStream_t stream)
{
    if (m < 8 || m > kMaxNormDim || m % 8 != 0 || sh.waves != kNormWaves || sh.unroll != 4 ||
        !w8_lanes_supported(sh))
        return hipErrorInvalidValue;
    int n_max = 0;
    for (int k = 0; k < count; ++k) n_max = n[k] > n_max ? n[k] : n_max;
    const GemvGeometry g = gemv_geometry(m, n_max, sh, FmtW8::kElemsPerLane, 64);
    MultiArgs<FmtW8> ma{};
    ma.count = count;
    ma.tile_begin[0] = 0;
    for (int k = 0; k < count; ++k) {
        ma.a[k].W = Wq[k];
        ma.a[k].ld = row_pitch ? row_pitch[k] : 0;
        ma.a[k].scale = static_cast<const __half *>(scale_f16[k]);
        ma.y[k] = y[k];
        ma.t[k] = t[k];
        ma.n[k] = n[k];
        ma.tile_begin[k + 1] = ma.tile_begin[k] + (n[k] + g.tile_cols - 1) / g.tile_cols;
    }
    const int tiles = ma.tile_begin[count];
#define TEAL_LAUNCH_N(LPR)                                                                     \
    hipLaunchKernelGGL((sparse_gemv_rmsnorm_multi_kernel<FmtW8, LPR, 4>),                      \
                       dim3(tiles * g.splits), dim3(kNormWaves * 64), g.lds, stream, ma, h,    \
                       gamma, eps, partial, counters, m, g.ks, g.tile_cols, g.splits)
    if (sh.lanes_per_row == 64) TEAL_LAUNCH_N(64);
    else if (sh.lanes_per_row == 32) TEAL_LAUNCH_N(32);
    else if (sh.lanes_per_row == 16) TEAL_LAUNCH_N(16);
    else TEAL_LAUNCH_N(8);
#undef TEAL_LAUNCH_N
    return hipGetLastError();
}

hipError_t launch_gemv_w4(const uint8_t *Wq, const void *scale_f16, const void *x_f16, float t,
                          float *y, int m, int n, float *partial, int *counters,
                          const GemvShape &sh, hipStream_t stream)
{
    GemvShape w4 = sh;
    w4.waves = kW4Waves;                          // the int4 kernel is built for 8 wavefronts
    const GemvGeometry g = gemv_geometry(m, n, w4, FmtW4::kElemsPerLane, kGroup);
    FmtW4::Args a{Wq, static_cast<const __half *>(scale_f16)};
    const __half *x = static_cast<const __half *>(x_f16);
#define TEAL_LAUNCH_W4(LPR)                                                                    \
    hipLaunchKernelGGL((sparse_gemv_w4_kernel<LPR, kW4Waves, kW4Unroll>),                      \
                       dim3(g.tiles * g.splits), dim3(kW4Waves * 64), g.lds, stream, a, x, t,  \
                       partial, counters, y, m, n, g.ks, g.tiles, g.tile_cols, g.splits)
    // A lane covers 32 columns: 16 lanes per row (tiles up to 512 columns) or 32 lanes
    // per row (up to 1024 columns).
    if (sh.lanes_per_row == 32) TEAL_LAUNCH_W4(32);
    else TEAL_LAUNCH_W4(16);
#undef TEAL_LAUNCH_W4
    return hipGetLastError();
}

hipError_t launch_gemv_w4_swiglu(const uint8_t *Wq, const void *scale_f16, const float *gate,
                                 const float *up, float t, float *y, int m, int n, float *partial,
                                 int *counters, const GemvShape &sh, hipStream_t stream)
{
    GemvShape w4 = sh;
    w4.waves = kW4Waves;
    const GemvGeometry g = gemv_geometry(m, n, w4, FmtW4::kElemsPerLane, kGroup);
    FmtW4::Args a{Wq, static_cast<const __half *>(scale_f16)};
#define TEAL_LAUNCH_W4S(LPR)                                                                   \
    hipLaunchKernelGGL((sparse_gemv_w4_swiglu_kernel<LPR, kW4Waves, kW4Unroll>),               \
                       dim3(g.tiles * g.splits), dim3(kW4Waves * 64), g.lds, stream, a, gate,  \
                       up, t, partial, counters, y, m, n, g.ks, g.tiles, g.tile_cols, g.splits)
    if (sh.lanes_per_row == 32) TEAL_LAUNCH_W4S(32);
    else TEAL_LAUNCH_W4S(16);
#undef TEAL_LAUNCH_W4S
    return hipGetLastError();
}

hipError_t launch_gemv_w4_rmsnorm_multi(int count, const uint8_t *const *Wq,
                                        const void *const *scale_f16, const float *t,
                                        float *const *y, const int *n, const float *h,
                                        const float *gamma, float eps, int m, float *partial,
                                        int *counters, const GemvShape &sh, hipStream_t stream)
{
    if (m < 8 || m > kMaxNormDim || m % kGroup != 0 || kW4Waves != kNormWaves)
        return hipErrorInvalidValue;
    int n_max = 0;
    for (int k = 0; k < count; ++k) n_max = n[k] > n_max ? n[k] : n_max;
    GemvShape w4 = sh;
    w4.waves = kW4Waves;
    const GemvGeometry g = gemv_geometry(m, n_max, w4, FmtW4::kElemsPerLane, kGroup);
    MultiArgs<FmtW4> ma{};
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
#define TEAL_LAUNCH_W4N(LPR)                                                                   \
    hipLaunchKernelGGL((sparse_gemv_w4_rmsnorm_multi_kernel<LPR, kW4Unroll>),                  \
                       dim3(tiles * g.splits), dim3(kNormWaves * 64), g.lds, stream, ma, h,    \
                       gamma, eps, partial, counters, m, g.ks, g.tile_cols, g.splits)
    if (sh.lanes_per_row == 32) TEAL_LAUNCH_W4N(32);
    else TEAL_LAUNCH_W4N(16);
#undef TEAL_LAUNCH_W4N
    return hipGetLastError();
}

hipError_t launch_gemv_w4_multi(int count, const uint8_t *const *Wq, const void *const *scale_f16,
                                const float *t, float *const *y, const int *n, const void *x_f16,
                                int m, float *partial, int *counters, const GemvShape &sh,
                                hipStream_t stream)
{
    int n_max = 0;
    for (int k = 0; k < count; ++k) n_max = n[k] > n_max ? n[k] : n_max;
    GemvShape w4 = sh;
    w4.waves = kW4Waves;
    const GemvGeometry g = gemv_geometry(m, n_max, w4, FmtW4::kElemsPerLane, kGroup);
    MultiArgs<FmtW4> ma{};
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
#define TEAL_LAUNCH_W4M(LPR)                                                                   \
    hipLaunchKernelGGL((sparse_gemv_w4_multi_kernel<LPR, kW4Waves, kW4Unroll>),                \
                       dim3(tiles * g.splits), dim3(kW4Waves * 64), g.lds, stream, ma, x,      \
                       partial, counters, m, g.ks, g.tile_cols, g.splits)
    if (sh.lanes_per_row == 32) TEAL_LAUNCH_W4M(32);
    else TEAL_LAUNCH_W4M(16);
#undef TEAL_LAUNCH_W4M
    return hipGetLastError();
}

// The int4 block body for the one-launch MLP.
struct W4Body {
    typedef FmtW4 Format;
    template <int LPR, class XS>
    static __device__ __forceinline__ bool run(const FmtW4::Args &a, const XS &x, float t,
                                               float *partial, int *counters, float *y, int m,
                                               int n, int ks, int tile, int s, int tile_cols,
                                               int splits, const SurvivorReport &report)
    {
        static_assert(LPR == 16 || LPR == 32, "a lane covers 32 int4 columns");
        return w4_block<LPR, kW4Waves, kW4Unroll>(a, x, t, partial, counters, y, m, n, ks, tile,
                                                  s, tile_cols, splits, report);
    }
};

static void set_wq_args(const void *&W, const __half *&scale, const void *w, const void *sc)
{
    W = w;
    scale = static_cast<const __half *>(sc);
}

hipError_t launch_mlp_w8(const MlpHostArgs &h, const MlpLaunch &L, hipStream_t stream)
{
    if (!mlp_shape_ok(L.gu, 16) || !mlp_shape_ok(L.down, 16)) return hipErrorInvalidValue;
    MlpArgs<FmtW8> A{};
    size_t lds;
    if (!fill_mlp_args<FmtW8>(A, lds, h, L, 64, [](FmtW8::Args &a, const void *W, const void *sc, int pitch) {
            set_wq_args(a.W, a.scale, W, sc);
            a.ld = pitch;
        }))
        return hipErrorInvalidValue;
    return launch_mlp_kernel<GemvBody<FmtW8>, true>(A, L.gu.lanes_per_row, L.down.lanes_per_row,
                                                    lds, stream);
}

hipError_t launch_mlp_w4(const MlpHostArgs &h, const MlpLaunch &L, hipStream_t stream)
{
    if (!mlp_shape_ok(L.gu, 32) || !mlp_shape_ok(L.down, 32)) return hipErrorInvalidValue;
    if (h.m % kGroup != 0 || h.f % kGroup != 0) return hipErrorInvalidValue;
    if (h.gu_pitch != 0 || h.down_pitch != 0) return hipErrorInvalidValue;   // rows are packed
    const auto lanes_ok = [](int l) { return l == 16 || l == 32; };
    if (!lanes_ok(L.gu.lanes_per_row) || !lanes_ok(L.down.lanes_per_row))
        return hipErrorInvalidValue;
    MlpArgs<FmtW4> A{};
    size_t lds;
    if (!fill_mlp_args<FmtW4>(A, lds, h, L, kGroup,
                              [](FmtW4::Args &a, const void *W, const void *sc, int) {
                                  set_wq_args(a.W, a.scale, W, sc);
                              }))
        return hipErrorInvalidValue;
    const dim3 grid(mlp_blocks(A.grid)), block(kW4Waves * 64);
#define TEAL_MLP_W4(LG, LD)                                                                    \
    hipLaunchKernelGGL((sparse_mlp_kernel<W4Body, LG, LD>), grid, block, lds, stream, A)
    if (L.gu.lanes_per_row == 32) {
        if (L.down.lanes_per_row == 32) TEAL_MLP_W4(32, 32);
        else TEAL_MLP_W4(32, 16);
    } else {
        if (L.down.lanes_per_row == 32) TEAL_MLP_W4(16, 32);
        else TEAL_MLP_W4(16, 16);
    }
#undef TEAL_MLP_W4
    return hipGetLastError();
}

}  // namespace teal

#ifdef TEAL_TRACE_BLOCKS
// The trace build's read-out for the kernels of this file (see trace_mark in gemv_common.h).
extern "C" int teal_trace_read_wq(unsigned long long *host, size_t count)
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
