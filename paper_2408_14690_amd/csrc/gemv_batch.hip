// Small-batch variant of the thresholded product (Section 5.4.4): one set of
// channels is dropped for the whole batch, chosen by the magnitude averaged
// over the batch dimension, and every row of the batch is multiplied with the
// surviving rows of the input-channel-major weights.  The weight stream is the
// same as for one vector (each surviving row is read once); a block keeps one
// accumulator set per batch row.
#include "gemv_common.h"

namespace teal {

namespace {

// Channel i survives iff (1 / batch) * sum_b |X[b][i]| > t.  Evaluated as
// sum > batch * t in fp64: fp16 -> fp32 -> fp64 and |.| are exact, a sum of
// up to kMaxBatch fp16 magnitudes is exact in fp64 and so is batch * t, so the
// decision involves no rounding and does not depend on the order of the batch.
// A NaN makes the sum NaN, which compares false (the channel is dropped).
template <int NB>
__device__ __forceinline__ bool survives_batch(const float (&xv)[NB], double bound)
{
    double s = 0.0;
#pragma unroll
    for (int b = 0; b < NB; ++b) s += (double)fabsf(xv[b]);
    return s > bound;
}

// compact_slice for a batch: list_idx[] receives the surviving channels of
// [k0, k1) in ascending order and list_x[] their NB activations each (rows at
// or past `batch` are zero).  Same scheme: ballots and popcounts per
// 64-channel segment, segment counts through LDS, every wavefront scans them.
template <int NB, int WAVES>
__device__ __forceinline__ int compact_slice_batch(const __half *__restrict__ X, int batch, int m,
                                                   double bound, int k0, int k1, int *list_idx,
                                                   float *list_x, int *seg_cnt)
{
    constexpr int PER_WAVE = kMaxSliceBatch / 64 / WAVES;
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int nseg = (k1 - k0 + 63) >> 6;

    float xv[PER_WAVE][NB];
    unsigned long long bal[PER_WAVE];
    // Unconditional loads from clamped positions (k1 > k0, batch >= 1), zeroed afterwards
    // where out of range, so that all loads are in flight together.
#pragma unroll
    for (int j = 0; j < PER_WAVE; ++j) {
        const int i = k0 + (w + j * WAVES) * 64 + lane;
        const int ic = min(i, k1 - 1);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const float v = __half2float(X[(size_t)min(b, batch - 1) * m + ic]);
            xv[j][b] = (i < k1 && b < batch) ? v : 0.f;
        }
    }
#pragma unroll
    for (int j = 0; j < PER_WAVE; ++j) {
        const int seg = w + j * WAVES;
        bal[j] = __ballot(survives_batch<NB>(xv[j], bound));
        if (lane == 0 && seg < nseg) seg_cnt[seg] = __popcll(bal[j]);
    }
    __syncthreads();
    const int c = lane < nseg ? seg_cnt[lane] : 0;
    const int incl = wave_inclusive_scan(c);
    const int seg_excl = incl - c;
    const int total = __builtin_amdgcn_readlane(incl, 63);
#pragma unroll
    for (int j = 0; j < PER_WAVE; ++j) {
        const int seg = w + j * WAVES;
        if (seg < nseg) {                              // wavefront-uniform
            const int base = __builtin_amdgcn_readlane(seg_excl, seg);
            if ((bal[j] >> lane) & 1ull) {
                const int slot = base + lanes_below(bal[j]);
                list_idx[slot] = k0 + seg * 64 + lane;
#pragma unroll
                for (int b = 0; b < NB; ++b) list_x[slot * NB + b] = xv[j][b];
            }
        }
    }
    __syncthreads();
    return total;
}

// The accumulators of one lane: a[bb][e] belongs to batch row bb and to column e
// of the lane's 8 columns.  Plain fp32 FMAs; products are exact in fp32 (8 + 11
// significand bits) and each accumulator sees its rows in list order.  (An
// outer-product formulation on the matrix cores, v_mfma_f32_4x4x1_16b_f32 with
// the weights as A and the batch's activations as B, computes the same sums
// but measured slower than the FMAs at 4 and 8 rows.)
template <int NB>
struct BatchAcc {
    float a[NB][8];
    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int bb = 0; bb < NB; ++bb)
#pragma unroll
            for (int e = 0; e < 8; ++e) a[bb][e] = 0.f;
    }
};

// The NB activations of one surviving row.
template <int NB>
struct RowX {
    float v[NB];
};

template <int NB>
__device__ __forceinline__ RowX<NB> load_row_x(const float *entry)
{
    RowX<NB> r;
    if constexpr (NB == 2) {
        const float2 f = *reinterpret_cast<const float2 *>(entry);
        r.v[0] = f.x; r.v[1] = f.y;
    } else {
#pragma unroll
        for (int q = 0; q < NB / 4; ++q) {
            const float4 f = *reinterpret_cast<const float4 *>(entry + 4 * q);
            r.v[4 * q] = f.x; r.v[4 * q + 1] = f.y; r.v[4 * q + 2] = f.z; r.v[4 * q + 3] = f.w;
        }
    }
    return r;
}

template <int NB>
__device__ __forceinline__ void multiply_row(BatchAcc<NB> &acc, u32x4 w, const RowX<NB> &x)
{
    float wv[8];                       // bf16 -> fp32 is a 16-bit shift
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        wv[2 * q] = __uint_as_float(w[q] << 16);
        wv[2 * q + 1] = __uint_as_float(w[q] & 0xffff0000u);
    }
#pragma unroll
    for (int bb = 0; bb < NB; ++bb)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc.a[bb][e] = fmaf(x.v[bb], wv[e], acc.a[bb][e]);
}

// stream_rows for a batch: per surviving row one 16-byte load per lane.  Slots
// past the end of the wavefront's share point at an all-zero entry (zero_slot).
template <int NB, int LPR, int U>
__device__ __forceinline__ void stream_rows_batch(BatchAcc<NB> &acc, const int *list_idx,
                                                  const float *list_x, int zero_slot, int start,
                                                  int mine,
                                                  const unsigned char *__restrict__ lane_base,
                                                  unsigned row_bytes)
{
    constexpr int R = 64 / LPR;
    if (mine <= 0) return;
    const int g = (threadIdx.x & 63) / LPR;
    const int last = mine - 1;
    const int batches = (mine + U * R - 1) / (U * R);

    struct Batch {
        u32x4 v[U];
        RowX<NB> x[U];
    };
    // The activations are fetched from LDS when the row load is issued, so that they
    // are in registers long before the weights arrive.
    auto issue = [&](Batch &b, int batch_no) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = (batch_no * U + u) * R + g;
            const int row = list_idx[start + min(e, last)];
            b.v[u] = load_stream16(lane_base + (size_t)(unsigned)row * row_bytes);
            b.x[u] = load_row_x<NB>(list_x + (e <= last ? start + e : zero_slot) * NB);
        }
    };
    auto consume = [&](const Batch &b) {
#pragma unroll
        for (int u = 0; u < U; ++u) multiply_row<NB>(acc, b.v[u], b.x[u]);
    };

    // Scheduling fences keep the two batches apart: without them the compiler issues both
    // batches back to back and drains the queue before the next pair.
    Batch b0, b1;
    issue(b0, 0);
    int it = 0;
    for (; it + 2 < batches; it += 2) {
        issue(b1, it + 1);
        __builtin_amdgcn_sched_barrier(0);
        consume(b0);
        __builtin_amdgcn_sched_barrier(0);
        issue(b0, it + 2);
        __builtin_amdgcn_sched_barrier(0);
        consume(b1);
        __builtin_amdgcn_sched_barrier(0);
    }
    if (it + 1 < batches) {
        issue(b1, it + 1);
        __builtin_amdgcn_sched_barrier(0);
        consume(b0);
        consume(b1);
    } else {
        consume(b0);
    }
}

// Leaves every lane's accumulators in red[], laid out [wavefront x row group]
// [batch row][tile column].
template <int NB, int LPR>
__device__ __forceinline__ void accumulators_to_lds(const BatchAcc<NB> &acc, float *red)
{
    constexpr int TN = LPR * 8;
    constexpr int R = 64 / LPR;
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int g = lane / LPR, l = lane % LPR;
    float *mine = red + (size_t)((w * R + g) * NB) * TN;
#pragma unroll
    for (int bb = 0; bb < NB; ++bb) {
        float4 *dst = reinterpret_cast<float4 *>(mine + bb * TN + l * 8);
        dst[0] = make_float4(acc.a[bb][0], acc.a[bb][1], acc.a[bb][2], acc.a[bb][3]);
        dst[1] = make_float4(acc.a[bb][4], acc.a[bb][5], acc.a[bb][6], acc.a[bb][7]);
    }
}

// block_finish for a batch.  red[] (WAVES x 64 lanes x NB x 8 floats) lies over the list,
// which is dead once every wavefront has left the row stream.  Partial rows are
// laid out [split][batch row][n]; the block that arrives last at the tile's
// counter adds them in split order for every batch row and writes Y.
template <int NB, int LPR, int WAVES>
__device__ __forceinline__ void block_finish_batch(const BatchAcc<NB> &acc, float *red,
                                                   float *partial, int *counters, float *Y,
                                                   int tile, int col0, int cols, int s, int splits,
                                                   int n, int batch, int cnt,
                                                   const SurvivorReport &report)
{
    constexpr int TN = LPR * 8;
    constexpr int THREADS = WAVES * 64;
    constexpr int R = 64 / LPR;
    __shared__ int last_flag;
    if (cols > n - col0) cols = n - col0;
    __syncthreads();                   // every wavefront is done with the list
    // Every lane leaves its accumulators in LDS: WAVES x R row groups per output.  (Folding
    // the R row groups of a wavefront with lane shuffles first costs more than the extra
    // LDS reads below once there are several accumulator sets.)
    accumulators_to_lds<NB, LPR>(acc, red);
    __syncthreads();
    const int total = batch * cols;
    auto wave_sum = [&](int bb, int c) {
        float sum = 0.f;
#pragma unroll
        for (int q = 0; q < WAVES * R; ++q) sum += red[(q * NB + bb) * TN + c];
        return sum;
    };
    if (tile == 0 && threadIdx.x == 0) report_slice(report, s, splits, cnt);
    if (splits == 1) {
        for (int k = threadIdx.x; k < total; k += THREADS) {
            const int bb = k / cols, c = k - bb * cols;
            store_coherent(Y + (size_t)bb * n + col0 + c, wave_sum(bb, c));
        }
        return;
    }
    for (int k = threadIdx.x; k < total; k += THREADS) {
        const int bb = k / cols, c = k - bb * cols;
        store_coherent(partial + ((size_t)s * batch + bb) * n + col0 + c, wave_sum(bb, c));
    }
    wait_vector_memory();
    __syncthreads();
    // the ticket wraps to zero with the last arrival: ready for the next call
    if (threadIdx.x == 0)
        last_flag = atomicInc(reinterpret_cast<unsigned *>(&counters[tile]), (unsigned)splits - 1u) ==
                    (unsigned)splits - 1u;
    __syncthreads();
    if (!last_flag) return;
    if (tile == 0 && threadIdx.x < 64) report_total(report, splits);

    // Second pass.  A thread owns up to OUT outputs (batch row, column) and keeps the
    // loads of MAXLD splits of all of them in flight at once; each output is summed in
    // split order, so the result does not depend on which block is last.
    constexpr int OUT = (NB * TN + THREADS - 1) / THREADS;
    constexpr int MAXLD = 16;
    const size_t split_stride = (size_t)batch * n;
    const float *p[OUT];
    float sum[OUT];
#pragma unroll
    for (int o = 0; o < OUT; ++o) {
        const int k = (int)threadIdx.x + o * THREADS;
        const int bb = k < total ? k / cols : 0, c = k < total ? k - bb * cols : 0;
        p[o] = partial + (size_t)bb * n + col0 + c;
        sum[o] = 0.f;
    }
    for (int k0 = 0; k0 < splits; k0 += MAXLD) {
        float v[OUT][MAXLD];
#pragma unroll
        for (int o = 0; o < OUT; ++o)
#pragma unroll
            for (int u = 0; u < MAXLD; ++u)
                v[o][u] = ((int)threadIdx.x + o * THREADS < total && k0 + u < splits)
                              ? load_coherent(p[o] + (size_t)(k0 + u) * split_stride) : 0.f;
#pragma unroll
        for (int o = 0; o < OUT; ++o)
#pragma unroll
            for (int u = 0; u < MAXLD; ++u) sum[o] += v[o][u];
    }
#pragma unroll
    for (int o = 0; o < OUT; ++o) {
        const int k = (int)threadIdx.x + o * THREADS;
        if (k < total) {
            const int bb = k / cols, c = k - bb * cols;
            store_coherent(Y + (size_t)bb * n + col0 + c, sum[o]);
        }
    }
}

// Work of one block: output tile `tile` x K-slice `s` of one matrix, all batch rows.
template <int NB, int LPR, int WAVES, int U>
__device__ __forceinline__ void batch_block(const void *__restrict__ W,
                                            const __half *__restrict__ X, int batch, double bound,
                                            float *partial, int *counters, float *Y, int m, int n,
                                            int ks, int tile, int s, int tile_cols, int splits,
                                            const SurvivorReport &report)
{
    extern __shared__ __align__(16) unsigned char smem[];
    // [list_x: (ks + 1) x NB floats][list_idx: ks ints]; red[] reuses the front.
    float *list_x = reinterpret_cast<float *>(smem);
    int *list_idx = reinterpret_cast<int *>(smem + (size_t)(ks + 1) * NB * sizeof(float));
    float *red = reinterpret_cast<float *>(smem);
    __shared__ int seg_cnt[kMaxSliceBatch / 64];

    const int k0 = s * ks;
    const int k1 = min(m, k0 + ks);
    if (threadIdx.x < NB) list_x[ks * NB + threadIdx.x] = 0.f;    // the all-zero entry
    const int cnt = compact_slice_batch<NB, WAVES>(X, batch, m, bound, k0, k1, list_idx, list_x,
                                                   seg_cnt);

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int start, mine;
    wave_share(cnt, w, WAVES, start, mine);

    const int col0 = tile * tile_cols;
    const int col = lane_column<8>(col0, tile_cols, n, lane % LPR);
    const unsigned row_bytes = (unsigned)n * 2u;
    const unsigned char *lane_base = static_cast<const unsigned char *>(W) + (size_t)col * 2;

    BatchAcc<NB> acc;
    acc.clear();
    stream_rows_batch<NB, LPR, U>(acc, list_idx, list_x, ks, start, mine, lane_base, row_bytes);
    block_finish_batch<NB, LPR, WAVES>(acc, red, partial, counters, Y, tile, col0, tile_cols, s,
                                       splits, n, batch, cnt, report);
}

template <int NB, int LPR, int WAVES, int U>
__global__ __launch_bounds__(WAVES * 64) void sparse_gemv_batch_kernel(
    const void *__restrict__ W, const __half *__restrict__ X, int batch, double bound,
    float *partial, int *counters, float *Y, int m, int n, int ks, int tiles, int tile_cols,
    int splits)
{
    batch_block<NB, LPR, WAVES, U>(W, X, batch, bound, partial, counters, Y, m, n, ks,
                                   blockIdx.x % tiles, blockIdx.x / tiles, tile_cols, splits,
                                   survivor_report(counters, 0, splits));
}

// Several matrices that read the same batch of hidden states (q/k/v, gate/up:
// Appendix A.3), each with its own threshold, in one launch; the block finds its
// matrix from its tile index as in sparse_gemv_multi_kernel.
struct BatchMultiArgs {
    const void *W[kMaxMulti];
    float *Y[kMaxMulti];
    double bound[kMaxMulti];          // batch * t_k
    int n[kMaxMulti];
    int tile_begin[kMaxMulti + 1];
    int count;
};

template <int NB, int LPR, int WAVES, int U>
__global__ __launch_bounds__(WAVES * 64) void sparse_gemv_batch_multi_kernel(
    BatchMultiArgs ma, const __half *__restrict__ X, int batch, float *partial, int *counters,
    int m, int ks, int tile_cols, int splits)
{
    const int tiles = ma.tile_begin[ma.count];
    const int gtile = blockIdx.x % tiles;
    const int s = blockIdx.x / tiles;
    int k = 0;
    size_t partial_off = 0;            // each matrix owns splits * batch * n floats of partial rows
#pragma unroll
    for (int j = 1; j < kMaxMulti; ++j) {
        if (j < ma.count && gtile >= ma.tile_begin[j]) {
            partial_off += (size_t)splits * batch * ma.n[j - 1];
            k = j;
        }
    }
    batch_block<NB, LPR, WAVES, U>(ma.W[k], X, batch, ma.bound[k], partial + partial_off,
                                   counters + ma.tile_begin[k], ma.Y[k], m, ma.n[k], ks,
                                   gtile - ma.tile_begin[k], s, tile_cols, splits,
                                   survivor_report(counters, k, splits));
}

constexpr int kBatchWaves = 8;
constexpr int kBatchUnroll = 4;

// One block thresholds the batch like sparsify_kernel does one vector: groups of 4 chunks
// of 1024 channels, the loads of a group (all batch rows) in flight together.
constexpr int kSparsifyWaves = 16;
constexpr int kSparsifyChunk = kSparsifyWaves * 64;
constexpr int kSparsifyGroup = 4;
__global__ __launch_bounds__(kSparsifyChunk) void sparsify_batch_kernel(
    const __half *__restrict__ X, int batch, int m, double bound, uint8_t *__restrict__ mask,
    int32_t *__restrict__ idx, int32_t *__restrict__ count)
{
    __shared__ int wave_cnt[2][kSparsifyGroup][kSparsifyWaves];
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    int base = 0;
    int buf = 0;
    for (int c0 = 0; c0 < m; c0 += kSparsifyGroup * kSparsifyChunk, buf ^= 1) {
        __half raw[kSparsifyGroup][kMaxBatch];
#pragma unroll
        for (int j = 0; j < kSparsifyGroup; ++j) {
            const int i = min(c0 + j * kSparsifyChunk + (int)threadIdx.x, m - 1);
#pragma unroll
            for (int b = 0; b < kMaxBatch; ++b)       // rows past the batch repeat the last row
                raw[j][b] = X[(size_t)min(b, batch - 1) * m + i];
        }
        unsigned long long bal[kSparsifyGroup];
#pragma unroll
        for (int j = 0; j < kSparsifyGroup; ++j) {
            const int i = c0 + j * kSparsifyChunk + (int)threadIdx.x;
            double s = 0.0;
#pragma unroll
            for (int b = 0; b < kMaxBatch; ++b)
                s += b < batch ? (double)fabsf(__half2float(raw[j][b])) : 0.0;
            const bool keep = i < m && s > bound;
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
        // wave_cnt is double-buffered: the next group writes the other half, and that
        // group's barrier orders it against this group's reads.
    }
    if (threadIdx.x == 0 && count) *count = base;
}

// The same result with eight channels per thread (one 16-byte load per batch row), for X on
// a 16-byte boundary and m a multiple of 8 (so that every row is): the block-wide prefix and
// the stores are shared by eight channels, as in the single-vector kernel of this shape.
constexpr int kVecChannels = 8;
constexpr int kVecPass = kSparsifyChunk * kVecChannels;

template <int P>
__global__ __launch_bounds__(kSparsifyChunk) void sparsify_batch_vec_kernel(
    const __half *__restrict__ X, int batch, int m, double bound, uint8_t *__restrict__ mask,
    bool mask_aligned, int32_t *__restrict__ idx, int32_t *__restrict__ count)
{
    __shared__ int wave_tot[2][P][kSparsifyWaves];
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    int base = 0;
    int buf = 0;
    for (int c0 = 0; c0 < m; c0 += P * kVecPass, buf ^= 1) {
        unsigned bits[P];
        int cnt[P], incl[P];
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int i0 = c0 + (p * kSparsifyChunk + (int)threadIdx.x) * kVecChannels;
            const int ic = min(i0, m - kVecChannels);     // m >= 8 and m % 8 == 0
            uint4 raw[kMaxBatch];
#pragma unroll
            for (int b = 0; b < kMaxBatch; ++b)           // rows past the batch repeat the last row
                raw[b] = *reinterpret_cast<const uint4 *>(X + (size_t)min(b, batch - 1) * m + ic);
            double sum[kVecChannels];
#pragma unroll
            for (int e = 0; e < kVecChannels; ++e) sum[e] = 0.0;
#pragma unroll
            for (int b = 0; b < kMaxBatch; ++b) {
                if (b < batch) {                          // block-uniform
                    const unsigned wd[4] = {raw[b].x, raw[b].y, raw[b].z, raw[b].w};
#pragma unroll
                    for (int e = 0; e < kVecChannels; ++e) {
                        const unsigned short h = (unsigned short)(wd[e >> 1] >> (16 * (e & 1)));
                        sum[e] += (double)fabsf(__half2float(__ushort_as_half(h)));
                    }
                }
            }
            unsigned bb = 0;
#pragma unroll
            for (int e = 0; e < kVecChannels; ++e) bb |= (sum[e] > bound ? 1u : 0u) << e;
            if (i0 >= m) bb = 0;
            bits[p] = bb;
            cnt[p] = __popc(bb);
            incl[p] = wave_inclusive_scan(cnt[p]);
            if (lane == 63) wave_tot[buf][p][w] = incl[p];
            if (mask && i0 < m) {
                if (mask_aligned) {
                    const unsigned lo = bb & 0xFu, hi = (bb >> 4) & 0xFu;
                    uint2 mv;
                    mv.x = (lo & 1u) | ((lo & 2u) << 7) | ((lo & 4u) << 14) | ((lo & 8u) << 21);
                    mv.y = (hi & 1u) | ((hi & 2u) << 7) | ((hi & 4u) << 14) | ((hi & 8u) << 21);
                    *reinterpret_cast<uint2 *>(mask + i0) = mv;
                } else {
#pragma unroll
                    for (int e = 0; e < kVecChannels; ++e) mask[i0 + e] = (uint8_t)((bb >> e) & 1u);
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int p = 0; p < P; ++p) {
            if (c0 + p * kVecPass < m) {                  // block-uniform
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
    }
    if (threadIdx.x == 0 && count) *count = base;
}

}  // namespace

bool gemv_batch_shape_supported(int batch, const GemvShape &s)
{
    if (batch < 1 || batch > kMaxBatch) return false;
    const int nb = batch <= 2 ? 2 : batch <= 4 ? 4 : 8;
    const bool lpr = s.lanes_per_row == 64 || s.lanes_per_row == 32 || s.lanes_per_row == 16;
    const bool tc = s.tile_cols >= 0 && s.tile_cols % 8 == 0 && s.tile_cols <= s.lanes_per_row * 8;
    // a thread of the second pass owns at most 4 outputs: nb x (8 * lanes) <= 2048
    const bool fits = nb * s.lanes_per_row <= 256;
    return lpr && tc && fits && s.waves == kBatchWaves && s.unroll == kBatchUnroll &&
           s.splits >= 1;
}

hipError_t launch_gemv_bf16_batch(const void *Wt, const void *X_f16, int batch, float t, float *Y,
                                  int m, int n, float *partial, int *counters,
                                  const GemvShape &sh, hipStream_t stream)
{
    const GemvGeometry g = gemv_geometry(m, n, sh, 8, 64);
    if (g.ks > kMaxSliceBatch || !gemv_batch_shape_supported(batch, sh)) return hipErrorInvalidValue;
    const int nb = batch <= 2 ? 2 : batch <= 4 ? 4 : 8;
    const size_t list_bytes = (size_t)(g.ks + 1) * nb * sizeof(float) + (size_t)g.ks * sizeof(int);
    const size_t red_bytes = (size_t)kBatchWaves * 64 * nb * 8 * sizeof(float);
    const size_t lds = list_bytes > red_bytes ? list_bytes : red_bytes;
    const double bound = (double)batch * (double)t;
    const __half *X = static_cast<const __half *>(X_f16);
#define TEAL_LAUNCH_B(NB, LPR)                                                                   \
    hipLaunchKernelGGL((sparse_gemv_batch_kernel<NB, LPR, kBatchWaves, kBatchUnroll>),           \
                       dim3(g.tiles * g.splits), dim3(kBatchWaves * 64), lds, stream, Wt, X,     \
                       batch, bound, partial, counters, Y, m, n, g.ks, g.tiles, g.tile_cols,     \
                       g.splits)
    const int lpr = sh.lanes_per_row;
    if (nb == 2) {
        if (lpr == 64) TEAL_LAUNCH_B(2, 64);
        else if (lpr == 32) TEAL_LAUNCH_B(2, 32);
        else TEAL_LAUNCH_B(2, 16);
    } else if (nb == 4) {
        if (lpr == 64) TEAL_LAUNCH_B(4, 64);
        else if (lpr == 32) TEAL_LAUNCH_B(4, 32);
        else TEAL_LAUNCH_B(4, 16);
    } else {
        if (lpr == 32) TEAL_LAUNCH_B(8, 32);
        else TEAL_LAUNCH_B(8, 16);
    }
#undef TEAL_LAUNCH_B
    return hipGetLastError();
}

hipError_t launch_gemv_bf16_batch_multi(int count, const void *const *Wt, const float *t,
                                        float *const *Y, const int *n, const void *X_f16,
                                        int batch, int m, float *partial, int *counters,
                                        const GemvShape &sh, hipStream_t stream)
{
    int n_max = 0;
    for (int k = 0; k < count; ++k) n_max = n[k] > n_max ? n[k] : n_max;
    const GemvGeometry g = gemv_geometry(m, n_max, sh, 8, 64);
    if (g.ks > kMaxSliceBatch || !gemv_batch_shape_supported(batch, sh)) return hipErrorInvalidValue;
    const int nb = batch <= 2 ? 2 : batch <= 4 ? 4 : 8;
    const size_t list_bytes = (size_t)(g.ks + 1) * nb * sizeof(float) + (size_t)g.ks * sizeof(int);
    const size_t red_bytes = (size_t)kBatchWaves * 64 * nb * 8 * sizeof(float);
    const size_t lds = list_bytes > red_bytes ? list_bytes : red_bytes;
    BatchMultiArgs ma{};
    ma.count = count;
    ma.tile_begin[0] = 0;
    for (int k = 0; k < count; ++k) {
        ma.W[k] = Wt[k];
        ma.Y[k] = Y[k];
        ma.bound[k] = (double)batch * (double)t[k];
        ma.n[k] = n[k];
        ma.tile_begin[k + 1] = ma.tile_begin[k] + (n[k] + g.tile_cols - 1) / g.tile_cols;
    }
    const int tiles = ma.tile_begin[count];
    const __half *X = static_cast<const __half *>(X_f16);
#define TEAL_LAUNCH_BM(NB, LPR)                                                                  \
    hipLaunchKernelGGL((sparse_gemv_batch_multi_kernel<NB, LPR, kBatchWaves, kBatchUnroll>),     \
                       dim3(tiles * g.splits), dim3(kBatchWaves * 64), lds, stream, ma, X,       \
                       batch, partial, counters, m, g.ks, g.tile_cols, g.splits)
    const int lpr = sh.lanes_per_row;
    if (nb == 2) {
        if (lpr == 64) TEAL_LAUNCH_BM(2, 64);
        else if (lpr == 32) TEAL_LAUNCH_BM(2, 32);
        else TEAL_LAUNCH_BM(2, 16);
    } else if (nb == 4) {
        if (lpr == 64) TEAL_LAUNCH_BM(4, 64);
        else if (lpr == 32) TEAL_LAUNCH_BM(4, 32);
        else TEAL_LAUNCH_BM(4, 16);
    } else {
        if (lpr == 32) TEAL_LAUNCH_BM(8, 32);
        else TEAL_LAUNCH_BM(8, 16);
    }
#undef TEAL_LAUNCH_BM
    return hipGetLastError();
}

hipError_t launch_sparsify_batch(const void *X_f16, int batch, int m, float t, uint8_t *mask,
                                 int32_t *idx, int32_t *count, hipStream_t stream)
{
    const __half *X = static_cast<const __half *>(X_f16);
    const double bound = (double)batch * (double)t;
    if (m >= kVecChannels && m % kVecChannels == 0 && (reinterpret_cast<uintptr_t>(X_f16) & 15) == 0) {
        const bool mask_aligned = (reinterpret_cast<uintptr_t>(mask) & 7) == 0;
        if (m <= kVecPass)
            hipLaunchKernelGGL(sparsify_batch_vec_kernel<1>, dim3(1), dim3(kSparsifyChunk), 0, stream,
                               X, batch, m, bound, mask, mask_aligned, idx, count);
        else
            hipLaunchKernelGGL(sparsify_batch_vec_kernel<2>, dim3(1), dim3(kSparsifyChunk), 0, stream,
                               X, batch, m, bound, mask, mask_aligned, idx, count);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(sparsify_batch_kernel, dim3(1), dim3(kSparsifyWaves * 64), 0, stream, X,
                       batch, m, bound, mask, idx, count);
    return hipGetLastError();
}

}  // namespace teal
