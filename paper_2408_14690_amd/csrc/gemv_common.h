// Device-side building blocks of the fused threshold + sparse GEMV kernels
// (gfx950, wave64).  One thread block owns an output tile and a slice of the
// input dimension (split-K, Section 4.4).  It (1) builds the mask
// s = [|x| > t] of its slice in-kernel (Definition 1; Section 4.4 fuses the
// mask creation) and compacts the survivors into an LDS list with wavefront
// ballots and an LDS prefix sum, (2) streams only the surviving rows of the
// input-channel-major weights with 16-byte non-temporal loads and fp32 FMAs,
// (3) sums its wavefronts' accumulators through LDS and writes one fp32
// partial row; the last block to finish a tile adds that tile's partial rows
// in split order and writes y (second pass, same launch).
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "teal_internal.h"
#include <map>
#include <mutex>
#include <utility>

namespace teal {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kMaxSegs = kMaxSlice / 64;   // 64-channel segments per slice

// Measurement aid, compiled in only with -DTEAL_TRACE_BLOCKS (a separate build of the library
// used to look at where the time of a launch goes; the library proper contains none of it):
// thread 0 of a block leaves the 100 MHz device clock at up to 8 marks in a device array (one
// per source file; teal_trace_read copies out that of the bf16 kernels).
#ifdef TEAL_TRACE_BLOCKS
constexpr int kTraceBlocks = 8192, kTraceMarks = 8;
static __device__ unsigned long long teal_trace[kTraceBlocks * kTraceMarks];
__device__ __forceinline__ void trace_mark(int slot)
{
    if (threadIdx.x == 0 && blockIdx.x < kTraceBlocks)
        teal_trace[blockIdx.x * kTraceMarks + slot] = wall_clock64();
}
__device__ __forceinline__ void trace_mark_thread(int slot, int thread)
{
    if ((int)threadIdx.x == thread && blockIdx.x < kTraceBlocks)
        teal_trace[blockIdx.x * kTraceMarks + slot] = wall_clock64();
}
#else
__device__ __forceinline__ void trace_mark(int) {}
__device__ __forceinline__ void trace_mark_thread(int, int) {}
#endif

// Weight bytes are used exactly once: load them non-temporal so they do not
// displace x and the partial sums from the caches (the counterpart of the
// eviction-policy hint of Section 4.4).
__device__ __forceinline__ u32x4 load_stream16(const void *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}

// Device-scope coherent accesses for data that one block writes and a block on
// another XCD reads within the same launch.  The outputs are stored this way too
// (write-through): lines left dirty in an L2 are written back at the end of the
// kernel, which was measured to add 0.15-0.2 us to every call.
__device__ __forceinline__ void store_coherent(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_coherent(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_coherent(int *p, int v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int load_coherent(const int *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// s_waitcnt vmcnt(0): every vector-memory operation this wavefront has issued
// has completed (expcnt and lgkmcnt fields left at their maxima = no wait).
__device__ __forceinline__ void wait_vector_memory()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0x0F70);
}

// Number of set bits of a wavefront ballot in lanes below the calling lane.
__device__ __forceinline__ int lanes_below(unsigned long long b)
{
    return (int)__builtin_amdgcn_mbcnt_hi((unsigned)(b >> 32),
                                          __builtin_amdgcn_mbcnt_lo((unsigned)b, 0u));
}

// Inclusive prefix sum over the 64 lanes of a wavefront with data-parallel
// primitives (no LDS round trips): shifts by 1, 2, 4, 8 within each row of 16
// lanes, then lane 15 of row 0 / 2 is added to row 1 / 3 and lane 31 to rows
// 2 and 3.  Lanes shifted in from outside a row contribute zero.
__device__ __forceinline__ int wave_inclusive_scan(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, true);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, true);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, true);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, true);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, true);   // row_bcast:15 -> rows 1, 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, true);   // row_bcast:31 -> rows 2, 3
    return v;
}

// Every call leaves the number of input channels that survived its threshold in the
// workspace: the realised sparsity of a call (Section 4.2 fixes a target p per matrix
// and a threshold estimated offline, so the two can drift apart).  The blocks of a
// matrix's first output tile each know the count of their K-slice; they travel like
// the partial rows (write-through store, then the arrival counter), and the block that
// finishes that tile last adds them.  The report area follows the arrival counters:
// int total[kMaxMatrices] (padded to kReportHeaderInts), then one row of `splits`
// slice counts per matrix.
struct SurvivorReport {
    int *total;        // this matrix's slot
    int *per_split;    // this matrix's row of slice counts
};

__device__ __forceinline__ SurvivorReport survivor_report(int *counters_base, int matrix, int splits)
{
    int *area = counters_base + kCounterBytes / sizeof(int);
    return SurvivorReport{area + matrix, area + kReportHeaderInts + matrix * splits};
}

// Called by thread 0 of a block of tile 0 before the block's arrival (or instead of it
// when there is one split).
__device__ __forceinline__ void report_slice(const SurvivorReport &r, int s, int splits, int cnt)
{
    store_coherent(splits == 1 ? r.total : r.per_split + s, cnt);
}

// Called by the first wavefront of the block that arrived last at tile 0.
__device__ __forceinline__ void report_total(const SurvivorReport &r, int splits)
{
    const int lane = threadIdx.x & 63;
    int sum = 0;
    for (int k = lane; k < splits; k += 64) sum += load_coherent(r.per_split + k);
    sum = __builtin_amdgcn_readlane(wave_inclusive_scan(sum), 63);
    if (lane == 0) store_coherent(r.total, sum);
}

// Where a block's activations come from.  A source loads what it needs for
// channel i (load) and turns it into an fp32 value that is exactly an fp16 value
// (value); kHeavy says that value() is worth skipping for segments past the slice.
// Between the loads and the first value() every thread of the block calls prepare()
// once: block-wide work whose result value() needs (it may contain barriers) runs
// there, with the slice's own loads already in flight.
struct HalfSource {                   // the hidden state itself, fp16 in memory
    static constexpr bool kHeavy = false;
    static constexpr bool kPlainHalf = true;
    typedef __half Raw;
    const __half *x;
    __device__ __forceinline__ Raw load(int i) const { return x[i]; }
    __device__ __forceinline__ float prepare() const { return 0.f; }
    __device__ __forceinline__ float value(Raw r, float) const { return __half2float(r); }
};

// SiLU(g) * u rounded to fp16 (Appendix A.3: the input of W_down), in stated
// binary32 arithmetic, because this value decides the mask: clamp -g to
// [-80, 80]; exp by k = rint(z log2 e), r = z - k ln2 (two fmas, ln2 split
// high / low), the degree-7 Taylor polynomial by Horner's rule with fmas, exact
// scaling by 2^k; sigma = 1 / (1 + e) (correctly rounded division);
// SiLU = g * sigma; times u; round to nearest even.  NaN in, NaN out.
__device__ __forceinline__ float swiglu_value(float g, float u)
{
#pragma clang fp contract(off)
    float z = -g;
    z = z > 80.0f ? 80.0f : z;
    z = z < -80.0f ? -80.0f : z;
    const float k = rintf(z * 1.44269502f);
    float r = fmaf(k, -0.693145752f, z);
    r = fmaf(k, -1.42860677e-06f, r);
    float p = 1.0f / 5040.0f;
    p = fmaf(p, r, 1.0f / 720.0f);
    p = fmaf(p, r, 1.0f / 120.0f);
    p = fmaf(p, r, 1.0f / 24.0f);
    p = fmaf(p, r, 1.0f / 6.0f);
    p = fmaf(p, r, 0.5f);
    p = fmaf(p, r, 1.0f);
    p = fmaf(p, r, 1.0f);
    const float e = ldexpf(p, (int)k);
    const float sg = 1.0f / (1.0f + e);
    const float silu = g != g ? g : g * sg;
    float h32 = silu * u;
    // The product is rounded to binary32 first and to binary16 second.  Without this
    // fence the compiler folds the two into one mixed-precision instruction that rounds
    // the exact product once, which differs from the stated arithmetic near ties.
    asm volatile("" : "+v"(h32));
    return __half2float(__float2half_rn(h32));
}

struct SwigluSource {                 // gate = x W_gate^T and up = x W_up^T, fp32 in memory
    static constexpr bool kHeavy = true;
    static constexpr bool kPlainHalf = false;
    typedef float2 Raw;
    const float *gate;
    const float *up;
    __device__ __forceinline__ Raw load(int i) const { return make_float2(gate[i], up[i]); }
    __device__ __forceinline__ float prepare() const { return 0.f; }
    __device__ __forceinline__ float value(Raw r, float) const { return swiglu_value(r.x, r.y); }
};

// ---- the normalised hidden state (the input of W_q/W_k/W_v and W_gate/W_up) ----
//
// x_i = gamma_i h_i / sqrt(mean(h^2) + eps), in stated arithmetic because x decides the
// mask: the squares are exact in binary64 and are added by pairwise summation over the
// index range padded with zeros to a power of two (halve the range, add the two halves'
// sums, every addition rounded to binary64); v = ss / m + eps, r = binary32(1 / sqrt(v))
// in binary64; a = h_i r, b = a gamma_i in binary32, each rounded; x_i = binary16(b).
//
// A block of kNormWaves wavefronts sums kNormChunk entries per pass, thread T entries
// 8T .. 8T+7 of the chunk: index bits 0-2 are added inside the thread, bits 3-8 across the
// wavefront's lanes, bits 9-11 across the wavefronts, the rest across chunks, which is
// the halving order read from the leaves up.  Adding zero is exact, so padding further
// than the next power of two changes nothing.
constexpr int kNormWaves = 8;
constexpr int kNormChunk = kNormWaves * 64 * 8;
constexpr int kMaxNormChunks = 4;
constexpr int kMaxNormDim = kNormChunk * kMaxNormChunks;

template <int CTRL>
__device__ __forceinline__ double lane_exchange(double v)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double read_lane(double v, int lane)
{
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), lane),
                            __builtin_amdgcn_readlane(__double2loint(v), lane));
}

// Sum over the 64 lanes in halving order (lane l next to l ^ 1, pairs next to pairs, ...).
// After each step all lanes of a group hold the group's sum, so the partner group may be
// read through a mirror instead of an exchange; a + b == b + a bit for bit.  All 64 lanes
// must be active.
__device__ __forceinline__ double wave_tree_sum(double s)
{
    s += lane_exchange<0xB1>(s);      // quad_perm [1,0,3,2]: lane ^ 1
    s += lane_exchange<0x4E>(s);      // quad_perm [2,3,0,1]: lane ^ 2
    s += lane_exchange<0x141>(s);     // row_half_mirror: the other quad of each 8 lanes
    s += lane_exchange<0x140>(s);     // row_mirror: the other half of each row of 16
    const double r0 = read_lane(s, 0), r1 = read_lane(s, 16);
    const double r2 = read_lane(s, 32), r3 = read_lane(s, 48);
    return (r0 + r1) + (r2 + r3);
}

// Sums of squares of the first C chunks' entries, one per wavefront and chunk, into
// wave_sums[c * kNormWaves + w].  All of a thread's loads are issued before the first is
// used; a chunk past the end of h is loaded from a clamped position and counted as zeros.
template <int C>
__device__ __forceinline__ void chunk_wave_sums(const float *__restrict__ h, int m,
                                                double *wave_sums)
{
#pragma clang fp contract(off)
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    float4 v[C][2];
#pragma unroll
    for (int c = 0; c < C; ++c) {
        const int j = min(c * kNormChunk + (int)threadIdx.x * 8, m - 8);
        const float4 *p = reinterpret_cast<const float4 *>(h + j);
        v[c][0] = p[0];
        v[c][1] = p[1];
    }
#pragma unroll
    for (int c = 0; c < C; ++c) {
        const bool live = c * kNormChunk + (int)threadIdx.x * 8 < m;
        const float e[8] = {v[c][0].x, v[c][0].y, v[c][0].z, v[c][0].w,
                            v[c][1].x, v[c][1].y, v[c][1].z, v[c][1].w};
        double q[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const double d = live ? (double)e[k] : 0.0;
            q[k] = d * d;
        }
        double s = ((q[0] + q[1]) + (q[2] + q[3])) + ((q[4] + q[5]) + (q[6] + q[7]));
        s = wave_tree_sum(s);
        if (lane == 0) wave_sums[c * kNormWaves + w] = s;
    }
}

// r = binary32(1 / sqrt(mean(h^2) + eps)) as stated above.  All kNormWaves * 64 threads of
// the block call it; wave_sums is LDS for kMaxNormChunks * kNormWaves doubles.  Needs
// 8 <= m <= kMaxNormDim, m % 8 == 0, h 16-byte aligned.  Contains one barrier.
__device__ __forceinline__ float rms_scale(const float *__restrict__ h, int m, float eps,
                                           double *wave_sums)
{
#pragma clang fp contract(off)
    const int chunks = (m + kNormChunk - 1) / kNormChunk;      // block-uniform
    if (chunks == 1) chunk_wave_sums<1>(h, m, wave_sums);
    else if (chunks == 2) chunk_wave_sums<2>(h, m, wave_sums);
    else chunk_wave_sums<4>(h, m, wave_sums);
    __syncthreads();
    double cs[kMaxNormChunks];
#pragma unroll
    for (int c = 0; c < kMaxNormChunks; ++c) {
        const double *ws = wave_sums + c * kNormWaves;
        cs[c] = c < (chunks == 3 ? 4 : chunks)
                    ? ((ws[0] + ws[1]) + (ws[2] + ws[3])) + ((ws[4] + ws[5]) + (ws[6] + ws[7]))
                    : 0.0;
    }
    const double ss = (cs[0] + cs[1]) + (cs[2] + cs[3]);
    const double var = ss / (double)m + (double)eps;
    return (float)(1.0 / sqrt(var));
}

__device__ __forceinline__ float rmsnorm_value(float h, float gamma, float r)
{
#pragma clang fp contract(off)
    float a = h * r;
    asm volatile("" : "+v"(a));       // a and b are rounded to binary32 one by one,
    float b = a * gamma;
    asm volatile("" : "+v"(b));       // and b to binary16 after that (no fused forms)
    return __half2float(__float2half_rn(b));
}

struct RmsnormSource {                // hidden state and norm weights, fp32 in memory
    static constexpr bool kHeavy = false;
    static constexpr bool kPlainHalf = false;
    typedef float2 Raw;
    const float *h;
    const float *gamma;
    int m;
    float eps;
    double *wave_sums;                // LDS, kMaxNormChunks * kNormWaves doubles
    __device__ __forceinline__ Raw load(int i) const { return make_float2(h[i], gamma[i]); }
    __device__ __forceinline__ float prepare() const { return rms_scale(h, m, eps, wave_sums); }
    __device__ __forceinline__ float value(Raw raw, float r) const
    {
        return rmsnorm_value(raw.x, raw.y, r);
    }
};

// Definition 1 on one element: fp16 -> fp32 is exact, the compare is fp32.
__device__ __forceinline__ bool survives(float xv, float t) { return fabsf(xv) > t; }

// Compacts the survivors of channels [k0, k1) into list[] as (channel, x as
// fp32 bits), ascending.  Each wavefront ballots its 64-channel segments and
// leaves their popcounts in seg_cnt[] (LDS, kMaxSegs ints); after one barrier
// every wavefront computes the exclusive prefix over the segment counts
// itself (lane j holds the prefix of segment j in `seg_excl`; lanes past the
// last segment hold the total) and scatters its survivors.  The x values and
// ballots stay in registers between the two steps, and all of a wavefront's
// loads of x are issued together.  Returns the total (same in all threads).
// Needs k1 - k0 <= kMaxSlice.  All threads of the block must call it; ends
// with a barrier after which list[] is complete.  `prepared`, when given, carries
// what the source prepares once per block (the scale of the normalisation) from
// one piece of a long slice to the next: computed when `have_prepared` is false
// (block-uniform), reused otherwise.
template <int WAVES, class XS>
__device__ __forceinline__ int compact_slice(const XS &x, float t, int k0,
                                             int k1, int2 *list, int *seg_cnt, int &seg_excl,
                                             float *prepared_io = nullptr,
                                             bool have_prepared = false)
{
    constexpr int PER_WAVE = kMaxSegs / WAVES;
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int nseg = (k1 - k0 + 63) >> 6;

    float xv[PER_WAVE];
    unsigned long long bal[PER_WAVE];
    // Unconditional loads from a clamped position (k1 > k0), the out-of-range lanes zeroed
    // afterwards: a load inside a branch is waited for before the next one is issued.
    typename XS::Raw raw[PER_WAVE];
#pragma unroll
    for (int j = 0; j < PER_WAVE; ++j)
        raw[j] = x.load(min(k0 + (w + j * WAVES) * 64 + lane, k1 - 1));
    float prepared;
    if (prepared_io && have_prepared) prepared = *prepared_io;
    else prepared = x.prepare();
    if (prepared_io) *prepared_io = prepared;
    const int w_uniform = __builtin_amdgcn_readfirstlane(w);
#pragma unroll
    for (int j = 0; j < PER_WAVE; ++j) {
        const int i = k0 + (w + j * WAVES) * 64 + lane;
        float v = 0.f;
        if (!XS::kHeavy || w_uniform + j * WAVES < nseg)          // wavefront-uniform
            v = x.value(raw[j], prepared);
        xv[j] = i < k1 ? v : 0.f;                     // x = 0 never survives (t >= 0)
    }
#pragma unroll
    for (int j = 0; j < PER_WAVE; ++j) {
        const int seg = w + j * WAVES;
        bal[j] = __ballot(survives(xv[j], t));
        if (lane == 0 && seg < nseg) seg_cnt[seg] = __popcll(bal[j]);
    }
    __syncthreads();
    const int c = lane < nseg ? seg_cnt[lane] : 0;
    const int incl = wave_inclusive_scan(c);
    seg_excl = incl - c;
    const int total = __builtin_amdgcn_readlane(incl, 63);
#pragma unroll
    for (int j = 0; j < PER_WAVE; ++j) {
        const int seg = w + j * WAVES;
        if (seg < nseg) {                              // wavefront-uniform
            const int base = __builtin_amdgcn_readlane(seg_excl, seg);
            if (survives(xv[j], t))
                list[base + lanes_below(bal[j])] =
                    make_int2(k0 + seg * 64 + lane, __float_as_int(xv[j]));
        }
    }
    __syncthreads();
    return total;
}

// Wavefront-uniform contiguous share of `cnt` items for wavefront w of WAVES.
__device__ __forceinline__ void wave_share(int cnt, int w, int waves, int &start, int &mine)
{
    const int per = cnt / waves, rem = cnt - per * waves;
    start = w * per + min(w, rem);
    mine = per + (w < rem ? 1 : 0);
}

// compact_slice for short slices (at most P segments of 64 channels) of an fp16 state,
// without a barrier: every wavefront ballots ALL segments of the slice itself (P loads per
// lane, the same number compact_slice issues), so it knows every count and writes exactly
// those entries of list[] that fall into its own share [start, start + mine) -- the entries
// it alone will read.  The result (list contents, total, seg_excl) is that of compact_slice.
template <int P, int WAVES>
__device__ __forceinline__ int compact_slice_private(const __half *__restrict__ x, float t, int k0,
                                                     int k1, int2 *list, int &seg_excl)
{
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    __half raw[P];
#pragma unroll
    for (int j = 0; j < P; ++j) raw[j] = x[min(k0 + j * 64 + lane, k1 - 1)];
    float xv[P];
    unsigned long long bal[P];
    int base[P + 1];
    base[0] = 0;
#pragma unroll
    for (int j = 0; j < P; ++j) {
        const int i = k0 + j * 64 + lane;
        xv[j] = i < k1 ? __half2float(raw[j]) : 0.f;          // x = 0 never survives (t >= 0)
        bal[j] = __ballot(survives(xv[j], t));
        base[j + 1] = base[j] + __popcll(bal[j]);
    }
    const int total = base[P];
    seg_excl = total;                                         // lane j: prefix of segment j
#pragma unroll
    for (int j = 0; j < P; ++j) seg_excl = lane == j ? base[j] : seg_excl;
    int start, mine;
    wave_share(total, w, WAVES, start, mine);
    const int end = start + mine;
#pragma unroll
    for (int j = 0; j < P; ++j) {
        if (base[j] < end && base[j + 1] > start) {           // wavefront-uniform
            const int rank = base[j] + lanes_below(bal[j]);
            if (survives(xv[j], t) && rank >= start && rank < end)
                list[rank] = make_int2(k0 + j * 64 + lane, __float_as_int(xv[j]));
        }
    }
    return total;
}

// One batch of row loads in flight: U 16-byte vectors per lane and the
// activations they are to be multiplied with.
template <int U>
struct RowBatch {
    u32x4 v[U];
    float xv[U];
};

// Streams `mine` consecutive list entries starting at list[start] and adds
// x_i * W[i][cols of this lane] into acc.  LPR lanes share one row per load
// (64 / LPR rows per wavefront load).  Two batches of U loads are kept in
// flight per wavefront: while one batch is multiplied out, the next is
// already on its way.  Slots past the end of the share repeat the last row
// with a zero multiplier (same address as a live load: no new traffic).
// `start` and `mine` are wavefront-uniform; lane_base = weights + this
// lane's column offset.
template <class F, int LPR, int U>
__device__ __forceinline__ void stream_rows(float (&acc)[F::kElemsPerLane], const int2 *list,
                                            int start, int mine,
                                            const unsigned char *__restrict__ lane_base,
                                            unsigned row_bytes)
{
    constexpr int R = 64 / LPR;
    if (mine <= 0) return;
    const int g = (threadIdx.x & 63) / LPR;
    const int last = mine - 1;
    const int batches = (mine + U * R - 1) / (U * R);

    auto issue = [&](RowBatch<U> &b, int batch) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e = (batch * U + u) * R + g;
            const int2 ent = list[start + min(e, last)];
            b.xv[u] = e <= last ? __int_as_float(ent.y) : 0.f;
            b.v[u] = load_stream16(lane_base + (size_t)(unsigned)ent.x * row_bytes);
        }
    };
    auto consume = [&](const RowBatch<U> &b) {
#pragma unroll
        for (int u = 0; u < U; ++u) F::fma(acc, b.v[u], b.xv[u]);
    };

    // The steady-state loop has no conditional issue, so that each consume
    // waits only for its own batch while the other batch stays in flight.
    RowBatch<U> b0, b1;
    issue(b0, 0);
    int it = 0;
    for (; it + 2 < batches; it += 2) {
        issue(b1, it + 1);
        consume(b0);
        issue(b0, it + 2);
        consume(b1);
    }
    if (it + 1 < batches) {
        issue(b1, it + 1);
        consume(b0);
        consume(b1);
    } else {
        consume(b0);
    }
}

// Where column c of a tile lies in a wavefront's row of the LDS combine buffer.  Lanes
// write their sums one float at a time (see store_wave_sums), EPL columns apart from their
// neighbours; one float of padding per EPL columns keeps those writes off a common bank.
template <int EPL, int LPR>
__device__ __forceinline__ int combine_index(int c)
{
    return LPR == 64 ? c : c + c / EPL;
}
template <int EPL, int LPR>
constexpr int combine_row = LPR == 64 ? LPR * EPL : LPR * EPL + LPR;

// Two accumulators a and b of a lane are exchanged with the partner lane 16 (or 32) lanes
// away such that one addition leaves a's pair sum in the even rows of 16 lanes (lower 32
// lanes) and b's pair sum in the odd rows (upper 32 lanes).  Register moves only: a lane
// shuffle goes through the LDS crossbar, which the 8 wavefronts of a block saturate
// (measured: 0.85 us for the 64 shuffles per lane of the int4 kernel).
__device__ __forceinline__ float pair_sum16(float a, float b)
{
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false,
                                                    false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float pair_sum32(float a, float b)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false,
                                                    false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Adds the accumulators of the 64 / LPR row groups of a wavefront (lanes that share their
// columns: lane = group * LPR + l) and leaves the sums in this wavefront's row `dst` of the
// combine buffer.  The row groups are added in the order ((g0 + g1) + (g2 + g3)) + ...;
// every exchange halves the number of registers, so that in the end each sum is held by
// exactly one lane: with R = 64 / LPR, register k of lane (rho, l), rho = lane / 16 (for
// LPR = 32: lane / 32), holds column l * N + R' * k + rho of the tile, R' = min(R, 4).
template <int LPR, int N>
__device__ __forceinline__ void store_wave_sums(const float (&acc)[N], float *dst)
{
    const int lane = threadIdx.x & 63;
    if constexpr (LPR == 64) {
        float4 *d4 = reinterpret_cast<float4 *>(dst + lane * N);
#pragma unroll
        for (int q = 0; q < N / 4; ++q)
            d4[q] = make_float4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
    } else if constexpr (LPR == 32) {
        const int l = lane & 31, rho = lane >> 5;
#pragma unroll
        for (int j = 0; j < N / 2; ++j)
            dst[combine_index<N, LPR>(l * N + 2 * j + rho)] = pair_sum32(acc[2 * j], acc[2 * j + 1]);
    } else {
        float v[N];
#pragma unroll
        for (int e = 0; e < N; ++e) v[e] = acc[e];
        if constexpr (LPR == 8) {          // groups 8 lanes apart: a rotation within the row of 16
#pragma unroll
            for (int e = 0; e < N; ++e)
                v[e] += __uint_as_float((unsigned)__builtin_amdgcn_update_dpp(
                    0, (int)__float_as_uint(v[e]), 0x128 /* row_ror:8 */, 0xF, 0xF, false));
        }
        const int l = lane & (LPR - 1), rho = lane >> 4;
        const bool writer = LPR == 16 || (lane & 8) == 0;   // with LPR = 8 both halves of a row hold the sums
#pragma unroll
        for (int k = 0; k < N / 4; ++k) {
            const float r0 = pair_sum16(v[4 * k], v[4 * k + 1]);
            const float r1 = pair_sum16(v[4 * k + 2], v[4 * k + 3]);
            // rows 0, 2: columns 4k (r0) and 4k + 2 (r1); rows 1, 3: 4k + 1 and 4k + 3
            const float s = pair_sum32(r0, r1);
            // lower 32 lanes: r0's columns (4k + row), upper 32 lanes: r1's (4k + 2 + row - 2)
            if (writer) dst[combine_index<N, LPR>(l * N + 4 * k + ((rho & 1) | (rho & 2)))] = s;
        }
    }
}

// Sums the wavefronts' accumulators through LDS.  With one split the sums are
// the outputs.  Otherwise the block writes its fp32 partial row, and the block
// that arrives last at the tile's counter adds the partial rows of all splits
// in a fixed order (results do not depend on which block is last) and writes
// y.  The split-K combine of Section 4.4, without atomics on y and without a
// second launch.  The tile is columns [col0, col0 + cols) of y, cols <= TN.
// Returns (block-uniform) whether this block wrote the tile's outputs.
template <class F, int LPR, int WAVES>
__device__ __forceinline__ bool block_finish(float *red,
                                             float *partial, int *counters, float *y, int tile,
                                             int col0, int cols, int s, int splits, int n,
                                             const typename F::Args &a, int cnt,
                                             const SurvivorReport &report)
{
    constexpr int EPL = F::kElemsPerLane;
    constexpr int TN = LPR * EPL;
    constexpr int THREADS = WAVES * 64;
    constexpr int OWN = (TN + THREADS - 1) / THREADS;     // columns c = thread + k * THREADS
    __shared__ int last_flag;
    const int w = threadIdx.x >> 6;
    if (cols > n - col0) cols = n - col0;
    // What finish() needs per output column (the int8 scales) is loaded now, so that its
    // latency lies under the combine and not after the last sum.
    typename F::ColumnScale scale[OWN];
#pragma unroll
    for (int k = 0; k < OWN; ++k)
        scale[k] = F::column_scale(a, col0 + min((int)threadIdx.x + k * THREADS, cols - 1));
    __syncthreads();                   // every wavefront has left its sums in red[]
    trace_mark(7);
    constexpr int ROW = combine_row<EPL, LPR>;
    if (tile == 0 && threadIdx.x == 0) report_slice(report, s, splits, cnt);
    if (splits == 1) {
#pragma unroll
        for (int k = 0; k < OWN; ++k) {
            const int c = (int)threadIdx.x + k * THREADS;
            if (c < cols) {
                float sum = 0.f;
#pragma unroll
                for (int ww = 0; ww < WAVES; ++ww) sum += red[ww * ROW + combine_index<EPL, LPR>(c)];
                store_coherent(y + col0 + c, F::finish(sum, scale[k]));
            }
        }
        return true;
    }

    // The 8 XCDs have separate L2s.  A device-wide fence would write back and
    // invalidate a whole L2 per block; instead the partial rows themselves move
    // with device-coherent accesses (write-through stores, cache-bypassing
    // loads), ordered by the arrival counter: every thread waits for its stores
    // to complete, the block synchronises, then one thread takes the ticket.
    float *row = partial + (size_t)s * n + col0;
    for (int c = threadIdx.x; c < cols; c += THREADS) {
        float sum = 0.f;
#pragma unroll
        for (int ww = 0; ww < WAVES; ++ww) sum += red[ww * ROW + combine_index<EPL, LPR>(c)];
        store_coherent(row + c, sum);
    }
    wait_vector_memory();   // this thread's write-through stores have completed
    __syncthreads();
    trace_mark(4);
    // The ticket wraps: the arrival that finds splits - 1 puts the counter back to zero in the
    // same atomic, so the counter is ready for the next call without a second access.
    // (Relaxed: an agent-scope release here makes the compiler write the whole L2 back, an
    // acquire invalidates it; measured +1.0 .. +5 us and +0.5 .. +0.9 us per call.  The data
    // this ticket orders never sits in an L2: see store_coherent / load_coherent.)
    if (threadIdx.x == 0)
        last_flag = atomicInc(reinterpret_cast<unsigned *>(&counters[tile]), (unsigned)splits - 1u) ==
                    (unsigned)splits - 1u;
    __syncthreads();
    trace_mark(5);
    if (!last_flag) return false;
    if (tile == 0 && w == 0) report_total(report, splits);

    // Second pass.  A thread owns a column and adds its partial rows in split order (a fixed
    // order, whichever block happens to be last), up to 16 loads in flight at once.  (Spreading
    // the splits of a column over several threads and adding their sums through LDS costs two
    // more barriers and was measured slower by 0.3 us per Llama-2-7B block.)
    constexpr int MAXLD = 16;
#pragma unroll
    for (int k = 0; k < OWN; ++k) {
        const int c = k * THREADS + (int)threadIdx.x;
        if (c < cols) {
            const float *p = partial + col0 + c;
            float sum = 0.f;
            for (int j = 0; j < splits; j += MAXLD) {
                float v[MAXLD];
#pragma unroll
                for (int u = 0; u < MAXLD; ++u)
                    v[u] = j + u < splits ? load_coherent(p + (size_t)(j + u) * n) : 0.f;
#pragma unroll
                for (int u = 0; u < MAXLD; ++u) sum += v[u];
            }
            store_coherent(y + col0 + c, F::finish(sum, scale[k]));
        }
    }
    return true;
}

// This lane's first column: lane l of a row group covers EPL columns starting at
// col0 + l * EPL.  Lanes past the tile's (or the matrix's) right edge re-read
// the last valid vector: same cache line as a live lane, and their sums are
// never written.
template <int EPL>
__device__ __forceinline__ int lane_column(int col0, int cols, int n, int l)
{
    int c = l * EPL;
    if (c > cols - EPL) c = cols - EPL;
    int col = col0 + c;
    if (col > n - EPL) col = n - EPL;
    return col;
}

// Work of one block for formats with no per-group state (bf16, int8): output
// tile `tile` (tile_cols columns) x K-slice `s` (ks channels) of one matrix.
// Returns (block-uniform) whether this block wrote the tile's outputs.
template <class F, int LPR, int WAVES, int U, class XS>
__device__ __forceinline__ bool gemv_block(const typename F::Args &a, const XS &x,
                                           float t, float *partial, int *counters, float *y, int m,
                                           int n, int ks, int tile, int s, int tile_cols,
                                           int splits, const SurvivorReport &report)
{
    constexpr int EPL = F::kElemsPerLane;
    extern __shared__ __align__(16) unsigned char smem[];
    int2 *list = reinterpret_cast<int2 *>(smem);
    float *red = reinterpret_cast<float *>(smem + (size_t)ks * sizeof(int2));
    __shared__ int seg_cnt[kMaxSegs];

    const int k0 = s * ks;
    const int k1 = min(m, k0 + ks);
    int cnt;
    if constexpr (XS::kPlainHalf) {
        // short slices: each wavefront compacts its own share, no barrier before the stream
        const int nseg = (k1 - k0 + 63) >> 6;                 // block-uniform
        int seg_excl;
        if (nseg <= 8) {
            cnt = compact_slice_private<8, WAVES>(x.x, t, k0, k1, list, seg_excl);
        } else {
            // a slice longer than kMaxSlice is compacted in pieces of that length, one
            // behind the other in the list (block-uniform trip count)
            cnt = 0;
            for (int c0 = k0; c0 < k1; c0 += kMaxSlice)
                cnt += compact_slice<WAVES>(x, t, c0, min(k1, c0 + kMaxSlice), list + cnt, seg_cnt,
                                            seg_excl);
        }
    } else {
        int seg_excl;
        float prepared = 0.f;
        cnt = 0;
        for (int c0 = k0; c0 < k1; c0 += kMaxSlice)
            cnt += compact_slice<WAVES>(x, t, c0, min(k1, c0 + kMaxSlice), list + cnt, seg_cnt,
                                        seg_excl, &prepared, c0 != k0);
    }

    trace_mark(2);
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    int start, mine;
    wave_share(cnt, w, WAVES, start, mine);

    const int col0 = tile * tile_cols;
    const int col = lane_column<EPL>(col0, tile_cols, n, lane % LPR);
    const unsigned row_bytes = (unsigned)((size_t)(a.ld ? a.ld : n) * F::kBitsPerElem / 8);
    const unsigned char *lane_base =
        static_cast<const unsigned char *>(a.W) + (size_t)col * F::kBitsPerElem / 8;

    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
    stream_rows<F, LPR, U>(acc, list, start, mine, lane_base, row_bytes);
    trace_mark(3);
    trace_mark_thread(1, (WAVES - 1) * 64);
    store_wave_sums<LPR>(acc, red + (threadIdx.x >> 6) * combine_row<EPL, LPR>);
    return block_finish<F, LPR, WAVES>(red, partial, counters, y, tile, col0, tile_cols, s, splits,
                                       n, a, cnt, report);
}

// One matrix per launch.  Grid: tiles * splits blocks; block id -> (tile,
// split) with the tile index fastest, so that the blocks dealt round-robin to
// the 8 XCDs at any moment read neighbouring column ranges of the same rows,
// and every XCD gets the same number of blocks (+-1).  tile_cols (a multiple
// of EPL, <= LPR * EPL) is the width of an output tile.
template <class F, int LPR, int WAVES, int U>
__global__ __launch_bounds__(WAVES * 64) void sparse_gemv_kernel(
    typename F::Args a, const __half *__restrict__ x, float t, float *partial, int *counters,
    float *y, int m, int n, int ks, int tiles, int tile_cols, int splits)
{
    trace_mark(0);
    gemv_block<F, LPR, WAVES, U>(a, HalfSource{x}, t, partial, counters, y, m, n, ks,
                                 blockIdx.x % tiles, blockIdx.x / tiles, tile_cols, splits,
                                 survivor_report(counters, 0, splits));
    trace_mark(6);
}

// The W_down step with its input formed in the kernel from the two products that
// precede it (Appendix A.3): one launch instead of an element-wise kernel plus
// the product, and the intermediate never travels through HBM.
template <class F, int LPR, int WAVES, int U>
__global__ __launch_bounds__(WAVES * 64) void sparse_gemv_swiglu_kernel(
    typename F::Args a, const float *__restrict__ gate, const float *__restrict__ up, float t,
    float *partial, int *counters, float *y, int m, int n, int ks, int tiles, int tile_cols,
    int splits)
{
    gemv_block<F, LPR, WAVES, U>(a, SwigluSource{gate, up}, t, partial, counters, y, m, n, ks,
                                 blockIdx.x % tiles, blockIdx.x / tiles, tile_cols, splits,
                                 survivor_report(counters, 0, splits));
}

// Several matrices that read the same hidden state (q/k/v, or gate/up:
// Appendix A.3), each with its own threshold (the per-matrix sparsity levels of
// Section 4.2), in one launch: the launch latency and the serial ends of a
// call are paid once.  The matrices' tiles are laid side by side; a block
// finds its matrix from its tile index.
constexpr int kMaxMulti = 4;

template <class F>
struct MultiArgs {
    typename F::Args a[kMaxMulti];
    float *y[kMaxMulti];
    float t[kMaxMulti];
    int n[kMaxMulti];
    int tile_begin[kMaxMulti + 1];   // first tile of each matrix; [count] = all tiles
    int count;
};

template <class F, int LPR, int WAVES, int U, class XS>
__device__ __forceinline__ void multi_block(const MultiArgs<F> &ma, const XS &x, float *partial,
                                            int *counters, int m, int ks, int tile_cols, int splits,
                                            int block)
{
    const int tiles = ma.tile_begin[ma.count];
    const int gtile = block % tiles;
    const int s = block / tiles;
    int k = 0;
    size_t partial_off = 0;            // each matrix owns splits * n floats of partial rows
#pragma unroll
    for (int j = 1; j < kMaxMulti; ++j) {
        if (j < ma.count && gtile >= ma.tile_begin[j]) {
            partial_off += (size_t)splits * ma.n[j - 1];
            k = j;
        }
    }
    gemv_block<F, LPR, WAVES, U>(ma.a[k], x, ma.t[k], partial + partial_off,
                                 counters + ma.tile_begin[k], ma.y[k], m, ma.n[k], ks,
                                 gtile - ma.tile_begin[k], s, tile_cols, splits,
                                 survivor_report(counters, k, splits));
}

template <class F, int LPR, int WAVES, int U>
__global__ __launch_bounds__(WAVES * 64) void sparse_gemv_multi_kernel(
    MultiArgs<F> ma, const __half *__restrict__ x, float *partial, int *counters, int m, int ks,
    int tile_cols, int splits)
{
    multi_block<F, LPR, WAVES, U>(ma, HalfSource{x}, partial, counters, m, ks, tile_cols, splits,
                                  (int)blockIdx.x);
}

// The grouped launch with its shared input formed in the kernel from the hidden state
// before the normalisation layer: one launch instead of a normalisation kernel plus the
// products, and the normalised state never travels through HBM.  Every block reads all
// of h (from L2 after the first block of its XCD) for the scale, and its own slice of h
// and gamma, whose loads are issued first.
template <class F, int LPR, int U>
__global__ __launch_bounds__(kNormWaves * 64) void sparse_gemv_rmsnorm_multi_kernel(
    MultiArgs<F> ma, const float *__restrict__ h, const float *__restrict__ gamma, float eps,
    float *partial, int *counters, int m, int ks, int tile_cols, int splits)
{
    __shared__ double wave_sums[kMaxNormChunks * kNormWaves];
    multi_block<F, LPR, kNormWaves, U>(ma, RmsnormSource{h, gamma, m, eps, wave_sums}, partial,
                                       counters, m, ks, tile_cols, splits, (int)blockIdx.x);
}

// Several grouped calls that do not depend on each other (the projections of a bare stack
// of decoder blocks, Appendix A.3, each group with its own input) in one launch.  The
// groups' blocks follow each other in the grid, so the hardware starts a group's blocks
// as the blocks of the one before it retire: the ends of a call that leave most of the
// chip idle (compaction before the first weight load, the split-K combine, the gap to the
// next kernel) lie under another group's row stream.  Each group runs the block body of
// its own grouped launch with its own shape, workspace region and report.
constexpr int kMaxStack = kMaxStackGroups;

template <class F>
struct StackGroup {
    MultiArgs<F> ma;
    const __half *x;
    float *partial;
    int *counters;
    int m, ks, tile_cols, splits;
    int lanes_per_row;               // 16, 32 or 64
};

template <class F>
struct StackArgs {
    StackGroup<F> g[kMaxStack];
    int block_begin[kMaxStack + 1];  // first block of each group; [count] = grid size
    int count;
};

// The group of a block of a stack launch, and the block's index inside the group.
template <class F>
__device__ __forceinline__ int stack_group_of_block(const StackArgs<F> &sa, int &block)
{
    int k = 0;
#pragma unroll
    for (int j = 1; j < kMaxStack; ++j)
        if (j < sa.count && (int)blockIdx.x >= sa.block_begin[j]) k = j;
    block = (int)blockIdx.x - sa.block_begin[k];
    return k;
}

// LANES8: the format's launch shapes include 8 lanes per row (int8 weights).
template <class F, int WAVES, int U, bool LANES8>
__global__ __launch_bounds__(WAVES * 64) void sparse_gemv_stack_kernel(StackArgs<F> sa)
{
    int block;
    const StackGroup<F> &sg = sa.g[stack_group_of_block(sa, block)];
    const HalfSource x{sg.x};
    if (sg.lanes_per_row == 64)
        multi_block<F, 64, WAVES, U>(sg.ma, x, sg.partial, sg.counters, sg.m, sg.ks, sg.tile_cols,
                                     sg.splits, block);
    else if (sg.lanes_per_row == 32)
        multi_block<F, 32, WAVES, U>(sg.ma, x, sg.partial, sg.counters, sg.m, sg.ks, sg.tile_cols,
                                     sg.splits, block);
    else if (!LANES8 || sg.lanes_per_row == 16)
        multi_block<F, 16, WAVES, U>(sg.ma, x, sg.partial, sg.counters, sg.m, sg.ks, sg.tile_cols,
                                     sg.splits, block);
    else if constexpr (LANES8)
        multi_block<F, 8, WAVES, U>(sg.ma, x, sg.partial, sg.counters, sg.m, sg.ks, sg.tile_cols,
                                    sg.splits, block);
}

// A launch that asks for more dynamic LDS than the 64 KiB every kernel may use has to raise
// the kernel's limit first (a list of more than kMaxSlice entries).  Host side; false when
// the runtime refuses.
// The limit is raised once per kernel and device and remembered, so that later launches
// (also those recorded into a graph after a first eager call) make no runtime call here.
inline bool allow_large_lds_of(const void *kernel, size_t lds_bytes)
{
    if (lds_bytes <= 64 * 1024) return true;
    static std::mutex lock;
    static std::map<std::pair<int, const void *>, size_t> granted;
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return false;
    std::lock_guard<std::mutex> hold(lock);
    size_t &have = granted[{device, kernel}];
    if (have >= lds_bytes) return true;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) !=
        hipSuccess)
        return false;
    have = lds_bytes;
    return true;
}
template <class Kernel>
inline bool allow_large_lds(Kernel kernel, size_t lds_bytes)
{
    return allow_large_lds_of(reinterpret_cast<const void *>(kernel), lds_bytes);
}

// Host-side launch geometry shared by the formats.
struct GemvGeometry {
    int tiles;         // blocks along the output dimension
    int tile_cols;     // output columns per tile
    int ks;            // input channels per block
    int splits;        // blocks along the input dimension (may be below the request)
    size_t lds;        // dynamic LDS bytes
};

inline GemvGeometry gemv_geometry(int m, int n, const GemvShape &sh, int elems_per_lane,
                                  int ks_multiple, int max_slice = kMaxSlice)
{
    GemvGeometry g;
    const int tn = sh.lanes_per_row * elems_per_lane;
    g.tile_cols = sh.tile_cols > 0 ? sh.tile_cols : tn;
    g.tiles = (n + g.tile_cols - 1) / g.tile_cols;
    int splits = sh.splits < 1 ? 1 : sh.splits;
    int ks = (m + splits - 1) / splits;
    ks = (ks + ks_multiple - 1) / ks_multiple * ks_multiple;
    if (ks > max_slice) ks = max_slice;
    g.ks = ks;
    g.splits = (m + ks - 1) / ks;
    // list + one row of the combine buffer per wavefront (padded by one float per lane)
    g.lds = (size_t)ks * sizeof(int2) + (size_t)sh.waves * (tn + sh.lanes_per_row) * sizeof(float);
    return g;
}

// Host side of a stack launch, shared by the formats: checks the groups' shapes, orders the
// groups and fills the kernel's arguments; set_args(F::Args &, group, k) copies matrix k's
// format-specific pointers.  The groups are independent, so their place in the grid is
// free: those with the most weight bytes per block go first and the launch ends on short
// blocks (measured on Llama-2-7B shapes, bf16: 37 us against 40 us in q+k+v, o, gate+up,
// down order, and 42-46 us with gate+up last).
template <class F, class SetArgs>
hipError_t fill_stack_args(StackArgs<F> &sa, size_t &lds, int groups, const StackGroupDesc *d,
                           int ks_multiple, int min_lanes, int max_lanes, SetArgs set_args)
{
    if (groups < 1 || groups > kMaxStack) return hipErrorInvalidValue;
    sa.count = groups;
    sa.block_begin[0] = 0;
    lds = 0;
    GemvGeometry geo[kMaxStack];
    int order[kMaxStack];
    for (int gi = 0; gi < groups; ++gi) {
        const StackGroupDesc &dg = d[gi];
        GemvShape sh = dg.shape;
        const int lanes = sh.lanes_per_row;
        if (dg.count < 1 || dg.count > kMaxMulti || sh.unroll != 4 || sh.splits < 1 ||
            lanes < min_lanes || lanes > max_lanes || (lanes & (lanes - 1)) != 0 ||
            sh.tile_cols < 0 || sh.tile_cols % F::kElemsPerLane != 0 ||
            sh.tile_cols > lanes * F::kElemsPerLane)
            return hipErrorInvalidValue;
        sh.waves = 8;
        int n_max = 0;
        for (int k = 0; k < dg.count; ++k) n_max = dg.n[k] > n_max ? dg.n[k] : n_max;
        geo[gi] = gemv_geometry(dg.m, n_max, sh, F::kElemsPerLane, ks_multiple);
        const long long work = (long long)geo[gi].ks * geo[gi].tile_cols;
        int at = gi;                       // insertion sort, descending, stable
        while (at > 0 && (long long)geo[order[at - 1]].ks * geo[order[at - 1]].tile_cols < work) {
            order[at] = order[at - 1];
            --at;
        }
        order[at] = gi;
    }
    for (int gi = 0; gi < groups; ++gi) {
        const StackGroupDesc &dg = d[order[gi]];
        const GemvGeometry &g = geo[order[gi]];
        StackGroup<F> &sg = sa.g[gi];
        sg.ma.count = dg.count;
        sg.ma.tile_begin[0] = 0;
        for (int k = 0; k < dg.count; ++k) {
            set_args(sg.ma.a[k], dg, k);
            sg.ma.y[k] = dg.y[k];
            sg.ma.t[k] = dg.t[k];
            sg.ma.n[k] = dg.n[k];
            sg.ma.tile_begin[k + 1] =
                sg.ma.tile_begin[k] + (dg.n[k] + g.tile_cols - 1) / g.tile_cols;
        }
        sg.x = static_cast<const __half *>(dg.x_f16);
        sg.partial = dg.partial;
        sg.counters = dg.counters;
        sg.m = dg.m;
        sg.ks = g.ks;
        sg.tile_cols = g.tile_cols;
        sg.splits = g.splits;
        sg.lanes_per_row = dg.shape.lanes_per_row;
        const long long blocks = (long long)sg.ma.tile_begin[dg.count] * g.splits;
        if (sa.block_begin[gi] + blocks > 0x7fffffffLL) return hipErrorInvalidValue;
        sa.block_begin[gi + 1] = sa.block_begin[gi] + (int)blocks;
        lds = g.lds > lds ? g.lds : lds;
    }
    return hipSuccess;
}

}  // namespace teal
