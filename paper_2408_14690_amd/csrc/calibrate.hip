// Threshold calibration (Section 4.2): t_p is read off an empirical
// distribution of |x| built from activations collected offline.  fp16
// magnitudes have only 32768 bit patterns and non-negative fp16 values order
// like their bit patterns, so an exact histogram over the patterns yields the
// exact order statistic: no sorting, any number of batches.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>

#include "teal_internal.h"

namespace teal {

namespace {

constexpr int kBins = 32768;              // fp16 magnitude bit patterns
constexpr int kHistThreads = 1024;
constexpr int kHistBlocks = 256;          // one per compute unit: the 128 KB of counters fill most of its LDS
constexpr int kHistLoads = 8;             // 16-byte loads per batch; a thread keeps two batches in flight
constexpr unsigned kDumpBin = 0x7C01u;    // every NaN is counted here, and this counter is never flushed

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct HistBatch {
    u32x4 d[kHistLoads];
    __device__ __forceinline__ void load(const u32x4 *p, size_t stride)
    {
#pragma unroll
        for (int u = 0; u < kHistLoads; ++u) d[u] = __builtin_nontemporal_load(p + u * stride);
    }
};

// Every block counts its share of x in a private histogram of all 32768
// patterns in LDS (32-bit counters: a block never sees 2^32 values, the
// entry point bounds count), then adds the non-empty counters to the global
// 64-bit histogram.  NaNs are left out.  The next batch of loads is issued
// before the current one is counted, so the stream never drains.
__global__ __launch_bounds__(kHistThreads) void abs_histogram_kernel(
    const uint16_t *__restrict__ x, size_t count, unsigned long long *__restrict__ hist)
{
    extern __shared__ unsigned int lds_hist[];   // kBins counters
    for (int b = threadIdx.x; b < kBins; b += kHistThreads) lds_hist[b] = 0u;
    __syncthreads();

    // branch-free: patterns above +Inf (NaNs) collapse onto the dump counter
    auto add = [&](unsigned mag) { atomicAdd(&lds_hist[min(mag, kDumpBin)], 1u); };
    auto add8 = [&](const u32x4 d) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            add(d[q] & 0x7FFFu);
            add((d[q] >> 16) & 0x7FFFu);
        }
    };
    const size_t tid = (size_t)blockIdx.x * kHistThreads + threadIdx.x;
    const size_t nthreads = (size_t)gridDim.x * kHistThreads;
    // 16-byte loads over the aligned body, scalar loads over the ragged head and tail
    const size_t head = (size_t)((16 - ((uintptr_t)x & 15)) & 15) / 2;
    const size_t lead = head < count ? head : count;
    const size_t vecs = (count - lead) / 8;
    const u32x4 *xv = reinterpret_cast<const u32x4 *>(x + lead);
    // batch b of this thread covers vectors tid + (b kHistLoads + u) nthreads, u < kHistLoads
    const size_t stride = (size_t)kHistLoads * nthreads;
    const size_t reach = tid + (size_t)(kHistLoads - 1) * nthreads;     // last vector of batch 0
    const size_t batches = reach < vecs ? (vecs - 1 - reach) / stride + 1 : 0;
    if (batches) {
        HistBatch cur, nxt;
        cur.load(xv + tid, nthreads);
        for (size_t b = 1; b < batches; ++b) {
            nxt.load(xv + tid + b * stride, nthreads);
#pragma unroll
            for (int u = 0; u < kHistLoads; ++u) add8(cur.d[u]);
            cur = nxt;
        }
#pragma unroll
        for (int u = 0; u < kHistLoads; ++u) add8(cur.d[u]);
    }
    for (size_t v = tid + batches * stride; v < vecs; v += nthreads)
        add8(__builtin_nontemporal_load(xv + v));
    const size_t tail0 = lead + vecs * 8;
    for (size_t i = tid; i < lead; i += nthreads) add(x[i] & 0x7FFFu);
    for (size_t i = tail0 + tid; i < count; i += nthreads) add(x[i] & 0x7FFFu);
    __syncthreads();
    for (int b = threadIdx.x; b <= 0x7C00; b += kHistThreads) {
        const unsigned c = lds_hist[b];
        if (c) atomicAdd(&hist[b], (unsigned long long)c);
    }
}

constexpr int kMaxLevels = 16;
static_assert(kBins == 1024 * 32, "the threshold kernel gives 32 bins to each of 1024 threads");

struct Levels {
    double p[kMaxLevels];
    int count;
};

// One block.  Thread i owns bins [32 i, 32 i + 32); an LDS scan over the 1024
// per-thread totals gives each thread the number of samples below its bins;
// for each level the thread whose range contains rank k walks its 32 bins.
__global__ __launch_bounds__(1024) void histogram_thresholds_kernel(
    const unsigned long long *__restrict__ hist, Levels lv, float *__restrict__ t_out)
{
    __shared__ unsigned long long part[1024];
    const int tid = threadIdx.x;
    unsigned long long own[32];
    unsigned long long sum = 0;
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        own[j] = hist[tid * 32 + j];
        sum += own[j];
    }
    part[tid] = sum;
    __syncthreads();
    // Hillis-Steele inclusive scan over 1024 entries
    for (int d = 1; d < 1024; d <<= 1) {
        const unsigned long long v = tid >= d ? part[tid - d] : 0ull;
        __syncthreads();
        part[tid] += v;
        __syncthreads();
    }
    const unsigned long long total = part[1023];
    const unsigned long long below = part[tid] - sum;
    for (int l = 0; l < lv.count; ++l) {
        // rank k = ceil(p N - 1e-9), each operation rounded once (no fused multiply-add), so
        // that the integer decision is the one plain IEEE double arithmetic makes anywhere
        double k_real = ceil(__dadd_rn(__dmul_rn(lv.p[l], (double)total), -1e-9));
        if (k_real < 0.0) k_real = 0.0;
        if (k_real > (double)total) k_real = (double)total;
        const unsigned long long k = (unsigned long long)k_real;
        if (k == 0) {
            if (tid == 0) t_out[l] = 0.f;
            continue;
        }
        if (k > below && k <= below + sum) {
            unsigned long long c = below;
            int bin = tid * 32;
#pragma unroll
            for (int j = 0; j < 32; ++j) {
                c += own[j];
                if (c >= k) {
                    bin = tid * 32 + j;
                    break;
                }
            }
            t_out[l] = __half2float(__ushort_as_half((unsigned short)bin));
        }
    }
}

}  // namespace

hipError_t launch_abs_histogram(const void *x_f16, size_t count, unsigned long long *hist,
                                hipStream_t stream)
{
    if (count == 0) return hipSuccess;
    size_t want = (count / 8 + kHistThreads - 1) / kHistThreads;
    int blocks = want < 1 ? 1 : want > (size_t)kHistBlocks ? kHistBlocks : (int)want;
    hipLaunchKernelGGL(abs_histogram_kernel, dim3(blocks), dim3(kHistThreads),
                       kBins * sizeof(unsigned int), stream,
                       static_cast<const uint16_t *>(x_f16), count, hist);
    return hipGetLastError();
}

hipError_t launch_histogram_thresholds(const unsigned long long *hist, const double *p, int np,
                                       float *t_out, hipStream_t stream)
{
    Levels lv{};
    lv.count = np;
    for (int l = 0; l < np; ++l) lv.p[l] = p[l];
    hipLaunchKernelGGL(histogram_thresholds_kernel, dim3(1), dim3(1024), 0, stream, hist, lv, t_out);
    return hipGetLastError();
}

}  // namespace teal
