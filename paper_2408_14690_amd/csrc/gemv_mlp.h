// The MLP of a Transformer block in ONE launch (Appendix A.3):
//     MLP(x) = (SiLU(x W_gate^T) . x W_up^T) W_down^T,
// every product thresholded as in Section 4.2 (x for W_gate and W_up, each with its own
// threshold; the intermediate h = SiLU(gate) . up for W_down).  The three products keep the
// block bodies of their own kernels, so results are bitwise those of the grouped gate + up
// call followed by the W_down call with its input formed in the kernel, for the same launch
// shapes.  What changes is when things run: the blocks of W_down follow those of gate / up
// in the same grid and wait, per K-slice, for exactly the gate / up tiles they read
// (mlp_schedule.h), so the gap between two dependent launches disappears and the ends of
// the gate / up product that leave the chip idle (wavefront skew, split-K combine) lie
// under W_down's row stream, whose own start-up lies under theirs.
//
// Waiting is bounded: a block that does not see its inputs within `spin_limit` polls (or
// that sees that another block gave up) sets the status word and leaves; the call's outputs
// are then invalid and the workspace has to be zero-filled again.  Producers never wait, and
// every producer precedes its consumers in block order, so with blocks dispatched in index
// order every wait ends whatever the number of resident blocks.
#pragma once

#include "gemv_common.h"
#include "mlp_schedule.h"

namespace teal {

// Control area at the end of an MLP call's workspace: the status word (0 = fine, 1 = a wait
// expired), then one readiness counter per thread block of the W_down product, each on a
// 128-byte line of its own.  A counter is polled by exactly one block, so no two pollers ever
// ask for the same line (many pollers on one line were measured to slow every coherent
// access of the launch: the split-K publish of the producers took 3 us instead of 1.3), and
// the block that has seen its counter reach the value it waits for puts it back to zero
// itself: nothing else is needed to leave the area ready for the next call.
constexpr int kMlpLineInts = 32;
__host__ __device__ inline int mlp_ready_index(int consumer) { return kMlpLineInts * (1 + consumer); }

// gate and up as written by other blocks of the same launch: read past the local L2.
struct SwigluReadySource {
    static constexpr bool kHeavy = true;
    static constexpr bool kPlainHalf = false;
    typedef float2 Raw;
    const float *gate;
    const float *up;
    __device__ __forceinline__ Raw load(int i) const
    {
        return make_float2(load_coherent(gate + i), load_coherent(up + i));
    }
    __device__ __forceinline__ float prepare() const { return 0.f; }
    __device__ __forceinline__ float value(Raw r, float) const { return swiglu_value(r.x, r.y); }
};

template <class F>
struct MlpArgs {
    MlpGrid grid;
    // gate (0) and up (1)
    typename F::Args a_gu[2];
    float *y_gu[2];
    float t_gu[2];
    const __half *x;
    int m;                       // input channels of gate / up
    int ks_gu;
    float *partial_gu;           // [2][splits_gu][f]
    int *counters_gu;            // region of the gate / up products: counters, survivor report
    // down
    typename F::Args a_d;
    float *y_d;
    float t_d;
    int n_d;                     // output channels of W_down
    int tile_cols_d;
    float *partial_d;
    int *counters_d;             // region of the W_down product
    int *control;
    unsigned spin_limit;
};

// The block body of the formats without per-group state.
template <class F>
struct GemvBody {
    typedef F Format;
    template <int LPR, class XS>
    static __device__ __forceinline__ bool run(const typename F::Args &a, const XS &x, float t,
                                               float *partial, int *counters, float *y, int m,
                                               int n, int ks, int tile, int s, int tile_cols,
                                               int splits, const SurvivorReport &report)
    {
        return gemv_block<F, LPR, 8, 4>(a, x, t, partial, counters, y, m, n, ks, tile, s,
                                        tile_cols, splits, report);
    }
};

// Body::run<LPR>(...) is the format's block body (gemv_block or w4_block) and returns
// whether the block wrote its tile's outputs.
template <class Body, int LPR_GU, int LPR_D>
__global__ __launch_bounds__(8 * 64) void sparse_mlp_kernel(MlpArgs<typename Body::Format> A)
{
    const MlpGrid &g = A.grid;
    const MlpBlock blk = mlp_block(g, (int)blockIdx.x);
    trace_mark(0);
#ifdef TEAL_TRACE_BLOCKS
    // where the block runs: XCC_ID (hardware register 20, bits 3:0) and HW_ID (register 4)
    if (threadIdx.x == 0 && blockIdx.x < kTraceBlocks)
        teal_trace[blockIdx.x * kTraceMarks + 1] =
            ((unsigned long long)__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) << 32) |
            (unsigned)__builtin_amdgcn_s_getreg(4 | (0 << 6) | (31 << 11));
#endif
    if (blk.kind != kMlpDown) {
        const int k = blk.kind;
        const bool wrote = Body::template run<LPR_GU>(
            A.a_gu[k], HalfSource{A.x}, A.t_gu[k], A.partial_gu + (size_t)k * g.splits_gu * g.f,
            A.counters_gu + k * g.tiles_gu, A.y_gu[k], A.m, g.f, A.ks_gu, blk.tile, blk.split,
            g.tile_cols_gu, g.splits_gu, survivor_report(A.counters_gu, k, g.splits_gu));
        trace_mark(6);
        if (!wrote) return;
        // The tile's columns of gate / up are written (write-through stores): once every
        // thread's stores are acknowledged, tell the K-slices of W_down that read them.
        wait_vector_memory();
        __syncthreads();
        if (threadIdx.x < 64) {
            int lo, hi;
            mlp_signal_range(g, blk.tile, lo, hi);
            for (int s = lo; s <= hi; ++s)
                for (int j = threadIdx.x; j < g.tiles_d; j += 64)
                    __hip_atomic_fetch_add(A.control + mlp_ready_index(s * g.tiles_d + j), 1,
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        trace_mark(7);
        return;
    }

    __shared__ int inputs_ready;
    if (threadIdx.x == 0) {
        const int expected = mlp_expected(g, blk.split);
        int *ready = A.control + mlp_ready_index(blk.split * g.tiles_d + blk.tile);
        unsigned spins = 0;
        int ok = 0;
        for (;;) {
            if (load_coherent(ready) == expected) {
                ok = 1;
                break;
            }
            // the shared status word only now and then: it is one line for all blocks
            if (spins >= A.spin_limit || ((spins & 255u) == 255u && load_coherent(A.control) != 0))
                break;
            ++spins;
            __builtin_amdgcn_s_sleep(2);
        }
        if (ok) store_coherent(ready, 0);      // every producer has told: ready for the next call
        else store_coherent(A.control, 1);
        inputs_ready = ok;
    }
    __syncthreads();
    trace_mark(7);
    if (!inputs_ready) return;

    const bool wrote = Body::template run<LPR_D>(
        A.a_d, SwigluReadySource{A.y_gu[0], A.y_gu[1]}, A.t_d, A.partial_d, A.counters_d, A.y_d,
        g.f, A.n_d, g.ks_d, blk.tile, blk.split, A.tile_cols_d, g.splits_d,
        survivor_report(A.counters_d, 0, g.splits_d));
    trace_mark(6);
    (void)wrote;
}

// Host side.  Geometry of the two products from their launch shapes, argument block.
inline bool mlp_grid(MlpGrid &g, GemvGeometry &ggu, GemvGeometry &gd, const MlpLaunch &L, int m,
                     int f, int d, int elems_per_lane, int ks_multiple, int max_slice_gu = kMaxSlice)
{
    ggu = gemv_geometry(m, f, L.gu, elems_per_lane, ks_multiple, max_slice_gu);
    gd = gemv_geometry(f, d, L.down, elems_per_lane, ks_multiple);
    if ((long long)gd.tiles * gd.splits > kMlpMaxConsumers) return false;
    g.f = f;
    g.tiles_gu = ggu.tiles;
    g.tile_cols_gu = ggu.tile_cols;
    g.splits_gu = ggu.splits;
    g.phase_tiles = L.phase_tiles > 0 && L.phase_tiles < ggu.tiles ? L.phase_tiles : ggu.tiles;
    g.tiles_d = gd.tiles;
    g.splits_d = gd.splits;
    g.ks_d = gd.ks;
    const long long blocks = 2LL * ggu.tiles * ggu.splits + (long long)gd.tiles * gd.splits;
    return blocks <= 0x7fffffffLL;
}

template <class F, class SetArgs>
bool fill_mlp_args(MlpArgs<F> &A, size_t &lds, const MlpHostArgs &h, const MlpLaunch &L,
                   int ks_multiple, SetArgs set_args)
{
    GemvGeometry ggu, gd;
    // gate / up slices of up to kMaxLongSlice channels where the block body compacts in pieces
    if (!mlp_grid(A.grid, ggu, gd, L, h.m, h.f, h.d, F::kElemsPerLane, ks_multiple,
                  F::kBitsPerElem == 4 ? kMaxSlice : kMaxLongSlice))
        return false;
    set_args(A.a_gu[0], h.W_gate, h.scale_gate, h.gu_pitch);
    set_args(A.a_gu[1], h.W_up, h.scale_up, h.gu_pitch);
    set_args(A.a_d, h.W_down, h.scale_down, h.down_pitch);
    A.y_gu[0] = h.gate;
    A.y_gu[1] = h.up;
    A.t_gu[0] = h.t_gate;
    A.t_gu[1] = h.t_up;
    A.x = static_cast<const __half *>(h.x_f16);
    A.m = h.m;
    A.ks_gu = ggu.ks;
    A.partial_gu = h.partial_gu;
    A.counters_gu = h.counters_gu;
    A.y_d = h.y;
    A.t_d = h.t_down;
    A.n_d = h.d;
    A.tile_cols_d = gd.tile_cols;
    A.partial_d = h.partial_d;
    A.counters_d = h.counters_d;
    A.control = h.control;
    A.spin_limit = L.spin_limit;
    lds = (ggu.lds > gd.lds ? ggu.lds : gd.lds) + (size_t)(L.extra_lds > 0 ? L.extra_lds : 0);
    return true;
}

// Launch for lanes-per-row pairs out of {16, 32, 64} (LANES8: also 8, int8 weights).
template <class Body, bool LANES8>
hipError_t launch_mlp_kernel(const MlpArgs<typename Body::Format> &A, int lanes_gu, int lanes_d,
                             size_t lds, hipStream_t stream)
{
    const dim3 grid(mlp_blocks(A.grid)), block(8 * 64);
#define TEAL_MLP_LAUNCH(LG, LD)                                                                \
    do {                                                                                       \
        if (!allow_large_lds(sparse_mlp_kernel<Body, LG, LD>, lds)) return hipErrorInvalidValue; \
        hipLaunchKernelGGL((sparse_mlp_kernel<Body, LG, LD>), grid, block, lds, stream, A);   \
    } while (0)
#define TEAL_MLP_DOWN(LG)                                                                      \
    do {                                                                                       \
        if (lanes_d == 64) TEAL_MLP_LAUNCH(LG, 64);                                            \
        else if (lanes_d == 32) TEAL_MLP_LAUNCH(LG, 32);                                       \
        else if (lanes_d == 16) TEAL_MLP_LAUNCH(LG, 16);                                       \
        else if constexpr (LANES8) TEAL_MLP_LAUNCH(LG, 8);                                     \
    } while (0)
    const auto ok = [](int l) { return l == 64 || l == 32 || l == 16 || (LANES8 && l == 8); };
    if (!ok(lanes_gu) || !ok(lanes_d)) return hipErrorInvalidValue;
    if (lanes_gu == 64) TEAL_MLP_DOWN(64);
    else if (lanes_gu == 32) TEAL_MLP_DOWN(32);
    else if (lanes_gu == 16) TEAL_MLP_DOWN(16);
    else if constexpr (LANES8) TEAL_MLP_DOWN(8);
#undef TEAL_MLP_DOWN
#undef TEAL_MLP_LAUNCH
    return hipGetLastError();
}

// Checks of a launch shape for this kernel: 8 wavefronts, 4 loads per batch, tiles that fit
// the lanes.
inline bool mlp_shape_ok(const GemvShape &s, int elems_per_lane)
{
    return s.waves == 8 && s.unroll == 4 && s.splits >= 1 && s.tile_cols >= 0 &&
           s.tile_cols % elems_per_lane == 0 && s.tile_cols <= s.lanes_per_row * elems_per_lane;
}

}  // namespace teal
