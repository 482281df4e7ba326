// Block schedule of the one-launch MLP (Appendix A.3: MLP(x) = (SiLU(x W_gate^T) . x W_up^T)
// W_down^T): which thread block does what, which blocks of W_down wait for which output
// tiles of W_gate / W_up.  Plain integer arithmetic shared by the kernel and the host (the
// host side is what the CPU tests of the schedule exercise), so the two cannot drift apart.
//
// Grid order.  First every block of the gate / up products, in phases: a phase covers
// `phase_tiles` consecutive output tiles of BOTH matrices (the same column range of gate and
// up, which is one contiguous range of the input of W_down) over all their K-slices; inside
// a phase the K-slice index is the slow one and the tiles (gate, up, gate, up, ...) the fast
// one.  Then every block of the W_down product, K-slice slow and output tile fast, so that
// the blocks that need the first columns of gate / up come first.  A consumer never
// precedes, in block order, a producer it waits for.
//
// Readiness.  A gate / up tile is finished when the block that combines its K-slices has
// written its columns of y; that block then adds one to the readiness counter of every
// block of W_down whose K-slice reads any of those columns (one counter per W_down block:
// a counter polled by one block only).  A block of W_down with K-slice s waits until its
// counter equals mlp_expected(s) = the number of gate and up tiles that overlap the slice.
#pragma once

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define TEAL_HD __host__ __device__
#else
#define TEAL_HD
#endif

namespace teal {

struct MlpGrid {
    int f;              // MLP width: columns of gate / up, input channels of W_down
    int tiles_gu;       // output tiles per matrix of the gate / up products
    int tile_cols_gu;
    int splits_gu;      // K-slices of the gate / up products
    int phase_tiles;    // tiles of each matrix per phase, 1..tiles_gu
    int tiles_d;        // output tiles of the W_down product
    int splits_d;       // its K-slices
    int ks_d;           // input channels per K-slice of W_down
};

enum MlpKind { kMlpGate = 0, kMlpUp = 1, kMlpDown = 2 };

struct MlpBlock {
    int kind;           // MlpKind
    int tile;           // output tile (of its matrix)
    int split;          // K-slice
};

TEAL_HD inline int mlp_blocks_gu(const MlpGrid &g) { return 2 * g.tiles_gu * g.splits_gu; }
TEAL_HD inline int mlp_blocks(const MlpGrid &g) { return mlp_blocks_gu(g) + g.tiles_d * g.splits_d; }

TEAL_HD inline MlpBlock mlp_block(const MlpGrid &g, int b)
{
    MlpBlock out;
    const int gu = mlp_blocks_gu(g);
    if (b < gu) {
        const int per_phase = 2 * g.phase_tiles * g.splits_gu;
        const int p = b / per_phase;
        const int r = b - p * per_phase;
        const int left = g.tiles_gu - p * g.phase_tiles;          // tiles of this and later phases
        const int here = left < g.phase_tiles ? left : g.phase_tiles;
        out.split = r / (2 * here);
        const int j = r - out.split * 2 * here;
        out.kind = j & 1;
        out.tile = p * g.phase_tiles + (j >> 1);
    } else {
        const int bd = b - gu;
        out.kind = kMlpDown;
        out.split = bd / g.tiles_d;
        out.tile = bd - out.split * g.tiles_d;
    }
    return out;
}

// K-slices [lo, hi] of W_down that read a column of gate / up tile `tile`.
TEAL_HD inline void mlp_signal_range(const MlpGrid &g, int tile, int &lo, int &hi)
{
    const int c0 = tile * g.tile_cols_gu;
    int c1 = c0 + g.tile_cols_gu;
    if (c1 > g.f) c1 = g.f;
    lo = c0 / g.ks_d;
    hi = (c1 - 1) / g.ks_d;
}

// Number of gate and up tiles a block of W_down with K-slice s waits for.
TEAL_HD inline int mlp_expected(const MlpGrid &g, int s)
{
    const int k0 = s * g.ks_d;
    int k1 = k0 + g.ks_d;
    if (k1 > g.f) k1 = g.f;
    return 2 * ((k1 - 1) / g.tile_cols_gu - k0 / g.tile_cols_gu + 1);
}

}  // namespace teal
