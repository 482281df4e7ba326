// Picks the kernel instantiation for a launch shape.  KERNEL(F, LPR, WAVES, U)
// must expand to a statement that launches that instantiation.
#pragma once

#define TEAL_DISPATCH_WU(KERNEL, F, LPR, sh)                                   \
    do {                                                                       \
        if ((sh).waves == 4 && (sh).unroll == 4) { KERNEL(F, LPR, 4, 4); }     \
        else if ((sh).waves == 4 && (sh).unroll == 8) { KERNEL(F, LPR, 4, 8); }\
        else if ((sh).waves == 8 && (sh).unroll == 4) { KERNEL(F, LPR, 8, 4); }\
        else if ((sh).waves == 8) { KERNEL(F, LPR, 8, 8); }                    \
        else { KERNEL(F, LPR, 16, 4); }                                        \
    } while (0)

#define TEAL_DISPATCH(KERNEL, F, sh)                                           \
    do {                                                                       \
        if ((sh).lanes_per_row == 64) TEAL_DISPATCH_WU(KERNEL, F, 64, sh);     \
        else if ((sh).lanes_per_row == 32) TEAL_DISPATCH_WU(KERNEL, F, 32, sh);\
        else if ((sh).lanes_per_row == 16) TEAL_DISPATCH_WU(KERNEL, F, 16, sh);\
        else TEAL_DISPATCH_WU(KERNEL, F, 8, sh);                               \
    } while (0)
