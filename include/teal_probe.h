/*
 * teal_probe.h -- measurement aids of the library, kept apart from the method's
 * interface (teal.h): nothing here is needed to use the sparse products.
 */
#ifndef TEAL_PROBE_H
#define TEAL_PROBE_H

#include "teal.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Measurement aid, not part of the method: a plain streaming read of `bytes`
 * bytes at `buf` with the 16-byte non-temporal loads of the row stream and no
 * other work, by `blocks` thread blocks of 512 threads.  Section 3 argues that
 * decoding is bound by the rate at which weights can be moved; this gives the
 * rate a kernel that only reads reaches on the part for a launch of that
 * size, to set beside the published peak.  Each thread folds the words it
 * reads with XOR (which keeps the loads alive); a thread whose fold equals
 * `match` stores `match` to sink[its block index], so with a value that does
 * not occur nothing is written.
 *   buf    device memory, 16-byte aligned; bytes a multiple of 16, >= 16.
 *   blocks 1..65536.
 *   sink   [blocks] uint32, device memory.
 */
teal_status teal_stream_read_probe(const void *buf, size_t bytes, int blocks, uint32_t match,
                                   uint32_t *sink, void *stream);

#ifdef __cplusplus
}
#endif

#endif /* TEAL_PROBE_H */
