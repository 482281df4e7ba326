/*
 * teal.h -- C ABI of the MI355X (gfx950) library for TEAL's decode-time hot
 * path: magnitude thresholding of a hidden state fused with a matrix-vector
 * product that reads from HBM only the weight channels whose activation
 * survived.
 *
 * Notation (Section 3): x in R^m is the hidden state, W in R^{n x m} the
 * weight matrix ("out x in"), y = x W^T in R^n.  The sparsification function
 * of Definition 1 (Section 4.2) is s_t(x)_i = 0 if |x_i| <= t, else x_i, and
 * the layer forward is Y = s_t(x) W^T (Section 4.2).
 *
 * Storage.  W is kept input-channel-major ("column-major" in the wording of
 * Sections 3 and 4.4): Wt[m][n], row i = the n weights of input channel i,
 * contiguous.  A dropped channel is then one contiguous row that is never
 * fetched.
 *
 * Conventions for every call.
 *   - Every pointer is DEVICE memory owned by the caller, unless it says
 *     "host".  The library never allocates, frees or keeps a pointer.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work; results are valid once the caller has
 *     synchronised the stream.  Calls on one stream run in order.
 *   - x is IEEE binary16 (fp16).  t is fp32, finite and >= 0 (it is a
 *     quantile of |x|, Definition 1).  The comparison |x_i| > t is done in
 *     fp32 on exactly converted values, so it involves no rounding.  NaN in x
 *     compares false (dropped); +-Inf is kept.  t = 0 is the dense product
 *     (only entries equal to zero are skipped).
 *   - y is fp32, fully overwritten (all zeros when nothing survives).
 *     Products are formed and summed in fp32, in a fixed order: results are
 *     bitwise reproducible from run to run for a given shape.
 *   - All argument checks happen on the host before any GPU work and return
 *     a status; nothing aborts, throws or prints.
 *   - `workspace` is caller-provided device scratch of at least
 *     teal_workspace_bytes(m, n) bytes, 256-byte aligned.  It must be
 *     zero-filled once before its first use (hipMemset, torch.zeros); every
 *     call that returns TEAL_OK leaves it ready for the next call, of any
 *     shape that fits.  Its contents are otherwise the library's (the one
 *     part a caller may read is described under teal_survivors_offset).
 *     Calls that may run concurrently need distinct workspaces.
 *   - No global state; any host thread may call with any current device, as
 *     long as the pointers belong to it.
 */
#ifndef TEAL_H
#define TEAL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum teal_status {
    TEAL_OK = 0,
    TEAL_ERR_NULL = 1,        /* a required pointer is NULL */
    TEAL_ERR_SHAPE = 2,       /* m or n out of range or not a multiple of the format's vector width */
    TEAL_ERR_ALIGN = 3,       /* a pointer is not aligned as required */
    TEAL_ERR_THRESHOLD = 4,   /* t (or eps) is negative, NaN or infinite; a level p is outside [0, 1] */
    TEAL_ERR_WORKSPACE = 5,   /* workspace too small */
    TEAL_ERR_UNSUPPORTED = 6, /* group size or launch parameters not supported */
    TEAL_ERR_HIP = 7,         /* the HIP runtime reported an error at launch */
    TEAL_ERR_STATIC_LIMIT = 8 /* m or n beyond teal_static_scratch_limit() (static-scratch call) */
} teal_status;

/* Static, NUL-terminated description of a status (host memory, never freed). */
const char *teal_status_string(teal_status s);

/* Library version: major * 10000 + minor * 100 + patch. */
int teal_version(void);

/* Device scratch needed by any teal_sparse_gemv_* call with these dimensions.
 * Returns 0 if m or n is out of range. */
size_t teal_workspace_bytes(int m, int n);

/*
 * Realised sparsity of a call.  Section 4.2 fixes a target sparsity p per
 * matrix and estimates its threshold offline, so the share of entries a call
 * actually zeroes can drift from p with the inputs.  Every teal_sparse_gemv_*
 * call (all formats, grouped, batched, fused producer) leaves the number of
 * input channels that survived the threshold of its matrix k (k = 0 for calls
 * with one matrix) as an int32 at byte offset teal_survivors_offset() + 4 * k
 * of its workspace; realised sparsity = 1 - count / m.  The values are
 * complete when the call has completed on its stream and stay until the next
 * call on that workspace; the caller reads them as it reads any device memory.
 * They cost no extra launch and no extra pass over x: the thread blocks of a
 * matrix's first output tile report the counts of their slices, and the block
 * that finishes that tile adds them.
 */
size_t teal_survivors_offset(void);

/*
 * Definition 1 (Section 4.2) alone, as the mask s = [|x| > t] of Section 4.4.
 *   x_f16 [m] fp16 (2-byte aligned), 1 <= m < 2^31 (m = 0 is accepted: count = 0).
 *   mask  [m] bytes, 1 = kept, 0 = zeroed.                 May be NULL.
 *   idx   [m] int32 capacity; the first `count` entries are the kept
 *         positions in ascending order, the rest is untouched. May be NULL.
 *   count one int32: number of kept entries.               May be NULL.
 */
teal_status teal_sparsify(const void *x_f16, int m, float t,
                          uint8_t *mask, int32_t *idx, int32_t *count,
                          void *stream);

/*
 * y = s_t(x) W^T (Section 4.2), computed as in Section 4.4: the mask is built
 * inside the kernel from x and t, only rows Wt[i][:] with |x_i| > t are read,
 * the input dimension is split across thread blocks, and the per-split
 * partial sums (fp32) are combined in a fixed order by the block that
 * finishes a tile last (one kernel launch per call).
 *   Wt_bf16 [m][n] bfloat16, input-channel-major, 16-byte aligned.
 *   x_f16   [m] fp16, 2-byte aligned.
 *   y       [n] fp32, 4-byte aligned.
 *   1 <= m <= 2^24, 8 <= n <= 2^24, n % 8 == 0.
 */
teal_status teal_sparse_gemv_bf16(const void *Wt_bf16, const void *x_f16, float t,
                                  float *y, int m, int n,
                                  void *workspace, size_t workspace_bytes,
                                  void *stream);

/*
 * teal_sparse_gemv_bf16 for callers that cannot allocate device memory and so
 * have no workspace to hand over: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  The split-K scratch (arrival
 * counters, survivor report, fp32 partial rows) lives in an array of the
 * library's own, a file-scope device array of about 5.3 MB that every GPU the
 * library is used on holds until the process ends; the call itself calls no
 * hipMalloc, hipFree or other allocating routine, and no memset.  The device
 * address of the array is looked up once per device and kept: by
 * teal_static_scratch_init() (no arguments; the device to set up must be
 * current; TEAL_OK or TEAL_ERR_HIP), which a caller that captures graphs
 * calls before the capture, else by the device's first
 * teal_sparse_gemv_bf16_static call.
 *   Arguments, checks, launch shape and result as for teal_sparse_gemv_bf16
 *   (y is bitwise the same), except: m and n at most
 *   teal_static_scratch_limit() = 65536, beyond which the call returns
 *   TEAL_ERR_STATIC_LIMIT and does nothing.
 *   All calls on one GPU share that GPU's array: calls that may overlap in
 *   time on one GPU (different streams, different host threads) race on it and
 *   are NOT allowed; calls on one stream run in order and are fine.  The array
 *   keeps the last call's contents; what must be zero at the start of a call
 *   (one arrival counter per output tile) is left at zero by the call before
 *   it, and nothing else is read before it is written.  The survivor count of
 *   the call is not available to the caller.
 */
size_t teal_static_scratch_limit(void);
teal_status teal_static_scratch_init(void);
teal_status teal_sparse_gemv_bf16_static(const void *Wt_bf16, const void *x_f16, float t,
                                         float *y, int m, int n, void *stream);

/*
 * Several matrices that read the same hidden state, in one kernel launch:
 * y_k = s_{t_k}(x) W_k^T for k = 0 .. count-1.  Within a Transformer block
 * W_q, W_k, W_v share their input, and so do W_gate and W_up (Appendix A.3);
 * each matrix keeps its own threshold (the per-matrix sparsity levels of
 * Section 4.2).  Results are bitwise those of count separate calls of
 * teal_sparse_gemv_bf16_ex with the same launch shape.
 *   count   1..4.
 *   Wt_bf16, t, y, n   HOST arrays of length count: device pointers to the
 *           matrices ([m][n_k] bf16, 16-byte aligned), thresholds, device
 *           pointers to the outputs (y_k: n_k fp32) and the output widths
 *           (n_k % 8 == 0).  Read during the call only.
 *   x_f16   [m] fp16, shared.
 *   workspace  at least teal_workspace_bytes(m, n_0 + ... + n_{count-1}).
 */
teal_status teal_sparse_gemv_bf16_multi(int count, const void *const *Wt_bf16, const float *t,
                                        float *const *y, const int *n, const void *x_f16, int m,
                                        void *workspace, size_t workspace_bytes, void *stream);
/*
 * The same on matrices stored with padded rows (the layout
 * teal_pack_bf16_pitch writes; Sections 3 and 4.4 fix only that a channel's
 * weights are contiguous).  row_pitch is a HOST array of length count:
 * elements from one row of matrix k to the next, >= n_k and a multiple of 8
 * (else TEAL_ERR_SHAPE); matrix k spans (m - 1) * row_pitch[k] + n_k elements
 * and the padding is never read.  Same sums as the packed call; the launch
 * shape may differ (teal_gemv_plan_multi_pitch): with every row pitch an odd
 * multiple of 256 bytes (n + 128 elements where 2 n is a multiple of 1024) a
 * 256-byte tile of a row falls on a different quarter of a KiB on every row,
 * all tiles stream at the same speed, and a group with about one such tile
 * (of 256 bytes, else 512, else 128 for m <= 4096) per compute unit and
 * m <= 8192 runs without split-K.  A pitch that is not a multiple of 256
 * bytes is accepted but puts the wider tiles of other launch shapes off the
 * 128-byte lines of the memory system (measured 20-30 % slower).
 */
teal_status teal_sparse_gemv_bf16_multi_pitch(int count, const void *const *Wt_bf16,
                                              const int *row_pitch, const float *t,
                                              float *const *y, const int *n, const void *x_f16,
                                              int m, void *workspace, size_t workspace_bytes,
                                              void *stream);

/*
 * Several grouped calls that do not depend on each other, in one kernel
 * launch.  Group g is what teal_sparse_gemv_bf16_multi computes for its
 * counts[g] matrices and its own input x_g of length m_g; the results are
 * bitwise those of the groups' separate calls.  The case is a bare stack of
 * projections timed as kernels in isolation (as Section 4.4 times one
 * product; the shapes of Appendix A.3, every group with an input of its own,
 * nothing between the products): a group's
 * thread blocks start as those of the group before it retire, so the ends of
 * a call during which little memory traffic flows lie under another group's
 * weight rows.  There is NO ordering between the groups: no group may read
 * what another group of the same call writes, and no two outputs may overlap.
 * (Inside a decoder the projections do depend on each other and are issued as
 * separate grouped calls.)
 *   groups  1..16.
 *   counts  HOST array [groups]: matrices in each group, 1..4.
 *   Wt_bf16, t, y, n   HOST arrays over all matrices, group after group
 *           (length counts[0] + ... + counts[groups-1]), as for
 *           teal_sparse_gemv_bf16_multi.
 *   x_f16, m  HOST arrays [groups]: device pointer to each group's input and
 *           its length.
 *   workspace  at least teal_workspace_bytes_stack(groups, counts, n, m), zero
 *           before first use like every workspace.  The groups' regions follow
 *           each other; region g is laid out and sized like the workspace of
 *           group g's own call (teal_workspace_bytes(m_g, sum of its n)), so
 *           its survivor report sits teal_survivors_offset() bytes into it.
 * teal_workspace_bytes_stack returns 0 for dimensions out of range.
 */
size_t teal_workspace_bytes_stack(int groups, const int *counts, const int *n, const int *m);
teal_status teal_sparse_gemv_bf16_stack(int groups, const int *counts,
                                        const void *const *Wt_bf16, const float *t,
                                        float *const *y, const int *n, const void *const *x_f16,
                                        const int *m, void *workspace, size_t workspace_bytes,
                                        void *stream);
/*
 * The same for the quantised formats (Section 5.3): group g is what
 * teal_sparse_gemv_w8_multi / teal_sparse_gemv_w4_multi computes for it, bit
 * for bit.  Wq and scale_f16 are HOST arrays over all matrices, group after
 * group, with the layouts, alignments and width multiples (16 / 32) of those
 * calls; group == 128 and every m_g % 128 == 0 for int4 (else
 * TEAL_ERR_UNSUPPORTED).  Workspace as above.
 */
teal_status teal_sparse_gemv_w8_stack(int groups, const int *counts, const int8_t *const *Wq,
                                      const void *const *scale_f16, const float *t,
                                      float *const *y, const int *n, const void *const *x_f16,
                                      const int *m, void *workspace, size_t workspace_bytes,
                                      void *stream);
teal_status teal_sparse_gemv_w4_stack(int groups, const int *counts, const uint8_t *const *Wq,
                                      const void *const *scale_f16, int group, const float *t,
                                      float *const *y, const int *n, const void *const *x_f16,
                                      const int *m, void *workspace, size_t workspace_bytes,
                                      void *stream);

/*
 * The grouped call with its shared input formed on the fly from the hidden
 * state before the normalisation layer.  Appendix A.3 feeds W_q, W_k, W_v (and
 * W_gate, W_up) with the block's normalised hidden state (Section 4.1 relates
 * the zero-mean shape of these inputs to the normalisation); the paper prints
 * no formula for the layer, and the one taken here is the root-mean-square
 * normalisation of the models it evaluates (Section 5):
 *     x_i = gamma_i * h_i / sqrt(mean_j(h_j^2) + eps).
 * x decides the mask, so its arithmetic is part of the interface.  With h and
 * gamma binary32: ss = sum of the squares h_j^2 in binary64 (the squares are
 * exact there) by pairwise summation -- the index range [0, P), P the smallest
 * power of two >= m and entries past m zero, is halved recursively and the two
 * halves' sums are added, every addition rounded to binary64;
 * v = ss / m + eps and r = binary32(1 / sqrt(v)), both in binary64 with
 * correctly rounded division and square root; a = h_i * r, b = a * gamma_i in
 * binary32, each rounded to nearest even; x_i = binary16(b).  A NaN in h makes
 * every x_i NaN (all dropped); a NaN in gamma_i only x_i.
 *
 * teal_rmsnorm_f16: the producer alone, x_f16[i] for i < m.
 *   h [m] fp32, 16-byte aligned; gamma [m] fp32; x_f16 [m] fp16.
 *   8 <= m <= 16384, m % 8 == 0; eps finite and >= 0 (else TEAL_ERR_THRESHOLD).
 *
 * teal_sparse_gemv_bf16_rmsnorm_multi: y_k = s_{t_k}(x) W_k^T for
 * k = 0 .. count-1, bitwise what teal_rmsnorm_f16 followed by
 * teal_sparse_gemv_bf16_multi gives, in one launch and without x travelling
 * through memory (every thread block computes r from all of h, then forms only
 * the x_i of its slice).  Arguments as for teal_sparse_gemv_bf16_multi, with
 * h, gamma, eps and the range of m as above in place of x_f16.
 */
teal_status teal_rmsnorm_f16(const float *h, const float *gamma, float eps, void *x_f16, int m,
                             void *stream);
teal_status teal_sparse_gemv_bf16_rmsnorm_multi(int count, const void *const *Wt_bf16,
                                                const float *t, float *const *y, const int *n,
                                                const float *h, const float *gamma, float eps,
                                                int m, void *workspace, size_t workspace_bytes,
                                                void *stream);
/* On matrices with padded rows (row_pitch as for teal_sparse_gemv_bf16_multi_pitch): bitwise
 * teal_rmsnorm_f16 followed by teal_sparse_gemv_bf16_multi_pitch wherever that call's launch
 * shape has at least 16 lanes per row, else the sums of the packed call's shape. */
teal_status teal_sparse_gemv_bf16_rmsnorm_multi_pitch(int count, const void *const *Wt_bf16,
                                                      const int *row_pitch, const float *t,
                                                      float *const *y, const int *n,
                                                      const float *h, const float *gamma,
                                                      float eps, int m, void *workspace,
                                                      size_t workspace_bytes, void *stream);

/*
 * The W_down step with its input formed on the fly (Appendix A.3:
 * MLP(x) = (SiLU(x W_gate^T) . x W_up^T) W_down^T; Section 4.2 thresholds the
 * intermediate h = SiLU(g) . u like any other input).
 *
 * h_i = fp16(SiLU(gate_i) * up_i) in the following binary32 arithmetic, every
 * operation rounded to nearest even (the value decides the mask, so it is part
 * of the interface): z = clamp(-g, -80, 80); k = rint(z * 1.44269502f);
 * r = fma(k, -0.693145752f, z); r = fma(k, -1.42860677e-06f, r);
 * p = the degree-7 Taylor polynomial of exp at r by Horner's rule with fma;
 * e = p * 2^k; sigma = 1 / (1 + e); SiLU = g * sigma; h32 = SiLU * u;
 * h = binary16(h32).  NaN in g or u gives NaN (dropped).
 *
 * teal_swiglu_f16: the producer alone, h_f16[i] for i < m (0 <= m <= 2^24).
 *   gate, up [m] fp32, 4-byte aligned; h_f16 [m] fp16.
 *
 * teal_sparse_gemv_bf16_swiglu: y = s_t(h) W_down^T in one launch; results are
 * bitwise those of teal_swiglu_f16 followed by teal_sparse_gemv_bf16, without
 * the element-wise launch and without h travelling through HBM.
 *   Wt_bf16, t, y, m, n, workspace as for teal_sparse_gemv_bf16 (m = the MLP
 *   width, n = the model width).
 */
teal_status teal_swiglu_f16(const float *gate, const float *up, void *h_f16, int m, void *stream);
teal_status teal_sparse_gemv_bf16_swiglu(const void *Wt_bf16, const float *gate, const float *up,
                                         float t, float *y, int m, int n,
                                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same product for 8-bit channel-wise quantised weights (Section 5.3):
 * W[j][i] = Wq[i][j] * scale[j].
 *   Wq    [m][n] int8 (symmetric, two's complement), 16-byte aligned.
 *   scale [n] fp16, one per output channel, 2-byte aligned.
 *   n % 16 == 0; x, y and the ranges of m, n as for teal_sparse_gemv_bf16.
 */
teal_status teal_sparse_gemv_w8(const int8_t *Wq, const void *scale_f16,
                                const void *x_f16, float t, float *y, int m, int n,
                                void *workspace, size_t workspace_bytes,
                                void *stream);

/*
 * teal_sparse_gemv_bf16_multi for 8-bit channel-wise weights: count matrices
 * (1..4) that read the same hidden state, one kernel launch.  Wq, scale_f16, t,
 * y, n are HOST arrays of length count (device pointers / values per matrix,
 * formats as for teal_sparse_gemv_w8, n_k % 16 == 0).  Results are bitwise
 * those of separate calls with the same launch shape.  workspace of at least
 * teal_workspace_bytes(m, n_0 + ... + n_{count-1}).
 */
teal_status teal_sparse_gemv_w8_multi(int count, const int8_t *const *Wq,
                                      const void *const *scale_f16, const float *t,
                                      float *const *y, const int *n, const void *x_f16, int m,
                                      void *workspace, size_t workspace_bytes, void *stream);
/* With padded rows, as teal_sparse_gemv_bf16_multi_pitch: row_pitch[k] >= n_k
 * elements (bytes), a multiple of 16. */
teal_status teal_sparse_gemv_w8_multi_pitch(int count, const int8_t *const *Wq,
                                            const int *row_pitch, const void *const *scale_f16,
                                            const float *t, float *const *y, const int *n,
                                            const void *x_f16, int m, void *workspace,
                                            size_t workspace_bytes, void *stream);

/*
 * The 8-bit calls with their input formed on the fly, as for bf16 weights
 * (Section 5.3 combines the method with weight quantisation; Appendix A.3
 * gives the inputs): teal_sparse_gemv_w8_swiglu is teal_sparse_gemv_w8 on
 * h = fp16(SiLU(gate) * up), teal_sparse_gemv_w8_rmsnorm_multi is
 * teal_sparse_gemv_w8_multi on the normalised hidden state, both in the
 * arithmetic stated for teal_sparse_gemv_bf16_swiglu and
 * teal_sparse_gemv_bf16_rmsnorm_multi, in one launch, with results bitwise those
 * of the producer call followed by the plain 8-bit call.  Arguments as for those
 * calls, with Wq / scale_f16 in place of Wt_bf16 (n % 16 == 0).
 */
teal_status teal_sparse_gemv_w8_swiglu(const int8_t *Wq, const void *scale_f16, const float *gate,
                                       const float *up, float t, float *y, int m, int n,
                                       void *workspace, size_t workspace_bytes, void *stream);
teal_status teal_sparse_gemv_w8_rmsnorm_multi(int count, const int8_t *const *Wq,
                                              const void *const *scale_f16, const float *t,
                                              float *const *y, const int *n, const float *h,
                                              const float *gamma, float eps, int m,
                                              void *workspace, size_t workspace_bytes,
                                              void *stream);

/*
 * The same product for 4-bit group-quantised weights (Section 5.3):
 * W[j][i] = nibble(i, j) * scale[i / group][j].
 *   Wq    [m][n/2] bytes, two two's-complement nibbles per byte along the
 *         output axis, low nibble = even j; 16-byte aligned.
 *   scale [m/group][n] fp16, 16-byte aligned.
 *   group == 128, m % 128 == 0, n % 32 == 0; x, y and the ranges of m, n as
 *   for teal_sparse_gemv_bf16.
 */
teal_status teal_sparse_gemv_w4(const uint8_t *Wq, const void *scale_f16, int group,
                                const void *x_f16, float t, float *y, int m, int n,
                                void *workspace, size_t workspace_bytes,
                                void *stream);

/*
 * The 4-bit calls with their input formed on the fly, as for the other formats:
 * teal_sparse_gemv_w4_swiglu is teal_sparse_gemv_w4 on h = fp16(SiLU(gate) * up),
 * teal_sparse_gemv_w4_rmsnorm_multi is teal_sparse_gemv_w4_multi on the normalised
 * hidden state (arithmetic as stated for the bf16 calls), in one launch, with
 * results bitwise those of the producer call followed by the plain 4-bit call.
 * group == 128, m % 128 == 0 (and m <= 16384 for the normalised input).
 */
teal_status teal_sparse_gemv_w4_swiglu(const uint8_t *Wq, const void *scale_f16, int group,
                                       const float *gate, const float *up, float t, float *y,
                                       int m, int n, void *workspace, size_t workspace_bytes,
                                       void *stream);
teal_status teal_sparse_gemv_w4_rmsnorm_multi(int count, const uint8_t *const *Wq,
                                              const void *const *scale_f16, int group,
                                              const float *t, float *const *y, const int *n,
                                              const float *h, const float *gamma, float eps,
                                              int m, void *workspace, size_t workspace_bytes,
                                              void *stream);

/*
 * teal_sparse_gemv_bf16_multi for 4-bit group-quantised weights: count matrices
 * (1..4) that read the same hidden state, one kernel launch.  Wq, scale_f16, t,
 * y, n are HOST arrays of length count (device pointers / values per matrix,
 * formats as for teal_sparse_gemv_w4, n_k % 32 == 0); group == 128,
 * m % 128 == 0.  workspace of at least
 * teal_workspace_bytes(m, n_0 + ... + n_{count-1}).
 */
teal_status teal_sparse_gemv_w4_multi(int count, const uint8_t *const *Wq,
                                      const void *const *scale_f16, int group, const float *t,
                                      float *const *y, const int *n, const void *x_f16, int m,
                                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * The MLP of a Transformer block in ONE kernel launch (Appendix A.3):
 *     MLP(x) = (SiLU(x W_gate^T) . x W_up^T) W_down^T,
 * with every product thresholded (Section 4.2): gate = s_{t_gate}(x) W_gate^T,
 * up = s_{t_up}(x) W_up^T, h = fp16(SiLU(gate) * up) in the arithmetic stated for
 * teal_sparse_gemv_bf16_swiglu, y = s_{t_down}(h) W_down^T.  The results (gate,
 * up and y) are bitwise those of the separate calls with the same launch
 * shapes: teal_sparse_gemv_bf16_ex on W_gate and on W_up, teal_swiglu_f16, and
 * teal_sparse_gemv_bf16_ex on W_down (equally teal_sparse_gemv_bf16_multi and
 * teal_sparse_gemv_bf16_swiglu when the shapes are the ones those calls pick;
 * the shape the library picks here when `shape` is NULL is teal_mlp_plan's,
 * which for the gate / up products may differ from theirs).  The thread
 * blocks of the W_down product follow those of gate and up in the same grid and
 * each waits only for the gate / up output tiles that cover its own slice of h,
 * so nothing separates the dependent products but those waits.
 *   Wt_gate, Wt_up [m][f] bf16, Wt_down [f][d] bf16, input-channel-major,
 *           16-byte aligned.  m = model width, f = MLP width, d = output width.
 *   x_f16   [m] fp16.
 *   gate, up [f] fp32: written by the call (the intermediates; they must not
 *           overlap anything else the call reads or writes), y [d] fp32.
 *   1 <= m <= 2^24, 8 <= f <= 2^23, 8 <= d <= 2^24, f % 8 == 0, d % 8 == 0
 *   (16 for int8, 32 for int4 weights).
 *   workspace  at least teal_workspace_bytes_mlp(m, f, d) bytes, zero before
 *           first use like every workspace: the workspace of the gate + up
 *           call (survivor counts of gate and up at teal_survivors_offset()),
 *           that of the W_down call at byte teal_mlp_down_region_offset(m, f)
 *           (its survivor count teal_survivors_offset() bytes further), then
 *           the readiness counters and a status word.
 *   shape   HOST pointer, read during the call; NULL = the library's choice
 *           (teal_mlp_plan).  For tuning and tests: lanes per row, tile width
 *           and split count of the gate / up products and of the W_down
 *           product as for teal_sparse_gemv_bf16_ex (8 wavefronts, 4 loads per
 *           batch); gu_phase_tiles > 0 orders the gate / up blocks in phases
 *           of that many output tiles of each matrix, so that the first
 *           columns of gate and up are finished first (0 = one phase);
 *           extra_lds_bytes (0..49152) of unused shared memory per block lower
 *           the number of blocks resident per compute unit; spin_limit is the
 *           number of polls after which a waiting block gives up;
 *           gu_row_pitch / down_row_pitch: elements from one row of W_gate and
 *           W_up (of W_down) to the next, for matrices stored with padded
 *           rows: 0 = f (d), else >= f (d) and a multiple of 8 (16 for int8;
 *           int4 rows are always packed: must be 0).  The matrices then
 *           span m * gu_row_pitch (f * down_row_pitch) elements, the last
 *           row included.  A pitch of an odd multiple of 256 bytes (f + 128
 *           bf16 elements when 2 f is a multiple of 1024) spreads every
 *           block's reads evenly over the memory channels; shape == NULL
 *           means packed rows.
 * Waits are bounded.  A block of W_down that does not see its inputs within
 * spin_limit polls stores 1 to the int32 status word at byte
 * teal_mlp_status_offset(m, f, d) of the workspace and leaves, and so does
 * every block that then finds the word set: the kernel always ends.  A caller
 * that wants the guarantee reads the word after synchronising; when it is not
 * zero, gate / up / y are invalid and the workspace must be zero-filled again.
 * With thread blocks dispatched in index order (every producer precedes its
 * consumers in the grid, and producers never wait) no wait can expire.
 *
 * teal_sparse_mlp_w8 / teal_sparse_mlp_w4: the same for the quantised formats
 * (Section 5.3), matrices and scales as for teal_sparse_gemv_w8 /
 * teal_sparse_gemv_w4 (int4: group == 128, m % 128 == 0, f % 128 == 0), bitwise
 * the format's grouped call followed by its _swiglu call.
 *
 * teal_mlp_plan: the shape the library picks (HOST pointer, in and out): on entry
 * gu_row_pitch and down_row_pitch say how the caller stores the matrices (0 =
 * packed rows; they are left as they are, and a pitch the call would refuse
 * gives TEAL_ERR_UNSUPPORTED), the other fields are written.  On rows an odd
 * multiple of 256 bytes apart the gate / up products get the shape of
 * teal_sparse_gemv_bf16_multi_pitch where this kernel has it (narrow tiles
 * without split-K, slices of up to 8192 channels).
 * teal_mlp_block_info: host-only description of thread block `block` of the
 * launch a shape gives, for checking the schedule without a GPU.  info is a
 * HOST array of 8 ints: [0] blocks in the grid (always set; the rest is -1 when
 * `block` is out of range), [1] 0 = gate, 1 = up, 2 = down, [2] output tile,
 * [3] K-slice; for a gate / up block [4], [5] = the columns [c0, c1) of its
 * tile and [6], [7] = the first and last K-slice of W_down told when the tile
 * is finished; for a block of W_down [4], [5] = the input channels [k0, k1) of
 * its slice, [6] = its K-slice and [7] = the number of gate and up tiles it
 * waits for.
 */
typedef struct teal_mlp_shape {
    int gu_lanes_per_row, gu_tile_cols, gu_splits, gu_phase_tiles;
    int down_lanes_per_row, down_tile_cols, down_splits;
    int extra_lds_bytes;
    int spin_limit;
    int gu_row_pitch, down_row_pitch;
} teal_mlp_shape;
size_t teal_workspace_bytes_mlp(int m, int f, int d);
size_t teal_mlp_down_region_offset(int m, int f);
size_t teal_mlp_status_offset(int m, int f, int d);
teal_status teal_mlp_plan(int weight_bits, int m, int f, int d, teal_mlp_shape *shape);
teal_status teal_mlp_block_info(int weight_bits, int m, int f, int d, const teal_mlp_shape *shape,
                                int block, int *info);
teal_status teal_sparse_mlp_bf16(const void *Wt_gate, const void *Wt_up, const void *Wt_down,
                                 const void *x_f16, float t_gate, float t_up, float t_down,
                                 float *gate, float *up, float *y, int m, int f, int d,
                                 void *workspace, size_t workspace_bytes, void *stream,
                                 const teal_mlp_shape *shape);
teal_status teal_sparse_mlp_w8(const int8_t *Wq_gate, const int8_t *Wq_up, const int8_t *Wq_down,
                               const void *scale_gate, const void *scale_up,
                               const void *scale_down, const void *x_f16, float t_gate,
                               float t_up, float t_down, float *gate, float *up, float *y, int m,
                               int f, int d, void *workspace, size_t workspace_bytes,
                               void *stream, const teal_mlp_shape *shape);
teal_status teal_sparse_mlp_w4(const uint8_t *Wq_gate, const uint8_t *Wq_up,
                               const uint8_t *Wq_down, const void *scale_gate,
                               const void *scale_up, const void *scale_down, int group,
                               const void *x_f16, float t_gate, float t_up, float t_down,
                               float *gate, float *up, float *y, int m, int f, int d,
                               void *workspace, size_t workspace_bytes, void *stream,
                               const teal_mlp_shape *shape);

/*
 * One-time layout step (Sections 3 and 4.4: weights used under input sparsity
 * must be stored channel-contiguous): canonical row-major W[n][m] bf16 ->
 * Wt[m][n].  Device to device, out of place; both 2-byte aligned; any m, n >= 1.
 */
teal_status teal_pack_bf16(const void *W_rowmajor, void *Wt, int m, int n,
                           void *stream);
/*
 * The same with padded rows: element (i, j) of Wt goes to Wt[i * row_pitch + j],
 * row_pitch >= n elements (the layout teal_mlp_shape's row pitches describe).
 * Wt spans (m - 1) * row_pitch + n elements; the padding is left untouched.
 */
teal_status teal_pack_bf16_pitch(const void *W_rowmajor, void *Wt, int m, int n, int row_pitch,
                                 void *stream);

/*
 * teal_sparse_gemv_bf16 with the launch shape chosen by the caller instead
 * of by the library; for tuning and for tests that walk the kernel variants.
 * Results are identical in meaning (the summation order differs with the
 * shape).  0 means "library's choice" for each field.
 *   lanes_per_row  64, 32, 16 or 8: lanes that share one weight row per load
 *                  (each lane reads 16 bytes), i.e. an output tile of up to
 *                  512, 256, 128 or 64 columns per thread block.
 *   tile_cols      output columns per thread block: a multiple of 8, at most
 *                  8 * lanes_per_row.
 *   splits         1..128: thread blocks along the input dimension (split-K,
 *                  Section 4.4).  A block takes at most 8192 input channels
 *                  (the library's own choice stays at 4096 or fewer), so a
 *                  request below ceil(m / 8192) runs with that many splits.
 *   waves          4, 8 or 16 wavefronts per thread block.
 *   unroll         4 or 8 row loads per batch (two batches in flight per
 *                  wavefront); 4 with 16 wavefronts.
 * Unsupported combinations return TEAL_ERR_UNSUPPORTED.
 */
teal_status teal_sparse_gemv_bf16_ex(const void *Wt_bf16, const void *x_f16, float t,
                                     float *y, int m, int n,
                                     void *workspace, size_t workspace_bytes,
                                     void *stream,
                                     int lanes_per_row, int tile_cols, int splits, int waves,
                                     int unroll);

/*
 * Threshold calibration (Section 4.2: t_p is estimated from an empirical
 * distribution of activations collected offline).  fp16 magnitudes have 32768
 * bit patterns, ordered like the values, so an exact histogram over them gives
 * exact order statistics over any number of batches.
 *
 * teal_abs_histogram adds to hist[b] the number of entries of x whose
 * magnitude has bit pattern b (NaNs are left out; +-Inf is pattern 0x7C00).
 *   x_f16 [count] fp16, 0 <= count <= 2^38 (more returns TEAL_ERR_SHAPE).
 *   hist  [TEAL_HIST_BINS] uint64, device memory, 8-byte aligned, zero-filled
 *         by the caller before the first batch.
 *
 * teal_histogram_thresholds reads, for each level p[l] in [0, 1], the
 * threshold t[l] = the k-th smallest magnitude of the N samples counted,
 * k = ceil(p[l] N) (so that the fraction of samples with |x| <= t reaches p,
 * Definition 1); t[l] = 0 when k = 0.
 *   p  HOST array of np doubles, 1 <= np <= 16.
 *   t  device array of np floats (each an fp16 value, exactly).
 */
#define TEAL_HIST_BINS 32768
teal_status teal_abs_histogram(const void *x_f16, size_t count, uint64_t *hist, void *stream);
teal_status teal_histogram_thresholds(const uint64_t *hist, const double *p, int np, float *t,
                                      void *stream);

/*
 * Small batches (Section 5.4.4).  One set of channels is dropped for the whole
 * batch, chosen by the magnitude of the activations averaged over the batch
 * dimension; the criterion is still one threshold:
 *     channel i is kept  iff  (1 / batch) * sum_b |X[b][i]| > t.
 * It is evaluated as sum_b |X[b][i]| > batch * t in fp64, which is exact for
 * fp16 data (no division, no rounding, independent of the order of the rows).
 * A NaN in any row of a channel drops the channel; +-Inf keeps it.
 *   X_f16 [batch][m] fp16, one hidden state per row, 2-byte aligned.
 *   1 <= batch <= TEAL_MAX_BATCH.  batch = 1 is Definition 1.
 *
 * teal_sparsify_batch: mask / idx / count as for teal_sparsify, one mask for
 * the batch.
 *
 * teal_sparse_gemv_bf16_batch: Y[b][:] = (X[b][:] . s) W^T for every row b with
 * the batch-wide mask s; each surviving weight row is read once for the whole
 * batch.  Y is [batch][n] fp32, fully overwritten.  Wt, m, n as for
 * teal_sparse_gemv_bf16; workspace of at least
 * teal_workspace_bytes_batch(m, n, batch) bytes, same rules as above.
 *
 * teal_sparse_gemv_bf16_batch_ex: the same with a caller-chosen launch shape
 * (0 = library's choice): lanes_per_row 64, 32 or 16 with
 * lanes_per_row * B <= 256, B = batch rounded up to 2, 4 or 8; tile_cols a
 * multiple of 8, at most 8 * lanes_per_row; splits such that a block's slice,
 * ceil(m / splits) rounded up to 64, is at most 2048 channels.
 *
 * teal_sparse_gemv_bf16_batch_multi: count (1..4) matrices that read the same
 * batch, one kernel launch, each matrix with its own threshold; Wt_bf16, t, Y, n
 * are HOST arrays of length count as for teal_sparse_gemv_bf16_multi (Y_k is
 * [batch][n_k]).  workspace of at least
 * teal_workspace_bytes_batch(m, n_0 + ... + n_{count-1}, batch).
 */
#define TEAL_MAX_BATCH 8
size_t teal_workspace_bytes_batch(int m, int n, int batch);
teal_status teal_sparsify_batch(const void *X_f16, int batch, int m, float t,
                                uint8_t *mask, int32_t *idx, int32_t *count, void *stream);
teal_status teal_sparse_gemv_bf16_batch(const void *Wt_bf16, const void *X_f16, int batch,
                                        float t, float *Y, int m, int n,
                                        void *workspace, size_t workspace_bytes, void *stream);
teal_status teal_sparse_gemv_bf16_batch_ex(const void *Wt_bf16, const void *X_f16, int batch,
                                           float t, float *Y, int m, int n,
                                           void *workspace, size_t workspace_bytes, void *stream,
                                           int lanes_per_row, int tile_cols, int splits);
teal_status teal_sparse_gemv_bf16_batch_multi(int count, const void *const *Wt_bf16,
                                              const float *t, float *const *Y, const int *n,
                                              const void *X_f16, int batch, int m,
                                              void *workspace, size_t workspace_bytes,
                                              void *stream);

/*
 * The launch shape the library chooses for teal_sparse_gemv_{bf16,w8,w4} at
 * these dimensions (weight_bits = 16, 8 or 4), in the terms of
 * teal_sparse_gemv_bf16_ex.  Host-only; every output pointer is HOST memory
 * and may be NULL.  Split-K (Section 4.4) is `splits` blocks along the input
 * dimension; the grid is ceil(n / tile_cols) * splits blocks.
 */
teal_status teal_gemv_plan(int weight_bits, int m, int n, int *lanes_per_row, int *tile_cols,
                           int *splits, int *waves, int *unroll);

/*
 * The same for a grouped launch (teal_sparse_gemv_{bf16,w8,w4}_multi) of count
 * matrices of widths n[0..count-1] (HOST array): the tile width is chosen so that
 * the matrices divide evenly and the blocks fill the chip once.
 */
teal_status teal_gemv_plan_multi(int weight_bits, int m, const int *n, int count,
                                 int *lanes_per_row, int *tile_cols, int *splits, int *waves,
                                 int *unroll);
/* The same for teal_sparse_gemv_{bf16,w8}_multi_pitch (weight_bits 16 or 8;
 * row_pitch a HOST array of length count). */
teal_status teal_gemv_plan_multi_pitch(int weight_bits, int m, const int *n, const int *row_pitch,
                                       int count, int *lanes_per_row, int *tile_cols, int *splits,
                                       int *waves, int *unroll);

#ifdef __cplusplus
}
#endif

#endif /* TEAL_H */
