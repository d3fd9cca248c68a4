/*
 * libzipml -- double-sampled low-precision minibatch SGD for least squares on AMD MI355X (gfx950).
 *
 * The method is that of "ZipML: Training Models with End-to-End Low Precision"
 * (arXiv 1611.05402): every sample row is stochastically quantised twice, independently, to
 * b-bit per-feature levels (Sec. 2.1, Supp. A.3), and each minibatch step uses the unbiased
 * double-sampled gradient  g = mean_i Q1(a_i) (Q2(a_i)^T x - b_i)  (Sec. 2.2, eq. (5)), optionally
 * with the model and the gradient stochastically quantised as well (Supp. C-E).
 *
 * General conventions
 *   - Plain C ABI.  Pointers named *_dev are DEVICE pointers owned by the caller; the library never
 *     allocates or frees device memory and keeps no pointer after a call returns.  Pointers named
 *     *_host are host pointers.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All device work is
 *     enqueued on it.  Calls that return a host value (zipml_loss, zipml_sgd_status, the OPTIMAL
 *     mode of zipml_levels) synchronise that stream; every other call is asynchronous.
 *   - Every call returns ZIPML_OK (0) or a negative error code; nothing aborts or throws across the
 *     boundary.  Argument errors are detected before any work is enqueued.
 *   - A is row-major fp32 with leading dimension lda >= d.  Level tables are [d][2^bits] fp32,
 *     non-decreasing along the second axis.  All device pointers must be 16-byte aligned.
 *   - The packed layout of the quantised copies is private to the library (copy 1 is stored
 *     feature-major for the gradient pass, copy 2 sample-major for the dot-product pass, both in
 *     units of 32 codes); zipml_unpack_codes is its only definition.
 *   - Random numbers: Philox4x32-10, key = seed, counter = (row, feature / 4, epoch * 256 + stream),
 *     output word feature % 4, the top 24 bits as a uniform in [0,1).  Streams 1, 2 are the two
 *     sample quantisations (row = sample index), 3 and 4 the model and gradient quantisations
 *     (row = step index within the epoch).  epoch must be < 2^24.
 */
#ifndef ZIPML_H
#define ZIPML_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- status codes ------------------------------------------------------------------------- */
#define ZIPML_OK            0
#define ZIPML_EINVAL       -1   /* bad argument value (sizes, bits, batch, NULL pointer)          */
#define ZIPML_EALIGN       -2   /* a device pointer is not 16-byte aligned                        */
#define ZIPML_ERANGE       -3   /* integer dot product could overflow int32 for these sizes       */
#define ZIPML_EWORKSPACE   -4   /* workspace missing or smaller than zipml_workspace_bytes()      */
#define ZIPML_ELAUNCH      -5   /* the HIP runtime refused a launch or copy                       */
#define ZIPML_EUNSUPPORTED -6   /* valid request that this build does not implement               */
#define ZIPML_ETIMEOUT     -7   /* a grid-wide wait inside the epoch kernel gave up               */

/* ---- modes and flags ---------------------------------------------------------------------- */
#define ZIPML_UNIFORM 0          /* 2^bits evenly spaced levels on [lo_j, hi_j]    (Sec. 2.1)     */
#define ZIPML_OPTIMAL 1          /* variance-optimal levels by dynamic programming (Sec. 3)       */
#define ZIPML_GREEDY 2           /* the same over the candidates a greedy search leaves (Sec. 3.2) */

#define ZIPML_RANGE_GIVEN 1      /* zipml_levels: lo_dev / hi_dev are inputs                      */
#define ZIPML_SYMMETRIC   2      /* zipml_levels: range [-M_j, M_j], M_j = max(|min|, |max|)
                                    (Supp. A.3 "Column Scaling")                                  */

#define ZIPML_SGD_STEPWISE 1     /* zipml_sgd_epoch: two launches per step instead of one
                                    persistent launch per epoch (same arithmetic)                 */
#define ZIPML_SGD_AVERAGED 2     /* zipml_sgd_epoch: the averaged estimator
                                    1/2 [Q1 (Q2^T x - b) + Q2 (Q1^T x - b)]  (Supp. B.2, footnote) */
#define ZIPML_SGD_PRODUCTION 4   /* zipml_debug_step: run the step in the launch and step loop that
                                    zipml_sgd_epoch takes for this shape (see zipml_debug_step)     */

const char *zipml_strerror(int code);

/* Bytes of ONE packed copy of an n x d matrix at `bits` bits per value, padding included
 * (n is rounded up to a multiple of 64, d to a multiple of 32).  0 if the arguments are invalid. */
size_t zipml_packed_bytes(int64_t n, int64_t d, int bits);

/* Bytes of device workspace that zipml_levels, zipml_sgd_epoch, zipml_debug_step and zipml_loss
 * need for a problem of this shape (one buffer serves all of them, one call at a time).
 * n_candidates may be 0 if neither ZIPML_OPTIMAL nor ZIPML_GREEDY is used (with it, the size
 * includes the bin moments, 24 d n_candidates bytes, and 64 MiB for partial copies of them). */
size_t zipml_workspace_bytes(int64_t n, int64_t d, int bits, int64_t batch, int n_candidates);

/* Per-feature quantisation levels.
 *   Sec. 2.1 (levels partition the scaled range), Supp. A.3 "Column Scaling" (one range per
 *   feature from the column min/max), Sec. 3.1-3.2 (variance-optimal levels: one scan of the data
 *   into n_candidates equal bins per feature, then the dynamic program T(k,m) on the bin edges).
 * Unless ZIPML_RANGE_GIVEN, lo_dev[d] / hi_dev[d] are written with the column ranges.
 * levels_dev[d][2^bits] is written.  grid_idx_dev[d][2^bits] (optional, may be NULL) receives the
 * integer grid position of every level: c for UNIFORM, the chosen bin edge for OPTIMAL, so that
 * level = lo_j + (hi_j - lo_j) * grid_idx / grid_max with grid_max = 2^bits - 1 or n_candidates.
 * mean_variance_host (optional, OPTIMAL and GREEDY only) receives the objective of eq. (6)
 * averaged over features.  UNIFORM is asynchronous.  OPTIMAL runs the dynamic program on the device
 * when its tables fit in on-chip memory (then only a request for mean_variance_host synchronises
 * the stream); otherwise it copies the bin moments to the host, runs the dynamic program on the
 * host cores and copies the levels back, which synchronises the stream.
 * GREEDY (Sec. 3.2, "2-Approximation in Almost-Linear Time"; supplement, Algorithm 1 with
 * gamma = 1, delta = 1): the bins are first merged greedily into at most 4 (2^bits - 1) + 1
 * intervals per feature, whose end points are the only candidates of the dynamic program; the
 * levels are within the factor the paper gives of OPTIMAL's, for a dynamic program over ~4 * 2^bits
 * instead of n_candidates points.  With n_candidates <= 4 (2^bits - 1) + 1 it is OPTIMAL.  Device
 * only: ZIPML_EUNSUPPORTED if the tables do not fit (8 bits with more than 1021 candidates).
 * bits in 1..8; OPTIMAL and GREEDY need 2^bits - 1 <= n_candidates <= 4096. */
int zipml_levels(void *stream, const float *A_dev, int64_t n, int64_t d, int64_t lda, int bits,
                 int mode, int flags, int n_candidates, float *lo_dev, float *hi_dev,
                 float *levels_dev, uint16_t *grid_idx_dev, double *mean_variance_host,
                 void *workspace_dev, size_t workspace_bytes);

/* Two independent stochastic quantisations of rows [row0, row0 + n_rows) of an n_total x d matrix
 * (Sec. 2.1: value v between neighbouring levels l <= v <= u goes to u with probability
 * (v - l)/(u - l), evaluated in fp32; Sec. 2.2: two independent copies).  A_dev points at the
 * first of the n_rows rows.  Values outside the level range are clamped to it.  packed1_dev and
 * packed2_dev each hold zipml_packed_bytes(n_total, d, bits) bytes; calls for disjoint row ranges
 * fill disjoint parts, so a large matrix can be quantised chunk by chunk.  row0 must be a multiple
 * of 32, and so must n_rows unless the chunk ends at n_total. */
int zipml_quantize(void *stream, const float *A_dev, int64_t n_rows, int64_t d, int64_t lda,
                   int64_t row0, int64_t n_total, const float *levels_dev, int bits, uint64_t seed,
                   uint32_t epoch, void *packed1_dev, void *packed2_dev);

/* The same two copies in the other layout each, for the symmetrised estimator: packed1s_dev gets
 * copy 2 in the layout of packed1, packed2s_dev copy 1 in the layout of packed2.  The draws are
 * those of zipml_quantize with the same (seed, epoch): zipml_unpack_codes(packed1s, copy = 1)
 * returns the codes of copy 2, and (packed2s, copy = 2) those of copy 1. */
int zipml_quantize_swapped(void *stream, const float *A_dev, int64_t n_rows, int64_t d, int64_t lda,
                           int64_t row0, int64_t n_total, const float *levels_dev, int bits,
                           uint64_t seed, uint32_t epoch, void *packed1s_dev, void *packed2s_dev);

/* Compact storage of the two samples (Sec. 2.2, "Overhead of Storing Samples"): the two
 * quantisations of a value differ by at most one level, so a base level and one bit per sample
 * hold both, bits + 2 bits per value instead of 2 * bits.  packed_a_dev and packed_b_dev are the
 * two copies in the SAME layout -- (packed2s, packed2): copy 1 and copy 2 sample-major, or
 * (packed1, packed1s): copy 1 and copy 2 feature-major, see zipml_quantize_swapped -- and
 * compact_dev holds zipml_compact_bytes(n, d, bits) bytes in two planes: first the smaller of the
 * two codes of every value, a packed array in the layout of the copies (bits / (bits + 2) of the
 * record); then, per unit of 32 values in the same order, a pair of dwords of bits saying which
 * values of copy a / copy b sit one level above it.  A storage and transfer format, restored bit
 * for bit by zipml_compact_decode; zipml_sgd_epoch_compact runs on the sample-major record as it is.  zipml_compact_encode synchronises the stream and
 * returns ZIPML_EINVAL if some pair of codes differs by more than one level (the arrays are then
 * not two samples of the same values); it uses 256 bytes of workspace. */
size_t zipml_compact_bytes(int64_t n, int64_t d, int bits);
int zipml_compact_encode(void *stream, const void *packed_a_dev, const void *packed_b_dev, int64_t n,
                         int64_t d, int bits, void *compact_dev, void *workspace_dev,
                         size_t workspace_bytes);
int zipml_compact_decode(void *stream, const void *compact_dev, int64_t n, int64_t d, int bits,
                         void *packed_a_dev, void *packed_b_dev);

/* zipml_sgd_epoch for very large minibatches reading the COMPACT record alone (Sec. 2.2, "Overhead
 * of Storing Samples"): compact_dev is what zipml_compact_encode writes for the two copies in the
 * sample-major layout, (packed2s, packed2) -- copy 1 from zipml_quantize_swapped, copy 2 from
 * zipml_quantize.  A step then reads bits + 2 instead of 2 * bits bits per value; the gradient pass
 * turns its operand on the chip.  Same estimator and arithmetic as zipml_sgd_epoch on the packed
 * copies (the model after the epoch is bit-identical).  Built for bits = 8, evenly spaced levels,
 * the fp32 model, minibatches of at least 16384 samples (a multiple of 64) and 513 to 2048
 * features; ZIPML_EUNSUPPORTED otherwise (for level tables that turn out not to be evenly spaced:
 * through zipml_sgd_status).  Asynchronous; workspace as for zipml_sgd_epoch. */
int zipml_sgd_epoch_compact(void *stream, const void *compact_dev, const float *levels_dev,
                            const float *b_dev, int64_t n, int64_t d, int bits, float *x_dev,
                            int64_t batch, float lr, void *workspace_dev, size_t workspace_bytes);

/* One epoch of double-sampled minibatch SGD on F(x) = 1/(2n) sum_i (a_i^T x - b_i)^2
 * (Sec. 2 and eq. (5); the minibatch gradient is the mean over `batch` consecutive samples; the
 * n / batch steps run in storage order).  x_dev[d] is the fp32 master model, updated in place:
 * x <- x - lr * g every step (Supp. E: the update is in full precision).
 *   model_bits = grad_bits = 0: full-precision (fp32) model, residuals and gradient.  The sums
 *     over features and over samples are accumulated as integers (fixed-point partial sums, and
 *     for evenly spaced 2-, 4- or 8-bit levels exact integer sums of codes times fixed-point
 *     digits), so the result does not depend on the order in which workgroups finish: two calls
 *     with the same arguments give the same bits.
 *   model_bits in 2..8: the model is stochastically quantised each step with row scaling
 *     (Supp. A.3 eq. (quant2), Supp. C), s = 2^(model_bits-1) - 1 magnitude intervals, and the dot
 *     product becomes an exact integer sum of grid_idx * model code; this needs grid_idx_dev and a
 *     level grid shared by all features: level value = grid_lo + grid_step * grid_idx.
 *   grad_bits in 2..8 (needs model_bits > 0): the mean gradient is quantised the same way before
 *     the update (Supp. D, E).
 * grid_max is the largest grid index (2^bits - 1 for UNIFORM levels, n_candidates for OPTIMAL);
 * ZIPML_ERANGE if grid_max * s * d could exceed int32.
 * batch must divide n and be 4, 8, 16 or a multiple of 32.  A minibatch of up to 2048 / GQ samples
 * (GQ = 1, 2 or 4 groups of 32 features per workgroup; 1024 samples at d = 2048) is one exchange
 * between the workgroups; larger ones -- up to the whole data set, i.e. gradient descent with
 * double sampling -- are supported for the fp32 model with evenly spaced 2-, 4- or 8-bit levels
 * and batch a multiple of 64 (taken in chunks by replicas of the workgroups, or by workgroups that
 * own samples instead of features); otherwise ZIPML_EUNSUPPORTED, which for level tables that
 * turn out not to be evenly spaced arrives through zipml_sgd_status with x_dev left untouched.
 * The call is asynchronous; a failed grid-wide wait is reported by zipml_sgd_status (ZIPML_ETIMEOUT):
 * the kernel then still runs to its end, and x_dev holds undefined values afterwards.
 * The workgroups of an epoch kernel wait for each other, so they must all be resident at once: the
 * library sizes the grid for that and refuses the launch (ZIPML_ELAUNCH) if the device cannot hold
 * it, but kernels of other streams that occupy the compute units at the same time can still keep
 * workgroups out -- two epoch calls on different streams of one device must not overlap; if they do,
 * the waits give up (ZIPML_ETIMEOUT) rather than hang. */
int zipml_sgd_epoch(void *stream, const void *packed1_dev, const void *packed2_dev,
                    const float *levels_dev, const uint16_t *grid_idx_dev, float grid_lo,
                    float grid_step, int grid_max, const float *b_dev, int64_t n, int64_t d,
                    int bits, float *x_dev, int64_t batch, float lr, int grad_bits, int model_bits,
                    uint64_t seed, uint32_t epoch, int flags, void *workspace_dev,
                    size_t workspace_bytes);

/* The same epoch for the least-squares SVM objective
 *   1/(2n) sum_i (a_i^T x - b_i)^2 + (c/2) ||x||^2,  b_i in {-1, +1}
 * ("Extension to Classification Models", Least Squares Support Vector Machines): the gradient of a
 * step gets the additional term c * x, taken in full precision:  x <- x - lr * (g + l2 * x).
 * Full-precision (fp32) model only; l2 >= 0; everything else as in zipml_sgd_epoch. */
int zipml_sgd_epoch_l2(void *stream, const void *packed1_dev, const void *packed2_dev,
                       const float *levels_dev, const float *b_dev, int64_t n, int64_t d, int bits,
                       float *x_dev, int64_t batch, float lr, float l2, int flags,
                       void *workspace_dev, size_t workspace_bytes);

/* The same epoch with the proximal step of the general update of Sec. 2,
 *   x <- prox_{lr R}( x - lr * (g + l2 * x) ),  prox_{lr R}(v) = argmin_u 1/2 ||u - v||^2 + lr R(u),
 * for the regularisers that act coordinate by coordinate:
 *   ZIPML_PROX_L1    R(x) = prox_coef * ||x||_1          (soft threshold at lr * prox_coef)
 *   ZIPML_PROX_L2SQ  R(x) = prox_coef / 2 * ||x||_2^2    (v / (1 + lr * prox_coef))
 *   ZIPML_PROX_BOX   the constraint ||x||_inf <= prox_coef (clamp)
 *   ZIPML_PROX_NONE  R = 0 (then the call is zipml_sgd_epoch_l2).
 * Full-precision (fp32) model only; prox_coef >= 0; everything else as in zipml_sgd_epoch_l2.
 * (Regularisers that need a norm of the whole model -- the unsquared l2 norm, an l2 ball -- are
 * not provided.) */
#define ZIPML_PROX_NONE 0
#define ZIPML_PROX_L1   1
#define ZIPML_PROX_L2SQ 2
#define ZIPML_PROX_BOX  3
int zipml_sgd_epoch_prox(void *stream, const void *packed1_dev, const void *packed2_dev,
                         const float *levels_dev, const float *b_dev, int64_t n, int64_t d, int bits,
                         float *x_dev, int64_t batch, float lr, float l2, int prox, float prox_coef,
                         int flags, void *workspace_dev, size_t workspace_bytes);

/* The same epoch with the symmetrised estimator (Supp. B.2 "Double Sampling", footnote: lower variance at no extra
 * randomness; the form the authors report running):
 *   g = 1/2 mean_i [ Q1(a_i) (Q2(a_i)^T x - b_i) + Q2(a_i) (Q1(a_i)^T x - b_i) ],
 * which needs both copies in both layouts: packed1s_dev / packed2s_dev from
 * zipml_quantize_swapped.  fp32 model; 2-, 4- or 8-bit evenly spaced levels; batch a multiple
 * of 64; more than 256 features (otherwise ZIPML_EUNSUPPORTED, through the status word if it is
 * the level tables that do not qualify).  l2 as in zipml_sgd_epoch_l2 (0 for plain least squares).
 * Large minibatches are taken as in zipml_sgd_epoch (chunks, replicas, sample owners). */
int zipml_sgd_epoch_avg(void *stream, const void *packed1_dev, const void *packed2_dev,
                        const void *packed1s_dev, const void *packed2s_dev, const float *levels_dev,
                        const float *b_dev, int64_t n, int64_t d, int bits, float *x_dev,
                        int64_t batch, float lr, float l2, int flags, void *workspace_dev,
                        size_t workspace_bytes);

/* For callers that cannot allocate device memory -- code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc: zipml_sgd_epoch with its workspace taken from a fixed
 * array of ZIPML_STATIC_WORKSPACE_BYTES bytes that is part of the library's code object (every GPU
 * the library runs on holds its own copy until the process ends).  The call allocates and frees
 * nothing and calls no allocating routine; the address of the array on the current device is
 * looked up on the first call on that device (make that call outside a capture).
 * Arguments as zipml_sgd_epoch, without the workspace.  status_dev (device, one int, 4-byte
 * aligned, required) receives what zipml_sgd_status would return for the call -- ZIPML_OK,
 * ZIPML_ETIMEOUT or ZIPML_EUNSUPPORTED -- once the work enqueued on the stream is done.
 * ZIPML_EWORKSPACE (with a line on stderr that names both sizes) if
 * zipml_workspace_bytes(n, d, bits, batch, 0) exceeds ZIPML_STATIC_WORKSPACE_BYTES.
 * All calls on one GPU share the one array, and it keeps what the last call left in it (a call
 * clears what it needs cleared): calls that overlap in time on one GPU -- two streams, two host
 * threads -- race and give undefined results; serialise them or use zipml_sgd_epoch. */
#define ZIPML_STATIC_WORKSPACE_BYTES (8u << 20)
int zipml_sgd_epoch_static(void *stream, const void *packed1_dev, const void *packed2_dev,
                           const float *levels_dev, const uint16_t *grid_idx_dev, float grid_lo,
                           float grid_step, int grid_max, const float *b_dev, int64_t n, int64_t d,
                           int bits, float *x_dev, int64_t batch, float lr, int grad_bits,
                           int model_bits, uint64_t seed, uint32_t epoch, int flags, int *status_dev);

/* Waits for the stream and returns the status word the last zipml_sgd_epoch / zipml_debug_step
 * left in this workspace: ZIPML_OK or ZIPML_ETIMEOUT. */
int zipml_sgd_status(void *stream, const void *workspace_dev, size_t workspace_bytes);

/* Loss F(x) = 1/(2n) sum_i (a_i^T x - b_i)^2 (Sec. 1 eq. (1) with the square loss).  With A_dev
 * the exact fp32 rows are used; with A_dev == NULL the rows are decoded from one packed copy
 * (`copy` = 1 or 2) and levels_dev.  Dot products in fp32, squares and their sum in fp64.
 * Synchronises the stream and writes *loss_host. */
int zipml_loss(void *stream, const float *A_dev, int64_t lda, const void *packed_dev, int copy,
               const float *levels_dev, int bits, const float *b_dev, const float *x_dev,
               int64_t n, int64_t d, double *loss_host, void *workspace_dev,
               size_t workspace_bytes);

/* ---- parity / debug exports (not on the timed path) --------------------------------------- */

/* Canonical codes of one packed copy (`copy` = 1 or 2): codes_dev[n][d], row-major uint8. */
int zipml_unpack_codes(void *stream, const void *packed_dev, int copy, int64_t n, int64_t d,
                       int bits, uint8_t *codes_dev);

/* Runs the single step `step` of the epoch from the model in x_dev (updated in place) and exposes
 * its intermediates; any output pointer may be NULL.  model_codes_dev[d] and grad_codes_dev[d] are
 * the signed integer codes of Q3 / Q4, acc_dev[batch] the int32 dot products (integer mode only),
 * r_dev[batch] the residuals Q2(a_i)^T x - b_i, g_dev[d] the mean gradient before Q4.
 * Without flags the step runs in a launch of its own kind (the vector loop).  With
 * ZIPML_SGD_PRODUCTION it runs in the persistent launch and on the step loop that zipml_sgd_epoch
 * uses: the matrix-core loop for evenly spaced 2-, 4- or 8-bit levels and an fp32 model (only r_dev
 * and g_dev may be asked for then, ZIPML_EINVAL otherwise), or the end-to-end loop for
 * model_bits > 0 on more than one workgroup (all five outputs).  Shapes or level tables that
 * zipml_sgd_epoch would not run on one of these loops return ZIPML_EUNSUPPORTED (for the level
 * tables through zipml_sgd_status, with x_dev left untouched). */
int zipml_debug_step(void *stream, const void *packed1_dev, const void *packed2_dev,
                     const float *levels_dev, const uint16_t *grid_idx_dev, float grid_lo,
                     float grid_step, int grid_max, const float *b_dev, int64_t n, int64_t d,
                     int bits, float *x_dev, int64_t batch, float lr, int grad_bits,
                     int model_bits, uint64_t seed, uint32_t epoch, int64_t step, int flags,
                     int32_t *model_codes_dev, int32_t *acc_dev, float *r_dev, float *g_dev,
                     int32_t *grad_codes_dev, void *workspace_dev, size_t workspace_bytes);

/* A plain streaming pass of known size, for measurements: reads `bytes` bytes (a multiple of 16)
 * at src_dev once, XORs all their 32-bit words into *sink_dev (which the caller clears beforehand)
 * and, if dst_dev is not NULL, also stores them there (a copy).  Asynchronous.  It gives the
 * streaming-read rate of the machine for a roofline, and a launch whose HBM traffic is known, by
 * which hardware byte counters can be scaled. */
int zipml_debug_stream(void *stream, const void *src_dev, void *dst_dev, size_t bytes,
                       uint32_t *sink_dev);

/* Development knobs: process-wide overrides of choices the library otherwise makes by itself, for
 * sweeps, A/B measurements and tests that steer kernel selection (the library never reads the
 * environment).  value = -1 restores the automatic choice.  Values out of a knob's range are
 * ignored by the code that consults it.  Returns ZIPML_EINVAL for an unknown knob. */
#define ZIPML_KNOB_TARGET_WORKGROUPS 0  /* preferred number of feature-owner workgroups (default 32)  */
#define ZIPML_KNOB_NO_MATRIX_CORES   1  /* 1: evenly spaced levels stay on the vector-ALU step loop    */
#define ZIPML_KNOB_CHUNK_SAMPLES     2  /* chunk size of minibatches taken in chunks                    */
#define ZIPML_KNOB_MAX_REPLICAS      3  /* most replicas of the workgroups that share the chunks        */
#define ZIPML_KNOB_ROWS_MIN_BATCH    4  /* smallest minibatch for the sample-owner kernel (>= 16384)    */
#define ZIPML_KNOB_ROWS_ITEM_BLOCKS  5  /* 64-feature blocks per wave and item of that kernel (at 2 bits any
                                            value keeps the integer kernel; 101, 102: the 4-bit floating-point
                                            dot pass with tiles of 64, 128 samples)                      */
#define ZIPML_KNOB_ROWS_WORKGROUPS   6  /* its number of workgroups                                     */
#define ZIPML_KNOB_SPIN_LIMIT        7  /* polls before a device-wide wait gives up (0: at once)        */
#define ZIPML_KNOB_HOST_DP           8  /* 1: the dynamic program of zipml_levels runs on the host     */
#define ZIPML_KNOB_HIST_FEATURES     9  /* features per workgroup of the bin-moment kernel              */
#define ZIPML_KNOB_STORE_EXCHANGE_MIN 10 /* smallest (workgroups x samples of one exchange) from which
                                            the sums travel through tagged stores and reducer
                                            workgroups instead of atomics (0: wherever the loop can; a
                                            huge value: never; by itself the library asks for 32768
                                            and at least 128 workgroups)                           */
#define ZIPML_KNOB_COOPERATIVE_LAUNCH 11 /* 1: the epoch kernels go through the runtime's cooperative
                                            launch (it checks that the grid can be resident, as the
                                            library does itself, and queues such launches apart from
                                            the stream's other work: some 20 us per call)          */
#define ZIPML_KNOB_REDUCER_WORKGROUPS 12 /* workgroups that only reduce the tagged partial sums, on
                                            compute units the launch leaves idle (0: none; 100 + n: n
                                            of them with pieces of four words instead of eight)   */
#define ZIPML_KNOB_PREFETCH_WORKGROUPS 13 /* workgroups that only read the packed codes of a later chunk
                                            into the cache, on compute units still idle (0: none)  */
#define ZIPML_KNOB_COUNT            14
int zipml_debug_set(int knob, int64_t value);

#ifdef __cplusplus
}
#endif
#endif /* ZIPML_H */
