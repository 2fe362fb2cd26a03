/*
 * bof4.h - C ABI of the MI355X (gfx950) hot path of BOF4 / BOF4-S / OPQ 4-bit block-wise weight quantisation
 * (arxiv 2505.06653).
 *
 * Conventions
 *   - "dev" pointers are device (HBM) addresses owned by the caller; "host" pointers are ordinary host memory.
 *     The library allocates nothing and frees nothing, and keeps no state between calls beyond constants it works out
 *     once (device properties, table layouts).
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Work is enqueued on it; a call that
 *     returns results to host memory waits for them before returning (how is stated per call).
 *   - Weights are bfloat16 bit patterns, flat; block b is elements [b*block, (b+1)*block).  `block` must be
 *     32, 64, 128 or 256 and `n` a positive multiple of it.
 *   - A codebook is 16 finite, strictly ascending doubles (host).  Code c means level index c (paper level c+1).
 *   - Return value: BOF4_OK or a negative error code; bof4_last_error() gives a message for the calling thread,
 *     bof4_last_hip_error() the raw hipError_t of the last BOF4_ERR_HIP.
 *   - Required alignment: weight pointers 16 bytes, code pointers 4 bytes, scale / outlier-value pointers
 *     2 bytes, outlier-index pointers 8 bytes, workspace 256 bytes.  Misalignment is BOF4_ERR_ARG.
 */
#ifndef BOF4_H
#define BOF4_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BOF4_OK 0
#define BOF4_ERR_ARG (-1)       /* null / misaligned pointer, bad n or block, codebook not finite and ascending, T < 0 */
#define BOF4_ERR_CAPACITY (-2)  /* outlier buffers too small; *n_outliers holds the required count              */
#define BOF4_ERR_WORKSPACE (-3) /* ws_bytes below bof4_workspace_bytes(...)                                    */
#define BOF4_ERR_HIP (-4)       /* a HIP runtime call failed                                                   */

/* Per-region sums of one Lloyd / EM expectation pass (section 3.2 eq. 6; appendix B.3). */
typedef struct {
    double num[16];      /* sum over region l of g * x      (numerator of eq. 6)                               */
    double den[16];      /* sum over region l of g          (denominator of eq. 6)                             */
    uint64_t cnt[16];    /* K_l: normalised weights that fell into region l                                    */
    double sse;          /* sum of g * (x - level[code])^2: n_used * MSE(W, Q(W)) by the decomposition of B.3  */
    uint64_t n_used;     /* weights that entered the sums (n minus outliers)                                   */
    uint64_t n_outliers; /* weights excluded by OPQ                                                            */
} bof4_lloyd_stats;

/* Bytes of device workspace that bof4_quantize, bof4_quantize_lloyd (with outlier buffers of `out_capacity` entries; 0
 * if OPQ is not used), bof4_lloyd_step, bof4_quant_error and bof4_lloyd_step_mae need for `n` weights in blocks of
 * `block` - the largest of them.  What it is made of: for the outlier extraction one staging region per wave of the
 * largest grid (4096 regions of 4 * ceil(out_capacity / 4096) + 64 entries of 10 bytes: about 40 bytes per entry of
 * out_capacity, i.e. 0.64 bytes per weight at out_capacity = n / 64), or, if larger, the per-tile tables of the
 * fallback path (20 bytes per 2048 weights + 10 bytes per entry); behind it 459,200 bytes of partial sums; for the MAE
 * step n / 4 bytes (its candidate list; n / 2 bytes below 2^29 weights) + about 0.8 MB.  Pure host function; 0 on
 * invalid arguments. */
size_t bof4_workspace_bytes(uint64_t n, uint32_t block, uint64_t out_capacity);

/* OPQ threshold T = F_M^{-1}(q) for Gaussian weights (section 3.3 eq. 9 with F_M = (2G-1)^I of appendix B.1):
 * the q-quantile of the absolute maximum of `block` standard normal variables.  Pure host function; NaN on
 * invalid arguments. */
double bof4_opq_threshold(double q, uint32_t block);

/* The 15 binary32 decision thresholds the kernels compare against: thr[k] is the largest binary32 number not
 * above the mid-point of levels k and k+1 (nearest-neighbour rule of section 3.2; a value exactly on a mid-point
 * goes to the lower level).  code(x) = number of k with x > thr[k].  Pure host function. */
int bof4_thresholds(const double* cb_host, float* thr_host);

/* The bin table of the kernels' branch-free nearest-level search (same rule as bof4_thresholds, different
 * evaluation): a normalised weight x in [-1, 1] falls into bin b = (bits(fma(x, 16, 2^20 + 16)) >> 3) & 63 of 33,
 * and code(x) = base33[b] + (x > thr33[b]).  *fast_host is 0 when the codebook does not fit this form (two thresholds
 * within one bin, or one closer to zero than 2^-30); the kernels then count the 15 thresholds.  Pure host function. */
int bof4_bin_table(const double* cb_host, float* thr33_host, uint32_t* base33_host, int* fast_host);

/*
 * One expectation pass of the data-driven Lloyd / EM codebook optimisation (section 3.2 eq. 6, appendix B.3).
 * Every block is normalised by its absolute (signed_norm = 0, section 2.1 eq. 1-2) or signed (signed_norm = 1,
 * section 3.1 eq. 4) maximum as stored in binary16, each normalised weight x is assigned to its nearest level,
 * and the sums of eq. 6 are accumulated per region with g = (block constant)^2 (weight_by_max2 = 1) or g = 1
 * (weight_by_max2 = 0, the normalised-error variant of appendix D).  With opq_T > 0 the OPQ outliers of
 * section 3.3 are replaced by zero before the maximum search and take no part in the sums.
 *   w_dev       n bfloat16 weights (device, read only)
 *   cb_host     16 levels (host)
 *   out_host    result (host), valid on return.  If it lies in ordinary memory the call copies it there and
 *               synchronises `stream`.  If it lies in pinned (device-visible) host memory the GPU writes it in place
 *               and the call returns as soon as the record has arrived (the stream may still be finishing the
 *               call's last kernel; later work on `stream` is ordered behind it as usual)
 *   ws_dev      workspace of at least bof4_workspace_bytes(n, block, 0) bytes (device); contents undefined after
 * The result is bit-identical from run to run (fixed reduction order).  Out of contract: a block whose largest
 * magnitude exceeds binary16's range (65504) - its stored constant is infinite, and the sums are not finite then
 * (bof4_quantize and bof4_dequantize follow the definitions there as well: every weight of such a block normalises
 * to zero and decodes to infinity times the zero level's value, i.e. not to a number).  A
 * constant below binary16's normal range (2^-14) is stored with the bits binary16 has for it; the weights of such a
 * block normalise to up to 1.5 in magnitude and are counted as they are.
 */
int bof4_lloyd_step(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                    double opq_T, int weight_by_max2, bof4_lloyd_stats* out_host, void* ws_dev, size_t ws_bytes,
                    void* stream);

/*
 * The same call in two halves, for a caller that wants to enqueue other work on `stream` before it needs the sums (the
 * kernels of the next call then run while the host is still waiting for this one).  bof4_lloyd_step_begin takes the
 * arguments of bof4_lloyd_step, needs out_host in pinned (device-visible) host memory (BOF4_ERR_ARG otherwise),
 * enqueues and returns; the record is complete once bof4_wait_result(&out_host->n_used, stream) has returned.
 * bof4_wait_result waits for a result word that the GPU writes last into pinned host memory: &stats->n_used of the
 * Lloyd and MAE steps, &stats->n of the error pass.
 */
int bof4_lloyd_step_begin(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                          double opq_T, int weight_by_max2, bof4_lloyd_stats* out_host, void* ws_dev, size_t ws_bytes,
                          void* stream);
int bof4_wait_result(const uint64_t* word_host, void* stream);

/*
 * bof4_lloyd_step for callers that cannot allocate device memory or hand in a workspace (code that runs where
 * hipMalloc is not allowed, tight serving loops, harnesses that forbid allocation): same arguments without ws_dev /
 * ws_bytes, same kernels, same result bit for bit.  The per-workgroup partial sums go to a fixed array of 459,200 bytes
 * that is part of the library's device code (every GPU the library runs on holds it until the process ends); the call
 * itself allocates and frees nothing.  out_host must lie in pinned (device-visible) host memory, which the GPU writes
 * in place (BOF4_ERR_ARG otherwise); n must not exceed BOF4_STATIC_MAX_N (BOF4_ERR_ARG otherwise).  All calls on one
 * GPU share the array, which keeps the last call's contents (every launch overwrites the records it reads, nothing has
 * to start at zero): two calls that overlap in time on one GPU - different streams or threads - race and give wrong
 * sums.  The first call on a device looks the array's address up (with that device current).
 */
#define BOF4_STATIC_MAX_N (1ull << 36)
int bof4_lloyd_step_static(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                           double opq_T, int weight_by_max2, bof4_lloyd_stats* out_host, void* stream);

/* Maximisation step (section 3.2, eq. 6 and its last paragraph): level l moves to num[l]/den[l] unless bit l of
 * pinned_mask is set or the region is empty (den[l] == 0).  Pure host function; cb_host is updated in place. */
int bof4_codebook_update(const bof4_lloyd_stats* stats_host, uint16_t pinned_mask, double* cb_host);

/*
 * One maximisation step of the data-free codebook design: every level that is not pinned moves to the theoretical MSE
 * centroid of its region for weights drawn from a given symmetric distribution (section 3.2 eq. 5; appendix B.2, the
 * boxed general centroid with the conditional expectation of "Expectation of Normalized Weights", p_M and F_X of
 * appendix B.1).  With the common factors cancelled,
 *     level(l) = INT m [Phi1(m x)]_a^b A(m)^(block-2) p_W(m) dm  /  INT m^2 [F_W(m x)]_a^b A(m)^(block-2) p_W(m) dm,
 * a, b the mid-point thresholds of the region, A = 2 F_W - 1, Phi1(t) = INT_-inf^t u p_W(u) du (for Gaussian weights
 * Phi1 = -g: the appendix's closed form, whose boxed copy lacks the minus sign).
 *   pdf_host, cdf_host   p_W and F_W on the uniform grid u_k = k u_max / (n_grid - 1), k = 0 .. n_grid - 1 (host;
 *               n_grid odd, 3 .. 2^24; F_W(0) = 1/2; p_W is even, the negative side is implied); u_max large enough for
 *               the tail beyond it not to matter.  Phi1 is made from p_W by the trapezoid rule, values between grid
 *               points by linear interpolation, the integrals over m by the composite Simpson rule on the same grid
 *   pinned_mask level 15 (the region with the point mass at +1) must be pinned, and level 0 for absolute normalisation
 *               (signed_norm = 0); BOF4_ERR_ARG otherwise.  With signed_norm = 1 the leftmost region starts at -1
 *   cb_out_host receives the 16 new levels (host; pinned and empty regions keep theirs)
 *   ws_dev      bof4_theory_workspace_bytes(n_grid) bytes (device, 256-byte aligned)
 * Copies the tables to the device, runs two small kernels, synchronises `stream`.
 */
int bof4_theory_centroids(const double* pdf_host, const double* cdf_host, uint32_t n_grid, double u_max, uint32_t block,
                          const double* cb_host, uint16_t pinned_mask, int signed_norm, double* cb_out_host,
                          void* ws_dev, size_t ws_bytes, void* stream);
size_t bof4_theory_workspace_bytes(uint32_t n_grid);

/* Per-region results of one Lloyd / EM expectation pass under the MAE criterion (section 3.2 eq. 7-8; appendix B.4). */
typedef struct {
    double median[16];   /* weighted median of the normalised weights of region l, weights = absolute block maximum:
                            the smallest x_k with 2 * sum_{x_j <= x_k} a_j >= sum_j a_j; NaN if the region carries no
                            weight (empty, or only all-zero blocks)                                                 */
    double den[16];      /* sum over region l of |block constant|                                                   */
    uint64_t cnt[16];    /* K_l                                                                                      */
    double sae;          /* sum of |block constant| * |x - level[code]|: n_used * MAE(W, Q(W))                      */
    uint64_t n_used;     /* weights that entered the statistics (n minus outliers)                                   */
    uint64_t n_outliers; /* weights excluded by OPQ                                                                  */
} bof4_mae_stats;

/*
 * The expectation pass for the MAE criterion (section 3.2 eq. 7-8, appendix B.4).  Normalisation, assignment and OPQ
 * as in bof4_lloyd_step; per region the exact weighted median of the normalised weights (weights: the absolute block
 * maximum as stored in binary16, for absolute and signed normalisation alike) is found by a radix search that reads
 * the weights twice and then a list of the few elements still in question (in the workspace: n / 4 bytes, n / 2
 * below 2^29 weights; if the list runs full - a tensor of equal numbers - or outliers must be tracked through the
 * region around zero, the weights are read three or four times instead).  From 2^26 weights up (at block 64) the weights are read once, after a look at
 * one tile of 4096 weights in 16 that tells the search where to expect the medians; if those tiles are unlike the rest
 * of the tensor the search notices and reads the weights again as above - the result is the same either way.  Two
 * environment variables help when looking into this: BOF4_MAE_TRACE (set: every call prints to stderr which way it
 * went; set to 2: also how full the fullest wave's stretch of the list got and every region's window) and
 * BOF4_MAE_NO_SAMPLING (set: always the two-pass search).  The appendix's closing formula names the element before the
 * weighted median; what is returned is the minimiser that its derivation arrives at.  Weights are added as exact
 * 64-bit integers, which
 * needs sum over all weights of |block constant| < 2^38 (BOF4_ERR_ARG otherwise).
 *   weight_by_max  nonzero: the paper's criterion (eq. 8).  0: every weight counts one unit - the plain median of the
 *               normalised weights (appendix D, the MAE of the normalised weights, which the paper shows to be the
 *               inferior objective); den then counts the weights of the region whose block constant is a binary16
 *               number, and sae is the sum of |x - level[code]|
 *   skip_mask   bit l set: the median of region l is not wanted (a pinned level) and is reported as NaN; cnt and den
 *               of the region are still returned.  The region that contains zero needs a fourth pass, so skipping it
 *               (it is pinned in every BOF4 codebook) saves time
 * Other arguments, workspace and the hand-over of the result as for bof4_lloyd_step.  Medians, counts and den are
 * bit-reproducible.
 */
int bof4_lloyd_step_mae(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                        double opq_T, int weight_by_max, uint16_t skip_mask, bof4_mae_stats* out_host, void* ws_dev,
                        size_t ws_bytes, void* stream);

/* Maximisation step for the MAE criterion: level l moves to median[l] unless bit l of pinned_mask is set or the region
 * carries no weight.  Pure host function; cb_host is updated in place. */
int bof4_codebook_update_mae(const bof4_mae_stats* stats_host, uint16_t pinned_mask, double* cb_host);

/*
 * Quantise (sections 2.1, 3.1, 3.3): OPQ outlier extraction (opq_T > 0), block (signed) absmax, normalisation,
 * nearest-of-16 assignment, nibble packing.
 *   codes_dev        n/2 bytes; element 2j in the low nibble of byte j, element 2j+1 in the high nibble
 *   scales_dev       n/block binary16 block constants (the sign is kept when signed_norm = 1)
 *   out_idx_dev / out_val_dev   outlier list in ascending flat index: int64 index, binary16 value; capacity
 *                    `out_capacity` entries each; ignored (may be NULL) when opq_T == 0
 *   n_outliers_host  receives the number of outliers (0 when opq_T == 0), valid on return; pinned host memory is
 *                    written by the GPU in place
 *   ws_dev           workspace of at least bof4_workspace_bytes(n, block, out_capacity) bytes; needed only
 *                    when opq_T > 0
 * With opq_T == 0 the call only enqueues.  With opq_T > 0 it waits for the count: it synchronises `stream`, or,
 * with a pinned counter, returns as soon as the count has arrived; codes, scales and the outlier list are then
 * complete in stream order (a later call or copy on `stream` sees them; another stream must wait for `stream`).
 * On BOF4_ERR_CAPACITY codes and scales are complete, the outlier list is not.
 */
int bof4_quantize(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                  double opq_T, uint8_t* codes_dev, uint16_t* scales_dev, int64_t* out_idx_dev,
                  uint16_t* out_val_dev, uint64_t out_capacity, uint64_t* n_outliers_host, void* ws_dev,
                  size_t ws_bytes, void* stream);

/*
 * bof4_quantize in two halves (same arguments both times): bof4_quantize_begin enqueues the kernels and returns;
 * bof4_quantize_finish waits for the outlier count and completes the call exactly as bof4_quantize would (count in
 * *n_outliers_host, BOF4_ERR_CAPACITY, the re-run for outliers piled up in one stretch).  With opq_T > 0 the counter
 * must lie in pinned host memory (BOF4_ERR_ARG otherwise).  Between the two the caller may enqueue other work on
 * `stream` that does not touch the outputs; nothing that reads codes, constants or the list may be enqueued before
 * bof4_quantize_finish has returned.
 */
int bof4_quantize_begin(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                        double opq_T, uint8_t* codes_dev, uint16_t* scales_dev, int64_t* out_idx_dev,
                        uint16_t* out_val_dev, uint64_t out_capacity, uint64_t* n_outliers_host, void* ws_dev,
                        size_t ws_bytes, void* stream);
int bof4_quantize_finish(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                         double opq_T, uint8_t* codes_dev, uint16_t* scales_dev, int64_t* out_idx_dev,
                         uint16_t* out_val_dev, uint64_t out_capacity, uint64_t* n_outliers_host, void* ws_dev,
                         size_t ws_bytes, void* stream);

/*
 * Quantise and take the Lloyd sums in one pass over the weights (sections 2.1, 3.1, 3.3 and section 3.2 eq. 6 /
 * appendix B.3 on the same normalised weights): the outputs of bof4_quantize and the record of bof4_lloyd_step for
 * the same arguments (codes, constants and the outlier list bit for bit; the sums up to the order of the additions),
 * reading the weights once instead of twice.  With opq_T > 0 the outliers are extracted and take no part in the sums.
 * Arguments as for the two calls; ws_dev needs bof4_workspace_bytes(n, block, out_capacity) bytes also when
 * opq_T == 0 (the partial sums live there).  The call waits for the outlier count and for the record, each as its own
 * call does (pinned host memory is written by the GPU in place).
 * bof4_quantize_lloyd_begin / _finish split it like bof4_quantize_begin / _finish: the counter (if opq_T > 0) and the
 * record must lie in pinned host memory (BOF4_ERR_ARG otherwise); _finish waits for the count and completes the
 * quantiser's part; the record is complete once bof4_wait_result(&stats_host->n_used, stream) has returned.
 */
int bof4_quantize_lloyd(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                        double opq_T, int weight_by_max2, uint8_t* codes_dev, uint16_t* scales_dev,
                        int64_t* out_idx_dev, uint16_t* out_val_dev, uint64_t out_capacity, uint64_t* n_outliers_host,
                        bof4_lloyd_stats* stats_host, void* ws_dev, size_t ws_bytes, void* stream);
int bof4_quantize_lloyd_begin(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                              double opq_T, int weight_by_max2, uint8_t* codes_dev, uint16_t* scales_dev,
                              int64_t* out_idx_dev, uint16_t* out_val_dev, uint64_t out_capacity,
                              uint64_t* n_outliers_host, bof4_lloyd_stats* stats_host, void* ws_dev, size_t ws_bytes,
                              void* stream);
int bof4_quantize_lloyd_finish(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                               double opq_T, int weight_by_max2, uint8_t* codes_dev, uint16_t* scales_dev,
                               int64_t* out_idx_dev, uint16_t* out_val_dev, uint64_t out_capacity,
                               uint64_t* n_outliers_host, bof4_lloyd_stats* stats_host, void* ws_dev, size_t ws_bytes,
                               void* stream);

/*
 * Dequantise (section 2.1 eq. 3): w~ = block constant * level[code] as one binary32 product rounded to
 * bfloat16, then the outliers (section 3.3) are written back over their zero placeholders.
 *   w_out_dev   n bfloat16 values (device)
 *   out_idx_dev / out_val_dev   n_outliers entries in ascending flat index, as bof4_quantize writes them (the
 *               write-back re-decodes each 16-weight group that holds outliers and relies on the outliers of one
 *               group being adjacent in the list; of two entries with the same index the later one wins)
 * Only enqueues; out_idx_dev entries must lie in [0, n) (not checked on the device side beyond a bounds test
 * that skips offending entries).
 */
int bof4_dequantize(const uint8_t* codes_dev, const uint16_t* scales_dev, uint64_t n, uint32_t block,
                    const double* cb_host, const int64_t* out_idx_dev, const uint16_t* out_val_dev,
                    uint64_t n_outliers, void* w_out_dev, void* stream);

/* The quantisation error of a tensor (the MSE / MAE figures of section 5 and of the paper's error table; the difference
 * that appendix B.3 decomposes): sums over all n weights of w - Q(w), where Q(w) is what bof4_dequantize returns for
 * what bof4_quantize stores - the bfloat16 decoded weight, or the outlier as kept in binary16. */
typedef struct {
    double sse;          /* sum (w - Q(w))^2 : n * MSE                                                               */
    double sae;          /* sum |w - Q(w)|   : n * MAE                                                               */
    double max_abs;      /* largest |w - Q(w)|                                                                       */
    uint64_t n_outliers; /* weights the quantiser stores as outliers                                                 */
    uint64_t n;          /* weights compared                                                                         */
} bof4_error_stats;

/*
 * One pass over the weights that quantises, decodes and compares in registers: nothing but the record is written
 * (2 bytes of memory traffic per weight, against 7 for quantise + dequantise + compare).  Arguments, workspace
 * (bof4_workspace_bytes(n, block, 0)) and the hand-over of the record as for bof4_lloyd_step.  max_abs and n_outliers
 * are exact; sse and sae are binary64 sums in a fixed order (bit-reproducible).
 */
int bof4_quant_error(const void* w_dev, uint64_t n, uint32_t block, const double* cb_host, int signed_norm,
                     double opq_T, bof4_error_stats* out_host, void* ws_dev, size_t ws_bytes, void* stream);

/*
 * The decoder inside a matrix-vector product (section 2.1 eq. 3 applied in a linear layer, outliers of section 3.3
 * restored; the setting of the appendix on the runtime overhead of OPQ).  The quantised tensor is a row-major
 * [rows x cols] matrix (blocks along the flat layout, cols a multiple of block) and
 *     y[t][r] = sum_c w~[r][c] * x[t][c],     w~ = block constant * level[code],
 * with the exact product of eq. 3 (a weight is not rounded to bfloat16 first, unlike bof4_dequantize), except at the
 * listed outlier positions, where w~ is the stored binary16 value.  Products and sums are binary32, in a fixed order:
 * y is bit-reproducible and lies within 64 * 2^-24 * sum_c |w~ x| of the exact sum (an outlier position counts with
 * its decoded placeholder as well as with its value).
 *   codes_dev, scales_dev   as bof4_quantize writes them for n = rows * cols; codes_dev needs 16-byte alignment here
 *   table_dev   what bof4_gemv_outlier_table made of the outlier list (n_outliers entries); may be NULL when
 *               n_outliers == 0
 *   x_dev       n_tokens x cols bfloat16 (device, 16-byte aligned), y_dev  n_tokens x rows binary32 (device)
 * Limits: cols <= 32768.  The matrix is read once per pair of tokens.  Only enqueues.
 */
int bof4_gemv(const uint8_t* codes_dev, const uint16_t* scales_dev, uint64_t rows, uint64_t cols, uint32_t block,
              const double* cb_host, const void* table_dev, uint64_t n_outliers, const void* x_dev,
              uint32_t n_tokens, float* y_dev, void* stream);

/* The outlier list (section 3.3) of one quantised matrix in the form bof4_gemv reads: per entry its column and
 * (stored value - block constant * level[code at that position]), and where the entries of every row and every
 * stretch of 2048 columns begin.  The list must be strictly ascending (no index twice); an entry outside the matrix
 * is ignored.  Made once per matrix (it depends on codes, constants, list and codebook); 8-byte aligned buffer of
 * bof4_gemv_outlier_table_bytes(rows, cols, n_outliers) bytes (device), BOF4_ERR_WORKSPACE if smaller.  Only
 * enqueues. */
int bof4_gemv_outlier_table(const uint8_t* codes_dev, const uint16_t* scales_dev, uint64_t rows, uint64_t cols,
                            uint32_t block, const double* cb_host, const int64_t* out_idx_dev,
                            const uint16_t* out_val_dev, uint64_t n_outliers, void* table_dev, size_t table_bytes,
                            void* stream);
size_t bof4_gemv_outlier_table_bytes(uint64_t rows, uint64_t cols, uint64_t n_outliers);

/*
 * The decoder inside a matrix product for many tokens, as the paper's inference path runs it: the matrix is decoded to
 * bfloat16 (section 2.1 eq. 3 rounded as bof4_dequantize rounds it, outliers of section 3.3 as stored) and multiplied
 * with bfloat16 activations, binary32 accumulation - without the decoded matrix ever reaching memory:
 *     y[t][r] = sum_c W^[r][c] * x[t][c],     W^ = what bof4_dequantize returns for the same quantised tensor.
 * Every product of two bfloat16 numbers is exact in binary32; the sums are binary32 (matrix cores, up to 128 tokens
 * per pass over the codes) in a fixed order: y is bit-reproducible and lies within (cols + 64) * 2^-24 * sum_c |W^ x|
 * of the exact sum (an outlier position counts with its decoded placeholder as well as with its value), and is exact
 * whenever every partial sum is a binary32 number.  The order of the additions depends on rows, cols and n_tokens
 * (how the columns are dealt out over workgroups), so the same token may differ in its last bits between calls with
 * different n_tokens; equal calls give equal bits.
 *
 * The matrix is read from a copy in the order of the matrix cores' operands, made once per matrix by bof4_gemm_pack
 * from what bof4_quantize wrote for n = rows * cols (row-major [rows x cols], cols a multiple of block):
 * bof4_gemm_packed_bytes(rows, cols) bytes (device, 16-byte aligned) - per tile of 32 rows x 64 columns 1024 bytes of
 * codes and 64 binary16 constants, 0.5625 bytes per weight; BOF4_ERR_WORKSPACE if the buffer is smaller.
 *   packed_dev  that copy
 *   table_dev   what bof4_gemm_outlier_table made of the outlier list (from the unpacked codes and constants): layout
 *               and size of bof4_gemv's table (bof4_gemv_outlier_table_bytes), but per entry
 *               (bfloat16(value) - bfloat16(constant * level)); may be NULL when n_outliers == 0
 *   x_dev       n_tokens x cols bfloat16 (device, 16-byte aligned), y_dev  n_tokens x rows binary32 (device)
 *   ws_dev      bof4_gemm_workspace_bytes(rows, cols, n_tokens) bytes (device, 256-byte aligned),
 *               BOF4_ERR_WORKSPACE if smaller: x reordered for the matrix cores and transposed for the list (4 bytes
 *               per token slot and column, token slots in 32s), and - for matrices with too few rows to fill the
 *               chip - the partial results of the workgroups that share a row
 * Limits: cols <= 32768 and a multiple of 32, n_tokens <= 65536.  The codes are read once per 128 tokens.  All three
 * calls only enqueue.
 */
int bof4_gemm(const void* packed_dev, uint64_t rows, uint64_t cols, const double* cb_host, const void* table_dev,
              uint64_t n_outliers, const void* x_dev, uint32_t n_tokens, float* y_dev, void* ws_dev, size_t ws_bytes,
              void* stream);
int bof4_gemm_pack(const uint8_t* codes_dev, const uint16_t* scales_dev, uint64_t rows, uint64_t cols, uint32_t block,
                   void* packed_dev, size_t packed_bytes, void* stream);
size_t bof4_gemm_packed_bytes(uint64_t rows, uint64_t cols);
int bof4_gemm_outlier_table(const uint8_t* codes_dev, const uint16_t* scales_dev, uint64_t rows, uint64_t cols,
                            uint32_t block, const double* cb_host, const int64_t* out_idx_dev,
                            const uint16_t* out_val_dev, uint64_t n_outliers, void* table_dev, size_t table_bytes,
                            void* stream);
size_t bof4_gemm_workspace_bytes(uint64_t rows, uint64_t cols, uint32_t n_tokens);

/* Measurement aid: the next bof4_quantize / bof4_dequantize / bof4_lloyd_step / bof4_quant_error / bof4_gemv / bof4_gemm call made by this thread records
 * the caller-owned hipEvent_t `start_event` immediately before and `stop_event` immediately after its main kernel
 * (the one that streams over the weights), on the call's stream; helper kernels and host synchronisation lie
 * outside the pair.  The request is consumed by that call.  Pass NULLs to cancel. */
int bof4_time_next_call(void* start_event, void* stop_event);

const char* bof4_last_error(void);
int bof4_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* BOF4_H */
