/*
 * cmpq.h - C ABI of the CMPQ quantization path for AMD MI355X (gfx950).
 *
 * CMPQ = Channel-Wise Mixed-Precision Quantization (arXiv 2410.13056).  The
 * library turns one linear layer's weight W and calibration activations X into
 * the paper's stored format: a bit-width per input channel, a look-up table of
 * 2^bits FP16 levels per channel, bit-packed codes grouped by width, and two
 * kinds of FP16 outliers.
 *
 * Orientation and notation follow the paper (Sec. 3.2.1):
 *   W in R^{d_in x d_out}, row-major with leading dimension ldw >= d_out;
 *   "channel i" is the row W[i,:], the d_out weights that multiply input
 *   feature i.  A framework that stores weights as [d_out, d_in] converts with
 *   cmpq_transpose first.  X in R^{n x d_in} (tokens by channels), row-major.
 *   The linear index of a weight is i*d_out + o and must stay below 2^31.
 *
 * Conventions for every entry point:
 *   - returns CMPQ_OK (0) or a negative CMPQ_E* code; cmpq_strerror names it.
 *     Argument errors are detected on the host before anything is enqueued.
 *   - every data pointer is a DEVICE pointer owned by the caller unless the
 *     comment says "host".  The library keeps nothing between calls (the two
 *     exceptions say so: cmpq_time_kernel, cmpq_act_stats_static) and
 *     allocates no device memory: scratch comes from the caller's workspace
 *     `ws` of `ws_bytes` bytes (256-byte aligned), at least
 *     cmpq_workspace_bytes(op, d_in, d_out, n) large, else CMPQ_EWORKSPACE.
 *   - work is enqueued on `stream` (a hipStream_t passed as void*, null = the
 *     default stream) and the call returns without waiting for it.
 *   - `status` (nullable device int32) receives bit flags OR-ed in by the
 *     kernels: CMPQ_STATUS_NONFINITE when an input held NaN or infinity.
 *   - results are bit-for-bit reproducible from run to run: no floating-point
 *     atomics, every cross-workgroup reduction has a fixed order.
 */
#ifndef CMPQ_H
#define CMPQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CMPQ_OK 0
#define CMPQ_EINVAL (-1)     /* null pointer, negative size, unknown enum value            */
#define CMPQ_ESHAPE (-2)     /* leading dimension too small, size beyond a documented limit */
#define CMPQ_EBUDGET (-3)    /* bit set not consecutive within 1..4, or avg_bits outside it */
#define CMPQ_ECOUNT (-4)     /* asked for more outliers than there are candidates           */
#define CMPQ_EWORKSPACE (-5) /* workspace missing, misaligned or too small                  */
#define CMPQ_EHIP (-6)       /* the HIP runtime refused a launch                            */

#define CMPQ_F16 0 /* IEEE binary16 */
#define CMPQ_F32 1 /* IEEE binary32 */

#define CMPQ_KMAX 16      /* levels per channel at the widest setting (4 bits)   */
#define CMPQ_PROTECTED 16 /* bits[i] of a channel of O_act: kept whole in FP16   */

#define CMPQ_STATUS_NONFINITE 1
#define CMPQ_STATUS_ARRANGEMENT 2 /* cmpq_kmeans_quantize_job was handed something that is no kept arrangement */

/* `op` of cmpq_workspace_bytes */
#define CMPQ_OP_ACT_STATS 0        /* n = tokens in the call                     */
#define CMPQ_OP_ALLOCATE_BITS 1    /* n ignored                                  */
#define CMPQ_OP_OUTLIER_CHANNELS 2 /* n = k                                      */
#define CMPQ_OP_OUTLIER_WEIGHTS 3  /* n = k                                      */
#define CMPQ_OP_KMEANS 4           /* n ignored                                  */
#define CMPQ_OP_PACK 5             /* n ignored                                  */
#define CMPQ_OP_DEQUANT_ERROR 6    /* n ignored                                  */
#define CMPQ_OP_OUTLIERS_BY_COLUMN 7 /* n = entries of O_q                        */
#define CMPQ_OP_LUT_MATVEC 8       /* n = tokens in the call                     */
#define CMPQ_OP_PACK_WITH_ERROR 9  /* n ignored                                  */
#define CMPQ_OP_LUT4 10            /* sizes ignored                              */
#define CMPQ_OP_KMEANS_ARRANGEMENT 11 /* bytes of cmpq_kmeans_job.arrangement; n ignored; 0: not available */

/* `mode` / `score` of cmpq_extract_outliers */
#define CMPQ_OUTLIER_CHANNELS 0
#define CMPQ_OUTLIER_WEIGHTS 1
#define CMPQ_SCORE_RESIDUAL 0  /* |W' - W'_q|: the criterion of Sec. 3.2.2           */
#define CMPQ_SCORE_MAGNITUDE 1 /* |W'|: the magnitude rule Sec. 3.2.2 contrasts with */
/* `scope` of cmpq_extract_outliers, weights mode */
#define CMPQ_SCOPE_LAYER 0   /* the k largest scores of the whole layer: Sec. 3.2.2 */
#define CMPQ_SCOPE_CHANNEL 1 /* the k largest scores of every channel (a variant)  */

/* `norm` of cmpq_act_stats_norm */
#define CMPQ_NORM_L2 0   /* sum of squares: the criterion of Sec. 3.2.1 */
#define CMPQ_NORM_L1 1   /* sum of magnitudes  (norm ablation, App. Tab. 13) */
#define CMPQ_NORM_LINF 2 /* largest magnitude  (norm ablation, App. Tab. 13) */

/* `init` of cmpq_kmeans_quantize */
#define CMPQ_INIT_QUANTILE 0
#define CMPQ_INIT_GIVEN 1

/* `algorithm` of cmpq_kmeans_job */
#define CMPQ_KMEANS_HISTOGRAM 0 /* rounds read cumulative tables of the channel (default)   */
#define CMPQ_KMEANS_DIRECT 1    /* rounds revisit every weight: K-1 compares, 2 accumulations */
/* `arrangement_use` of cmpq_kmeans_job */
#define CMPQ_ARRANGEMENT_NONE 0
#define CMPQ_ARRANGEMENT_KEEP 1  /* leave this run's per-channel tables in `arrangement`       */
#define CMPQ_ARRANGEMENT_REUSE 2 /* start from the tables an earlier run left in `arrangement` */

size_t cmpq_workspace_bytes(int op, int64_t d_in, int64_t d_out, int64_t n);
const char *cmpq_strerror(int code);

/* Outlier counts are integers: round_half_up(ppm * n / 1e6) in integer arithmetic
 * (Sec. 3.2.2 prints the fractions 0.45 % and 0.05 %, i.e. 4500 and 500 ppm). */
int64_t cmpq_count_ppm(int64_t ppm, int64_t n);

/*
 * Sec. 3.2.1, the L2 norm of each channel of X: acc[i] (+)= sum_t X[t,i]^2 in fp64 and
 * sumsq[i] = (float)acc[i].  The square of the paper's a_i is kept: it ranks
 * channels identically and is the channel weight of the output error (App. B.3).
 *   X      [n, d_in], dtype CMPQ_F16 or CMPQ_F32, leading dimension ldx >= d_in.
 *   acc    [d_in] fp64, in/out.  accumulate = 0 overwrites it (tokens of a first
 *          chunk), accumulate != 0 adds to it (later chunks); n = 0 is allowed.
 *   sumsq  [d_in] fp32, out, nullable.
 * Workspace: CMPQ_OP_ACT_STATS.  Status: CMPQ_STATUS_NONFINITE.
 */
int cmpq_act_stats(const void *X, int dtype, int64_t n, int64_t d_in, int64_t ldx, double *acc,
                   float *sumsq, int accumulate, void *ws, size_t ws_bytes, int32_t *status,
                   void *stream);

/*
 * The same statistic under another norm (the appendix compares the l1 and l-infinity norms
 * with the l2 norm as allocation criterion, Tab. 13): norm = CMPQ_NORM_L2 is cmpq_act_stats;
 * CMPQ_NORM_L1: acc[i] (+)= sum_t |X[t,i]|; CMPQ_NORM_LINF: acc[i] = max(acc[i], max_t |X[t,i]|)
 * (accumulate = 0 starts from 0).  stat[i] = (float)acc[i] is what cmpq_extract_outliers and
 * cmpq_allocate_bits rank; the error weight of cmpq_dequant_error stays the l2 statistic.
 * Arguments, workspace and status as cmpq_act_stats.
 */
int cmpq_act_stats_norm(const void *X, int dtype, int64_t n, int64_t d_in, int64_t ldx, int norm,
                        double *acc, float *stat, int accumulate, void *ws, size_t ws_bytes,
                        int32_t *status, void *stream);

/*
 * cmpq_act_stats for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving or calibration loops, harnesses that forbid
 * allocation.  Same arguments (without ws / ws_bytes), same results bit for bit; the
 * row-split partial sums go to a fixed array inside the library, (2048*512 + 262144) fp64
 * = 10 MiB of device memory per GPU that the process holds from the library's load on.
 * The call allocates and frees nothing and records no memset (nothing in the array has to
 * start at zero: every partial that is read was written by the same call).
 * Limits: d_in <= 262144, else CMPQ_ESHAPE.  CMPQ_EHIP when the runtime cannot name the
 * array's address on the current device.  All calls on one GPU share the array: two calls
 * that overlap on one GPU (different streams, or threads) race; calls on one stream do not.
 */
int cmpq_act_stats_static(const void *X, int dtype, int64_t n, int64_t d_in, int64_t ldx, double *acc,
                          float *sumsq, int accumulate, int32_t *status, void *stream);

/*
 * Orientation helper for Sec. 3.2.1's W in R^{d_in x d_out}: dst[c, r] = src[r, c].
 * src is [rows, cols] with ld_src >= cols, dst is [cols, rows] with ld_dst >= rows,
 * both of `dtype`; they must not overlap.  No workspace.
 */
int cmpq_transpose(const void *src, int dtype, int64_t rows, int64_t cols, int64_t ld_src,
                   void *dst, int64_t ld_dst, void *stream);

/*
 * Algorithm 1 (channel-wise precision allocation) with an integer budget.
 *   sumsq      [d_in] channel statistic (non-negative, finite).
 *   chan_mask  [d_in] nullable; 1 marks a channel of O_act.  Such channels get
 *              bits = CMPQ_PROTECTED and are left out of the ranking and the budget.
 *   n_protected  number of ones in chan_mask (the caller chose it; 0 when null).
 *   bit_set    host, n_set consecutive widths within 1..4, ascending (the paper: {2,3,4}).
 *   avg_bits   b, within [bit_set[0], bit_set[n_set-1]].
 * With d_eff = d_in - n_protected and T = floor(b*d_eff + 1e-9):
 *   s < b < s+1: the T - s*d_eff channels with the largest statistic get s+1, the rest s
 *     (for {2,3,4} these are the b > 3 and b < 3 branches of Algorithm 1);
 *   b = s with s-1 and s+1 in the set (the b = 3 branch): the ceil(0.01*(d_eff-1)) lowest
 *     get s-1 and as many highest get s+1; otherwise every channel gets s.
 * Ranking: larger statistic first, equal statistics by smaller channel index.
 *   bits        [d_in] out.
 *   counts_host host, [n_set] out, nullable: channels per width, written before returning
 *               (they follow from the sizes alone).
 * Workspace: CMPQ_OP_ALLOCATE_BITS.
 */
int cmpq_allocate_bits(const float *sumsq, int64_t d_in, const uint8_t *chan_mask,
                       int64_t n_protected, const int32_t *bit_set, int n_set, double avg_bits,
                       uint8_t *bits, int64_t *counts_host, void *ws, size_t ws_bytes,
                       void *stream);

/*
 * The two outlier extractions of Sec. 3.2.2.  Both pick the k largest keys under the
 * order "larger key first, equal keys by smaller index" and return indices ascending.
 *
 * mode CMPQ_OUTLIER_CHANNELS (O_act): keys are sumsq[d_in].
 *   idx_out [k] int32 channel indices; chan_mask_out [d_in] (nullable) 1 = selected.
 *   scope, W, centroids, codes, bits, val_out are ignored.  k > d_in: CMPQ_ECOUNT.
 *
 * mode CMPQ_OUTLIER_WEIGHTS (O_q): candidates are the entries of channels with bits in
 *   1..4 (W' = W - O_act).  Key = fp32 |w - centroids[i][codes[i,o]]| for
 *   CMPQ_SCORE_RESIDUAL (needs centroids [d_in,16] from a first cmpq_kmeans_quantize, and
 *   its codes [d_in,d_out] or null), or fp32 |w| for CMPQ_SCORE_MAGNITUDE.  With codes
 *   null the key is the smallest fp32 |w - centroids[i][j]| over the channel's 2^bits[i]
 *   levels: the preliminary quantization codes every weight by its nearest level (Sec. 3
 *   eq. Q(x)), so this is the same key, and the first run need not write codes at all.
 *   scope CMPQ_SCOPE_LAYER (the paper's rule): the k largest keys of the whole layer.
 *     idx_out [k] int32 linear indices i*d_out+o, ascending; val_out [k] (nullable) the
 *     weights as FP16 bit patterns.  k > d_in*d_out: CMPQ_ECOUNT.  The number of candidates
 *     depends on `bits`, which is device data: when k exceeds it, every candidate is
 *     returned and the rest of idx_out holds -1 (val_out there is left as it was).
 *   scope CMPQ_SCOPE_CHANNEL (a variant: the same count in every channel, so that no
 *     channel's slice of the sparse list is longer than another's): the k largest keys of
 *     EACH channel with bits in 1..4, same order and tie rule inside the channel (equal keys
 *     by smaller output index).  idx_out / val_out hold k entries per such channel, the
 *     channels in ascending order, i.e. [k * n_live] ascending linear indices with n_live =
 *     number of channels with bits in 1..4 (the sum of cmpq_allocate_bits' counts).
 *     k > d_out: CMPQ_ECOUNT.
 *   sumsq and chan_mask_out are ignored.
 * Workspace: CMPQ_OP_OUTLIER_CHANNELS / CMPQ_OP_OUTLIER_WEIGHTS (n = k).
 */
int cmpq_extract_outliers(int mode, int score, int scope, const float *sumsq, const void *W,
                          int dtype, int64_t d_in, int64_t d_out, int64_t ldw,
                          const float *centroids, const uint8_t *codes, const uint8_t *bits,
                          int64_t k, int32_t *idx_out, uint16_t *val_out, uint8_t *chan_mask_out,
                          void *ws, size_t ws_bytes, void *stream);

/*
 * Sec. 3.2.1, channel-wise non-uniform quantization: for every channel with bits[i] in
 * 1..4, K = 2^bits[i] levels by Lloyd's algorithm on W[i,:], then each weight is coded by
 * its nearest level (Sec. 3 eq. Q(x)).
 *   out_idx     [n_out] int32 nullable: linear indices, strictly ascending, of entries removed
 *               before clustering (O_q, Sec. 3.2.2); they weigh 0 but still get a code.
 *   elem_weight [d_in, d_out] fp32 nullable, leading dimension d_out: importance of each
 *               entry in the level update (null = 1).  Must be >= 0 and finite.
 *   iters       rounds of (assign, update), run in full; then one more assignment.
 *   init        CMPQ_INIT_QUANTILE: level j starts at the order statistic
 *               floor((2j+1)*M/(2K)) of the M entries with positive weight; 0 when M = 0.
 *               CMPQ_INIT_GIVEN (a variant; the paper names no start): level j starts at
 *               centroids[i][j] as found on entry, j < K, in any order and with repeats
 *               allowed; -0.0 reads as +0.0; the levels must be finite.  Sec. 3.2.2's final
 *               quantization can so continue from the preliminary one's levels.
 *   centroids   [d_in, 16] fp32 out (in/out with CMPQ_INIT_GIVEN): K levels, then +infinity;
 *               all +infinity for a channel with bits outside 1..4.
 *   codes       [d_in, d_out] uint8 out (0 for such a channel).  May be null for inputs the
 *               histogram kernel takes (fp16, unit importance, rows of whole groups of 4
 *               entries, 8-byte aligned): the call then leaves the levels alone and skips the
 *               last assignment, which is all the preliminary quantization of Sec. 3.2.2
 *               needs when cmpq_extract_outliers is given no codes.  Null otherwise: CMPQ_EINVAL.
 * Assignment: the nearest level in exact arithmetic, equal distances to the smaller level
 * index.  Update: level = sum(m*x)/sum(m) of its members, accumulated in fp64 and rounded
 * once to fp32; a level without members keeps its value.  -0.0 reads as +0.0.
 * Limits: d_out <= 32768 for CMPQ_F16, <= 16384 for CMPQ_F32 (CMPQ_ESHAPE beyond).
 * Workspace: CMPQ_OP_KMEANS.  Status: CMPQ_STATUS_NONFINITE (the levels and codes of a channel
 * that holds a non-finite weight, or is given a non-finite starting level, are unspecified, its
 * codes stay below K; the other channels are not affected).
 */
int cmpq_kmeans_quantize(const void *W, int dtype, int64_t d_in, int64_t d_out, int64_t ldw,
                         const uint8_t *bits, const int32_t *out_idx, int64_t n_out,
                         const float *elem_weight, int iters, int init, float *centroids,
                         uint8_t *codes, void *ws, size_t ws_bytes, int32_t *status,
                         void *stream);

/*
 * The preliminary quantization of Sec. 3.2.2 for a new budget, from runs kept per width.
 * Levels and codes of a channel depend on its own weights and width only, so after one
 * cmpq_kmeans_quantize per width b = bit_set[j] over ALL channels (bits[i] = b for every i, no
 * out_idx), the first pass for any allocation `bits` is a row-wise choice:
 *   centroids[i,:], codes[i,:] = those of run j with bit_set[j] == bits[i];
 *   +infinity / 0 for a channel whose width is outside 1..4 (O_act) or not in bit_set -
 * exactly what cmpq_kmeans_quantize(W, bits, no out_idx) writes.  This is what makes
 * retargeting a quantized layer to another average width cheap (the cost the paper's closing
 * section names): only the steps after the first pass run again.
 *   bit_set             [n_set] host, distinct widths in 1..4, n_set <= 4.
 *   centroids_by_width  host array of n_set device pointers to [d_in, 16] fp32.
 *   codes_by_width      host array of n_set device pointers to [d_in, d_out] u8.
 *   centroids [d_in, 16] fp32, codes [d_in, d_out] u8: out.
 * No workspace.  Errors: CMPQ_EINVAL for null pointers, a width outside 1..4 or listed twice.
 */
int cmpq_select_by_width(const uint8_t *bits, int64_t d_in, int64_t d_out, const int32_t *bit_set,
                         int n_set, const float *const *centroids_by_width,
                         const uint8_t *const *codes_by_width, float *centroids, uint8_t *codes,
                         void *stream);

/*
 * cmpq_kmeans_quantize with every choice spelled out per call: a plain C structure of
 * pointers and sizes.  The fields up to `status` mean what the arguments of the same name
 * of cmpq_kmeans_quantize mean; that call is this one with algorithm = CMPQ_KMEANS_HISTOGRAM
 * and nothing of the stored format asked for.
 *   algorithm   which implementation runs the Lloyd rounds of Sec. 3.2.1 for fp16 weights with
 *               unit importance.  Both give identical levels and codes: CMPQ_KMEANS_HISTOGRAM
 *               reads cumulative tables of the channel, CMPQ_KMEANS_DIRECT revisits every
 *               weight (K-1 compares, 2 accumulations; kept as the independent second
 *               implementation).  Other inputs (fp32, elem_weight, rows that are not a whole
 *               number of 4 entries) run on the general kernel whatever is named here, and so
 *               does init = CMPQ_INIT_GIVEN with CMPQ_KMEANS_DIRECT (on the histogram kernel).
 *   bit_set ... err_total   (all null / 0: not asked for.)  Sec. 3.2.2's final quantization is
 *               followed by the stored format (Sec. 5.1) and the error (App. B.3) of the very
 *               codes it produces; with these fields set, the call leaves what
 *               cmpq_pack_with_error(W, ..., codes, bits, centroids, bit_set, n_set,
 *               counts_host, packed, chan_idx, lut, out_idx, n_out, sumsq, err_ch, err_total)
 *               would leave after it - packed rows, channel lists and tables bit-identical,
 *               err_ch / err_total equal up to the order of the fp64 additions - and, where the
 *               histogram kernel runs, writes them from its coding pass instead of reading
 *               weights and codes again.  Every one of the fields must then be given as for
 *               that call (sumsq nullable).  `codes` may be null, here as in a call without these
 *               fields, only for inputs the histogram kernel takes (fp16, unit importance, rows
 *               of whole groups of 4 entries, 8-byte aligned; CMPQ_KMEANS_HISTOGRAM): the dense
 *               codes are then not written at all.
 *   arrangement, arrangement_use   (null / CMPQ_ARRANGEMENT_NONE: not used.)  Sec. 3.2.2 runs
 *               the quantizer twice on the same channels: the final quantization differs from
 *               the preliminary one only by the entries of O_q (0.05 % - 1 % of a layer).  The
 *               histogram kernel's rounds read per-channel tables (weights counted and ordered
 *               by 16-bit key) that do not depend on the width or on the levels, so the
 *               preliminary run can leave them (CMPQ_ARRANGEMENT_KEEP: n_out must be 0) in a
 *               caller buffer of cmpq_workspace_bytes(CMPQ_OP_KMEANS_ARRANGEMENT, d_in, d_out, 0)
 *               bytes, 16-byte aligned, and the final run (CMPQ_ARRANGEMENT_REUSE, with its
 *               out_idx) starts from them instead of fetching, keying, counting and ordering the
 *               weights again: it takes the entries of out_idx out of the tables.  Levels, codes
 *               and everything else come out bit for bit as without the buffer.  The later call
 *               must name the same W, d_in, d_out, ldw and bits as the one that kept the buffer;
 *               only inputs the histogram kernel takes (see `codes` above) can use it, otherwise
 *               CMPQ_EINVAL.  A buffer that holds no kept arrangement for a channel raises
 *               CMPQ_STATUS_ARRANGEMENT and leaves that channel's outputs as for a non-finite one.
 * The library reads the structure during the call only.  Errors as cmpq_kmeans_quantize and
 * cmpq_pack_with_error; CMPQ_EINVAL for a null job, an unknown algorithm, or a stored format
 * asked for in part.  Workspace: CMPQ_OP_KMEANS.
 */
typedef struct cmpq_kmeans_job {
    const void *W; /* device, [d_in, d_out] */
    int dtype;
    int64_t d_in, d_out, ldw;
    const uint8_t *bits;     /* device, [d_in] */
    const int32_t *out_idx;  /* device, [n_out], nullable */
    int64_t n_out;
    const float *elem_weight; /* device, nullable */
    int iters, init;
    float *centroids; /* device, [d_in, 16] */
    uint8_t *codes;   /* device, [d_in, d_out] */
    int32_t *status;  /* device, nullable */
    int algorithm;
    /* the stored format and the error, as in cmpq_pack_with_error */
    const int32_t *bit_set;     /* host */
    int n_set;
    const int64_t *counts_host; /* host */
    uint32_t *const *packed;    /* host array of device pointers */
    int32_t *const *chan_idx;   /* host array of device pointers */
    uint16_t *const *lut;       /* host array of device pointers */
    const float *sumsq;         /* device, nullable */
    double *err_ch;             /* device, [d_in] */
    double *err_total;          /* device, [2] */
    /* tables shared between the two quantizations of Sec. 3.2.2 */
    void *arrangement;          /* device */
    int arrangement_use;
} cmpq_kmeans_job;

int cmpq_kmeans_quantize_job(const cmpq_kmeans_job *job, void *ws, size_t ws_bytes, void *stream);

/*
 * Introspection for host-side checks: the launch shape the histogram K-means kernel uses for
 * fp16 channels of d_out weights (d_out a multiple of 4, at most 32768).  shape [6], host, out:
 * lanes per workgroup, groups of 4 weights per lane, low key bits that name the place inside a
 * bucket (64 or 128 places; 2^(16 - bits) buckets), bytes of the per-channel place array, bytes
 * of dynamic LDS per workgroup, bytes of static LDS per workgroup.  Launches nothing.
 * CMPQ_EINVAL for a null pointer or a length that is no positive multiple of 4, CMPQ_ESHAPE
 * beyond the limit.
 */
int cmpq_kmeans_launch_shape(int64_t d_out, int64_t *shape);

/*
 * Sec. 5.1 / Fig. 4, the stored format: one code matrix per width.  For j < n_set and
 * b = bit_set[j], the channels with bits == b in ascending index form the rows:
 *   chan_idx[j] [counts_host[j]] int32             channel of each row;
 *   packed[j]   [counts_host[j], ceil(d_out*b/32)] uint32; a row is a little-endian bit
 *               stream, code of output o in stream bits [o*b, (o+1)*b), stream bit s =
 *               bit (s mod 32) of word (s / 32), zero padded to whole words;
 *   lut[j]      [counts_host[j], 2^b] FP16 bit patterns of the levels (round to nearest even).
 * packed, chan_idx, lut are HOST arrays of n_set DEVICE pointers; bit_set and counts_host
 * (from cmpq_allocate_bits) are host arrays.  Channels of O_act store no row.
 * Workspace: CMPQ_OP_PACK.
 */
int cmpq_pack(const uint8_t *codes, int64_t d_in, int64_t d_out, const uint8_t *bits,
              const float *centroids, const int32_t *bit_set, int n_set,
              const int64_t *counts_host, uint32_t *const *packed, int32_t *const *chan_idx,
              uint16_t *const *lut, void *ws, size_t ws_bytes, void *stream);

/*
 * App. A.2 (Tab. 10): CMPQ with the uniform quantizer of Sec. 3 in place of K-means.  Widths
 * still come from cmpq_allocate_bits, channels of O_act (bits outside 1..4) stay FP16, there
 * is no O_q.  Channel i is cut into groups of `group` consecutive outputs (a power of two in
 * 8..512; the last group of a channel may be shorter) and per group, with N = bits[i],
 *     Delta = (max - min) / (2^N - 1),  code = Clamp(round((w - min) / Delta), 0, 2^N - 1),
 * decided in fp32 (one IEEE division each, ties to even); Delta = 0 gives code 0.  The weight
 * is rebuilt as zero + code * scale.
 *   W       [d_in, d_out], CMPQ_F16 or CMPQ_F32, leading dimension ldw >= d_out.
 *   bits    [d_in] u8 from cmpq_allocate_bits.
 *   codes   [d_in, d_out] u8 out, dense (0 on channels of O_act).
 *   scale, zero  [d_in, ceil(d_out / group)] fp32 out: Delta and min of each group (0, 0 on
 *           channels of O_act).
 *   err_ch  [d_in] fp64 out, nullable: sum_o (w - (zero + code * scale))^2 with the rebuilt
 *           value exact; on channels of O_act the error of rounding to FP16.
 * All pointers are device pointers.  No workspace.  Status: CMPQ_STATUS_NONFINITE (the codes of
 * a group that holds a non-finite weight are unspecified).  Errors: CMPQ_EINVAL for a null
 * pointer, an unknown dtype or a group size that is not a power of two in 8..512; CMPQ_ESHAPE
 * for ldw < d_out.
 */
int cmpq_rtn_quantize(const void *W, int dtype, int64_t d_in, int64_t d_out, int64_t ldw,
                      const uint8_t *bits, int64_t group, uint8_t *codes, float *scale, float *zero,
                      double *err_ch, int32_t *status, void *stream);

/*
 * Reconstruction W_hat = W_q + O (Sec. 3.2.2) and the output error of App. B.3,
 * Delta Y = X (W - W_hat), with cross-channel products of X dropped:
 *   W_hat[i,o] = fp16(W[i,o]) for channels with bits outside 1..4 and for the entries of
 *                out_idx [n_out] (ascending linear indices, nullable), else
 *                centroids[i][codes[i,o]];
 *   err_ch[i]     = sum_o (W - W_hat)^2                    [d_in] fp64 out
 *   err_total[0]  = sum_i sumsq[i] * err_ch[i]  (sumsq null: weight 1);  err_total[1] = sum_i err_ch[i].
 * Workspace: CMPQ_OP_DEQUANT_ERROR.
 */
int cmpq_dequant_error(const void *W, int dtype, int64_t d_in, int64_t d_out, int64_t ldw,
                       const float *centroids, const uint8_t *codes, const uint8_t *bits,
                       const int32_t *out_idx, int64_t n_out, const float *sumsq, double *err_ch,
                       double *err_total, void *ws, size_t ws_bytes, void *stream);

/*
 * cmpq_pack (Sec. 5.1) and cmpq_dequant_error (App. B.3) in one pass over the codes, for a
 * caller that wants both: every argument means what it means in those two calls, the packed
 * rows, channel lists and tables are bit-identical to cmpq_pack's, err_ch and err_total equal
 * cmpq_dequant_error's up to the order of the fp64 additions.  HBM traffic per weight: the
 * weight and one code byte in, bits/8 bytes out (the two calls read the code byte twice).
 * Errors: those of the two calls.  Workspace: CMPQ_OP_PACK_WITH_ERROR.
 */
int cmpq_pack_with_error(const void *W, int dtype, int64_t d_in, int64_t d_out, int64_t ldw,
                         const uint8_t *codes, const uint8_t *bits, const float *centroids,
                         const int32_t *bit_set, int n_set, const int64_t *counts_host,
                         uint32_t *const *packed, int32_t *const *chan_idx, uint16_t *const *lut,
                         const int32_t *out_idx, int64_t n_out, const float *sumsq, double *err_ch,
                         double *err_total, void *ws, size_t ws_bytes, void *stream);

/*
 * ---- Sec. 6 / Fig. 4: the product with the deployed weight --------------------------------
 *
 * Fig. 4 splits a layer by precision: per width a table-driven product of the input with
 * the packed codes, plus the outlier matrices multiplied in FP16 with the same input, all
 * summed into one output.  The three calls below are that consumer of cmpq_pack's format.
 * The deployed weight is
 *   W_hat[i,o] = FP16 table level lut[row(i)][code(i,o)]   for a quantized entry,
 *              = fp16(W[i,o])                               for channels of O_act and entries of O_q
 * (an outlier overrides its level: a table cannot store the exact zero that "W_q + O" of
 * Sec. 3.2.2 would need), and Y[t,o] = sum_i X[t,i] * W_hat[i,o].
 */

/*
 * The rows of O_act as they are deployed: W_act[j, :] = fp16(W[act_idx[j], :]) for
 * j < k_act (act_idx from cmpq_extract_outliers, CHANNELS mode).  W_act is FP16
 * [k_act, d_out] with leading dimension ld_act >= d_out.  No workspace.
 */
int cmpq_gather_channels(const void *W, int dtype, int64_t d_in, int64_t d_out, int64_t ldw,
                         const int32_t *act_idx, int64_t k_act, uint16_t *W_act, int64_t ld_act,
                         void *stream);

/*
 * O_q in the form the product reads: a compressed sparse matrix (Sec. 6) whose rows are
 * the outputs, so that every output is one sequential sum.
 * Input: out_idx [n_out] ascending linear indices i*d_out+o with their FP16 values out_val
 * (from cmpq_extract_outliers), and the final centroids / codes of the layer.  Output:
 *   colptr  [d_out+1] int32: entries of column o are colptr[o] .. colptr[o+1]-1;
 *   row_idx [n_out]   int32: input channel of each entry, ascending inside a column;
 *   delta   [n_out]   fp32 : out_val - FP16 table level of the entry's code.  Adding
 *                            X[t,i]*delta to the table product makes the outlier override
 *                            its level.
 * Workspace: CMPQ_OP_OUTLIERS_BY_COLUMN.  d_out < 2^20.
 */
int cmpq_outliers_by_column(const int32_t *out_idx, const uint16_t *out_val, int64_t n_out,
                            int64_t d_in, int64_t d_out, const float *centroids,
                            const uint8_t *codes, int32_t *colptr, int32_t *row_idx, float *delta,
                            void *ws, size_t ws_bytes, void *stream);

/*
 * Y[t,o] = sum_i X[t,i] * W_hat[i,o] for t < m: X FP16 [m, d_in] (ldx), Y fp32 [m, d_out]
 * (ldy).  The weight arrives as stored:
 *   bit_set, n_set, counts_host, packed, chan_idx, lut   as written by cmpq_pack (host
 *       arrays of device pointers; a width with no channels may have null pointers);
 *   act_idx [k_act], W_act [k_act, d_out] (ld_act)       the channels of O_act, FP16;
 *   colptr, row_idx, delta                               O_q from cmpq_outliers_by_column
 *                                                        (colptr null: no such outliers).
 * Products and sums are fp32: per output the table products are summed over slabs of 128
 * rows of one width in a fixed order, then the O_act rows, then the column's O_q entries;
 * the result is reproducible bit for bit.  Workspace: CMPQ_OP_LUT_MATVEC with n = m.
 * Limits: m <= 65535, d_out < 2^20.
 */
int cmpq_lut_matvec(const void *X, int64_t m, int64_t d_in, int64_t ldx, int64_t d_out,
                    const int32_t *bit_set, int n_set, const int64_t *counts_host,
                    const uint32_t *const *packed, const int32_t *const *chan_idx,
                    const uint16_t *const *lut, const int32_t *act_idx, const uint16_t *W_act,
                    int64_t k_act, int64_t ld_act, const int32_t *colptr, const int32_t *row_idx,
                    const float *delta, float *Y, int64_t ldy, void *ws, size_t ws_bytes,
                    void *stream);

/*
 * Sec. 5.1 / Tab. 7: the look-up tables held in 4 bits, (1*4 + 8*4)/4096 bits of overhead per
 * weight for a 3-bit channel.  The paper does not say how the centres are quantized; the
 * figure leaves 4 bits per table entry and nothing per channel.
 *   mode CMPQ_LUT4_CODEBOOK (the reading taken): the 4 bits index one 16-entry table per
 *     layer, found by the non-uniform quantizer of Sec. 3 (K-means with K = 16, as
 *     cmpq_kmeans_quantize runs it: quantile start, `iters` rounds, nearest level in exact
 *     arithmetic with ties to the smaller index, fp64 means rounded once to fp32) over all
 *     centres of the layer as the stored format holds them, v = FP16(centroids[i][j]) for
 *     j < 2^bits[i] and bits[i] in 1..4 (-0 as +0; a non-finite centre takes no part).
 *       table       [16] fp32 out, device: the levels (all 0 when no channel is quantized);
 *       codes4      [d_in, 16] u8 out: the level of every table entry (0 in unused slots);
 *       centroids_q [d_in, 16] fp32 out: FP16(table[codes4]) - what a stored FP16 table of
 *                   the layer gives back; +infinity in unused slots and on channels of O_act.
 *     Workspace: CMPQ_OP_LUT4.
 *   mode CMPQ_LUT4_UNIFORM (an alternative): one uniform 16-level grid per layer, the uniform
 *     quantizer of Sec. 3 with N = 4 over all centres (fp32 values, not rounded to FP16):
 *       lo = min, hi = max, Delta = (hi - lo) / 15, code = Clamp(round((c - lo) / Delta), 0, 15)
 *       in fp32 with ties to even, c_q = lo + code * Delta formed exactly and rounded once to
 *       fp32; Delta = 0: code 0.  table[0] = lo, table[1] = Delta (0, 0 when no channel is
 *       quantized), the other entries are left alone.  `iters` is ignored; no workspace.
 * centroids [d_in, 16] fp32 in (from cmpq_kmeans_quantize), bits [d_in] u8.  centroids_q goes
 * to cmpq_pack, cmpq_dequant_error and the deployed product in place of `centroids`.
 * d_in <= 2^27.
 */
#define CMPQ_LUT4_CODEBOOK 0
#define CMPQ_LUT4_UNIFORM 1
int cmpq_lut4_quantize(int mode, const float *centroids, const uint8_t *bits, int64_t d_in, int iters,
                       uint8_t *codes4, float *table, float *centroids_q, void *ws, size_t ws_bytes,
                       void *stream);

/*
 * Several products in one pair of launches (Sec. 6 / Fig. 4 for the products that can run
 * side by side: the query, key and value projections read the same input, so do the gate and
 * up projections).  Single-token products are short, so a launch per layer is dominated by
 * launch and first-load latency; grouped, the short layers run beside the long ones.
 * Every field has the meaning of the argument of the same name of cmpq_lut_matvec; all
 * products of a group share the number of tokens m.  Results are bit-identical to one
 * cmpq_lut_matvec call per layer.
 * Workspace: the sum over the layers of cmpq_workspace_bytes(CMPQ_OP_LUT_MATVEC, d_in, d_out, m)
 * is always enough.  Limits: n_layers <= CMPQ_MAX_GROUP; those of cmpq_lut_matvec per layer; the
 * partial rows of all layers together stay below 65536 (CMPQ_ESHAPE beyond).
 * Errors are those of cmpq_lut_matvec; nothing is launched when one layer is rejected.
 */
#define CMPQ_MAX_GROUP 8
typedef struct cmpq_deployed_layer {
    const void *X; /* device, FP16 [m, d_in] */
    int64_t d_in, ldx, d_out;
    const int32_t *bit_set; /* host */
    int n_set;
    const int64_t *counts_host;          /* host */
    const uint32_t *const *packed;       /* host array of device pointers */
    const int32_t *const *chan_idx;      /* host array of device pointers */
    const uint16_t *const *lut;          /* host array of device pointers */
    const int32_t *act_idx;              /* device */
    const uint16_t *W_act;               /* device */
    int64_t k_act, ld_act;
    const int32_t *colptr, *row_idx;     /* device, colptr nullable */
    const float *delta;                  /* device */
    float *Y;                            /* device, fp32 [m, d_out] */
    int64_t ldy;
} cmpq_deployed_layer;

int cmpq_lut_matvec_group(const cmpq_deployed_layer *layers, int n_layers, int64_t m, void *ws,
                          size_t ws_bytes, void *stream);

/*
 * The same products with the packed rows added up in FP16 (Sec. 6 / Fig. 4: the paper's
 * kernel keeps FP16 throughout; cmpq_lut_matvec_group above adds in fp32).  Arguments, limits,
 * workspace and errors are those of cmpq_lut_matvec_group.  What differs:
 *   - a product X[t,i] * level is rounded to FP16 (to nearest even);
 *   - the products of a run of R consecutive packed rows of one width (in the order of that
 *     width's chan_idx; R = 32, halved while that leaves fewer than 512 workgroups, down to
 *     8: the run length of the launch) are added in FP16, one after the other, starting from 0;
 *   - the run sums, the rows of O_act (fp32 products) and the entries of O_q are then added
 *     in fp32 in a fixed order, as in cmpq_lut_matvec_group: results are reproducible bit for
 *     bit, and equal an emulation of the three steps up to the fp32 rounding of the last one.
 * Against the exact product: |Y - Y_exact| <= (R + 1) * 2^-11 * sum_i |X[t,i] * W_hat[i,o]| over
 * the packed rows, plus the fp32 rounding of cmpq_lut_matvec_group (a worst-case bound; errors of
 * either sign mostly cancel).  There is no overflow check: a run whose partial sum leaves the
 * FP16 range (|sum| > 65504) gives infinities, as FP16 arithmetic does - callers keep
 * 32 * max|X| * max|level| below that.
 */
int cmpq_lut_matvec_group_fp16acc(const cmpq_deployed_layer *layers, int n_layers, int64_t m, void *ws,
                                  size_t ws_bytes, void *stream);

/*
 * Measurement hook (for a benchmark that wants the duration of one kernel rather than of an
 * entry point, which may launch several).  Arms the CALLING THREAD: the next launch of the
 * named kernel from this thread records event_begin (a hipEvent_t passed as void*) on the
 * launch stream right before the kernel and event_end right after it, and the hook is
 * disarmed again.  Null events disarm.  The elapsed time between the two events, once both
 * have completed, is the kernel's duration on that stream (plus what else shares the GPU
 * with it when other streams are busy).  This is the one piece of state the library keeps,
 * and it is per thread; it changes no result.  CMPQ_EINVAL for an unknown kernel.
 */
#define CMPQ_KERNEL_ACT_STATS 0     /* the streaming pass of cmpq_act_stats over X (aligned input)     */
#define CMPQ_KERNEL_TRANSPOSE 1     /* cmpq_transpose, fp16 with aligned rows                           */
#define CMPQ_KERNEL_KMEANS 2        /* the k-means kernel of cmpq_kmeans_quantize (histogram algorithm) */
#define CMPQ_KERNEL_OUTLIER_STAGE 3 /* the one pass over the layer of the layer-wide O_q selection      */
#define CMPQ_KERNEL_PACK_ERROR 4    /* the one-pass kernel of cmpq_pack_with_error                      */
#define CMPQ_KERNEL_COUNT 5
int cmpq_time_kernel(int kernel, void *event_begin, void *event_end);

/*
 * Measurement helper (for a benchmark that prices a kernel against a peak that depends on the
 * clock): the shader clock under a vector-ALU load.  Enqueues one kernel on `stream`:
 * n_workgroups workgroups of 256 lanes each run `iters` rounds of 64 dependent fused
 * multiply-adds on four independent chains per lane and read two counters before and after,
 * the shader-clock counter and the constant-rate wall counter.
 *   ticks     [n_workgroups, 2] u64 out, device: per workgroup the two differences
 *             (shader ticks, wall ticks);
 *   wall_khz  host out: the rate of the wall counter in kHz.
 * clock = shader ticks / wall ticks * wall rate, per workgroup; the caller reads `ticks`
 * after synchronising.  With n_workgroups a multiple of the number of compute units the
 * whole GPU is busy while the counters run.  It changes nothing else and keeps nothing.
 * CMPQ_EINVAL: null pointer, iters < 1, n_workgroups outside 1..65536; CMPQ_EHIP when the
 * runtime does not report the wall counter's rate.
 */
int cmpq_shader_clock_probe(int iters, int n_workgroups, uint64_t *ticks, int *wall_khz, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CMPQ_H */
