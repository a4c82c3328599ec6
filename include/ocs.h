/*
 * ocs.h - C ABI of the OCS-expanded quantized layer for AMD MI355X (gfx950).
 *
 * Outlier channel splitting (Zhao et al., "Improving Neural Network Quantization without
 * Retraining using Outlier Channel Splitting"): input channels that hold outliers are
 * duplicated and halved (Sec. 3.2, Eq. 3 and Eq. 4), chosen greedily one at a time
 * (Sec. 3.4); weights and activations are put on a symmetric k-bit linear grid (Sec. 3.1,
 * Eq. 1), optionally narrowed by a clip threshold (Sec. 1, Sec. 5.2); the expanded layer
 * (Eq. 2 over the expanded channel set) then runs as an integer GEMM with 32-bit
 * accumulation followed by the trailing scale factors of Eq. 1.
 *
 * Conventions (all entry points unless stated otherwise)
 *  - Return value: OCS_OK (0) or a negative OCS_E_* code; nothing is thrown across the ABI.
 *    ocs_strerror() turns a code into text.  Arguments are validated on the host before any
 *    device work, so every argument error is reported without touching the GPU.
 *  - Every tensor / index / scale pointer is a DEVICE pointer owned by the caller.  The
 *    library allocates nothing; scratch space comes from the caller's `workspace`
 *    (device memory, 256-byte aligned), at least ocs_workspace_bytes() bytes.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *    enqueue work on that stream and never synchronise; results (including scalar results
 *    such as thresholds) are written to device memory so that the chain
 *    split -> quantize -> gemm needs no host round trip.
 *  - Layout: a tensor T of a layer is [rows, C*g] row-major with a leading dimension in
 *    elements; K-columns are channel-major: input channel c owns columns c*g .. c*g+g-1
 *    (g = 1 for a fully connected layer or a 1x1 convolution, g = kh*kw for a convolution
 *    lowered by im2col; Sec. 3.2: a split duplicates a whole 2-D activation channel and
 *    every 2-D filter attached to it).  Activations X are [M, C*g], weights W are [N, C*g]
 *    (both operands K-contiguous), outputs Y are [M, N].
 *  - Code tensors (int8) have a 16-byte aligned base and a leading dimension that is a
 *    multiple of OCS_CALIGN; for rows longer than OCS_SHORT_K bytes ocs_qgemm additionally
 *    needs a multiple of OCS_KALIGN (its K-step).  The producer writes zeros into every pad
 *    column (columns (C+s)*g .. ld-1) and the consumers rely on those zeros.
 *  - fp32 inputs may have any leading dimension >= the row length and any float-aligned
 *    base: rows are read with 16-byte loads at whatever alignment they have.
 *  - `clip_ratio` (Sec. 4: the grid's threshold as a fraction of the largest magnitude) must be
 *    positive and finite wherever the call derives the threshold itself: OCS_E_CLIP otherwise.
 *    It is ignored when the caller passes a threshold.
 *  - NaN / Inf inputs give unspecified codes (no fault).  Index arrays read from device
 *    memory are clamped into range before use, so bad indices cannot cause a fault.
 *  - Two calls that share a workspace or an output must be ordered on one stream.
 */
#ifndef OCS_H
#define OCS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define OCS_KALIGN 64 /* leading dimension of the code tensors ocs_qgemm reads is a multiple of this */
#define OCS_ROWALIGN 128 /* what ocs_padded_cols rounds to: rows then start on cache-line boundaries
                            and ocs_qgemm can walk K in 128-byte steps (the zero padding joins in) */
#define OCS_CALIGN 16 /* leading dimension of any int8 code tensor is a multiple of this */
#define OCS_SHORT_K 320 /* rows of at most this many bytes (rounded up to OCS_KALIGN): ocs_qgemm reads
                           them in one go and accepts any leading dimension that is a multiple of
                           OCS_CALIGN and holds the row */

#define OCS_OK 0
#define OCS_E_NULL (-1)      /* a required pointer is NULL                                  */
#define OCS_E_SHAPE (-2)     /* non-positive dimension, leading dimension too small, too big */
#define OCS_E_ALIGN (-3)     /* code tensor base / leading dimension / workspace misaligned  */
#define OCS_E_BITS (-4)      /* bit width outside 2..8                                       */
#define OCS_E_SPLITS (-5)    /* num_splits negative or beyond the supported maximum          */
#define OCS_E_OVERFLOW (-6)  /* Kexp * qmax_x * qmax_w does not fit a 32-bit accumulator     */
#define OCS_E_WORKSPACE (-7) /* workspace NULL or smaller than ocs_workspace_bytes()         */
#define OCS_E_HIP (-8)       /* a HIP call failed; ocs_last_hip_error() has the text         */
#define OCS_E_MODE (-9)      /* unknown mode                                                 */
#define OCS_E_CLIP (-10)     /* clip_ratio is not a positive finite number                   */

#define OCS_MODE_HALVE 0 /* choose channels on this tensor and halve both copies (Eq. 3)     */
#define OCS_MODE_DUP 1   /* channel choice given; copy channels un-halved (Eq. 4, weights)   */

#define OCS_MAX_EXPANDED_CHANNELS 8000  /* C + num_splits may not exceed this                */

/* Text for an OCS_E_* code (static storage, never NULL). */
const char *ocs_strerror(int code);

/* Text of the last HIP error seen by the calling thread ("" if none). */
const char *ocs_last_hip_error(void);

/*
 * Split budget of Sec. 3.4: ceil(r * C), evaluated in double precision.
 * r <= 0 or C <= 0 gives 0.  Host-only, no device work.
 */
int ocs_num_splits(int C, double r);

/* Bytes per pixel of un-lowered activation codes for ocs_qconv: channels rounded up to OCS_CALIGN. */
int64_t ocs_padded_channels(int64_t channels);

/*
 * Recommended leading dimension of the code tensor of an expanded layer: (C+s)*g rounded up to
 * OCS_ROWALIGN, or, for rows of at most OCS_SHORT_K bytes, only to OCS_CALIGN: the GEMM streams
 * such rows once and the pass that writes them is bound by memory, so padding there is only more
 * bytes (a 68-code row of the paper's 64-channel layers takes 80 bytes, not 128).  For longer rows
 * any multiple of OCS_KALIGN that holds the row is accepted by ocs_qgemm; with this one the rows
 * of both operands are whole cache lines, which measured 10 % (operands in cache) to 25 %
 * (operands in HBM) faster on the 3x3 layer shapes.
 */
int64_t ocs_padded_cols(int64_t cols);

/* Row length of the tap-major weight tensor of ocs_qconv: g*ldc rounded up to OCS_KALIGN. */
int64_t ocs_conv_weight_cols(int g, int64_t ldc);

/*
 * Scratch bytes that any call below needs for a tensor of `rows` x `cols` fp32 elements
 * (cols = C*g of the unexpanded tensor).  Host-only.  Returns 0 for non-positive sizes.
 */
size_t ocs_workspace_bytes(int64_t rows, int64_t cols);

/*
 * Channel selection of Sec. 3.4 on a tensor T [rows, C*g]: num_splits times, take the
 * expanded channel that currently holds the largest magnitude (lowest expanded index on
 * ties; the two halves of a split channel are equal, so ties always occur), halve it, and
 * append its copy at expanded index C+i.
 *   split_src  [num_splits]   out: expanded index split at step i
 *   chan_src   [C+num_splits] out: original channel that expanded channel j descends from
 *   chan_depth [C+num_splits] out: number of halvings applied to expanded channel j
 *   max_out    device float   out: largest magnitude after all splits (may be NULL)
 * T is only read.  Used on weights (weight OCS) or on a batch of activations
 * (activation OCS with the channels chosen on that batch, Sec. 5.3).
 */
int ocs_select_channels(const float *T, int64_t rows, int C, int g, int64_t ld, int num_splits,
                        int32_t *split_src, int32_t *chan_src, int32_t *chan_depth,
                        float *max_out, void *workspace, size_t ws_bytes, void *stream);

/*
 * Weight side of OCS (Sec. 3.2 Eq. 3 / Eq. 4, Sec. 3.4), done off-line per Sec. 3.5.
 *   mode OCS_MODE_HALVE: select channels on W as ocs_select_channels does, then
 *        W'[n, j*g+t] = W[n, chan_src[j]*g+t] * 2^-chan_depth[j]        (Eq. 3)
 *        split_src, chan_src, chan_depth are outputs.
 *   mode OCS_MODE_DUP:   split_src [num_splits] is an INPUT (chosen on activations);
 *        W'[n, j*g+t] = W[n, chan_src[j]*g+t]                            (Eq. 4)
 *        chan_src, chan_depth are outputs.
 * Optional outputs (each may be NULL):
 *   W_out [N, (C+s)*g] fp32, leading dimension ldo: the expanded weights.
 *   wmax_out device float: max|W'|.
 *   Wq [N, ldq] int8 codes of W' on the `bits`-bit grid with threshold
 *        clip_ratio * max|W'| (Eq. 1; clip after OCS as in Sec. 5.2), pad columns zero;
 *        scale_w_out device float[2] = {threshold, threshold / qmax} (required with Wq).
 * W is only read.
 */
int ocs_split_weights(const float *W, int64_t N, int C, int g, int64_t ldw, int num_splits,
                      int mode, int32_t *split_src, int32_t *chan_src, int32_t *chan_depth,
                      float *W_out, int64_t ldo, float *wmax_out, int bits, float clip_ratio,
                      int8_t *Wq, int64_t ldq, float *scale_w_out, void *workspace,
                      size_t ws_bytes, void *stream);

/*
 * Quantization-aware splitting of the weights (Sec. 3.3), done off-line like ocs_split_weights.
 * In units of the grid step a QA split replaces w by the pair ((w - 1/2)/2, (w + 1/2)/2), whose
 * members, rounded with that section's Q(x) = floor(x + 1/2), add up to Q(w).
 *   Selection and threshold: as ocs_split_weights in mode OCS_MODE_HALVE on the same W
 *        (split_src, chan_src, chan_depth are outputs with the same values);
 *        T = clip_ratio * max|plainly halved W'|, step = T / qmax, qmax = 2^(bits-1) - 1.
 *   Members: the split list is replayed on W; at each split the channel that keeps its index
 *        becomes (v - step/2)/2 and the appended copy (v + step/2)/2, in fp32, one
 *        add/subtract and one exact halving per split.
 *   chan_path [C + num_splits] uint32, output: the history of expanded channel j, one bit per
 *        split of its lineage, first split in bit 0 (0: kept its index, 1: appended copy);
 *        chan_depth[j] bits are used.
 *   W_out [N, (C+s)*g] fp32 (leading dimension ldo; may be NULL): the QA-split weights.
 *   Wq [N, ldq] int8 (may be NULL): codes clamp(floor(w' * (qmax / T) + 1/2), -qmax, qmax), pad
 *        columns zero.  At least one of W_out, Wq is required.
 *   scale_w_out device float[2] = {T, step} (required).
 * Activations are duplicated as for Eq. 3 (ocs_split_act with chan_depth = NULL).
 * W is only read.
 */
int ocs_split_weights_qa(const float *W, int64_t N, int C, int g, int64_t ldw, int num_splits,
                         int32_t *split_src, int32_t *chan_src, int32_t *chan_depth,
                         uint32_t *chan_path, float *W_out, int64_t ldo, int bits,
                         float clip_ratio, int8_t *Wq, int64_t ldq, float *scale_w_out,
                         void *workspace, size_t ws_bytes, void *stream);

/*
 * Clip threshold of least mean squared error over a histogram (Sec. 4.1), for calibration.
 *   x [rows, cols] fp32 (leading dimension ldx), only read.
 *   Histogram of |x|: num_bins (1..8192) equal bins on [0, m], m = max|x|; a value falls in bin
 *        min(num_bins-1, floor(|x| * (num_bins / m))) (fp32: one division, one multiply); a bin
 *        counts at its centre x_i = (i + 1/2) * (m / num_bins).
 *   Candidates T_c = m * (c / num_candidates), c = 1..num_candidates (1..65536).
 *   Error of a candidate: 1/num_bins * sum_i h_i * (x_i - code_i * T_c/qmax)^2 with code_i the
 *        code of x_i under ocs_quantize's arithmetic contract for threshold T_c and `bits`;
 *        evaluated in fp64, bins in increasing order.  The first candidate of least error wins.
 *   threshold_out device float[2] = {chosen threshold, m}; element 0 can be handed to
 *        ocs_quantize / ocs_split_act as their `threshold`.
 *   hist_out device uint64[num_bins] and mse_out device double[num_candidates], both required:
 *        the frequencies and the error of every candidate (outputs, and the routine's scratch).
 * workspace as for ocs_quantize on the same shape.
 */
int ocs_mse_clip_threshold(const float *x, int64_t rows, int64_t cols, int64_t ldx, int bits,
                           int num_bins, int num_candidates, float *threshold_out,
                           unsigned long long *hist_out, double *mse_out, void *workspace,
                           size_t ws_bytes, void *stream);

/*
 * Sec. 3.3 on the activation side (Eq. 4 with the quantization-aware pair), per batch.
 * split_src / chan_src / chan_depth: the choice made on this batch by ocs_select_channels
 * (plain halving); threshold: device float, the activation grid's range T (with no clipping:
 * the max_out of that same call), step = T / qmax.  The split list is replayed on X: at each
 * split the channel that keeps its index becomes (x - step/2)/2, the appended copy
 * (x + step/2)/2 (fp32, one add/subtract and one exact halving per split); codes
 * clamp(floor(x' * (qmax / T) + 1/2), -qmax, qmax).  chan_path [C + num_splits] uint32 is an
 * output (the histories, as in ocs_split_weights_qa).  Xq [M, ldq] int8, pad columns zero;
 * scale_out device float[2] = {T, step}, must not be `threshold`.  The weights are duplicated
 * un-halved (ocs_split_weights, OCS_MODE_DUP) as for Eq. 4.  A plain, non-streaming kernel:
 * the paper finds activation splitting ineffective (Sec. 5.3) and this variant is provided for
 * completeness, not tuned.
 */
int ocs_split_act_qa(const float *X, int64_t M, int C, int g, int64_t ldx, const int32_t *split_src,
                     const int32_t *chan_src, const int32_t *chan_depth, uint32_t *chan_path,
                     int num_splits, int bits, const float *threshold, int8_t *Xq, int64_t ldq,
                     float *scale_out, void *stream);

/*
 * Linear quantization of Sec. 3.1 Eq. 1 with optional clipping (Sec. 1).
 *   x [rows, cols] fp32 -> q [rows, ldq] int8, q = clamp(rne(x * (qmax / T)), -qmax, qmax),
 *   qmax = 2^(bits-1) - 1 (a grid of 2^bits - 1 points), columns cols .. ldq-1 zero.
 *   threshold != NULL: T = *threshold (device float, T >= 0; a static or clipped grid).
 *   threshold == NULL: T = clip_ratio * max|x| (clip_ratio = 1 spans the whole range).
 *   T == 0 gives all-zero codes and a zero step.
 *   scale_out device float[2] = {T, T / qmax}.
 * Arithmetic contract: qmax / T is one correctly rounded fp32 division, x * (qmax / T) one
 * fp32 multiply, rne = round half to even.
 */
int ocs_quantize(const float *x, int64_t rows, int64_t cols, int64_t ldx, int bits,
                 const float *threshold, float clip_ratio, int8_t *q, int64_t ldq,
                 float *scale_out, void *workspace, size_t ws_bytes, void *stream);

/*
 * Activation side of OCS, per batch (Sec. 3.5: a layer that copies and scales the chosen
 * channels), fused with Eq. 1:
 *   Xq[i, j*g+t] = Q( X[i, chan_src[j]*g+t] * f_j ),  j < C+num_splits,  pad columns zero,
 *   f_j = 1 when chan_depth == NULL (Eq. 3: the weights carry the halving) and
 *   f_j = 2^-chan_depth[j] otherwise (Eq. 4).
 * chan_src may be NULL only when num_splits == 0.
 * Threshold as in ocs_quantize; with threshold == NULL it is clip_ratio times the largest
 * magnitude of the EXPANDED activations (i.e. after halving).
 *   scale_out device float[2] = {T, T / qmax}.
 */
int ocs_split_act(const float *X, int64_t M, int C, int g, int64_t ldx, const int32_t *chan_src,
                  const int32_t *chan_depth, int num_splits, int bits, const float *threshold,
                  float clip_ratio, int8_t *Xq, int64_t ldq, float *scale_out, void *workspace,
                  size_t ws_bytes, void *stream);

/*
 * ocs_split_act for callers that cannot allocate device memory and so have no workspace to
 * pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Arguments, arithmetic and results are those of ocs_split_act; the scratch space (partial and
 * column maxima of the per-batch grid) is an array of OCS_STATIC_SCRATCH_BYTES bytes that is part
 * of the library's device image: each GPU the library runs on holds its own copy from the first
 * call on that GPU until the process ends.  The call allocates and frees nothing.
 *  - A tensor whose scratch need, ocs_workspace_bytes(M, C*g), exceeds OCS_STATIC_SCRATCH_BYTES is
 *    refused with OCS_E_WORKSPACE before any device work (every layer shape of the paper's
 *    networks fits).
 *  - All calls on one GPU share that GPU's array: two calls that may overlap there (different
 *    streams, different threads) race and give undefined thresholds; order them on one stream.
 *    Nothing in the array has to start at zero and nothing is carried from one call to the next.
 *  - The first call on a device looks the array's address up (hipGetSymbolAddress); make that
 *    call outside a graph capture.
 */
#define OCS_STATIC_SCRATCH_BYTES (2 * 1024 * 1024)
int ocs_split_act_static(const float *X, int64_t M, int C, int g, int64_t ldx, const int32_t *chan_src,
                         const int32_t *chan_depth, int num_splits, int bits, const float *threshold,
                         float clip_ratio, int8_t *Xq, int64_t ldq, float *scale_out, void *stream);

/*
 * The dynamic threshold of ocs_split_act on its own (Eq. 1's max|x| over the expanded
 * activations, times clip_ratio): scale_out device float[2] = {T, T / qmax}.  Calling this
 * and then ocs_split_act with threshold = scale_out is what ocs_split_act does by itself
 * when its threshold is NULL; the split lets a caller reuse one threshold for several
 * batches, or time the two passes separately.
 */
int ocs_act_threshold(const float *X, int64_t M, int C, int g, int64_t ldx, const int32_t *chan_src,
                      const int32_t *chan_depth, int num_splits, int bits, float clip_ratio,
                      float *scale_out, void *workspace, size_t ws_bytes, void *stream);

/*
 * The expanded layer of Eq. 2 on integer codes, then the trailing factors of Eq. 1:
 *   acc[i,n] = sum_{k < Kexp} Xq[i,k] * Wq[n,k]   (int8 x int8 -> int32, exact)
 *   Y[i,n]   = float(acc[i,n]) * (scale_x[1] * scale_w[1])
 * Xq [M, ldx], Wq [N, ldw] int8; ldx, ldw >= Kexp rounded up to OCS_KALIGN and multiples of it,
 * or, when that rounded extent is at most OCS_SHORT_K, >= Kexp rounded up to OCS_CALIGN and
 * multiples of that (OCS_E_SHAPE / OCS_E_ALIGN otherwise; what such a row lacks up to its last
 * K-step counts as zero codes); scale_x, scale_w are the device float[2] written by the producers;
 * bits_x / bits_w are the grids' bit widths, used only for the overflow check
 * Kexp * qmax_x * qmax_w < 2^31.  acc_out [M, ldacc] int32 is optional (NULL = not
 * stored); Y [M, ldy] fp32 is required.  workspace may be NULL (none is needed).
 * Every column Kexp .. ld-1 of both operands must hold zero codes (the producers' contract): on
 * rows longer than 320 bytes the kernels walk K in 128-byte steps whenever both leading
 * dimensions reach the next multiple of 128, and those columns then enter the sums.
 */
int ocs_qgemm(const int8_t *Xq, int64_t ldx, const int8_t *Wq, int64_t ldw, int64_t M, int64_t N,
              int64_t Kexp, int bits_x, int bits_w, const float *scale_x, const float *scale_w,
              int32_t *acc_out, int64_t ldacc, float *Y, int64_t ldy, void *workspace,
              size_t ws_bytes, void *stream);

/*
 * ocs_split_act (static grid, copies un-scaled: the activation side of Eq. 3) and ocs_qgemm as ONE
 * launch: the GEMM's loader reads the fp32 rows of X [M, C*g] itself, puts them on the grid of
 * `threshold` (Eq. 1, the arithmetic of ocs_split_act: the codes are the same), and takes the
 * copies of the split channels from the codes it has just produced, so the code tensor Xq never
 * reaches memory: 4 bytes are read per element of X instead of 4 read + (1 + r) written + (1 + r)
 * read again.  acc_out and Y are bit for bit those of the two calls.
 *   chan_src [C + num_splits]: as written by the weight side; only the appended entries are used.
 *   threshold: device float T > 0 (a profiled grid, Sec. 5).  scale_x_out: optional device
 *        float[2], receives {T, T / qmax} as ocs_split_act's scale_out would; must not be `threshold`.
 *   Wq [N, ldw], scale_w: the weight codes and grid of the expanded layer, ldw >= (C+num_splits)*g
 *        rounded up to OCS_CALIGN and a multiple of it, pad columns zero.
 * Serves the shapes ocs_split_act_qgemm_fits() accepts (host-only; 1 = yes): 64 <= C*g <= 8192,
 * at most 2048 appended columns num_splits*g, N <= 256 (one tile of output columns, so that X is
 * read once); X needs only its float alignment, at any ldx.  Other shapes: OCS_E_SHAPE, and the
 * two calls do the same work.
 */
int ocs_split_act_qgemm_fits(int64_t M, int C, int g, int num_splits, int64_t N, int64_t ldx);
/* 1 where it fits and was measured ahead of the two calls (rows of X of 256 values and more). */
int ocs_split_act_qgemm_pays(int64_t M, int C, int g, int num_splits, int64_t N, int64_t ldx);
int ocs_split_act_qgemm(const float *X, int64_t M, int C, int g, int64_t ldx, const int32_t *chan_src,
                        int num_splits, int bits_x, const float *threshold, const int8_t *Wq, int64_t ldw,
                        int64_t N, int bits_w, const float *scale_w, float *scale_x_out, int32_t *acc_out,
                        int64_t ldacc, float *Y, int64_t ldy, void *stream);

/*
 * ocs_qgemm with the K extent of every output tile shared between `parts` workgroups (2 .. 16, at
 * most one per 64-byte K-step): for shapes with far fewer output tiles than the chip has compute
 * units and a long K.  Each workgroup leaves the int32 partial sums of its 256 x 256 tile in the
 * workspace and signs in at a counter; the one that signs in last adds the others' sums to its
 * own and writes the output.  Integer sums do not depend on the order, so acc_out and Y are
 * bit-identical to ocs_qgemm's; nobody waits for anybody and there is no second launch.
 *   workspace: device memory, 256-byte aligned, at least ocs_qgemm_split_k_workspace_bytes(M, N,
 *        Kexp, parts) bytes (0 = this shape cannot be split: more than 128 tiles of 256 x 256, or
 *        parts out of range; the call then returns OCS_E_SHAPE).  Needs no initialisation.
 *   The arrival counters are part of the library's device image; at most 512 such calls may be
 *   in flight on one GPU at a time.
 * On MI355X this measured slower than ocs_qgemm on every layer shape of the paper's networks (the
 * partial sums cross between L2s through memory): ocs_qgemm never uses it by itself.
 */
size_t ocs_qgemm_split_k_workspace_bytes(int64_t M, int64_t N, int64_t Kexp, int parts);
int ocs_qgemm_split_k(const int8_t *Xq, int64_t ldx, const int8_t *Wq, int64_t ldw, int64_t M, int64_t N,
                      int64_t Kexp, int bits_x, int bits_w, const float *scale_x, const float *scale_w,
                      int32_t *acc_out, int64_t ldacc, float *Y, int64_t ldy, int parts, void *workspace,
                      size_t ws_bytes, void *stream);

/*
 * A convolution as the linear layer of Eq. 2 over its input channels (Sec. 3.2: a channel of a
 * convolution is a whole 2-D activation plane with the 2-D filters attached to it), with the
 * lowering to a GEMM done inside the kernel's operand loader instead of materialising the
 * lowered (im2col) activation.  The activation is split and quantized ONCE, un-lowered, by
 * ocs_split_act with g = 1 on its [B*H*W, C] view (kh*kw times less traffic than the lowered
 * matrix); every code of the lowered matrix is a code of that tensor, or zero outside the image.
 *
 * ocs_conv_weights_tap_major: weight codes Wq [N, ldq] as ocs_split_weights writes them for
 *   g = kh*kw (expanded channel j owns columns j*g .. j*g+g-1) -> Wt [N + 1, ldt],
 *   ldt = g*ldc rounded up to OCS_KALIGN, with Wt[n, t*ldc + j] = Wq[n, j*g + t] for
 *   j < C_exp = C + num_splits, zero everywhere else, and row N all zeros (the kernel reads it
 *   for taps outside the image).  ldc: bytes per pixel of the activation codes, a multiple of
 *   OCS_CALIGN, >= C_exp (ocs_padded_channels(C_exp) is the tightest).
 *
 * ocs_qconv: Aq [B, H, W, ldc] int8 (channels C_exp .. ldc-1 zero, as ocs_split_act pads),
 *   kernel kh x kw, stride, zero padding pad on every side; output pixel (b, yo, xo) is row
 *   (b*Ho + yo)*Wo + xo of Y [B*Ho*Wo, N] fp32 (and of acc_out, optional int32), Ho = (H + 2*pad
 *   - kh)/stride + 1.  acc = sum over taps and expanded channels of code products, exactly the
 *   accumulator ocs_qgemm gives on the lowered codes; Y = float(acc) * (scale_x[1]*scale_w[1]).
 *   Wt as written by ocs_conv_weights_tap_major for the same ldc.
 * Both calls: device pointers, asynchronous on `stream`, 16-byte aligned code tensors.
 */
int ocs_conv_weights_tap_major(const int8_t *Wq, int64_t N, int C_exp, int g, int64_t ldq,
                               int8_t *Wt, int64_t ldc, void *stream);
int ocs_qconv(const int8_t *Aq, int64_t ldc, int B, int H, int W, int C_exp, int kh, int kw,
              int stride, int pad, const int8_t *Wt, int64_t N, int bits_x, int bits_w,
              const float *scale_x, const float *scale_w, int32_t *acc_out, int64_t ldacc,
              float *Y, int64_t ldy, void *stream);

/*
 * ocs_qgemm / ocs_qconv with the output handed to the NEXT layer as codes instead of fp32: the
 * epilogue applies Eq. 1 with the next layer's static grid to the dequantized output (and the
 * activation side of the next layer's Eq. 3: the channels it splits are duplicated), so the
 * 4-byte output and the next layer's pass over it never touch memory.  Per element, in fp32:
 *   y = float(acc) * (scale_x[1] * scale_w[1]);  relu != 0: y = max(y, 0);
 *   code = clamp(rne(y * (qmax / T)), -qmax, qmax), T = *next_threshold (device float, the grid
 *   fixed from profiling as in Sec. 5), qmax = 2^(next_bits-1) - 1, arithmetic as in ocs_quantize.
 *   Yq[i, j] = code of output channel next_chan_src[j] for j < N + next_splits <= N + 512 (next_chan_src
 *   device int32 [N + next_splits] as the next layer's ocs_split_weights wrote it; its first N
 *   entries are the identity; NULL allowed when next_splits == 0).
 *   Yq [M, ldyq] int8, ldyq a multiple of OCS_CALIGN and >= N + next_splits.  Columns
 *   N + next_splits .. ldyq-1 are written as zero codes, like every producer's pad columns.
 *   next_scale_out device float[2] = {T, T / qmax} (may be NULL; must not be next_threshold).
 *   acc_out optional int32 [M, ldacc] as in ocs_qgemm.  Other arguments as in ocs_qgemm / ocs_qconv.
 */
int ocs_qgemm_requant(const int8_t *Xq, int64_t ldx, const int8_t *Wq, int64_t ldw, int64_t M,
                      int64_t N, int64_t Kexp, int bits_x, int bits_w, const float *scale_x,
                      const float *scale_w, int relu, const float *next_threshold, int next_bits,
                      const int32_t *next_chan_src, int next_splits, int8_t *Yq, int64_t ldyq,
                      float *next_scale_out, int32_t *acc_out, int64_t ldacc, void *stream);
int ocs_qconv_requant(const int8_t *Aq, int64_t ldc, int B, int H, int W, int C_exp, int kh, int kw,
                      int stride, int pad, const int8_t *Wt, int64_t N, int bits_x, int bits_w,
                      const float *scale_x, const float *scale_w, int relu,
                      const float *next_threshold, int next_bits, const int32_t *next_chan_src,
                      int next_splits, int8_t *Yq, int64_t ldyq, float *next_scale_out,
                      int32_t *acc_out, int64_t ldacc, void *stream);

/*
 * Weight side of Eq. 4 on codes, for a channel choice that changes with every batch (Sec. 5.3).
 * The copies of a duplicated weight channel are not scaled, so max|W'| = max|W|, the codes of
 * the first C*g columns are those of the un-expanded weights whatever the choice, and an appended
 * channel's codes are byte copies of its source's.  Given Wq [N, ldq] whose first C*g columns hold
 * the codes of W (ocs_quantize on W with ldq >= (C + num_splits)*g, once), this call rewrites
 * only columns C*g .. ldq-1 for the batch's chan_src [C + num_splits] (device int32, from
 * ocs_select_channels): Wq[n, j*g + t] = Wq[n, chan_src[j]*g + t] for C <= j < C + num_splits,
 * zero beyond.  Result = what ocs_split_weights in OCS_MODE_DUP writes, without reading W.
 */
int ocs_duplicate_weight_codes(int8_t *Wq, int64_t ldq, int64_t N, int C, int g, int num_splits,
                               const int32_t *chan_src, void *stream);

/*
 * The expanded layer of Eq. 3 run WITHOUT expanding it (off-line preparation).  In Eq. 2 on
 * codes a duplicated activation channel multiplies each of its weight copies by the same
 * activation code, so the expanded layer's int32 accumulator equals that of an un-expanded layer
 * whose weight code for channel c is the sum of the codes of c's copies:
 *   Wf[n, c*g + t] = sum over j with chan_src[j] == c of Wq[n, j*g + t],   c < C.
 * Wq [N, ldq]: the expanded weight codes (ocs_split_weights or ocs_split_weights_qa) with their
 * chan_src [C + num_splits].  Wf [N, ldf] int8, ldf >= C*g, pad columns zero.
 * max_abs_out device int32: the largest |sum|.  The sums fit int8 whenever (copies of a channel)
 * * qmax_w <= 127, which holds for every weight width below 8 bits at the paper's expansion
 * ratios; a sum beyond +-127 is stored saturated and makes Wf unusable, so check *max_abs_out
 * <= 127 once.  With Wf the layer is ocs_quantize (or ocs_split_act with num_splits = 0) on the
 * un-expanded activations and ocs_qgemm with Kexp = C*g and the same scale_w: accumulators and
 * outputs are bit-identical to the expanded layer's, with no duplicated channels anywhere.
 */
int ocs_fold_weights(const int8_t *Wq, int64_t ldq, int64_t N, int C, int g, int num_splits,
                     const int32_t *chan_src, int8_t *Wf, int64_t ldf, int32_t *max_abs_out,
                     void *stream);

/*
 * Measurement helper (no passage of the paper).  Arms a pair of caller-created hipEvent_t
 * (created with timing enabled) for the calling thread's NEXT launch of one kernel family:
 * OCS_TIME_SPLIT_QUANTIZE (the streaming pass of ocs_split_act / ocs_quantize /
 * ocs_split_weights), OCS_TIME_GEMM (ocs_qgemm) or OCS_TIME_ABSMAX (the pass that takes the
 * largest magnitude for a per-batch grid).  That launch stamps the events with the kernel's
 * own begin and end, so hipEventElapsedTime(start, stop) is the kernel's duration as a
 * profiler reports it.  One pair may be pending per family; a pair is used once.  Returns
 * OCS_E_MODE for an unknown family.
 */
#define OCS_TIME_SPLIT_QUANTIZE 1
#define OCS_TIME_GEMM 2
#define OCS_TIME_ABSMAX 3
int ocs_time_next(int family, void *start_event, void *stop_event);

/*
 * Measurement helper (no passage of the paper): a plain device-to-device copy of `bytes`
 * bytes (multiple of 16, both pointers 16-byte aligned) with 16-byte accesses, as a grid-stride
 * loop of `workgroups` workgroups of 256 lanes, or, with workgroups == 0, in the one-shot form:
 * one 16-byte group per lane, one workgroup per 4 KB, no loop (the form the chip streams
 * fastest; the split+quantize pass is built the same way).  Profiling runs use the copy to scale
 * HBM byte counters against a transfer of known size.
 */
int ocs_calib_copy(const void *src, void *dst, size_t bytes, int workgroups, void *stream);

/*
 * Further measurement helpers (no passage of the paper; the path never calls them): plain kernels
 * of known work whose rates are this chip's own ceilings for the kernels of the path.  workgroups
 * == 0 selects the one-shot form everywhere (see ocs_calib_copy).
 *   ocs_calib_pack: the split+quantize pass's traffic pattern without its arithmetic: 16 bytes read
 *        and 4 written per lane (`bytes` = bytes read, multiple of 16; dst holds bytes / 4).
 *   ocs_calib_read: `passes` read-only sweeps with 16-byte loads over `bytes` bytes at src
 *        (multiple of 16, 16-byte aligned; with passes > 1 a power of two, and workgroups >= 1).
 *        A buffer far larger than the caches with one pass gives the HBM read rate; a buffer of a
 *        megabyte or two with many passes stays in every L2 and gives the rate at which the compute
 *        units draw from their L2s.  sink: device int32 [max(workgroups, 1)] (practically never
 *        written).
 *   ocs_calib_fill: writes `bytes` bytes at dst with 16-byte stores of `value` (nontemporal != 0:
 *        with the streaming hint).
 *   ocs_calib_mfma: `workgroups` (>= 1) workgroups of 4 waves; every wave issues iters * 4
 *        instructions v_mfma_i32_32x32x32_i8 (the GEMM's) on fragments taken from `operands`
 *        (device, 16 KB, 16-byte aligned: zeros, a constant, or random bytes), with no memory access
 *        inside the loop: workgroups * 4 * iters * 4 * 65536 integer operations per launch.
 *        sink: device int32 [workgroups * 256], written.
 * All are asynchronous on `stream`; time them with events around the call.
 */
int ocs_calib_pack(const void *src, void *dst, size_t bytes, int workgroups, void *stream);
int ocs_calib_read(const void *src, size_t bytes, int passes, int workgroups, void *sink, void *stream);
int ocs_calib_fill(void *dst, size_t bytes, int value, int nontemporal, int workgroups, void *stream);
int ocs_calib_mfma(const void *operands, int iters, int workgroups, void *sink, void *stream);

/*
 * Launch-shape overrides for benchmarking (no passage of the paper; results never depend
 * on them).  Keys: "act_grid", "act_nt", "act_un", "act_map", "act_wide", "act_dep", "act_tile",
 * "act_np" (the split+quantize pass; act_tile: the tile-ordered variant never (0) / wherever it
 * fits (1); act_np: the one-shot variant never (0) / with 1..8 loads per lane wherever that many
 * hold a row (1..8) / wherever it serves the shape (9); default: by shape), "max_flat", "max_grid",
 * "max_un", "max_bt" (the whole-tensor max|x|
 * pass; max_flat 2: the flat pass, and ocs_split_act folds its maxima in a launch of its own whatever the tensor's size), "sel_inline" (most splits for which ocs_split_weights runs the selection inside its
 * code pass instead of as a launch of its own; 0: never), "gemm_tile" (tile variant of
 * ocs_qgemm / ocs_qconv: 6, 7, 9, 10, 11, 12, 14, 16, 17, 18, 19, 23, 24, 25; an id a shape cannot use falls
 * back to one it can), "fused_variant" (ocs_split_act_qgemm with more than 128 output columns:
 * 1 = 64-row workgroups, 2 = 128-row ones), "fused_stride" (rows between that kernel's workgroups: 0 = a
 * whole tile always, n > 0 = n).  value < 0 restores the default.  Returns OCS_OK or OCS_E_MODE for an
 * unknown key.  The settings belong to the calling thread and affect its own calls only.
 */
int ocs_tune(const char *key, int value);

#ifdef __cplusplus
}
#endif
#endif /* OCS_H */
