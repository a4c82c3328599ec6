/*
 * CPU oracle for the OCS-expanded quantized layer (Zhao et al., "Improving Neural
 * Network Quantization without Retraining using Outlier Channel Splitting").
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, literal statement of what the
 * method computes; the GPU library never calls it, links it or shares a line with it.
 * Everything here works on host pointers, one element at a time, in the order the
 * paper describes the method:
 *
 *   Sec. 3.4   split budget ceil(r*C); splits are made one at a time, each on the
 *              channel that currently holds the largest |value| in the layer
 *   Sec. 3.2   Eq. 3 (duplicate the channel, halve both weight copies) and Eq. 4
 *              (duplicate the channel, halve both activation copies)
 *   Sec. 3.1   Eq. 1, symmetric k-bit linear grid with 2^k - 1 points
 *   Sec. 1     clipping = narrowing the grid, i.e. saturating beyond a threshold
 *   Sec. 5.2   OCS first, clip afterwards
 *   Sec. 3.2   Eq. 2, the linear layer, evaluated on the integer codes
 *   Sec. 3.3   quantization-aware splitting of the weights, with that section's
 *              rounding function floor(x + 1/2)
 *   Sec. 4.1   clip threshold of least mean squared error over a histogram
 *
 * Precision.  A code is an integer decided by floating point, so the decision is taken
 * in the arithmetic the GPU kernels use: fp32, one correctly rounded division
 * qmax / T, one multiply, round-half-to-even, saturate.  Halving is exact in any
 * binary format.  The dequantized output is evaluated in fp64.
 *
 * Parity pins live in tests/test_oracle_pins.py (functional identity of the split
 * layer, halving of every split channel's maximum, greedy == brute force, the grid's
 * definition, the s = 0 case against a library matmul, the w = 3 example of Sec. 3.3,
 * Table 4's weight-size row, the rounded QA pair adding up to the rounded original, the
 * histogram against a library histogram and the error against its element-wise definition).
 * Unpinned: nothing in this file; the paper's accuracy tables are not reproduced
 * (datasets and trained weights are needed for those).
 *
 * Build: gcc -O2 -std=c99 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC
 * OpenMP only partitions independent rows over threads; it changes no arithmetic.
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <omp.h>

#define REF_OK 0
#define REF_E_ARG (-1)
#define REF_E_OVERFLOW (-2)
#define REF_E_NOMEM (-3)

#define REF_MODE_HALVE 0 /* Eq. 3: greedy selection on this tensor, both copies halved   */
#define REF_MODE_DUP 1   /* Eq. 4, weight side: selection given, copies left un-halved   */

void ref_set_threads(int n) {
    if (n > 0) omp_set_num_threads(n);
}

int ref_get_threads(void) { return omp_get_max_threads(); }

/* Sec. 3.4: a layer with C channels receives ceil(r*C) splits. */
int ref_num_splits(int C, double r) {
    if (C <= 0 || !(r > 0.0)) return 0;
    return (int)ceil(r * (double)C);
}

/*
 * Sec. 3.4 + Eq. 3 / Eq. 4 (weight side), done literally.
 *
 * T is [rows, C*g] row-major with leading dimension ld; channel c owns columns
 * c*g .. c*g+g-1 (a 2-D filter of an im2col'd convolution, or one column of an FC
 * layer).  T_out is [rows, (C+s)*g] with leading dimension ldo and always receives
 * the expanded tensor.
 *
 * MODE_HALVE: for each of the s steps, scan every element of the current expanded
 * tensor, take the channel holding the largest magnitude (lowest expanded index on
 * ties), append a copy of that channel at index C+i and multiply both copies by one
 * half.  split_src[i] receives the expanded index that step i split.
 * MODE_DUP: split_src is an input; the chosen channel is copied without scaling
 * (the halving is applied to the activations instead).
 *
 * chan_src[j]  = original channel that expanded channel j descends from.
 * chan_depth[j] = number of halvings that expanded channel j has gone through.
 * max_out      = largest magnitude in the expanded tensor (may be NULL).
 */
int ref_split_weights(const float *T, int64_t rows, int C, int g, int64_t ld, int s, int mode,
                      int32_t *split_src, int32_t *chan_src, int32_t *chan_depth, float *T_out,
                      int64_t ldo, float *max_out) {
    if (!T || !T_out || !chan_src || !chan_depth || (s > 0 && !split_src)) return REF_E_ARG;
    if (rows <= 0 || C <= 0 || g <= 0 || s < 0) return REF_E_ARG;
    if (ld < (int64_t)C * g || ldo < (int64_t)(C + s) * g) return REF_E_ARG;

    for (int64_t n = 0; n < rows; ++n)
        for (int64_t k = 0; k < (int64_t)C * g; ++k) T_out[n * ldo + k] = T[n * ld + k];
    for (int j = 0; j < C; ++j) {
        chan_src[j] = j;
        chan_depth[j] = 0;
    }

    for (int i = 0; i < s; ++i) {
        int cur = C + i; /* channels present before this step */
        int pick;
        if (mode == REF_MODE_HALVE) {
            float best = -1.0f;
            pick = 0;
            for (int j = 0; j < cur; ++j)
                for (int64_t n = 0; n < rows; ++n)
                    for (int t = 0; t < g; ++t) {
                        float a = fabsf(T_out[n * ldo + (int64_t)j * g + t]);
                        if (a > best) {
                            best = a;
                            pick = j;
                        }
                    }
            split_src[i] = pick;
        } else {
            pick = split_src[i];
            if (pick < 0 || pick >= cur) return REF_E_ARG;
        }
        for (int64_t n = 0; n < rows; ++n)
            for (int t = 0; t < g; ++t) {
                float v = T_out[n * ldo + (int64_t)pick * g + t];
                if (mode == REF_MODE_HALVE) v = v * 0.5f;
                T_out[n * ldo + (int64_t)pick * g + t] = v;
                T_out[n * ldo + (int64_t)cur * g + t] = v;
            }
        chan_depth[pick] += 1;
        chan_src[cur] = chan_src[pick];
        chan_depth[cur] = chan_depth[pick];
    }

    if (max_out) {
        float m = 0.0f;
        for (int64_t n = 0; n < rows; ++n)
            for (int64_t k = 0; k < (int64_t)(C + s) * g; ++k) {
                float a = fabsf(T_out[n * ldo + k]);
                if (a > m) m = a;
            }
        *max_out = m;
    }
    return REF_OK;
}

/* One value onto the grid of Eq. 1 with range [-T, T]: fp32 decision (see header). */
static int8_t code_of(float v, float inv_step, float qmax) {
    float p = v * inv_step;
    float r = nearbyintf(p); /* round-half-to-even under the default rounding mode */
    if (r > qmax) r = qmax;
    if (r < -qmax) r = -qmax;
    return (int8_t)r;
}

/* qmax / T, kept finite: for T below about 1e-36 the fp32 quotient overflows, and an
 * infinite factor would send the value 0 to NaN although Eq. 1 maps 0 to the grid point 0. */
static float inv_step_of(float T, float qmax) {
    if (!(T > 0.0f)) return 0.0f;
    float inv = qmax / T;
    return inv > FLT_MAX ? FLT_MAX : inv;
}

/*
 * Eq. 1 with an optional clip threshold (Sec. 1; Sec. 5.2 for clip-after-OCS).
 * x [rows, cols] (ld ldx) -> codes q [rows, ldq], columns cols..ldq-1 set to zero.
 * threshold != NULL: T = *threshold.  Otherwise T = clip_ratio * max|x|.
 * scale_out = {T, T / qmax}.
 */
int ref_quantize(const float *x, int64_t rows, int64_t cols, int64_t ldx, int bits,
                 const float *threshold, float clip_ratio, int8_t *q, int64_t ldq,
                 float *scale_out) {
    if (!x || !q || !scale_out) return REF_E_ARG;
    if (rows <= 0 || cols <= 0 || ldx < cols || ldq < cols) return REF_E_ARG;
    if (bits < 2 || bits > 8) return REF_E_ARG;
    float qmax = (float)((1 << (bits - 1)) - 1);
    float T;
    if (threshold) {
        T = *threshold;
    } else {
        float m = 0.0f;
        for (int64_t i = 0; i < rows; ++i)
            for (int64_t k = 0; k < cols; ++k) {
                float a = fabsf(x[i * ldx + k]);
                if (a > m) m = a;
            }
        T = clip_ratio * m;
    }
    float inv = inv_step_of(T, qmax);
    scale_out[0] = T;
    scale_out[1] = T / qmax;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        for (int64_t k = 0; k < cols; ++k) q[i * ldq + k] = code_of(x[i * ldx + k], inv, qmax);
        for (int64_t k = cols; k < ldq; ++k) q[i * ldq + k] = 0;
    }
    return REF_OK;
}

/* Sec. 3.3's rounding function Q(x) = floor(x + 1/2) on the saturated fp32 product: one
 * fp32 add, then floor.  Used for quantization-aware split weights only. */
static int8_t code_of_half_up(float v, float inv_step, float qmax) {
    float p = v * inv_step;
    if (p > qmax) p = qmax;
    if (p < -qmax) p = -qmax;
    return (int8_t)floorf(p + 0.5f);
}

/*
 * Sec. 3.3, quantization-aware (QA) splitting of the weights, followed by Eq. 1 with the
 * rounding function of that section.
 *
 * In units of the grid step a QA split sends w to the pair ((w - 1/2)/2, (w + 1/2)/2), so
 * that the two rounded members add up to the rounded original.  The paper leaves open how
 * the grid step can be known before the splits that determine it, and which member stays
 * in place.  Reading taken here:
 *   1. the splits are chosen, and the threshold fixed, by the plain-halving procedure of
 *      Sec. 3.4 / Eq. 3 on the same tensor: T = clip_ratio * max|halved tensor|,
 *      step = T / qmax;
 *   2. the same split list is then replayed on the original tensor with the QA pair, in
 *      tensor units: the channel that keeps its index becomes (v - step/2)/2, the appended
 *      copy (v + step/2)/2 (the order in which the pair is written);
 *   3. fp32, one subtraction (or addition) and one exact halving per split step;
 *   4. codes by Q(x) = floor(x + 1/2) with the threshold T of step 1.
 * chan_path[j] records expanded channel j's history, one bit per split it went through,
 * first split in bit 0: 0 = kept its index (minus member), 1 = was the appended copy (plus
 * member).  A lineage grows only like log2(s) (equal copies are split in turn), so 32 bits
 * are ample; more than 31 splits on one lineage is refused all the same.
 * T_out [rows, (C+s)*g] receives the QA-split fp32 tensor, q its codes (pad columns zero),
 * scale_out = {T, step}.
 */
int ref_split_weights_qa(const float *T, int64_t rows, int C, int g, int64_t ld, int s, int bits,
                         float clip_ratio, int32_t *split_src, int32_t *chan_src,
                         int32_t *chan_depth, uint32_t *chan_path, float *T_out, int64_t ldo,
                         int8_t *q, int64_t ldq, float *scale_out) {
    if (!T || !T_out || !chan_src || !chan_depth || !chan_path || !q || !scale_out) return REF_E_ARG;
    if (s > 0 && !split_src) return REF_E_ARG;
    if (rows <= 0 || C <= 0 || g <= 0 || s < 0 || bits < 2 || bits > 8) return REF_E_ARG;
    int64_t K = (int64_t)C * g, Ke = (int64_t)(C + s) * g;
    if (ld < K || ldo < Ke || ldq < Ke) return REF_E_ARG;
    float qmax = (float)((1 << (bits - 1)) - 1);

    /* 1. selection and threshold from the plain-halving procedure */
    float *halved = (float *)malloc((size_t)rows * (size_t)Ke * sizeof(float));
    if (!halved) return REF_E_NOMEM;
    float m = 0.0f;
    int rc = ref_split_weights(T, rows, C, g, ld, s, REF_MODE_HALVE, split_src, chan_src,
                               chan_depth, halved, Ke, &m);
    free(halved);
    if (rc != REF_OK) return rc;
    float Tthr = clip_ratio * m;
    float step = Tthr / qmax;
    float half_step = step * 0.5f;

    /* 2./3. replay the list with the QA pair */
    for (int64_t n = 0; n < rows; ++n)
        for (int64_t k = 0; k < K; ++k) T_out[n * ldo + k] = T[n * ld + k];
    int *len = (int *)calloc((size_t)(C + s), sizeof(int));
    if (!len) return REF_E_NOMEM;
    for (int j = 0; j < C + s; ++j) chan_path[j] = 0u;
    for (int i = 0; i < s; ++i) {
        int pick = split_src[i], cur = C + i;
        if (len[pick] >= 31) {
            free(len);
            return REF_E_ARG;
        }
        for (int64_t n = 0; n < rows; ++n)
            for (int t = 0; t < g; ++t) {
                float v = T_out[n * ldo + (int64_t)pick * g + t];
                float lo = v - half_step;
                float hi = v + half_step;
                T_out[n * ldo + (int64_t)pick * g + t] = lo * 0.5f;
                T_out[n * ldo + (int64_t)cur * g + t] = hi * 0.5f;
            }
        chan_path[cur] = chan_path[pick] | (1u << len[pick]);
        len[pick] += 1;
        len[cur] = len[pick];
    }
    free(len);

    /* 4. codes */
    float inv = inv_step_of(Tthr, qmax);
    scale_out[0] = Tthr;
    scale_out[1] = step;
    for (int64_t n = 0; n < rows; ++n) {
        for (int64_t k = 0; k < Ke; ++k)
            q[n * ldq + k] = code_of_half_up(T_out[n * ldo + k], inv, qmax);
        for (int64_t k = Ke; k < ldq; ++k) q[n * ldq + k] = 0;
    }
    return REF_OK;
}

/*
 * Sec. 4.1: clip threshold by minimal mean squared error over a histogram.
 *
 * A histogram of the values is built (bin values x_i, frequencies h(x_i), i = 1..n), the
 * error of a candidate threshold T is MSE(T) = 1/n * sum_i h(x_i) * (x_i - Q_T(x_i))^2 with
 * Q_T the quantizer of Eq. 1 on the grid of range [-T, T], candidates are evenly spaced between
 * 0 and max|x|, and the candidate with the least error is taken.  The paper fixes neither the
 * number of bins nor the number of candidates ("a large number"), nor what a bin's value is.
 * Reading taken here:
 *   - the grid is symmetric, so the histogram is taken over |x|: n equal bins on [0, m],
 *     m = max|x|; a value falls in bin min(n-1, floor(|x| * (n / m))), decided in fp32 with
 *     one division n / m and one multiply;
 *   - a bin's value is its centre, x_i = (i + 1/2) * (m / n) in fp32 (i counted from 0);
 *   - candidates T_c = m * (c / n_cand), c = 1..n_cand, in fp32 (the last one is m itself);
 *   - Q_T(x_i) = code * step with the code decided in fp32 exactly as everywhere else
 *     (qmax / T, one multiply, saturate, round half to even) and step = T / qmax;
 *   - the error and the sum are evaluated in fp64, bins in increasing order;
 *   - the first candidate with the least error wins.
 * hist [n] (may be NULL) receives the frequencies, mse [n_cand] (may be NULL) the errors,
 * out = {chosen threshold, m}.  m = 0 gives threshold 0.
 */
int ref_mse_clip(const float *x, int64_t rows, int64_t cols, int64_t ldx, int bits, int n_bins,
                 int n_cand, uint64_t *hist, double *mse, float *out) {
    if (!x || !out) return REF_E_ARG;
    if (rows <= 0 || cols <= 0 || ldx < cols || bits < 2 || bits > 8) return REF_E_ARG;
    if (n_bins < 1 || n_cand < 1) return REF_E_ARG;
    float qmax = (float)((1 << (bits - 1)) - 1);
    float m = 0.0f;
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t k = 0; k < cols; ++k) {
            float a = fabsf(x[i * ldx + k]);
            if (a > m) m = a;
        }
    uint64_t *h = (uint64_t *)calloc((size_t)n_bins, sizeof(uint64_t));
    if (!h) return REF_E_NOMEM;
    float to_bin = m > 0.0f ? (float)n_bins / m : 0.0f;
    if (to_bin > FLT_MAX) to_bin = FLT_MAX;
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t k = 0; k < cols; ++k) {
            float p = fabsf(x[i * ldx + k]) * to_bin;
            int b = p >= (float)n_bins ? n_bins - 1 : (int)p;
            h[b] += 1;
        }
    float width = m / (float)n_bins;
    int best_c = 1;
    double best = 0.0;
    for (int c = 1; c <= n_cand; ++c) {
        float T = m * ((float)c / (float)n_cand);
        float inv = inv_step_of(T, qmax);
        float step = T / qmax;
        double sum = 0.0;
        for (int i = 0; i < n_bins; ++i) {
            float xi = ((float)i + 0.5f) * width;
            double e = (double)xi - (double)code_of(xi, inv, qmax) * (double)step;
            sum += (double)h[i] * (e * e);
        }
        double err = sum / (double)n_bins;
        if (mse) mse[c - 1] = err;
        if (c == 1 || err < best) {
            best = err;
            best_c = c;
        }
    }
    if (hist) memcpy(hist, h, (size_t)n_bins * sizeof(uint64_t));
    free(h);
    out[0] = m * ((float)best_c / (float)n_cand);
    out[1] = m;
    return REF_OK;
}

/*
 * Sec. 3.3 on the activation side (Eq. 4 with the quantization-aware pair): the split list
 * (chosen by the plain-halving procedure on the batch, as for the weights) is replayed on the
 * activations; at each split the channel that keeps its index becomes (x - step/2)/2 and the
 * appended copy (x + step/2)/2, step = T / qmax with the given threshold T of the activation
 * grid; codes by Q(x) = floor(x + 1/2).  Same fp32 order as ref_split_weights_qa.
 * Xf (may be NULL) receives the expanded fp32 activations [M, (C+s)*g].
 */
int ref_split_act_qa(const float *X, int64_t M, int C, int g, int64_t ldx, const int32_t *split_src,
                     int s, int bits, float T, int8_t *Xq, int64_t ldq, float *scale_out, float *Xf,
                     int64_t ldf) {
    if (!X || !Xq || !scale_out || (s > 0 && !split_src)) return REF_E_ARG;
    if (M <= 0 || C <= 0 || g <= 0 || s < 0 || bits < 2 || bits > 8) return REF_E_ARG;
    int64_t K = (int64_t)C * g, Ke = (int64_t)(C + s) * g;
    if (ldx < K || ldq < Ke || (Xf && ldf < Ke)) return REF_E_ARG;
    float qmax = (float)((1 << (bits - 1)) - 1);
    float step = T / qmax, half_step = step * 0.5f;
    float inv = inv_step_of(T, qmax);
    float *E = (float *)malloc((size_t)M * (size_t)Ke * sizeof(float));
    if (!E) return REF_E_NOMEM;
    for (int64_t i = 0; i < M; ++i)
        for (int64_t k = 0; k < K; ++k) E[i * Ke + k] = X[i * ldx + k];
    for (int i = 0; i < s; ++i) {
        int pick = split_src[i], cur = C + i;
        if (pick < 0 || pick >= cur) {
            free(E);
            return REF_E_ARG;
        }
        for (int64_t r = 0; r < M; ++r)
            for (int t = 0; t < g; ++t) {
                float v = E[r * Ke + (int64_t)pick * g + t];
                float lo = v - half_step;
                float hi = v + half_step;
                E[r * Ke + (int64_t)pick * g + t] = lo * 0.5f;
                E[r * Ke + (int64_t)cur * g + t] = hi * 0.5f;
            }
    }
    scale_out[0] = T;
    scale_out[1] = step;
    for (int64_t r = 0; r < M; ++r) {
        for (int64_t k = 0; k < Ke; ++k) {
            Xq[r * ldq + k] = code_of_half_up(E[r * Ke + k], inv, qmax);
            if (Xf) Xf[r * ldf + k] = E[r * Ke + k];
        }
        for (int64_t k = Ke; k < ldq; ++k) Xq[r * ldq + k] = 0;
    }
    free(E);
    return REF_OK;
}

/*
 * The activation side of Eq. 3 / Eq. 4 followed by Eq. 1 (Sec. 3.5: a layer that copies
 * and scales the chosen channels).  Expanded channel j of the output reads original
 * channel chan_src[j]; with chan_depth != NULL it is multiplied by 2^-chan_depth[j]
 * (Eq. 4), with chan_depth == NULL it is copied as is (Eq. 3: the weights carry the
 * halving).  Xf (may be NULL) receives the expanded fp32 activations [M, (C+s)*g].
 * Threshold: *threshold if given, else clip_ratio * max|expanded activations|.
 */
int ref_split_act(const float *X, int64_t M, int C, int g, int64_t ldx, const int32_t *chan_src,
                  const int32_t *chan_depth, int s, int bits, const float *threshold,
                  float clip_ratio, int8_t *Xq, int64_t ldq, float *scale_out, float *Xf,
                  int64_t ldf) {
    if (!X || !Xq || !scale_out || (s > 0 && !chan_src)) return REF_E_ARG;
    if (M <= 0 || C <= 0 || g <= 0 || s < 0) return REF_E_ARG;
    int64_t K = (int64_t)C * g, Ke = (int64_t)(C + s) * g;
    if (ldx < K || ldq < Ke || (Xf && ldf < Ke)) return REF_E_ARG;
    if (bits < 2 || bits > 8) return REF_E_ARG;
    for (int j = 0; j < C + s; ++j) {
        int src = chan_src ? chan_src[j] : j;
        if (src < 0 || src >= C) return REF_E_ARG;
        if (chan_depth && chan_depth[j] < 0) return REF_E_ARG;
    }
    float qmax = (float)((1 << (bits - 1)) - 1);

    float *E = (float *)malloc((size_t)M * (size_t)Ke * sizeof(float));
    if (!E) return REF_E_NOMEM;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int j = 0; j < C + s; ++j) {
            int src = chan_src ? chan_src[j] : j;
            float f = chan_depth ? ldexpf(1.0f, -chan_depth[j]) : 1.0f;
            for (int t = 0; t < g; ++t)
                E[i * Ke + (int64_t)j * g + t] = X[i * ldx + (int64_t)src * g + t] * f;
        }

    float T;
    if (threshold) {
        T = *threshold;
    } else {
        float m = 0.0f;
        for (int64_t e = 0; e < M * Ke; ++e) {
            float a = fabsf(E[e]);
            if (a > m) m = a;
        }
        T = clip_ratio * m;
    }
    float inv = inv_step_of(T, qmax);
    scale_out[0] = T;
    scale_out[1] = T / qmax;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t k = 0; k < Ke; ++k) {
            Xq[i * ldq + k] = code_of(E[i * Ke + k], inv, qmax);
            if (Xf) Xf[i * ldf + k] = E[i * Ke + k];
        }
        for (int64_t k = Ke; k < ldq; ++k) Xq[i * ldq + k] = 0;
    }
    free(E);
    return REF_OK;
}

/*
 * Eq. 2 on the codes of the expanded layer: acc[i,n] = sum_k Xq[i,k] * Wq[n,k],
 * accumulated in 64 bits and required to fit in 32; then the trailing factors of
 * Eq. 1 for both operands, in fp64: Y = acc * step_x * step_w.
 * acc_out and Y may each be NULL.
 */
int ref_qgemm(const int8_t *Xq, int64_t ldx, const int8_t *Wq, int64_t ldw, int64_t M, int64_t N,
              int64_t Kexp, float step_x, float step_w, int32_t *acc_out, int64_t ldacc, double *Y,
              int64_t ldy) {
    if (!Xq || !Wq) return REF_E_ARG;
    if (M <= 0 || N <= 0 || Kexp <= 0 || ldx < Kexp || ldw < Kexp) return REF_E_ARG;
    if ((acc_out && ldacc < N) || (Y && ldy < N)) return REF_E_ARG;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t n = 0; n < N; ++n) {
            int64_t a = 0;
            for (int64_t k = 0; k < Kexp; ++k)
                a += (int64_t)Xq[i * ldx + k] * (int64_t)Wq[n * ldw + k];
            if (a > INT32_MAX || a < INT32_MIN) bad |= 1;
            if (acc_out) acc_out[i * ldacc + n] = (int32_t)a;
            if (Y) Y[i * ldy + n] = (double)a * ((double)step_x * (double)step_w);
        }
    return bad ? REF_E_OVERFLOW : REF_OK;
}

/*
 * The layer's output handed to the next layer as codes instead of fp32: what Eq. 1 (and the
 * activation side of Eq. 3 for the NEXT layer's split channels) makes of the dequantized
 * output, with a static grid.  Per element, in fp32 as the GPU's epilogue computes it:
 * y = float(acc) * (step_x * step_w); optionally y = max(y, 0); code = Q(y) on the grid of
 * range [-T_next, T_next] with bits_next bits.  Expanded output channel j < N + s_next reads
 * output channel chan_src_next[j] (NULL: identity, s_next = 0).  Columns N + s_next .. ldq-1
 * are set to zero.  scale_out = {T_next, T_next / qmax}.
 */
int ref_requantize(const int32_t *acc, int64_t ldacc, int64_t M, int64_t N, float step_x, float step_w,
                   int relu, int bits_next, float T_next, const int32_t *chan_src_next, int s_next,
                   int8_t *Yq, int64_t ldq, float *scale_out) {
    if (!acc || !Yq || !scale_out || M <= 0 || N <= 0 || s_next < 0 || ldacc < N) return REF_E_ARG;
    if (ldq < N + s_next || bits_next < 2 || bits_next > 8) return REF_E_ARG;
    if (s_next > 0 && !chan_src_next) return REF_E_ARG;
    float qmax = (float)((1 << (bits_next - 1)) - 1);
    float inv = inv_step_of(T_next, qmax);
    float scale = step_x * step_w;
    scale_out[0] = T_next;
    scale_out[1] = T_next / qmax;
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N + s_next; ++j) {
            int64_t src = chan_src_next ? chan_src_next[j] : j;
            if (src < 0 || src >= N) return REF_E_ARG;
            float y = (float)acc[i * ldacc + src] * scale;
            if (relu && !(y > 0.0f)) y = 0.0f;
            Yq[i * ldq + j] = code_of(y, inv, qmax);
        }
        for (int64_t j = N + s_next; j < ldq; ++j) Yq[i * ldq + j] = 0;
    }
    return REF_OK;
}

/*
 * The expanded layer of Eq. 3 run without expanding it.  In Eq. 2 on codes, a duplicated
 * activation channel multiplies each of its weight copies by the same activation code, so
 *   sum_j Xq[i, src(j)] * Wq[n, j]  =  sum_c Xq[i, c] * (sum over the copies j of c of Wq[n, j]):
 * the integer accumulator of the expanded layer equals that of an un-expanded layer whose
 * weight code for channel c is the SUM of the codes of c's copies.  The sum needs more range
 * than one copy (up to copies * qmax), which int8 has to spare whenever the weights use fewer
 * than 8 bits.  Wf[n, c*g + t] = sum_{j: chan_src[j] == c} Wq[n, j*g + t]; columns C*g .. ldf-1
 * zero; *max_abs = the largest |sum|.  Sums beyond +-127 are stored saturated and make the
 * result unusable: the caller checks *max_abs <= 127.
 */
int ref_fold_weights(const int8_t *Wq, int64_t ldq, int64_t N, int C, int g, int s,
                     const int32_t *chan_src, int8_t *Wf, int64_t ldf, int32_t *max_abs) {
    if (!Wq || !Wf || !max_abs || N <= 0 || C <= 0 || g <= 0 || s < 0) return REF_E_ARG;
    if (s > 0 && !chan_src) return REF_E_ARG;
    if (ldq < (int64_t)(C + s) * g || ldf < (int64_t)C * g) return REF_E_ARG;
    int32_t worst = 0;
    for (int64_t n = 0; n < N; ++n) {
        for (int c = 0; c < C; ++c)
            for (int t = 0; t < g; ++t) {
                int32_t sum = 0;
                for (int j = 0; j < C + s; ++j) {
                    int src = chan_src ? chan_src[j] : j;
                    if (src == c) sum += Wq[n * ldq + (int64_t)j * g + t];
                }
                int32_t a = sum < 0 ? -sum : sum;
                if (a > worst) worst = a;
                Wf[n * ldf + (int64_t)c * g + t] = (int8_t)(sum > 127 ? 127 : (sum < -127 ? -127 : sum));
            }
        for (int64_t k = (int64_t)C * g; k < ldf; ++k) Wf[n * ldf + k] = 0;
    }
    *max_abs = worst;
    return REF_OK;
}

/*
 * Eq. 2 itself on real-valued operands, in fp64: Y[i,n] = sum_k X[i,k] * W[n,k].
 * Used to state the functional identity of Eq. 3 / Eq. 4 (split layer == unsplit layer).
 */
int ref_layer_f64(const float *X, int64_t ldx, const float *W, int64_t ldw, int64_t M, int64_t N,
                  int64_t K, double *Y, int64_t ldy) {
    if (!X || !W || !Y || M <= 0 || N <= 0 || K <= 0) return REF_E_ARG;
    if (ldx < K || ldw < K || ldy < N) return REF_E_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t n = 0; n < N; ++n) {
            double a = 0.0;
            for (int64_t k = 0; k < K; ++k) a += (double)X[i * ldx + k] * (double)W[n * ldw + k];
            Y[i * ldy + n] = a;
        }
    return REF_OK;
}
