/*
 * CPU oracle for the binary-HDC hot path of arXiv 2206.04746 (HDTorch).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the yardstick the GPU library is checked
 * against; it is never part of the product path.  It shares no code, header, table
 * or helper with the HIP library and is written for obviousness, not speed: every
 * hypervector is held one byte per dimension and every operation is the plain
 * definition (or, for online training, the algorithm step by step).  The only
 * concession to run time is an OpenMP "parallel for" over independent samples, which
 * changes no arithmetic.
 *
 * What follows the paper and where:
 *   - encoding: Sec. III, Eq. (1) - bind ID and level vectors by XOR, add over the
 *     features per dimension, majority vote back to bits;
 *   - classical training: Sec. III - one-pass accumulation of a class's encoded
 *     vectors, majority vote to a class vector;
 *   - online training: Sec. III, Eqs. (2),(3) and the caption of Fig. 1 - per
 *     datapoint, similarity-weighted add to the target class and subtract from the
 *     wrongly predicted class;
 *   - inference: Sec. III - Hamming distance to every class vector, nearest wins.
 *
 * Readings where the paper is silent (all listed with reasons in the design notes):
 *   bins are equal-width with floor and clamping; majority is strict and an exact tie
 *   takes the bit of a caller-supplied tie vector; bits are packed LSB first with
 *   zero pad bits; the online step uses the cosine between the fp32 accumulator row
 *   and the bipolar view s = 2h-1 of the sample, weight (1 - cos) for both the add and
 *   the subtract, learning rate on the subtract only, dot products and norms in fp64,
 *   a zero-norm row has cosine 0, ties in argmin/argmax go to the lowest class.
 *
 * Pin status: encode, classical training, binarisation, search and the quantiser are
 * pinned by closed forms, brute force and invariants (tests/test_oracle_*.py).
 * Online training is pinned only by hand-worked cases and closed forms for special
 * inputs; the paper prints no worked example, so beyond those: parity unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Threads the "parallel for" loops over samples will use (1 without OpenMP). */
int32_t orc_threads(void)
{
#ifdef _OPENMP
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---- layout helpers (Sec. IV-B1: bits are packed into 32-bit integers) -------- */

/* words[r][W] -> bits[r][D], dimension d = bit (d mod 32) of word (d div 32). */
void orc_unpack(const uint32_t *words, int64_t rows, int32_t D, uint8_t *bits)
{
    const int64_t W = (D + 31) / 32;
    for (int64_t r = 0; r < rows; ++r)
        for (int32_t d = 0; d < D; ++d)
            bits[r * D + d] = (uint8_t)((words[r * W + (d >> 5)] >> (d & 31)) & 1u);
}

/* bits[r][D] -> words[r][W]; bits D..32W-1 of the last word stay 0. */
void orc_pack(const uint8_t *bits, int64_t rows, int32_t D, uint32_t *words)
{
    const int64_t W = (D + 31) / 32;
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t w = 0; w < W; ++w)
            words[r * W + w] = 0u;
        for (int32_t d = 0; d < D; ++d)
            if (bits[r * D + d])
                words[r * W + (d >> 5)] |= (uint32_t)1u << (d & 31);
    }
}

/* ---- discretisation (Sec. III: feature values fall into a fixed number of bins) ---- */

/* Equal-width bins over [lo, hi): t = (x - lo) * scale with scale = float(L/(hi-lo)),
 * two separately rounded fp32 operations; bin = floor(t) clamped to [0, L-1];
 * anything that is not >= 0 (negative, NaN) goes to bin 0. */
void orc_quantize_f32(const float *x, int64_t N, int32_t F, const float *lo,
                      const float *scale, int32_t L, int32_t *q)
{
    for (int64_t n = 0; n < N; ++n)
        for (int32_t f = 0; f < F; ++f) {
            volatile float diff = x[n * F + f] - lo[f]; /* volatile: no fused multiply-add */
            float t = diff * scale[f];
            int32_t b;
            if (!(t >= 0.0f))
                b = 0;
            else if (t >= (float)L)
                b = L - 1;
            else
                b = (int32_t)t;
            q[n * F + f] = b;
        }
}

/* Byte features 0..255 split into L equal bins: bin = floor(x * L / 256). */
void orc_quantize_u8(const uint8_t *x, int64_t N, int32_t F, int32_t L, int32_t *q)
{
    for (int64_t n = 0; n < N; ++n)
        for (int32_t f = 0; f < F; ++f)
            q[n * F + f] = ((int32_t)x[n * F + f] * L) / 256;
}

/* ---- encoding, Eq. (1) -------------------------------------------------------- */

/* hv[n][d] = majority over f of ( item[f][d] XOR level[q[n][f]][d] ), strict
 * majority 2c > F; an exact tie 2c == F takes tie[d]. */
void orc_encode(const int32_t *q, int64_t N, int32_t F, int32_t D,
                const uint8_t *item, const uint8_t *level, const uint8_t *tie,
                uint8_t *hv)
{
#pragma omp parallel
    {
        int32_t *cnt = (int32_t *)malloc((size_t)D * sizeof(int32_t));
#pragma omp for schedule(static)
        for (int64_t n = 0; n < N; ++n) {
            for (int32_t d = 0; d < D; ++d)
                cnt[d] = 0;
            for (int32_t f = 0; f < F; ++f) {
                const uint8_t *id = item + (int64_t)f * D;
                const uint8_t *lv = level + (int64_t)q[n * F + f] * D;
                for (int32_t d = 0; d < D; ++d)
                    cnt[d] += id[d] ^ lv[d];
            }
            for (int32_t d = 0; d < D; ++d) {
                int32_t twice = 2 * cnt[d];
                hv[n * D + d] = twice > F ? 1 : twice < F ? 0 : tie[d];
            }
        }
        free(cnt);
    }
}

/* ---- classical training (Sec. III: single-pass accumulation per class) -------- */

/* acc[c][d] += hv[n][d] and class_n[c] += 1 for c = labels[n]; labels outside
 * [0, C) are skipped. acc / class_n are added to, so calls compose. */
void orc_train_classical(const uint8_t *hv, const int32_t *labels, int64_t N, int32_t D,
                         int32_t C, int32_t *acc, int64_t *class_n)
{
    for (int64_t n = 0; n < N; ++n) {
        int32_t c = labels[n];
        if (c < 0 || c >= C)
            continue;
        class_n[c] += 1;
        for (int32_t d = 0; d < D; ++d)
            acc[(int64_t)c * D + d] += hv[n * D + d];
    }
}

/* class vector = majority of the class's samples, same rule as in encoding. */
void orc_binarize_classical(const int32_t *acc, const int64_t *class_n, int32_t C,
                            int32_t D, const uint8_t *tie, uint8_t *class_bits)
{
    for (int32_t c = 0; c < C; ++c)
        for (int32_t d = 0; d < D; ++d) {
            int64_t twice = 2 * (int64_t)acc[(int64_t)c * D + d];
            class_bits[(int64_t)c * D + d] =
                twice > class_n[c] ? 1 : twice < class_n[c] ? 0 : tie[d];
        }
}

/* ---- online training, Eqs. (2),(3) -------------------------------------------- */

/* For each epoch, for each sample in the given order: cosine of every accumulator
 * row with s = 2h-1 (all from the rows as they are before this sample's update),
 * prediction = most similar class, then
 *      acc[y]    += (1 - cos_y) * s                      (always)
 *      acc[pred] -= lr * (1 - cos_pred) * s              (only if pred != y).
 * pred_log (may be NULL) receives the prediction made at every step,
 * margin_log (may be NULL) the gap between the best and second-best cosine. */
void orc_train_online(const uint8_t *hv, const int32_t *labels, int64_t N, int32_t D,
                      int32_t C, int32_t epochs, float lr, float *acc,
                      int32_t *pred_log, double *margin_log)
{
    double *cosv = (double *)malloc((size_t)C * sizeof(double));
    const double root_d = sqrt((double)D);
    int64_t step = 0;
    for (int32_t e = 0; e < epochs; ++e)
        for (int64_t n = 0; n < N; ++n, ++step) {
            const uint8_t *h = hv + n * D;
            const int32_t y = labels[n];
            if (y < 0 || y >= C) {
                if (pred_log) pred_log[step] = -1;
                if (margin_log) margin_log[step] = 0.0;
                continue;
            }
            for (int32_t c = 0; c < C; ++c) {
                const float *m = acc + (int64_t)c * D;
                double dot = 0.0, nrm = 0.0;
                for (int32_t d = 0; d < D; ++d) {
                    double v = (double)m[d];
                    dot += h[d] ? v : -v;
                    nrm += v * v;
                }
                cosv[c] = nrm == 0.0 ? 0.0 : dot / (sqrt(nrm) * root_d);
            }
            int32_t pred = 0;
            for (int32_t c = 1; c < C; ++c)
                if (cosv[c] > cosv[pred])
                    pred = c;
            if (pred_log) pred_log[step] = pred;
            if (margin_log) {
                double second = -2.0;
                for (int32_t c = 0; c < C; ++c)
                    if (c != pred && cosv[c] > second)
                        second = cosv[c];
                margin_log[step] = C > 1 ? cosv[pred] - second : 0.0;
            }
            const float w_y = (float)(1.0 - cosv[y]);
            const float w_p = (float)((double)lr * (1.0 - cosv[pred]));
            float *my = acc + (int64_t)y * D;
            for (int32_t d = 0; d < D; ++d)
                my[d] = h[d] ? my[d] + w_y : my[d] - w_y;
            if (pred != y) {
                float *mp = acc + (int64_t)pred * D;
                for (int32_t d = 0; d < D; ++d)
                    mp[d] = h[d] ? mp[d] - w_p : mp[d] + w_p;
            }
        }
    free(cosv);
}

/* ---- stand-alone summations (Sec. IV-B2) and cosine inference (Sec. III) ------------ */

/* Horizontal summation: out[n] = number of set dimensions of row n. */
void orc_hsum(const uint8_t *bits, int64_t N, int32_t D, int32_t *out)
{
    for (int64_t n = 0; n < N; ++n) {
        int32_t s = 0;
        for (int32_t d = 0; d < D; ++d)
            s += bits[n * D + d];
        out[n] = s;
    }
}

/* Vertical summation: out[d] = number of rows whose dimension d is set. */
void orc_vsum(const uint8_t *bits, int64_t N, int32_t D, int32_t *out)
{
    for (int32_t d = 0; d < D; ++d)
        out[d] = 0;
    for (int64_t n = 0; n < N; ++n)
        for (int32_t d = 0; d < D; ++d)
            out[d] += bits[n * D + d];
}

/* Cosine-similarity inference against real-valued class rows m[C][D]: with s = 2 h - 1,
 * cos[n][c] = <m_c, s> / (|m_c| sqrt(D)), 0 for an all-zero row (the same expression as inside
 * online training); pred[n] = lowest c with the largest cosine.  fp64. */
void orc_search_cosine(const uint8_t *hv, int64_t N, int32_t D, const float *m, int32_t C,
                       double *cosv, int32_t *pred)
{
    const double root_d = sqrt((double)D);
    double *nrm = (double *)malloc((size_t)C * sizeof(double));
    for (int32_t c = 0; c < C; ++c) {
        double s2 = 0.0;
        for (int32_t d = 0; d < D; ++d) {
            double v = (double)m[(int64_t)c * D + d];
            s2 += v * v;
        }
        nrm[c] = s2;
    }
    for (int64_t n = 0; n < N; ++n) {
        const uint8_t *h = hv + n * D;
        int32_t best = 0;
        for (int32_t c = 0; c < C; ++c) {
            const float *row = m + (int64_t)c * D;
            double dot = 0.0;
            for (int32_t d = 0; d < D; ++d) {
                double v = (double)row[d];
                dot += h[d] ? v : -v;
            }
            const double cs = nrm[c] == 0.0 ? 0.0 : dot / (sqrt(nrm[c]) * root_d);
            cosv[n * C + c] = cs;
            if (cs > cosv[n * C + best])
                best = c;
        }
        pred[n] = best;
    }
    free(nrm);
}

/* ---- batched online training (Sec. VI-D2) -------------------------------------- */

/* "Only updating class vectors after a batch size of n new datapoints are received":
 * the class accumulators stay frozen while a batch of `batch` consecutive samples is
 * scored exactly as in orc_train_online (cosines, prediction, weights from the frozen
 * rows); the batch's weighted +-s vectors are summed per class in fp64, in sample
 * order, and added to the rows in one step, acc = float(double(acc) + delta).
 * Reading where the paper is silent: the sum of a batch is formed in fp64 and rounded
 * to fp32 once.  The paper prints no worked example: parity unpinned beyond the
 * hand-worked and closed-form cases in the tests. */
void orc_train_online_batched(const uint8_t *hv, const int32_t *labels, int64_t N, int32_t D,
                              int32_t C, int32_t epochs, float lr, int64_t batch, float *acc)
{
    double *cosv = (double *)malloc((size_t)C * sizeof(double));
    double *nrm = (double *)malloc((size_t)C * sizeof(double));
    double *delta = (double *)malloc((size_t)C * D * sizeof(double));
    const double root_d = sqrt((double)D);
    for (int32_t e = 0; e < epochs; ++e)
        for (int64_t b0 = 0; b0 < N; b0 += batch) {
            const int64_t b1 = b0 + batch < N ? b0 + batch : N;
            for (int64_t i = 0; i < (int64_t)C * D; ++i)
                delta[i] = 0.0;
            for (int32_t c = 0; c < C; ++c) {
                double s2 = 0.0;
                for (int32_t d = 0; d < D; ++d) {
                    double v = (double)acc[(int64_t)c * D + d];
                    s2 += v * v;
                }
                nrm[c] = s2;
            }
            for (int64_t n = b0; n < b1; ++n) {
                const uint8_t *h = hv + n * D;
                const int32_t y = labels[n];
                if (y < 0 || y >= C)
                    continue;
                for (int32_t c = 0; c < C; ++c) {
                    const float *m = acc + (int64_t)c * D;
                    double dot = 0.0;
                    for (int32_t d = 0; d < D; ++d) {
                        double v = (double)m[d];
                        dot += h[d] ? v : -v;
                    }
                    cosv[c] = nrm[c] == 0.0 ? 0.0 : dot / (sqrt(nrm[c]) * root_d);
                }
                int32_t pred = 0;
                for (int32_t c = 1; c < C; ++c)
                    if (cosv[c] > cosv[pred])
                        pred = c;
                const double w_y = (double)(float)(1.0 - cosv[y]);
                const double w_p = (double)(float)((double)lr * (1.0 - cosv[pred]));
                double *dy = delta + (int64_t)y * D;
                for (int32_t d = 0; d < D; ++d)
                    dy[d] += h[d] ? w_y : -w_y;
                if (pred != y) {
                    double *dp = delta + (int64_t)pred * D;
                    for (int32_t d = 0; d < D; ++d)
                        dp[d] += h[d] ? -w_p : w_p;
                }
            }
            for (int64_t i = 0; i < (int64_t)C * D; ++i)
                acc[i] = (float)((double)acc[i] + delta[i]);
        }
    free(cosv);
    free(nrm);
    free(delta);
}

/* class bit = sign of the accumulator; exactly zero takes tie[d]. */
void orc_binarize_online(const float *acc, int32_t C, int32_t D, const uint8_t *tie,
                         uint8_t *class_bits)
{
    for (int32_t c = 0; c < C; ++c)
        for (int32_t d = 0; d < D; ++d) {
            float a = acc[(int64_t)c * D + d];
            class_bits[(int64_t)c * D + d] = a > 0.0f ? 1 : a < 0.0f ? 0 : tie[d];
        }
}

/* ---- inference (Sec. III: Hamming distance, most similar class) --------------- */

/* dist[n][c] = number of dimensions where hv[n] and class c differ;
 * pred[n] = lowest c attaining the minimum.  dist may be NULL. */
void orc_search(const uint8_t *hv, int64_t N, const uint8_t *class_bits, int32_t C,
                int32_t D, uint32_t *dist, int32_t *pred)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        uint32_t best = 0;
        int32_t arg = 0;
        for (int32_t c = 0; c < C; ++c) {
            uint32_t k = 0;
            for (int32_t d = 0; d < D; ++d)
                k += hv[n * D + d] != class_bits[(int64_t)c * D + d];
            if (dist)
                dist[n * C + c] = k;
            if (c == 0 || k < best) {
                best = k;
                arg = c;
            }
        }
        pred[n] = arg;
    }
}
