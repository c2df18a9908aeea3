/*
 * CPU oracle for the user-side network that AIF runs asynchronously, in
 * parallel with retrieval (Sec. 3.1, "Pre-Computation Phase", Eq. 1-3).
 *
 * TEST INFRASTRUCTURE ONLY, like the rest of this directory: only the tests,
 * the smoke check and the benchmark's cpu_baseline leg may call it; the GPU
 * library shares no code with it.
 *
 * Inputs: the user's profile embedding U_profile [1, d_raw], behaviour
 * sequence embeddings U_seq [l, d_raw], and the weights.  In the paper's order:
 *   Eq. 1  U^_profile = U_profile W_profile^T   [1, d]
 *          U^_seq     = U_seq W_seq^T           [l, d]
 *   Eq. 2  U_self_attention = Pooling(FFN(Softmax(U^_seq U^_seq^T / sqrt(d)) U^_seq))   [1, d]
 *   Eq. 3  U_profile_attention = Softmax(U^_profile U^_seq^T / sqrt(d)) U^_seq          [1, d]
 * and the user vector combined from them, which is cached for the real-time phase.
 *
 * The paper names FFN, Pooling and the combination without defining them.
 * Readings taken here (and by the GPU library):
 *   FFN(x)     = max(0, W_ffn x + b_ffn), one layer, d -> d, applied to every row;
 *   Pooling    = mean over the l sequence positions;
 *   combined   = [U_self_attention | U_profile_attention], width 2 d;
 *   no residual connection, normalisation, mask or dropout (none is printed);
 *   l = 0 gives zero vectors.
 * U^_seq is returned as well: it is the behaviour-sequence tensor (keys and
 * values) the real-time target attention reads.
 *
 * Everything in IEEE double over float inputs, plain loops.
 *
 * Pins (tests/test_user_oracle_pins.py): NumPy float64 matmul for Eq. 1;
 * softmax rows sum to one; l = 1 and equal-rows special cases; torch SDPA in
 * float64 for the attention cores of Eq. 2 and Eq. 3; identity / zero FFN
 * special cases; a hand-worked two-position case fixing the 1/sqrt(d) scale;
 * brute force against an independently written NumPy reference.  The paper
 * prints no number for Eq. 1-3: beyond these, parity unpinned by the paper.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Eq. 1: out[r, :] = W in[r, :],  in [rows, d_raw], W [d, d_raw]. */
void aifo_user_project(const float *in, int rows, int d_raw, const float *W, int d, double *out)
{
    for (int r = 0; r < rows; ++r)
        for (int n = 0; n < d; ++n) {
            double acc = 0.0;
            for (int m = 0; m < d_raw; ++m) acc += (double)W[(size_t)n * d_raw + m] * (double)in[(size_t)r * d_raw + m];
            out[(size_t)r * d + n] = acc;
        }
}

/* Attention core shared by Eq. 2 and Eq. 3: out[r, :] = Softmax_t(<Q_r, S_t> / sqrt(d)) S,
 * Q [rows, d], S [l, d] (keys and values are the same projected sequence). */
int aifo_user_attend(const double *Q, int rows, const double *S, int l, int d, double *out)
{
    for (size_t i = 0; i < (size_t)rows * d; ++i) out[i] = 0.0;
    if (l <= 0) return 0;
    double *p = (double *)malloc(sizeof(double) * (size_t)l);
    if (!p) return 3;
    for (int r = 0; r < rows; ++r) {
        double mx = -INFINITY;
        for (int t = 0; t < l; ++t) {
            double acc = 0.0;
            for (int m = 0; m < d; ++m) acc += Q[(size_t)r * d + m] * S[(size_t)t * d + m];
            p[t] = acc / sqrt((double)d);
            if (p[t] > mx) mx = p[t];
        }
        double den = 0.0;
        for (int t = 0; t < l; ++t) { p[t] = exp(p[t] - mx); den += p[t]; }
        for (int t = 0; t < l; ++t)
            for (int m = 0; m < d; ++m) out[(size_t)r * d + m] += p[t] / den * S[(size_t)t * d + m];
    }
    free(p);
    return 0;
}

/* FFN of Eq. 2 (reading: one layer with ReLU): y[r, :] = max(0, W_ffn x[r, :] + b_ffn). */
void aifo_user_ffn(const double *x, int rows, int d, const float *W, const float *b, double *y)
{
    for (int r = 0; r < rows; ++r)
        for (int n = 0; n < d; ++n) {
            double acc = b ? (double)b[n] : 0.0;
            for (int m = 0; m < d; ++m) acc += (double)W[(size_t)n * d + m] * x[(size_t)r * d + m];
            y[(size_t)r * d + n] = acc > 0.0 ? acc : 0.0;
        }
}

/* Pooling of Eq. 2 (reading: mean over positions). */
void aifo_user_pool(const double *y, int rows, int d, double *out)
{
    for (int n = 0; n < d; ++n) {
        double acc = 0.0;
        for (int r = 0; r < rows; ++r) acc += y[(size_t)r * d + n];
        out[n] = rows > 0 ? acc / rows : 0.0;
    }
}

/* Eq. 1-3 for one user.  user_vec [2 d] = [U_self_attention | U_profile_attention];
 * seq_hat [l, d] = U^_seq.  Either output may be NULL. */
int aifo_user_network(const float *profile, const float *seq, int l, int d_raw, int d,
                      const float *w_profile, const float *w_seq, const float *w_ffn, const float *b_ffn,
                      double *user_vec, double *seq_hat)
{
    if (l < 0 || d_raw <= 0 || d <= 0) return 1;
    size_t n = (size_t)(l > 0 ? l : 1) * d;
    double *sh = (double *)malloc(sizeof(double) * n), *att = (double *)malloc(sizeof(double) * n);
    double *ffn = (double *)malloc(sizeof(double) * n), *ph = (double *)malloc(sizeof(double) * (size_t)d);
    if (!sh || !att || !ffn || !ph) { free(sh); free(att); free(ffn); free(ph); return 3; }
    aifo_user_project(profile, 1, d_raw, w_profile, d, ph);             /* Eq. 1 */
    aifo_user_project(seq, l, d_raw, w_seq, d, sh);
    if (seq_hat) memcpy(seq_hat, sh, sizeof(double) * (size_t)l * d);
    if (user_vec) {
        aifo_user_attend(sh, l, sh, l, d, att);                         /* Eq. 2 */
        aifo_user_ffn(att, l, d, w_ffn, b_ffn, ffn);
        aifo_user_pool(ffn, l, d, user_vec);
        aifo_user_attend(ph, 1, sh, l, d, user_vec + d);                /* Eq. 3 */
    }
    free(sh); free(att); free(ffn); free(ph);
    return 0;
}
