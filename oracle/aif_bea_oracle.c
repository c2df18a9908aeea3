/*
 * CPU oracle for the Bridge Embedding Approximation (BEA) of AIF, Sec. 4.1,
 * Algorithm 1.
 *
 * TEST INFRASTRUCTURE ONLY, like the rest of this directory: only the tests,
 * the smoke check and the benchmark's cpu_baseline leg may call it; the GPU
 * library shares no code with it.
 *
 * Algorithm 1 has n bridge embeddings B [n, d].  Its four steps are
 *   1. user side (asynchronous):  W = Softmax(B U^T / sqrt(d))        [n, m]
 *   2. user side (asynchronous):  V = f(U, W | Theta_u)               [n, d']
 *      -- f is the user-side network; it is an input here, not computed.
 *   3. item side (nearline):      w^ = Softmax(I B^T / sqrt(d))       [b, n]
 *   4. online, at pre-ranking:    v^ = w^ V                           [b, d']
 * Steps 1 and 3 are the same operator (a softmax over the rows of the second
 * operand of the scaled dot products with the rows of the first), so one
 * function serves both.  Step 4 is the only one on the real-time path: the
 * weighted sum of the n user-side vectors with the item's n weights.
 *
 * Everything in IEEE double over float inputs, plain loops.
 *
 * Pins (tests/test_bea_oracle_pins.py): rows of a softmax sum to one; zero
 * item embeddings give uniform weights and hence the mean of V; a hand-worked
 * two-bridge case with e/(1+e); a dominant bridge gives a one-hot row;
 * scipy's softmax and NumPy float64 matmul as library cross-checks; one-hot
 * weights select a row of V; weights that sum to one keep every coordinate of
 * v^ between the smallest and largest of that coordinate over the rows of V;
 * the cross block of the whole scoring path equals step 4 on the row's
 * trailing n entries; brute force against a NumPy reference on tiny inputs.
 * The paper prints no number for Algorithm 1: beyond these, parity unpinned
 * by the paper itself.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

/* Steps 1 and 3: out[r, :] = Softmax_j( <X_r, Y_j> / sqrt(d) ), X [rows, d], Y [cols, d].
 * Step 3: X = item embeddings I, Y = bridges B.  Step 1: X = B, Y = user embeddings U. */
int aifo_bea_attention_weights(const float *X, int rows, const float *Y, int cols, int d, double *out)
{
    if (rows < 0 || cols <= 0 || d <= 0) return 1;
    for (int r = 0; r < rows; ++r) {
        double *o = out + (size_t)r * cols;
        double mx = -INFINITY;
        for (int j = 0; j < cols; ++j) {
            double acc = 0.0;
            for (int m = 0; m < d; ++m) acc += (double)X[(size_t)r * d + m] * (double)Y[(size_t)j * d + m];
            o[j] = acc / sqrt((double)d);
            if (o[j] > mx) mx = o[j];
        }
        double den = 0.0;
        for (int j = 0; j < cols; ++j) { o[j] = exp(o[j] - mx); den += o[j]; }
        for (int j = 0; j < cols; ++j) o[j] /= den;
    }
    return 0;
}

/* Step 4: v^[i, :] = sum_j w^[i, j] V[j, :],  w^ [b, n] (double), V [n, d'] (float). */
void aifo_bea_weighted_sum(const double *w_hat, int b, int n, const float *V, int d_out, double *v_hat)
{
    for (int i = 0; i < b; ++i)
        for (int m = 0; m < d_out; ++m) {
            double acc = 0.0;
            for (int j = 0; j < n; ++j) acc += w_hat[(size_t)i * n + j] * (double)V[(size_t)j * d_out + m];
            v_hat[(size_t)i * d_out + m] = acc;
        }
}
