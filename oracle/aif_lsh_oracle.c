/*
 * CPU oracle for the LSH-based long-sequence behaviour modelling of AIF
 * (Sec. 4.3, "Efficient User Behavior Modeling").
 *
 * TEST INFRASTRUCTURE ONLY, like aif_oracle.c: the tests, the smoke check and
 * the benchmark's cpu_baseline leg call it; the product shares no code with it.
 *
 * The steps, in the paper's order and notation:
 *
 *   Eq. 5   signature of an embedding M_i in R^d under d' shared Gaussian
 *           hyperplanes: bit k = [ (M_i W_hash^T)_k > 0 ]           (aifo_lsh_sign)
 *           d' bits are stored as d'/8 bytes; the first bit of a byte is its
 *           most significant one (the paper's example: 00110101 -> 53).
 *   Eq. 6   similarity of two signatures = number of equal bits / d', i.e.
 *           PopulationCount(XNOR) / d'                               (aifo_lsh_equal_bits)
 *   Eq. 7   M_sim [b, l] between the b candidates and the l history items.
 *   Eq. 8   LSH-DIN: M_sim times the projected history embeddings
 *           U~ = U_seq W_seq^T [l, d] (handed in ready-made; it is user-side
 *           work) -- NO softmax, the similarities are the weights.   (aifo_lsh_din)
 *   Eq. 9   SimTier: the similarities of one candidate are counted into N
 *           tiers.  The paper leaves the tier edges open; the reading taken
 *           is N equal intervals of [0, 1], the last one closed:
 *           tier(m) = min(N - 1, floor(m N)).                        (aifo_simtier)
 *   Table 3 cost of the similarity modules, b * l * (sum of the widths that
 *           enter them), from which the printed reductions follow.   (aifo_lsh_similarity_cost)
 *
 * Counts are integers, sums are IEEE double; nothing is blocked or reordered.
 *
 * Pins (tests/test_lsh_oracle_pins.py): the 53 example; a signature is fully
 * similar to itself and not at all to its complement; equal bits + differing
 * bits = d'; collision probability 1 - theta/pi per bit for two vectors at
 * angle theta (the textbook SimHash law) within three standard errors; DIN and
 * SimTier against NumPy float64 on bits unpacked by np.unpackbits (another
 * route to the same definition); histogram sums to l; the reductions 43.75 %,
 * 50 % and 93.75 % of Table 3.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { AIFO_OK = 0, AIFO_EINVAL = 1, AIFO_ERANGE = 5 };

/* d' bits -> d'/8 bytes, first bit = most significant (00110101 -> 53). */
void aifo_lsh_pack_bits(const uint8_t *bits, int n_bits, uint8_t *bytes)
{
    for (int b = 0; b < n_bits / 8; ++b) {
        unsigned v = 0;
        for (int k = 0; k < 8; ++k) v = (v << 1) | (bits[8 * b + k] ? 1u : 0u);
        bytes[b] = (uint8_t)v;
    }
}

/* Eq. 5: sig[i] = pack( [ sum_m M[i, m] W_hash[k, m] > 0 ]_k ), W_hash is [d', d]. */
int aifo_lsh_sign(const float *M, int n, int d, const float *w_hash, int d_bits, uint8_t *sig)
{
    if (d_bits <= 0 || d_bits % 8) return AIFO_EINVAL;
    uint8_t *bits = (uint8_t *)malloc((size_t)d_bits);
    if (!bits) return AIFO_EINVAL;
    for (int i = 0; i < n; ++i) {
        for (int k = 0; k < d_bits; ++k) {
            double s = 0.0;
            for (int m = 0; m < d; ++m) s += (double)M[(size_t)i * d + m] * (double)w_hash[(size_t)k * d + m];
            bits[k] = s > 0.0;
        }
        aifo_lsh_pack_bits(bits, d_bits, sig + (size_t)i * (d_bits / 8));
    }
    free(bits);
    return AIFO_OK;
}

/* Eq. 6, numerator: how many of the d' bits of two signatures are equal (XNOR, then count the ones). */
int aifo_lsh_equal_bits(const uint8_t *a, const uint8_t *b, int n_bytes)
{
    int equal = 0;
    for (int j = 0; j < n_bytes; ++j) {
        const unsigned x = (unsigned)(uint8_t)~(a[j] ^ b[j]);
        for (int k = 0; k < 8; ++k) equal += (x >> k) & 1u;
    }
    return equal;
}

/* Eq. 8 for one candidate: a = sum_t (equal_t / d') U~[t, :]. */
void aifo_lsh_din(const int32_t *equal, int L, int d_bits, const float *u_seq, int d, double *a)
{
    for (int m = 0; m < d; ++m) a[m] = 0.0;
    for (int t = 0; t < L; ++t) {
        const double w = (double)equal[t] / (double)d_bits;
        for (int m = 0; m < d; ++m) a[m] += w * (double)u_seq[(size_t)t * d + m];
    }
}

/* Eq. 9 for one candidate: tier(m) = min(N - 1, floor(m N)) with m = equal / d', counted over the history. */
void aifo_simtier(const int32_t *equal, int L, int d_bits, int n_tiers, int32_t *count)
{
    for (int j = 0; j < n_tiers; ++j) count[j] = 0;
    for (int t = 0; t < L; ++t) {
        int tier = (int)(((int64_t)equal[t] * n_tiers) / d_bits);     /* floor of a non-negative quotient */
        if (tier > n_tiers - 1) tier = n_tiers - 1;
        ++count[tier];
    }
}

/* One request: for every candidate, look its signature up in the table (Sec. 4.3: the signatures are kept
 * as a byte-valued index table), compare it with the signatures of the user's history (Eq. 7), then Eq. 8 and Eq. 9
 * from the SAME similarities (the reuse Table 3 counts on).
 * sig_table [n_items, d'/8], seq_sig [L, d'/8], u_seq [L, d]; out: din [n, d], tiers [n, n_tiers],
 * equal_out [n, L] (may be NULL). */
int aifo_lsh_request(const uint8_t *sig_table, int64_t n_items, int d_bits,
                     const int32_t *ids, int n,
                     const uint8_t *seq_sig, const float *u_seq, int L, int d,
                     int n_tiers, double *din, int32_t *tiers, int32_t *equal_out, int n_threads)
{
    if (d_bits <= 0 || d_bits % 8 || n_tiers <= 0 || L < 0 || d <= 0) return AIFO_EINVAL;
    const int nb = d_bits / 8;
    for (int i = 0; i < n; ++i)
        if (ids[i] < 0 || ids[i] >= n_items) return AIFO_ERANGE;
    int bad = 0;
#pragma omp parallel for schedule(static) num_threads(n_threads > 0 ? n_threads : 1)
    for (int i = 0; i < n; ++i) {
        int32_t *eq = (int32_t *)malloc(sizeof(int32_t) * (size_t)(L > 0 ? L : 1));
        if (!eq) {
            bad = 1;
            continue;
        }
        const uint8_t *h = sig_table + (size_t)ids[i] * nb;
        for (int t = 0; t < L; ++t) eq[t] = aifo_lsh_equal_bits(h, seq_sig + (size_t)t * nb, nb);
        aifo_lsh_din(eq, L, d_bits, u_seq, d, din + (size_t)i * d);
        aifo_simtier(eq, L, d_bits, n_tiers, tiers + (size_t)i * n_tiers);
        if (equal_out) memcpy(equal_out + (size_t)i * L, eq, sizeof(int32_t) * (size_t)L);
        free(eq);
    }
    return bad ? AIFO_EINVAL : AIFO_OK;
}

/* Table 3: cost of the attention / similarity modules = b * l * (sum of the vector widths they contract). */
double aifo_lsh_similarity_cost(double b, double l, const double *widths, int n_widths)
{
    double w = 0.0;
    for (int i = 0; i < n_widths; ++i) w += widths[i];
    return b * l * w;
}
