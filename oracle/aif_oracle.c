/*
 * CPU oracle for the real-time pre-ranking scoring path of AIF.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU
 * library is checked against.  Only the test-suite, the smoke check and the
 * benchmark's cpu_baseline leg may call it; the product path never does and
 * shares no code with it.
 *
 * Everything is computed in IEEE double over inputs handed in as float (the
 * storage types fp32 and bf16 both widen to float exactly), one candidate at
 * a time, in the order the paper lays the online phase out:
 *
 *   1. look the candidate's nearline item vector up in the index table
 *      (Sec. 3.2: item vectors are kept in an index table and meet the
 *      user vectors at pre-ranking),
 *   2. form the attention query from the item vector (projection of the
 *      Eq. 1 kind, or the leading slice when no projection is given),
 *   3. scaled dot-product attention of the candidate over the user's
 *      behaviour sequence: Softmax(q K^T / sqrt(d)) V, the operator of Eq. 3
 *      with the candidate in the place of the profile,
 *   4. real-time half of the cross features (Sec. 3.3): the cached user
 *      component combined with the item vector,
 *   5. model input = [user | item | attention | cross] (Sec. 1: the input
 *      tensor is assembled before the forward pass),
 *   6. shallow MLP head, ReLU between layers, linear last layer -> logit,
 *      sigmoid -> score (Sec. 1: the head is a small MLP),
 *   7. keep the best k of the request (Sec. 1: about 10^4 -> about 10^2).
 *
 * Pins (tests/test_oracle_pins.py): softmax weights sum to one; L = 1 returns
 * V_0; equal keys or q = 0 return the mean of V; adding one vector to every
 * key changes nothing; one dominant key returns its value row; H heads equal
 * H single-head calls; float64 NumPy / torch SDPA cross-checks; hand-worked
 * cross and MLP cases; top-k against a full stable sort; permutation
 * equivariance and mini-batch invariance of the whole path; brute force
 * against an independently written NumPy reference on tiny inputs.  The paper
 * prints no numeric value for this path, so beyond those the parity is
 * unpinned by the paper itself.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { AIFO_OK = 0, AIFO_EINVAL = 1, AIFO_ESHAPE = 2, AIFO_ENOMEM = 3, AIFO_ERANGE = 5 };
enum { AIFO_CROSS_NONE = 0, AIFO_CROSS_HADAMARD = 1, AIFO_CROSS_SEGDOT = 2, AIFO_CROSS_BEA = 3 };

/* aif_bea_oracle.c: step 4 of Algorithm 1 */
void aifo_bea_weighted_sum(const double *w_hat, int b, int n, const float *V, int d_out, double *v_hat);

/* Step 1 (Sec. 3.2): e_i = T[id_i, :].  An id outside the table is an error. */
int aifo_gather(const float *table, int64_t n_items, int d_item,
                const int32_t *ids, int n, double *e_out)
{
    for (int i = 0; i < n; ++i) {
        int64_t id = ids[i];
        if (id < 0 || id >= n_items) return AIFO_ERANGE;
        for (int m = 0; m < d_item; ++m)
            e_out[(size_t)i * d_item + m] = (double)table[(size_t)id * d_item + m];
    }
    return AIFO_OK;
}

/* Nearline maintenance of the index table (Sec. 3.4: the table of nearline results is replaced as a whole or
 * patched row by row).  Incremental update: row ids[i] of the table becomes rows[i, :], entries applied in
 * order (a later entry for the same id replaces an earlier one); ids outside the table are skipped and
 * counted in *n_skipped.  A full update is a new table: nothing to compute. */
void aifo_update_rows(float *table, int64_t n_items, int d_item,
                      const int32_t *ids, const float *rows, int n, int *n_skipped)
{
    int skipped = 0;
    for (int i = 0; i < n; ++i) {
        int64_t id = ids[i];
        if (id < 0 || id >= n_items) { ++skipped; continue; }
        for (int m = 0; m < d_item; ++m) table[(size_t)id * d_item + m] = rows[(size_t)i * d_item + m];
    }
    if (n_skipped) *n_skipped = skipped;
}

/* Step 2: q = W_q e (W_q is [d_attn, d_item], no bias; form of Eq. 1), or the
 * first d_attn coordinates of e when w_q is NULL. */
void aifo_query(const double *e, const float *w_q, int d_item, int d_attn, double *q)
{
    for (int r = 0; r < d_attn; ++r) {
        if (!w_q) { q[r] = e[r]; continue; }
        double s = 0.0;
        for (int m = 0; m < d_item; ++m) s += (double)w_q[(size_t)r * d_item + m] * e[m];
        q[r] = s;
    }
}

/* Step 3 (Eq. 3 with query := candidate): for each head h (a contiguous
 * d_h = d_attn / H wide slice of q, K and V)
 *   s_t = <q^h, K_t^h> / sqrt(d_h);  p = softmax_t(s);  a^h = sum_t p_t V_t^h.
 * seq_len == 0 gives a = 0.  p_out (may be NULL) receives the weights [H, L]. */
void aifo_attention(const double *q, const float *K, const float *V, int L,
                    int d_attn, int H, double *a, double *p_out)
{
    int dh = d_attn / H;
    for (int m = 0; m < d_attn; ++m) a[m] = 0.0;
    if (L <= 0) return;
    double *s = (double *)malloc(sizeof(double) * (size_t)L);
    for (int h = 0; h < H; ++h) {
        int o = h * dh;
        double mx = -INFINITY;
        for (int t = 0; t < L; ++t) {
            double acc = 0.0;
            for (int m = 0; m < dh; ++m) acc += q[o + m] * (double)K[(size_t)t * d_attn + o + m];
            s[t] = acc / sqrt((double)dh);
            if (s[t] > mx) mx = s[t];
        }
        double den = 0.0;
        for (int t = 0; t < L; ++t) { s[t] = exp(s[t] - mx); den += s[t]; }
        for (int t = 0; t < L; ++t) {
            double p = s[t] / den;
            if (p_out) p_out[(size_t)h * L + t] = p;
            for (int m = 0; m < dh; ++m) a[o + m] += p * (double)V[(size_t)t * d_attn + o + m];
        }
    }
    free(s);
}

/* Width of the cross block for a mode. */
int aifo_cross_width(int mode, int d_item, int n_cross, int d_c)
{
    if (mode == AIFO_CROSS_HADAMARD) return d_item;
    if (mode == AIFO_CROSS_SEGDOT) return (d_c > 0 && d_item % d_c == 0) ? n_cross * (d_item / d_c) : -1;
    if (mode == AIFO_CROSS_BEA) return (n_cross > 0 && n_cross <= d_item && d_c > 0) ? d_c : -1;
    return 0;
}

/* Step 4 (Sec. 3.3, real-time generation from the cached user component):
 *   HADAMARD: c_m = u_m * e_m          (user operand [d_item])
 *   SEGDOT:   c[j*S + s] = <Vc_j, e[s*d_c : (s+1)*d_c]>,  S = d_item / d_c,
 *             Vc is [n_cross, d_c].
 *   BEA:      (Sec. 4.1, Algorithm 1, step 4) the item row ends with the
 *             candidate's n = n_cross bridge weights w^ (the nearline pipeline
 *             stores them with the item vector); the user operand is V
 *             [n, d_c]; c = w^ V, width d_c. */
int aifo_cross(int mode, const float *uc, int n_cross, int d_c,
               const double *e, int d_item, double *c)
{
    if (mode == AIFO_CROSS_NONE) return AIFO_OK;
    if (mode == AIFO_CROSS_HADAMARD) {
        for (int m = 0; m < d_item; ++m) c[m] = (double)uc[m] * e[m];
        return AIFO_OK;
    }
    if (mode == AIFO_CROSS_SEGDOT) {
        if (d_c <= 0 || d_item % d_c) return AIFO_ESHAPE;
        int S = d_item / d_c;
        for (int j = 0; j < n_cross; ++j)
            for (int s = 0; s < S; ++s) {
                double acc = 0.0;
                for (int m = 0; m < d_c; ++m)
                    acc += (double)uc[(size_t)j * d_c + m] * e[s * d_c + m];
                c[j * S + s] = acc;
            }
        return AIFO_OK;
    }
    if (mode == AIFO_CROSS_BEA) {
        if (n_cross <= 0 || n_cross > d_item || d_c <= 0) return AIFO_ESHAPE;
        aifo_bea_weighted_sum(e + (d_item - n_cross), 1, n_cross, uc, d_c, c);
        return AIFO_OK;
    }
    return AIFO_EINVAL;
}

/* Step 6: h_0 = x; h_l = max(0, W_l h_{l-1} + b_l) for l < n_layers; the last
 * layer is linear.  dims has n_layers + 1 entries; w holds the W_l ([out, in]
 * row-major) back to back, b the biases back to back (NULL = zero biases).
 * Writes the dims[n_layers] outputs of the last layer to z. */
int aifo_mlp(const double *x, int n_layers, const int32_t *dims,
             const float *w, const float *b, double *z)
{
    int widest = 0;
    for (int l = 0; l <= n_layers; ++l) if (dims[l] > widest) widest = dims[l];
    double *h0 = (double *)malloc(sizeof(double) * (size_t)widest);
    double *h1 = (double *)malloc(sizeof(double) * (size_t)widest);
    if (!h0 || !h1) { free(h0); free(h1); return AIFO_ENOMEM; }
    memcpy(h0, x, sizeof(double) * (size_t)dims[0]);
    size_t wo = 0, bo = 0;
    for (int l = 0; l < n_layers; ++l) {
        int din = dims[l], dout = dims[l + 1];
        for (int r = 0; r < dout; ++r) {
            double acc = b ? (double)b[bo + r] : 0.0;
            for (int m = 0; m < din; ++m) acc += (double)w[wo + (size_t)r * din + m] * h0[m];
            if (l + 1 < n_layers && acc < 0.0) acc = 0.0;
            h1[r] = acc;
        }
        wo += (size_t)din * dout; bo += (size_t)dout;
        double *t = h0; h0 = h1; h1 = t;
    }
    memcpy(z, h0, sizeof(double) * (size_t)dims[n_layers]);
    free(h0); free(h1);
    return AIFO_OK;
}

double aifo_sigmoid(double z) { return 1.0 / (1.0 + exp(-z)); }

/* Steps 1-6 for every candidate of one request.  Optional outputs (NULL to
 * skip): a_out [n, d_attn], c_out [n, d_cross], y_out [n].  The candidate
 * loop is split over n_threads OpenMP threads when n_threads > 1; the loop
 * body is the same scalar code. */
int aifo_score(const float *table, int64_t n_items, int d_item,
               const float *w_q, int d_attn, int n_heads,
               const float *user_vec, int d_user,
               int cross_mode, const float *cross_vecs, int n_cross, int d_c,
               const float *seq_keys, const float *seq_vals, int seq_len,
               int n_layers, const int32_t *dims, const float *w, const float *b,
               const int32_t *ids, int n,
               double *z_out, double *y_out, double *a_out, double *c_out,
               int n_threads)
{
    if (n_heads <= 0 || d_attn % n_heads) return AIFO_ESHAPE;
    int d_cross = aifo_cross_width(cross_mode, d_item, n_cross, d_c);
    if (d_cross < 0) return AIFO_ESHAPE;
    if (cross_mode == AIFO_CROSS_HADAMARD && !cross_vecs) {
        if (d_user != d_item) return AIFO_ESHAPE;
        cross_vecs = user_vec;
    }
    if (!w_q && d_attn > d_item) return AIFO_ESHAPE;
    int d_in = d_user + d_item + d_attn + d_cross;
    if (dims[0] != d_in || dims[n_layers] != 1) return AIFO_ESHAPE;
    for (int i = 0; i < n; ++i)
        if (ids[i] < 0 || (int64_t)ids[i] >= n_items) return AIFO_ERANGE;

    int status = AIFO_OK;
    if (n_threads < 1) n_threads = 1;
#pragma omp parallel for schedule(static) num_threads(n_threads)
    for (int i = 0; i < n; ++i) {
        double *buf = (double *)malloc(sizeof(double) * (size_t)(d_item + 2 * d_attn + d_cross + d_in));
        double *e = buf, *q = e + d_item, *a = q + d_attn, *c = a + d_attn, *x = c + d_cross;
        aifo_gather(table, n_items, d_item, ids + i, 1, e);
        aifo_query(e, w_q, d_item, d_attn, q);
        aifo_attention(q, seq_keys, seq_vals, seq_len, d_attn, n_heads, a, NULL);
        aifo_cross(cross_mode, cross_vecs, n_cross, d_c, e, d_item, c);
        int o = 0;
        for (int m = 0; m < d_user; ++m) x[o++] = (double)user_vec[m];
        for (int m = 0; m < d_item; ++m) x[o++] = e[m];
        for (int m = 0; m < d_attn; ++m) x[o++] = a[m];
        for (int m = 0; m < d_cross; ++m) x[o++] = c[m];
        double z = 0.0;
        int rc = aifo_mlp(x, n_layers, dims, w, b, &z);
        if (rc != AIFO_OK) {
#pragma omp critical
            status = rc;
        }
        z_out[i] = z;
        if (y_out) y_out[i] = aifo_sigmoid(z);
        if (a_out) memcpy(a_out + (size_t)i * d_attn, a, sizeof(double) * (size_t)d_attn);
        if (c_out && d_cross) memcpy(c_out + (size_t)i * d_cross, c, sizeof(double) * (size_t)d_cross);
        free(buf);
    }
    return status;
}

/* Ordering used by step 7: a comes before b when z[a] is larger; a NaN is
 * smaller than every number; equal values (and -0 / +0) keep position order. */
static int before(const double *z, int32_t a, int32_t b)
{
    double za = z[a], zb = z[b];
    if (isnan(za)) return 0;
    if (isnan(zb)) return 1;
    return za > zb;
}

static void merge_sort(const double *z, int32_t *pos, int32_t *tmp, int lo, int hi)
{
    if (hi - lo < 2) return;
    int mid = lo + (hi - lo) / 2;
    merge_sort(z, pos, tmp, lo, mid);
    merge_sort(z, pos, tmp, mid, hi);
    int i = lo, j = mid, o = lo;
    while (i < mid && j < hi) {
        /* take from the right run only when it is strictly ahead: stable */
        if (before(z, pos[j], pos[i])) tmp[o++] = pos[j++]; else tmp[o++] = pos[i++];
    }
    while (i < mid) tmp[o++] = pos[i++];
    while (j < hi) tmp[o++] = pos[j++];
    memcpy(pos + lo, tmp + lo, sizeof(int32_t) * (size_t)(hi - lo));
}

/* Step 7 (Sec. 1): positions of the k largest logits, best first, from a
 * stable descending sort of all n positions.  k > n: the first n slots are
 * filled, the rest get idx = -1, val = -inf. */
int aifo_topk(const double *z, int n, int k, int32_t *idx, double *val)
{
    if (n < 0 || k <= 0) return AIFO_EINVAL;
    int32_t *pos = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    int32_t *tmp = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    if (!pos || !tmp) { free(pos); free(tmp); return AIFO_ENOMEM; }
    for (int i = 0; i < n; ++i) pos[i] = i;
    merge_sort(z, pos, tmp, 0, n);
    for (int j = 0; j < k; ++j) {
        if (j < n) { idx[j] = pos[j]; val[j] = z[pos[j]]; }
        else { idx[j] = -1; val[j] = -INFINITY; }
    }
    free(pos); free(tmp);
    return AIFO_OK;
}
