/*
 * aif_lsh.h -- C ABI of the LSH-based long-sequence behaviour modelling of AIF
 * on MI355X (gfx950): Sec. 4.3 of arXiv 2511.12934 ("Efficient User Behavior
 * Modeling"), the online part.
 *
 * Offline, every item's multi-modal embedding is hashed to a d'-bit signature
 * (Eq. 5) and the signatures form a byte-valued index table
 * (Sec. 4.3).  Online, for one request with about 10^4
 * candidates and a long behaviour sequence, the library
 *   - looks each candidate's signature up in that table,
 *   - compares it with the signatures of the user's l history items: the
 *     similarity is the number of equal bits over d', XNOR + population count
 *     (Eq. 6, Eq. 7),
 *   - LSH-DIN (Eq. 8): the similarity-weighted sum of the projected history
 *     embeddings U~ = U_seq W_seq^T, no softmax,
 *   - SimTier (Eq. 9): the histogram of the candidate's l similarities over N
 *     tiers; the tiers are N equal intervals of [0, 1], the last one closed:
 *     tier(m) = min(N - 1, floor(m N))  (the paper leaves the edges open).
 * Both outputs come from the same similarities (the reuse Table 3 counts on).
 *
 * Bit order of a signature byte: the first of its eight bits is the most
 * significant one (Sec. 4.3: 00110101 -> 53).  It only matters to whoever
 * builds the signatures; equal-bit counts do not depend on it.
 *
 * Conventions are those of aif.h: plain C, every call returns an aif_status
 * and enqueues nothing on failure, DEVICE pointers belong to the device that
 * was current at init, all work is asynchronous on the caller's stream, the
 * library owns only its context and workspace, borrows the signature table
 * for the life of the context and the request tensors until the enqueued work
 * has completed.  Not capturable into a HIP graph.
 */
#ifndef AIF_LSH_H
#define AIF_LSH_H

#include "aif.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct aif_lsh_ctx aif_lsh_ctx;

typedef struct {
    int64_t n_items;        /* rows of the signature table                                         */
    int32_t d_bits;         /* d' of Eq. 5: signature width in bits, a multiple of 32, 32..256      */
    int32_t d_out;          /* d of Eq. 8: width of U~ and of the DIN output, a multiple of 16, 16..256 */
    int32_t n_tiers;        /* N of Eq. 9, 1..8                                                    */
    aif_dtype dtype;        /* storage type of U~ (the DIN output is fp32 always)                  */
    int32_t max_seq_len;    /* longest history, in items                                           */
    int32_t max_candidates; /* per request                                                         */
    int32_t max_users;      /* requests per aif_lsh_batch call                                     */
} aif_lsh_config;

typedef struct {
    const uint8_t *seq_sigs;   /* DEVICE [seq_len, d_bits / 8]: signatures of the history items, 4-byte aligned */
    const void *seq_emb;       /* DEVICE [seq_len, d_out] row-major, config dtype: U~ = U_seq W_seq^T (user side), 16-byte aligned */
    int32_t seq_len;           /* 0..max_seq_len; 0 gives DIN = 0 and empty tiers                   */
    const int32_t *cand_ids;   /* DEVICE [n_cand]: rows of the signature table                      */
    int32_t n_cand;            /* 0..max_candidates                                                 */
    float *din_out;            /* DEVICE [n_cand, d_out] row-major fp32: Eq. 8, 16-byte aligned     */
    int32_t *tier_out;         /* DEVICE [n_cand, n_tiers] row-major: Eq. 9                         */
} aif_lsh_request;

/* Sec. 4.3.  Creates a context for one signature table (DEVICE, [n_items, d_bits / 8] row-major, 4-byte
 * aligned, borrowed until aif_lsh_destroy) and allocates the per-request workspace.  Synchronous. */
AIF_API aif_status aif_lsh_init(const aif_lsh_config *config, const uint8_t *sig_table, aif_lsh_ctx **out);

/* Eq. 6-9 for n_req requests (HOST array, read during the call) on hip_stream.  Per request the
 * user-side sums the DIN needs are formed once, then every candidate is served.  A candidate id outside
 * [0, n_items) cannot fault: it reads row 0, its DIN row is NaN, its tiers are -1 and a counter read by
 * aif_lsh_poll_device_errors is bumped.  Results do not depend on how a candidate list is cut into
 * requests.  Errors: AIF_EINVAL (NULL, negative sizes, misaligned tensors), AIF_ERANGE (beyond the limits
 * of the context), AIF_EDEVICE. */
AIF_API aif_status aif_lsh_batch(aif_lsh_ctx *ctx, const aif_lsh_request *reqs, int32_t n_req, void *hip_stream);

/* Frees the context and its workspace; the caller has synchronised its streams.  NULL is allowed. */
AIF_API void aif_lsh_destroy(aif_lsh_ctx *ctx);

/* Text of the last failure of this context (of the last failed aif_lsh_init when ctx is NULL). */
AIF_API const char *aif_lsh_last_error(const aif_lsh_ctx *ctx);

/* After the caller has synchronised the stream: number of out-of-range candidate ids seen since the
 * last poll (the counter is reset).  Synchronous device read. */
AIF_API aif_status aif_lsh_poll_device_errors(aif_lsh_ctx *ctx, int32_t *n_bad_ids);

/* Which kernel forms the equal-bit counts of Eq. 6-7 and the tier counts of Eq. 9 in this context:
 * 0 = vector ALU (XNOR + population count; any signature width and tier count), 1 = matrix cores (the
 * bits as +1 / -1 int8, the count as a dot product; signatures of 32, 64 or 128 bits whose tiers are
 * 2 d' / N = a power of two equal-bit counts wide).  Same counts either way.  -1 for a NULL context. */
AIF_API int32_t aif_lsh_simtier_kind(const aif_lsh_ctx *ctx);

/* Which kernel forms Eq. 8 in this context: 0 = vector ALU (one table row added per bit), 1 = matrix
 * cores (the candidates' bits one-hot against the fp32 tables cut exactly into three bf16 pieces;
 * d_out a multiple of 32 up to 128).  Same value up to the order of the fp32 additions.  -1 for a NULL
 * context. */
AIF_API int32_t aif_lsh_din_kind(const aif_lsh_ctx *ctx);

/* Per-kernel timing with HIP events on the caller's stream, as aif_profile_begin / _end of aif.h:
 * stages AIF_LSH_STAGE_USER (user-side sums), _DIN, _SIMTIER; ms[] and calls[] have AIF_LSH_N_STAGES
 * entries. */
typedef enum { AIF_LSH_STAGE_USER = 0, AIF_LSH_STAGE_DIN = 1, AIF_LSH_STAGE_SIMTIER = 2, AIF_LSH_N_STAGES = 3 } aif_lsh_stage;
AIF_API aif_status aif_lsh_profile_begin(aif_lsh_ctx *ctx, int32_t max_calls);
AIF_API aif_status aif_lsh_profile_end(aif_lsh_ctx *ctx, double *ms, int32_t *calls);

#ifdef __cplusplus
}
#endif
#endif /* AIF_LSH_H */
