/*
 * aif.h -- C ABI of the MI355X (gfx950) real-time pre-ranking scoring library.
 *
 * The library computes what the Asynchronous Inference Framework (AIF,
 * arXiv 2511.12934) leaves online, i.e. the second, real-time call of
 * Sec. 3.1 ("Real-Time Prediction Phase"): for one user request with about
 * 10^4 retrieved candidates (Sec. 1) it
 *   - indexes each candidate's nearline-precomputed item vector in the index
 *     table (Sec. 3.2),
 *   - combines it with the request's cached user-side tensors (Sec. 3.1, 3.2),
 *   - forms the interaction-dependent terms: a scaled dot-product attention
 *     of the candidate over the user's behaviour sequence (operator of Eq. 3
 *     with the candidate as the query) and the real-time half of the cross
 *     features (Sec. 3.3),
 *   - runs the shallow MLP head on [user | item | attention | cross] (Sec. 1),
 *   - and selects the best k candidates (Sec. 1: about 10^4 -> about 10^2).
 * Mini-batches (Sec. 1: a request's candidates are scored in slices of about a
 * thousand) are the caller's choice of how many aif_request slices a candidate
 * list is cut into; scores do not depend on the slicing.
 *
 * Conventions
 *   - Plain C, no exceptions.  Every call returns an aif_status; on failure
 *     nothing has been enqueued and aif_last_error() describes the reason.
 *   - "DEVICE" pointers are HIP device addresses on the device that was
 *     current at aif_score_init; "HOST" pointers are ordinary host memory
 *     read during the call only.
 *   - All work is enqueued on the caller's stream (hipStream_t passed as
 *     void*, NULL = default stream) and is asynchronous; the library never
 *     synchronises the stream.  One context serves one stream at a time.
 *   - The library owns the context, its workspace and its repacked weight
 *     copies (made in aif_score_init).  It borrows the item table for the
 *     life of the context, and the request tensors until the enqueued work
 *     has completed; it never frees caller memory.
 *   - Calls must not be made while the stream is being captured into a HIP
 *     graph (the calls stage descriptors through pinned memory and events).
 */
#ifndef AIF_H
#define AIF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AIF_API __attribute__((visibility("default")))

typedef struct aif_ctx aif_ctx;

typedef enum {
    AIF_OK = 0,
    AIF_EINVAL = 1,   /* NULL pointer, non-positive size, unknown enum            */
    AIF_ESHAPE = 2,   /* sizes inconsistent with each other or with the context   */
    AIF_ENOMEM = 3,   /* host or device allocation failed                         */
    AIF_EDEVICE = 4,  /* a HIP call failed                                        */
    AIF_ERANGE = 5    /* a request exceeds the limits the context was sized for   */
} aif_status;

typedef enum { AIF_F32 = 0, AIF_BF16 = 1 } aif_dtype;

typedef enum {
    AIF_CROSS_NONE = 0,
    AIF_CROSS_HADAMARD = 1, /* c = u (.) e, width d_item (Sec. 3.3)                        */
    AIF_CROSS_SEGDOT = 2,   /* c[j*S+s] = <Vc_j, e[s*d_c:(s+1)*d_c]>, S = d_item/d_c,
                               the shape of Sec. 4.1: n user-side vectors meet one item  */
    AIF_CROSS_BEA = 3       /* Bridge Embedding Approximation, Sec. 4.1, Algorithm 1 step 4
                               (the online weighted sum): the item row ENDS with the
                               candidate's n_cross bridge weights w^ (the nearline pipeline
                               stores them with the item vector), the request brings the n_cross
                               asynchronously inferred user-side vectors V [n_cross, d_cross_vec];
                               c = w^ V, width d_cross_vec.  The whole row, weights included,
                               is still the "item" block of the MLP input.                  */
} aif_cross;

/* Model and sizing.  Width rules: d_item, d_attn and the cross width must each
 * span a multiple of 16 bytes in the storage type (4 fp32 / 8 bf16 elements);
 * d_attn is a multiple of n_heads; without w_q, d_attn <= d_item;
 * layer_dims[0] = d_user + d_item + d_attn + d_cross and layer_dims[n_layers] = 1. */
typedef struct {
    aif_dtype dtype;          /* storage type of table, user tensors and weights          */
    int64_t n_items;          /* rows of the item table                                   */
    int32_t d_item;           /* row width                                                */
    int32_t d_user;           /* user vector width                                        */
    int32_t d_attn;           /* attention width = n_heads * head width                   */
    int32_t n_heads;
    int32_t max_seq_len;      /* largest behaviour-sequence length of any request         */
    aif_cross cross_mode;
    int32_t n_cross;          /* SEGDOT: number of user-side cross vectors; BEA: number of bridges (<= d_item); else 0 */
    int32_t d_cross_vec;      /* SEGDOT: their width (divides d_item); BEA: width d' of the user-side vectors; else 0 */
    int32_t n_layers;         /* MLP layers, >= 1                                         */
    const int32_t *layer_dims;/* HOST, n_layers + 1 entries [D_in, ..., 1]                */
    int32_t max_candidates;   /* largest n_cand of one request                            */
    int32_t max_users;        /* largest number of requests in one aif_score_batch        */
    uint32_t flags;           /* reserved, must be 0                                      */
} aif_config;

/* Model tensors, all DEVICE, storage type = config.dtype.  The table is
 * borrowed for the life of the context; the weights are read (and repacked)
 * during aif_score_init only. */
typedef struct {
    const void *item_table;   /* [n_items, d_item] row-major                              */
    const void *w_q;          /* [d_attn, d_item] row-major, q = W_q e; NULL: q = e[0:d_attn] */
    const void *const *w;     /* HOST array of n_layers DEVICE ptrs, W_l [d_out, d_in] row-major, y = W x + b */
    const void *const *b;     /* HOST array of n_layers DEVICE ptrs [d_out]; NULL array or NULL entry = zero bias */
} aif_weights;

/* One request (or one mini-batch slice of it).  Tensor pointers are DEVICE
 * and must stay valid until the enqueued work completes; user_vec,
 * cross_vecs, seq_keys and seq_vals must be 16-byte aligned. */
typedef struct {
    const void *user_vec;     /* [d_user]                                                 */
    const void *cross_vecs;   /* SEGDOT, BEA: [n_cross, d_cross_vec] row-major; HADAMARD: [d_item] or NULL = user_vec (needs d_user = d_item) */
    const void *seq_keys;     /* [seq_len, d_attn] row-major; heads are contiguous slices  */
    const void *seq_vals;     /* [seq_len, d_attn]; may alias seq_keys                    */
    int32_t seq_len;          /* 0 .. max_seq_len; 0 gives a zero attention block         */
    const int32_t *cand_ids;  /* [n_cand] table rows                                      */
    int32_t n_cand;           /* 0 .. max_candidates                                      */
    float *logits_out;        /* [n_cand] fp32 logits z                                   */
    float *scores_out;        /* [n_cand] sigmoid(z), or NULL                             */
} aif_request;

/* Create a context on the current device for one deployed model of the real-time
 * phase (Sec. 3.1, second call: the lightweight head and what it reads; Sec. 3.2:
 * the index table of nearline item vectors it indexes): validates the
 * configuration, sizes the workspace for max_users requests of max_candidates
 * candidates, repacks the weights.  Synchronous.  *out is set only on AIF_OK.
 * A bf16 model whose shapes the matrix-core kernels do not cover is still served,
 * by the shape-agnostic fp32 kernels, at a fraction of the speed: after AIF_OK
 * aif_last_error(*out) then holds a note that names the stage (empty string
 * otherwise), and aif_stage_kind() answers per stage. */
AIF_API aif_status aif_score_init(const aif_config *cfg, const aif_weights *weights, aif_ctx **out);

/* The real-time prediction call of Sec. 3.1 for one request (or one mini-batch
 * slice of it, Sec. 1): the cached user-side tensors meet the candidates' item
 * vectors (Sec. 3.2), the interaction-dependent terms are formed (Eq. 3's
 * operator with the candidate as query; Sec. 3.3) and the head scores every
 * candidate: logits (and optional sigmoid scores) in candidate order.
 * Equivalent to aif_score_batch with n_req = 1. */
AIF_API aif_status aif_score_request(aif_ctx *ctx, const aif_request *req, void *hip_stream);

/* The same for n_req requests (HOST array) in one pass -- concurrent users, or
 * the mini-batch slices of one user's candidate list, which Sec. 1 has scored
 * separately and in parallel: gather (Sec. 3.2) -> attention + cross (Eq. 3,
 * Sec. 3.3) -> MLP head (Sec. 1).  Each candidate's result depends only on its own row and its
 * request's user tensors, so any slicing of a candidate list into requests
 * yields the same numbers.  A candidate id outside [0, n_items) does not
 * fault: its logit and score are NaN and a device counter is bumped (see
 * aif_poll_device_errors).  Errors: AIF_EINVAL (NULL), AIF_ERANGE (n_req,
 * n_cand or seq_len above the context's limits). */
AIF_API aif_status aif_score_batch(aif_ctx *ctx, const aif_request *reqs, int32_t n_req, void *hip_stream);

/* The cut that is the purpose of the pre-ranking stage (Sec. 1: of about 10^4
 * retrieved candidates about 10^2 go on to ranking).  Per request r, the
 * positions (0-based, within its candidate list) of the k largest logits, best
 * first; equal logits keep the lower position first; a
 * NaN ranks below every number.  logits: HOST array of n_req DEVICE pointers;
 * n_cand: HOST array.  idx_out / val_out: DEVICE [n_req * k]; when
 * k > n_cand[r] the tail is idx = -1, val = -inf.  1 <= k <= 4096. */
AIF_API aif_status aif_topk(aif_ctx *ctx, const float *const *logits, const int32_t *n_cand, int32_t n_req,
                    int32_t k, int32_t *idx_out, float *val_out, void *hip_stream);

/* aif_score_batch followed by aif_topk over the same requests (Sec. 1: the purpose of the stage is the cut
 * from about 10^4 to about 10^2), as one call: request r's k best positions go to idx_out / val_out
 * [r * k, (r + 1) * k) (DEVICE), exactly as aif_topk would leave them from logits_out of request r.  One
 * descriptor upload instead of two: the shortest path for a single request.  For a candidate list cut into
 * mini-batch slices use aif_score_batch and one aif_topk over the whole list.  Errors as the two calls. */
AIF_API aif_status aif_score_topk(aif_ctx *ctx, const aif_request *reqs, int32_t n_req, int32_t k, int32_t *idx_out,
                                  float *val_out, void *hip_stream);

/* For callers that cannot allocate device memory at the time of the call -- code running under HIP graph capture,
 * tight serving loops, harnesses that forbid it: aif_score_topk for ONE request, with every per-call buffer
 * (descriptor tables, folded bias, packed K/V, the feature matrix [e | attention | cross], hidden activations of the
 * layer-by-layer MLP) inside a fixed array of AIF_STATIC_SCRATCH_BYTES that the library holds on each GPU it runs
 * on, from load until the process ends.  The call allocates and frees nothing, uses no pinned staging, event, copy
 * or memset command -- only kernel launches on hip_stream, so it may be captured into a HIP graph and replayed (the
 * request's pointers and sizes are then baked into the graph).  Same kernels and same bits as aif_score_topk; k = 0
 * scores without selecting (idx_out, val_out may then be NULL).  Errors: as aif_score_topk, and AIF_ERANGE with the
 * byte counts in aif_last_error when the request does not fit the array (about 10^4 candidates of configurations
 * C1-C4, fewer for wider rows).  ALL calls on one GPU share that one array, whatever context or stream they come
 * through: a call overwrites what the last one left, and calls that overlap in time on one GPU race -- order them
 * on one stream or with events.  aif_peek_features does not see this call's features. */
#define AIF_STATIC_SCRATCH_BYTES (16u << 20)
AIF_API aif_status aif_score_topk_static(aif_ctx *ctx, const aif_request *req, int32_t k, int32_t *idx_out,
                                         float *val_out, void *hip_stream);

/* Nearline maintenance of the item table (Sec. 3.4: the index table of nearline results is refreshed as a
 * whole and also row by row).
 *
 * Incremental: row ids[i] of the context's item table becomes rows[i, :] (ids: DEVICE [n] int32; rows: DEVICE
 * [n, d_item] row-major, config.dtype, 16-byte aligned).  The table handed to aif_score_init (or
 * aif_swap_table) is written: it must be writable device memory.  Asynchronous on hip_stream and ordered with
 * it: scoring calls enqueued earlier on the stream read the old rows, later ones the new rows.  The ids of
 * one call must be distinct (a nearline batch is keyed by item); with a repeated id the row holds pieces of
 * either source.  An id outside [0, n_items) writes nothing and bumps the counter read by
 * aif_poll_device_errors.  Errors: AIF_EINVAL (NULL with n > 0, negative n, misaligned rows). */
AIF_API aif_status aif_update_rows(aif_ctx *ctx, const int32_t *ids, const void *rows, int32_t n, void *hip_stream);

/* Full update: later calls on this context read new_table (DEVICE [n_items, d_item] row-major, config.dtype,
 * 16-byte aligned, borrowed like the first one).  Host-side only; calls already enqueued keep the old table,
 * which the caller keeps alive until they complete. */
AIF_API aif_status aif_swap_table(aif_ctx *ctx, const void *new_table, int64_t n_items);

/* Release the context, its workspace and weight copies.  The caller must
 * have synchronised every stream the context was used on.  NULL is a no-op. */
AIF_API void aif_score_destroy(aif_ctx *ctx);

/* Message for the last failing call on this context (never NULL); with
 * ctx = NULL, the last failing aif_score_init of the calling thread.  Right
 * after a successful aif_score_init: the fallback note described there. */
AIF_API const char *aif_last_error(const aif_ctx *ctx);

/* After the caller has synchronised the stream: number of out-of-range
 * candidate ids seen since the last poll (the counter is reset).
 * Synchronous device read. */
AIF_API aif_status aif_poll_device_errors(aif_ctx *ctx, int32_t *n_bad_ids);

/* Test hook: rows [first_row, first_row + n_rows) of the feature matrix
 * [e | attention | cross] that the last batch left for its request number
 * `request`, copied to the HOST buffer out as a row-major
 * [n_rows, d_item + d_attn + d_cross] matrix of config.dtype (the library's
 * own layout in device memory is not part of the interface).  Synchronous;
 * the caller has synchronised the stream of that batch.  Rows at or beyond
 * the request's n_cand are unspecified. */
AIF_API aif_status aif_peek_features(aif_ctx *ctx, int32_t request, int32_t first_row, int32_t n_rows, void *out);

/* Per-kernel timing with HIP events on the caller's stream (the service
 * metrics of Sec. 5.1 are response times; this is their per-kernel breakdown).
 * Between aif_profile_begin and aif_profile_end every aif_score_batch records
 * an event before and after each of its kernels, and every aif_topk around
 * its kernel, for at most max_calls calls of each kind (later calls are not
 * recorded).  aif_profile_end synchronises on the recorded events and returns
 * the summed milliseconds per stage in ms_sum[AIF_STAGE_COUNT] and the number
 * of recorded calls per stage in n_calls[AIF_STAGE_COUNT] (both HOST). */
enum { AIF_STAGE_GATHER = 0, AIF_STAGE_USER_FOLD = 1, AIF_STAGE_ATTENTION = 2, AIF_STAGE_MLP = 3,
       AIF_STAGE_TOPK = 4, AIF_STAGE_COUNT = 5 };
AIF_API aif_status aif_profile_begin(aif_ctx *ctx, int32_t max_calls);
/* The same for a subset of the stages: stage_mask has bit (1 << AIF_STAGE_x) set
 * for every stage to be timed; only the events that bound those stages are
 * recorded (an event costs a few microseconds on the stream), the others'
 * ms_sum and n_calls come back 0.  AIF_EINVAL if the mask names no stage. */
AIF_API aif_status aif_profile_begin_stages(aif_ctx *ctx, int32_t max_calls, uint32_t stage_mask);
/* The same, recording only every `every`-th scoring call (and every `every`-th
 * aif_topk) from the first on: max_calls bounds the RECORDED calls, n_calls of
 * aif_profile_end counts them.  For long runs, where the events of every call
 * would cost more stream time than the timing is worth.  AIF_EINVAL if every < 1. */
AIF_API aif_status aif_profile_begin_sampled(aif_ctx *ctx, int32_t max_calls, uint32_t stage_mask, int32_t every);
AIF_API aif_status aif_profile_end(aif_ctx *ctx, double *ms_sum, int32_t *n_calls);

/* Which kernel family serves a stage of this context: 0 = shape-agnostic fp32
 * kernels, 1 = bf16 MFMA kernels.  stage is one of the AIF_STAGE_* values.
 * For AIF_STAGE_GATHER the answer describes the LAST scoring call: 0 = the table
 * was indexed by a launch of its own (timed as that stage), 2 = by the attention
 * kernel, which then reads the item vectors from the table and writes them to the
 * workspace itself (the gather stage's time is then only the user fold and the
 * packing of K/V; the gather's bytes are moved under the attention stage). */
AIF_API int32_t aif_stage_kind(const aif_ctx *ctx, int32_t stage);

/* Number of distinct users the LAST scoring call staged (Sec. 3.1: user-side work is done per user, not per
 * mini-batch).  Requests of one call whose user_vec, cross_vecs, seq_keys, seq_vals and seq_len are all equal --
 * the slices of one candidate list -- count once: the user fold and the packing of K/V run once for them, and
 * every slice reads the shared result.  -1 for a NULL context, 0 before the first call. */
AIF_API int32_t aif_last_user_slots(const aif_ctx *ctx);

/* Width of the contraction that layer 1 of the MLP head computes PER CANDIDATE in this context (Sec. 2: what does
 * not depend on the candidate is done once).  D_in - d_user after the user fold; where the Hadamard cross block
 * (Sec. 3.3) is folded into each user's layer-1 weights as well -- its share sum_k W1c[n,k] u_k e_k is linear in the
 * item vector, so W'[n,k] = W1e[n,k] + u_k W1c[n,k] takes its place, once per user -- d_item + d_attn.  A
 * measurement that counts the head's arithmetic counts this width (no credit for avoided work).  -1 for NULL. */
AIF_API int32_t aif_mlp_layer1_width(const aif_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* AIF_H */
