/*
 * aif_user.h -- C ABI of the user-side network that AIF runs asynchronously,
 * in parallel with candidate retrieval, on MI355X (gfx950): Sec. 3.1 of
 * arXiv 2511.12934, "Pre-Computation Phase", Eq. 1-3.
 *
 * For each user the library takes the profile embedding U_profile [d_raw] and
 * the behaviour-sequence embeddings U_seq [l, d_raw] and computes
 *   Eq. 1  U^_profile = W_profile U_profile,  U^_seq[t] = W_seq U_seq[t]      (width d)
 *   Eq. 2  U_self_attention = Pooling(FFN(Softmax(U^_seq U^_seq^T / sqrt(d)) U^_seq))
 *   Eq. 3  U_profile_attention = Softmax(U^_profile U^_seq^T / sqrt(d)) U^_seq
 * and leaves, in caller memory, the tensors the real-time phase reads
 * (aif.h): the combined user vector and the projected sequence U^_seq, which
 * serves as keys and values of the target attention.
 *
 * The paper names FFN, Pooling and the combination without defining them;
 * this library takes
 *   FFN(x)   = max(0, W_ffn x + b_ffn), one layer d -> d, on every position,
 *   Pooling  = mean over the l positions,
 *   combined = [U_self_attention | U_profile_attention], width 2 d,
 * with no residual connection, normalisation, mask or dropout (none is
 * printed).  l = 0 gives a zero vector.
 *
 * Arithmetic: inputs and weights in the storage type, fp32 accumulation;
 * with bf16 storage U^_seq is rounded to bf16 once, when it is written, and
 * both attentions read the rounded values (the real-time phase reads the same
 * ones); attention outputs are rounded to the storage type before the FFN.
 *
 * Conventions are those of aif.h: plain C, every call returns an aif_status
 * and enqueues nothing on failure, DEVICE pointers belong to the device that
 * was current at init, all work is asynchronous on the caller's stream (the
 * point of the phase is to run beside other work: give it a stream of its
 * own), the library owns only its context, workspace and weight copies and
 * borrows the request tensors until the enqueued work has completed.  Not
 * capturable into a HIP graph.  One context serves one stream at a time.
 */
#ifndef AIF_USER_H
#define AIF_USER_H

#include "aif.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct aif_user_ctx aif_user_ctx;

typedef struct {
    aif_dtype dtype;        /* storage type of embeddings, weights and outputs                       */
    int32_t d_raw;          /* d^U of Sec. 3.1: width of the profile and behaviour embeddings, a multiple of 16 bytes */
    int32_t d;              /* common width after Eq. 1, a multiple of 16 bytes                      */
    int32_t max_seq_len;    /* longest behaviour sequence                                            */
    int32_t max_users;      /* users per aif_user_precompute call                                    */
} aif_user_config;

/* Weights, all DEVICE, storage type = config.dtype, row-major [out, in] (y = W x + b); read and
 * repacked during aif_user_init only. */
typedef struct {
    const void *w_profile;  /* [d, d_raw]  Eq. 1                                                     */
    const void *w_seq;      /* [d, d_raw]  Eq. 1                                                     */
    const void *w_ffn;      /* [d, d]      FFN of Eq. 2                                              */
    const void *b_ffn;      /* [d] or NULL = zero bias                                               */
} aif_user_weights;

/* One user.  DEVICE pointers, 16-byte aligned, valid until the enqueued work completes. */
typedef struct {
    const void *profile;    /* [d_raw]                                                               */
    const void *seq;        /* [seq_len, d_raw] row-major                                            */
    int32_t seq_len;        /* 0..max_seq_len                                                        */
    void *user_vec_out;     /* [2 d]: [U_self_attention | U_profile_attention]                       */
    void *seq_out;          /* [seq_len, d] row-major: U^_seq                                        */
} aif_user_request;

/* Sec. 3.1.  Creates a context on the current device, copies the weights, sizes the workspace for
 * max_users users of max_seq_len positions.  Synchronous.  *out is set only on AIF_OK. */
AIF_API aif_status aif_user_init(const aif_user_config *config, const aif_user_weights *weights, aif_user_ctx **out);

/* Eq. 1-3 for n_users users (HOST array, read during the call) on hip_stream.  Errors: AIF_EINVAL
 * (NULL, negative sizes, misaligned tensors), AIF_ERANGE (beyond the limits of the context),
 * AIF_EDEVICE. */
AIF_API aif_status aif_user_precompute(aif_user_ctx *ctx, const aif_user_request *users, int32_t n_users, void *hip_stream);

/* Frees the context, its workspace and weight copies; the caller has synchronised its streams.  NULL is allowed. */
AIF_API void aif_user_destroy(aif_user_ctx *ctx);

/* Text of the last failure of this context (of the last failed aif_user_init when ctx is NULL). */
AIF_API const char *aif_user_last_error(const aif_user_ctx *ctx);

/* Which kernel family serves the attentions of Eq. 2 and Eq. 3 in this context: 0 = shape-agnostic
 * fp32 kernel, 1 = bf16 MFMA kernels. */
AIF_API int32_t aif_user_attention_kind(const aif_user_ctx *ctx);

/* Per-kernel timing with HIP events on the caller's stream, as aif_profile_begin / _end of aif.h:
 * stages AIF_USER_STAGE_PROJECT (Eq. 1), _ATTENTION (the attentions of Eq. 2 and Eq. 3), _FFN_POOL
 * (FFN, pooling, combined vector); ms[] and calls[] have AIF_USER_N_STAGES entries. */
typedef enum { AIF_USER_STAGE_PROJECT = 0, AIF_USER_STAGE_ATTENTION = 1, AIF_USER_STAGE_FFN_POOL = 2, AIF_USER_N_STAGES = 3 } aif_user_stage;
AIF_API aif_status aif_user_profile_begin(aif_user_ctx *ctx, int32_t max_calls);
AIF_API aif_status aif_user_profile_end(aif_user_ctx *ctx, double *ms, int32_t *calls);

#ifdef __cplusplus
}
#endif
#endif /* AIF_USER_H */
