// MFMA (bf16) kernels of libaif: eligibility, packed weights, launchers.
#pragma once
#include "aif_dev.h"

namespace aif {

struct MfmaPlan {
    bool attn = false;                 // a3-a5 run on the MFMA attention kernel
    bool mlp = false;                  // a6-a7 run on the MFMA MLP chain
    int attn_variant = -1;
    int mlp_variant = -1;
    void *wpack[MAX_LAYERS] = {};      // hidden layers' bf16 weights in MFMA fragment order (owned)
    void *wq_pack = nullptr;           // bf16 W_q in fragment order (owned)
    float *zeros = nullptr;            // zero vector standing in for an absent bias (owned)
    char *kvpack = nullptr;            // per-request K/V in fragment order (owned workspace)
    float *kmax = nullptr;             // per request, head and 64-key stage: max |k_t| (owned workspace)
    size_t pack_stride = 0;            // bytes of kvpack per request
    int nktp = 0;                      // key tiles per head the pack layout is sized for
    char *hbuf[2] = {};                // layered MLP: hidden activations between launches, ping-pong (owned workspace)
    char *w0_user = nullptr;           // per user slot: layer 1's fragments with the Hadamard cross block folded in (owned workspace; Model::cross_in_mlp == 2)
    size_t w0_stride = 0;              // bytes per slot
};
constexpr int MLP_VARIANT_LAYERS = 100;   // mlp_variant of the one-launch-per-layer path (k_mlp_layers.hip)

struct MlpPack {
    const char *w[3];                  // hidden layers' weights in fragment order
    const float *bias[3];              // fp32 biases of hidden layers 2, 3 (index 1, 2), never null; [0] unused
    const float *wlast;                // fp32 weights of the final ->1 layer
    const float *blast;                // its bias (1 float), never null
    const char *w0_user;               // layer 1's fragments per user slot with the Hadamard cross block folded in (k_mlp_chain.h: UW), or null
    size_t w0_stride;                  // bytes per slot
};

// Decide which MFMA kernels can serve the model and pack their weights
// (w_q, w: the caller's device tensors, read here only).
hipError_t mfma_plan(const Model &m, int max_seq_len, int max_users, size_t x_rows, const void *w_q, const void *const *w,
                     MfmaPlan &plan, hipStream_t s);
void mfma_release(MfmaPlan &plan);

// Host side: which attention kernel serves which request.  A request whose packed K/V (all heads) fit in one
// CU's LDS goes to the resident kernel: such requests are cut into groups of tiles (about one group per CU), written to `out` (room for attn_max_groups() entries), their number returned.
// The others are the streaming kernels': *n_streamed says how many (requests with candidates).  The choice
// depends on the request alone, so its result does not depend on what else is in the batch.
// info (optional): what a device-side rebuild of the groups needs (few_fill): the tiles per group at most, and which
// of the first 32 requests are the resident kernel's.
struct AttnPlanInfo {
    int32_t per;
    uint32_t resident;
};
int attn_plan_groups(const Model &m, const ReqDesc *reqs /*host*/, int n_req, int n_cu, AttnGroup *out /*host*/,
                     int *n_streamed, AttnPlanInfo *info = nullptr);
size_t attn_max_groups(size_t x_rows, int max_users);

// kv_packed: the batch's K/V are already in fragment order (launch_stage did it)
// gather_table: non-null only when attn_gathers(m, b, plan): the attention kernel then reads the item vectors from
// the table itself (the caller has not run the gather) and counts ids outside the table in *bad
hipError_t launch_attn_mfma(const Model &m, const Batch &b, void *X, const MfmaPlan &plan, bool kv_packed, hipStream_t s,
                            const void *gather_table = nullptr, int32_t *bad = nullptr);
bool attn_gathers(const Model &m, const Batch &b, const MfmaPlan &plan);

// k_stage.hip: gather + user fold + K/V packing as one launch (bf16 models served by the MFMA attention kernel)
bool stage_fusable(const Model &m, const MfmaPlan &plan);
// Model::cross_in_mlp == 2 on a model whose staging is not launch_stage: the users' layer-1 weights as a launch of its own
hipError_t launch_fold_w0(const Model &m, const Batch &b, const MfmaPlan &plan, hipStream_t s);
// up (optional, only with gather == false): the same launch also carries the call's descriptor tables from mapped
// pinned host memory to the device (bytes rounded up to 16, as launch_upload); its own blocks then read the request
// descriptors through the mapping (reqs_mapped), every later kernel reads the device copy that `b` points to.
struct StageUpload {
    const void *src_mapped;
    void *dst;
    size_t bytes;
    const ReqDesc *reqs_mapped;
    const int32_t *slot_req_mapped;     // the batch's slot_req table through the same mapping
};
// few (optional, a batch of at most FEW_MAX requests, not with up): the requests' descriptors travel in the kernel's
// arguments, the launch's blocks read them there and its first blocks write the device tables of the batch (k_stage.h:
// FewFill), so no upload of any kind precedes the launch.
struct FewFill;
hipError_t launch_stage(const Model &m, const Batch &b, const void *table, void *X, int32_t *bad, const float *w1u,
                        const float *b1, float *bias1, const MfmaPlan &plan, bool gather, hipStream_t s,
                        const StageUpload *up = nullptr, const FewFill *few = nullptr);

// bias_f32[l] / wlast_f32: the context's fp32 copies (bias of layer l or null; last layer's weight row).
hipError_t launch_mlp_mfma(const Model &m, const Batch &b, const void *X, const MfmaPlan &plan,
                           const float *const *bias_f32, const float *wlast_f32, const float *bias1, hipStream_t s);

// k_mlp_mfma.hip
int mlp_mfma_variant(const Model &m);
bool mlp_chain_forms_cross(int variant, const Model &m);
bool mlp_chain_folds_cross(int variant, const Model &m);
// bytes per user slot of layer 1's weights with the Hadamard cross block folded in (k_stage.h: fold_w0_block)
inline size_t mlp_w0_user_bytes(const Model &m) { return (size_t)m.dims[1] * (m.d_item + m.d_attn) * 2; }
hipError_t launch_mlp_variant(int variant, const Model &m, const Batch &b, const void *X, const MlpPack &pk,
                              const float *bias1, hipStream_t s);
hipError_t pack_frag(const void *W, int n_in, int col0, int N, int K, bool from_mfma, void *dst, hipStream_t s);

// k_mlp_layers.hip: wide heads, one launch per layer
bool mlp_layers_ok(const Model &m);
size_t mlp_layers_buf_bytes(const Model &m, size_t x_rows, int which);
hipError_t launch_mlp_layers(const Model &m, const Batch &b, const void *X, const MlpPack &pk, const float *bias1,
                             char *const *hbuf, hipStream_t s);

// k_attn_mfma.hip
int attn_mfma_variant(const Model &m, bool has_wq);
size_t attn_pack_stride(const Model &m, int max_seq_len, int *nktp_out);
hipError_t launch_attn_variant(const Model &m, const Batch &b, void *X, const MfmaPlan &plan, bool kv_packed,
                               const void *gather_table, int32_t *bad, hipStream_t s);
constexpr int ATTN_VARIANT_PROJ = 2;      // attn_variant of the projection + 16-wide-heads kernel (k_attn_proj.hip)

// k_attn_proj.hip: query projection, 16-wide heads, Hadamard / segment-dot cross
bool attn_proj_ok(const Model &m, bool has_wq);
size_t attn_proj_pack_stride(const Model &m, int max_seq_len, int *nktp_out);
// gather_table, bad: as for launch_attn_mfma
hipError_t launch_attn_proj(const Model &m, const Batch &b, void *X, const MfmaPlan &plan, bool small, bool kv_packed,
                            hipStream_t s, const void *gather_table = nullptr, int32_t *bad = nullptr);
// the user-side staging of this attention kernel's models as one launch: K/V packing, user fold and (Model::cross_in_mlp
// == 2) the users' layer-1 weights; the attention launch that follows takes kv_packed = true
bool stage_proj_fusable(const Model &m, const MfmaPlan &plan);
hipError_t launch_stage_proj(const Model &m, const Batch &b, const float *w1u, const float *b1, float *bias1,
                             const MfmaPlan &plan, hipStream_t s);
struct FoldW0;
hipError_t fold_w0_args(const Model &m, const MfmaPlan &plan, FoldW0 &f);      // k_stage.hip

}  // namespace aif
