// MFMA (bf16) kernels of libaif: eligibility, packed weights, launchers.
#pragma once
#include "aif_dev.h"

namespace aif {

struct MfmaPlan {
    bool attn = false;                 // a3-a5 run on the MFMA attention kernel
    bool mlp = false;                  // a6-a7 run on the MFMA MLP chain
    int attn_variant = -1;
    int mlp_variant = -1;
    void *wpack[MAX_LAYERS] = {};      // bf16 weights in MFMA fragment order (owned)
    float *bias[MAX_LAYERS] = {};      // fp32 biases of layers >= 2 (owned)
    void *wq_pack = nullptr;           // bf16 W_q in fragment order (owned)
};

// Decide which MFMA kernels can serve the model and pack their weights.
hipError_t mfma_plan(const Model &m, int max_seq_len, const void *w_q, const void *const *w,
                     const void *const *b, MfmaPlan &plan, hipStream_t s);
void mfma_release(MfmaPlan &plan);

hipError_t launch_attn_mfma(const Model &m, const Batch &b, void *X, const MfmaPlan &plan, hipStream_t s);
hipError_t launch_mlp_mfma(const Model &m, const Batch &b, const void *X, const MfmaPlan &plan,
                           const float *bias1, hipStream_t s);

}  // namespace aif
