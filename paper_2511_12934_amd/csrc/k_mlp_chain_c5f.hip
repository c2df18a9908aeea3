// The fused MLP chain (k_mlp_chain.h), shape of k_mlp_chain_c5.hip, with the segment-dot cross block folded into the user's
// layer-1 weights (one set of layer-1 fragments per user slot): layer 1 contracts over [item | attention] = 384 columns.
#include "k_mlp_chain.h"

namespace aif {

hipError_t mlp_chain_c5f(const Model &m, const Batch &b, const void *X, const MlpPack &pk, const float *bias1, hipStream_t s)
{
    return launch_spec<384, 1024, 512, 256, 4, 16, 4, 1, 0, 1>(m, b, X, pk, bias1, s);
}

}  // namespace aif
