// The fused MLP chain (k_mlp_chain.h), shape of k_mlp_chain_c2.hip, with the Hadamard cross block folded into the user's layer-1
// weights (one set of layer-1 fragments per user slot, made by the staging launch): layer 1 contracts over [item | attention].
#include "k_mlp_chain.h"

namespace aif {

hipError_t mlp_chain_c2f(const Model &m, const Batch &b, const void *X, const MlpPack &pk, const float *bias1, hipStream_t s)
{
    return launch_spec<128, 256, 128, 0, 4, 16, 4, 2, 0, 1>(m, b, X, pk, bias1, s);
}

}  // namespace aif
