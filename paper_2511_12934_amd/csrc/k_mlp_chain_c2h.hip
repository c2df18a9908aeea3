// The fused MLP chain (k_mlp_chain.h), shape of k_mlp_chain_c2.hip, with the Hadamard cross block formed in the kernel from the item
// block (4 k-steps of 16): the workspace's cross block is neither written by the attention kernel nor read here.
#include "k_mlp_chain.h"

namespace aif {

hipError_t mlp_chain_c2h(const Model &m, const Batch &b, const void *X, const MlpPack &pk, const float *bias1, hipStream_t s)
{
    return launch_spec<192, 256, 128, 0, 4, 16, 4, 2, 4>(m, b, X, pk, bias1, s);
}

}  // namespace aif
