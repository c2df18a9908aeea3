// The fused MLP chain (k_mlp_chain.h) for one shape -- C3: 192 -> 512 -> 256 -> 1 after the user fold; waves per block, fragments per
// stage, ring slots: 4, 16, 4.
#include "k_mlp_chain.h"

namespace aif {

hipError_t mlp_chain_c3(const Model &m, const Batch &b, const void *X, const MlpPack &pk, const float *bias1, hipStream_t s)
{
    return launch_spec<192, 512, 256, 0, 4, 16, 4>(m, b, X, pk, bias1, s);
}

}  // namespace aif
