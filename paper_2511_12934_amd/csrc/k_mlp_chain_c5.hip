// The fused MLP chain (k_mlp_chain.h) for one shape -- C5: 448 -> 1024 -> 512 -> 256 -> 1 after the user fold; waves per block,
// fragments per stage, ring slots, blocks per compute unit: 4, 16, 4, 1 (one wave per SIMD with the whole register file).
#include "k_mlp_chain.h"

namespace aif {

hipError_t mlp_chain_c5(const Model &m, const Batch &b, const void *X, const MlpPack &pk, const float *bias1, hipStream_t s)
{
    return launch_spec<448, 1024, 512, 256, 4, 16, 4, 1>(m, b, X, pk, bias1, s);
}

}  // namespace aif
