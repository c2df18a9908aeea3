// MFMA kernels -- plan and launchers.
#include "k_mfma.h"

namespace aif {

hipError_t mfma_plan(const Model &, int, const void *, const void *const *, const void *const *, MfmaPlan &plan,
                     hipStream_t)
{
    plan.attn = false;
    plan.mlp = false;
    return hipSuccess;
}

void mfma_release(MfmaPlan &plan)
{
    for (auto &p : plan.wpack) { if (p) (void)hipFree(p); p = nullptr; }
    for (auto &p : plan.bias) { if (p) (void)hipFree(p); p = nullptr; }
    if (plan.wq_pack) (void)hipFree(plan.wq_pack);
    plan.wq_pack = nullptr;
}

hipError_t launch_attn_mfma(const Model &, const Batch &, void *, const MfmaPlan &, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_mlp_mfma(const Model &, const Batch &, const void *, const MfmaPlan &, const float *, hipStream_t) { return hipErrorNotSupported; }

}  // namespace aif
