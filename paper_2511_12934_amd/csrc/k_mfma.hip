// MFMA kernels -- plan (eligibility + weight packing) and launchers.
#include "k_mfma.h"

#include <cstdlib>

namespace aif {

hipError_t mfma_plan(const Model &m, int max_seq_len, int max_users, size_t x_rows, const void *w_q, const void *const *w,
                     MfmaPlan &plan, hipStream_t s)
{
    plan.attn = false;
    plan.mlp = false;
    const char *force = getenv("AIF_FORCE_GENERIC");
    if (force && force[0] == '1') return hipSuccess;

    plan.attn_variant = attn_mfma_variant(m, w_q != nullptr);
    if (plan.attn_variant >= 0) {
        plan.pack_stride = attn_pack_stride(m, max_seq_len, &plan.nktp);
        hipError_t e = hipMalloc((void **)&plan.kvpack, plan.pack_stride * max_users + 16);
        if (e != hipSuccess) return e;
        e = hipMalloc((void **)&plan.kmax, (size_t)max_users * m.n_heads * (plan.nktp / 2 + 1) * 4);
        if (e != hipSuccess) return e;
        if (plan.attn_variant == ATTN_VARIANT_PROJ) {
            e = hipMalloc(&plan.wq_pack, (size_t)m.d_attn * m.d_item * 2);
            if (e != hipSuccess) return e;
            e = pack_frag(w_q, m.d_item, 0, m.d_attn, m.d_item, false, plan.wq_pack, s);
            if (e != hipSuccess) return e;
        }
        plan.attn = true;
    }

    plan.mlp_variant = mlp_mfma_variant(m);
    {
        const char *lay = getenv("AIF_MLP_LAYERED");    // testing and measurement: one launch per layer even where a fused chain serves the shape
        if (lay && lay[0] == '1') plan.mlp_variant = -1;
    }
    if (plan.mlp_variant < 0 && mlp_layers_ok(m)) {
        plan.mlp_variant = MLP_VARIANT_LAYERS;
        for (int i = 0; i < 2; ++i) {
            const size_t bytes = mlp_layers_buf_bytes(m, x_rows, i);
            if (!bytes) continue;
            hipError_t e = hipMalloc((void **)&plan.hbuf[i], bytes);
            if (e != hipSuccess) return e;
        }
    }
    if (plan.mlp_variant >= 0) {
        const int nh = m.n_layers - 1;
        for (int l = 0; l < nh; ++l) {
            const int K = l == 0 ? m.k1 : m.dims[l], N = m.dims[l + 1];
            hipError_t e = hipMalloc(&plan.wpack[l], (size_t)N * K * 2);
            if (e != hipSuccess) return e;
            e = pack_frag(w[l], m.dims[l], l == 0 ? m.d_user : 0, N, K, l > 0, plan.wpack[l], s);
            if (e != hipSuccess) return e;
        }
        int widest = 0;
        for (int l = 1; l <= m.n_layers; ++l) widest = m.dims[l] > widest ? m.dims[l] : widest;
        hipError_t e = hipMalloc((void **)&plan.zeros, (size_t)widest * 4);
        if (e != hipSuccess) return e;
        e = hipMemsetAsync(plan.zeros, 0, (size_t)widest * 4, s);
        if (e != hipSuccess) return e;
        plan.mlp = true;
    }
    return hipSuccess;
}

void mfma_release(MfmaPlan &plan)
{
    for (auto &p : plan.wpack) {
        if (p) (void)hipFree(p);
        p = nullptr;
    }
    if (plan.wq_pack) (void)hipFree(plan.wq_pack);
    plan.wq_pack = nullptr;
    if (plan.zeros) (void)hipFree(plan.zeros);
    plan.zeros = nullptr;
    if (plan.kvpack) (void)hipFree(plan.kvpack);
    plan.kvpack = nullptr;
    if (plan.kmax) (void)hipFree(plan.kmax);
    plan.kmax = nullptr;
    for (auto &p : plan.hbuf) {
        if (p) (void)hipFree(p);
        p = nullptr;
    }
    if (plan.w0_user) (void)hipFree(plan.w0_user);
    plan.w0_user = nullptr;
}

hipError_t launch_attn_mfma(const Model &m, const Batch &b, void *X, const MfmaPlan &plan, bool kv_packed, hipStream_t s,
                            const void *gather_table, int32_t *bad)
{
    return launch_attn_variant(m, b, X, plan, kv_packed, gather_table, bad, s);
}

hipError_t launch_mlp_mfma(const Model &m, const Batch &b, const void *X, const MfmaPlan &plan,
                           const float *const *bias_f32, const float *wlast_f32, const float *bias1, hipStream_t s)
{
    MlpPack pk{};
    const int nh = m.n_layers - 1;
    for (int l = 0; l < nh && l < 3; ++l) {
        pk.w[l] = (const char *)plan.wpack[l];
        pk.bias[l] = bias_f32[l] ? bias_f32[l] : plan.zeros;
    }
    pk.wlast = wlast_f32;
    pk.blast = bias_f32[m.n_layers - 1] ? bias_f32[m.n_layers - 1] : plan.zeros;
    pk.w0_user = m.cross_in_mlp == 2 ? plan.w0_user : nullptr;
    pk.w0_stride = plan.w0_stride;
    if (plan.mlp_variant == MLP_VARIANT_LAYERS) return launch_mlp_layers(m, b, X, pk, bias1, plan.hbuf, s);
    return launch_mlp_variant(plan.mlp_variant, m, b, X, pk, bias1, s);
}

}  // namespace aif
