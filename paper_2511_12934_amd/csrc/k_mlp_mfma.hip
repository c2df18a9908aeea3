// a6-a7 on the matrix cores -- the MLP head (Sec. 1: a small MLP) as one
// fused bf16 MFMA chain.
//
// The products are formed transposed, H^T = W . X^T: the weights are the A
// operand (rows = output features) and the candidates are the columns of the
// B operand.  A 32x32x16 MFMA leaves, in lane (column c, half h), output rows
// 8q + 4h + i (q, i = 0..3) of column c -- sixteen features of ONE candidate.
// The B operand of the next layer wants, in lane (column c, half h), eight
// contraction indices of column c.  The contraction index may be assigned to
// (half, slot) in any way as long as both operands agree, so the sixteen
// values a lane already holds are used in place as two k-steps of the next
// layer (slot s of half h <-> feature 16j + 8(s/4) + 4h + s%4) and the next
// layer's weights are stored in that order once, at init.  Activations of all
// layers therefore stay in registers: no LDS round trip, no transpose.
//
// Weights stream through a ring in LDS, shared by the waves of the block; each
// wave owns one column tile of 32 candidates.  The user block of layer 1
// arrives as the per-request bias (user fold), the final ->1 layer is a dot
// product in the epilogue.
//
// Here: the weights' fragment order and the choice of a chain; the kernel is in k_mlp_chain.h, one translation unit
// per shape (k_mlp_chain_*.hip).
#include "k_mfma.h"
#include "mfma_util.h"

namespace aif {

hipError_t mlp_chain_c2(const Model &, const Batch &, const void *, const MlpPack &, const float *, hipStream_t);
hipError_t mlp_chain_c3(const Model &, const Batch &, const void *, const MlpPack &, const float *, hipStream_t);
hipError_t mlp_chain_c4(const Model &, const Batch &, const void *, const MlpPack &, const float *, hipStream_t);
hipError_t mlp_chain_c5(const Model &, const Batch &, const void *, const MlpPack &, const float *, hipStream_t);
hipError_t mlp_chain_c2h(const Model &, const Batch &, const void *, const MlpPack &, const float *, hipStream_t);
hipError_t mlp_chain_c3h(const Model &, const Batch &, const void *, const MlpPack &, const float *, hipStream_t);
hipError_t mlp_chain_c4h(const Model &, const Batch &, const void *, const MlpPack &, const float *, hipStream_t);
hipError_t mlp_chain_c2f(const Model &, const Batch &, const void *, const MlpPack &, const float *, hipStream_t);
hipError_t mlp_chain_c3f(const Model &, const Batch &, const void *, const MlpPack &, const float *, hipStream_t);
hipError_t mlp_chain_c4f(const Model &, const Batch &, const void *, const MlpPack &, const float *, hipStream_t);
hipError_t mlp_chain_c5f(const Model &, const Batch &, const void *, const MlpPack &, const float *, hipStream_t);

// Can the chain of this variant form the Hadamard cross block itself (Model::cross_in_mlp)?  Layer 1 after the user
// fold must be exactly [item | attention | item (.) u] with the item width the kernel was built for.
bool mlp_chain_forms_cross(int variant, const Model &m)
{
    if (m.dtype != 1 || m.cross_mode != 1 || m.k1 != 2 * m.d_item + m.d_attn) return false;
    if (variant == 0 || variant == 1) return m.d_item == 64;
    if (variant == 2) return m.d_item == 128;
    return false;
}

// Can the cross block be folded into each user's layer-1 weights (Model::cross_in_mlp == 2; k_stage.h: fold_w0_block)?
// It must be linear in the item vector with coefficients that depend on the user alone -- the Hadamard block
// u (.) e, and BEA's w^ V, whose weights w^ are the item row's last entries (Sec. 4.1) -- and layer 1 without it,
// [item | attention], must be a width the `f` chains are built for.
bool mlp_chain_folds_cross(int variant, const Model &m)
{
    if (m.dtype != 1) return false;
    if (m.cross_mode == 1) return mlp_chain_forms_cross(variant, m);
    if (m.cross_mode == 2)      // segment dots: whole k-steps per segment, what a staging block keeps of the vectors (k_stage.h)
        return variant == 3 && m.k1 == m.d_item + m.d_attn + m.d_cross && m.d_item + m.d_attn == 384 && m.d_cv % 16 == 0 &&
               m.d_item % m.d_cv == 0 && m.n_cross <= 32 && m.n_cross * m.d_cv <= 2048;
    if (m.cross_mode != 3 || m.k1 != m.d_item + m.d_attn + m.d_cv || m.d_cv % 16 || m.n_cross > m.d_item) return false;
    if (m.d_cv > 64 || m.n_cross * m.d_cv > 2048) return false;      // what a staging block keeps of the user's vectors (k_stage.h)
    const int k = m.d_item + m.d_attn;
    return ((variant == 0 || variant == 1) && k == 128) || (variant == 2 && k == 256);
}

// ---- weights into fragment order --------------------------------------------
// dst[((rt * KS + j) * 64 + lane) * 8 + s] = W[32 rt + lane % 32][col0 + k(j, lane / 32, s)]
// first layer (activations read from memory):   k = 16 j + 8 h + s
// later layers (activations left by an MFMA):   k = 16 j + 8 (s / 4) + 4 h + s % 4
__global__ void k_pack_frag(const uint16_t *__restrict__ W, int n_in, int col0, int N, int K, int from_mfma,
                            uint16_t *__restrict__ dst)
{
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)N * K) return;
    const int s = (int)(idx & 7), lane = (int)((idx >> 3) & 63);
    const int KS = K / 16;
    const int j = (int)((idx >> 9) % KS), rt = (int)((idx >> 9) / KS);
    const int n = 32 * rt + (lane & 31), h = lane >> 5;
    const int k = from_mfma ? 16 * j + 8 * (s >> 2) + 4 * h + (s & 3) : 16 * j + 8 * h + s;
    dst[idx] = W[(size_t)n * n_in + col0 + k];
}

hipError_t pack_frag(const void *W, int n_in, int col0, int N, int K, bool from_mfma, void *dst, hipStream_t s)
{
    const size_t total = (size_t)N * K;
    hipLaunchKernelGGL(k_pack_frag, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const uint16_t *)W, n_in,
                       col0, N, K, from_mfma ? 1 : 0, (uint16_t *)dst);
    return hipGetLastError();
}

// ---- dispatch -----------------------------------------------------------------
int mlp_mfma_variant(const Model &m)
{
    if (m.dtype != 1) return -1;
    const int nh = m.n_layers - 1;
    const int k1 = m.k1, h1 = nh >= 1 ? m.dims[1] : 0, h2 = nh >= 2 ? m.dims[2] : 0, h3 = nh >= 3 ? m.dims[3] : 0;
    if (nh == 2 && k1 == 192 && h1 == 256 && h2 == 128) return 0;
    if (nh == 2 && k1 == 192 && h1 == 512 && h2 == 256) return 1;
    if (nh == 1 && k1 == 384 && h1 == 256) return 2;
    if (nh == 3 && k1 == 448 && h1 == 1024 && h2 == 512 && h3 == 256) return 3;
    return -1;
}

hipError_t launch_mlp_variant(int variant, const Model &m, const Batch &b, const void *X, const MlpPack &pk,
                              const float *bias1, hipStream_t s)
{
    if (b.n_blk == 0) return hipSuccess;
    switch (variant) {
    // cross_in_mlp: 0 the cross block is in the workspace, 1 the chain forms it from the item block, 2 it is folded into
    // the user's layer-1 weights (the `f` chains: layer 1 over [item | attention])
    case 0: return m.cross_in_mlp == 2 ? mlp_chain_c2f(m, b, X, pk, bias1, s) : m.cross_in_mlp ? mlp_chain_c2h(m, b, X, pk, bias1, s) : mlp_chain_c2(m, b, X, pk, bias1, s);
    case 1: return m.cross_in_mlp == 2 ? mlp_chain_c3f(m, b, X, pk, bias1, s) : m.cross_in_mlp ? mlp_chain_c3h(m, b, X, pk, bias1, s) : mlp_chain_c3(m, b, X, pk, bias1, s);
    case 2: return m.cross_in_mlp == 2 ? mlp_chain_c4f(m, b, X, pk, bias1, s) : m.cross_in_mlp ? mlp_chain_c4h(m, b, X, pk, bias1, s) : mlp_chain_c4(m, b, X, pk, bias1, s);
    case 3: return m.cross_in_mlp == 2 ? mlp_chain_c5f(m, b, X, pk, bias1, s) : mlp_chain_c5(m, b, X, pk, bias1, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace aif
