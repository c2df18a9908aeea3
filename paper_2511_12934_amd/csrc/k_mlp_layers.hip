// a6-a7 for WIDE heads on the matrix cores -- the MLP head (Sec. 1: "shallow
// multilayer perceptron") one layer per launch, for models whose hidden layers
// are too wide for a candidate's activations to stay in registers across the
// chain (k_mlp_mfma): e.g. 448 -> 1024 -> 512 -> 256 -> 1.
//
// Each launch is a bf16 GEMM in the transposed form of the fused chain,
// H_out^T = W H_in^T, with a 256-feature x 256-candidate tile per block: eight
// waves as 2 (features) x 4 (candidates), each holding 4 x 2 MFMA tiles of
// 32 x 32.  Both operands reach LDS as ready-made 1 KB MFMA fragments by
// direct-to-LDS loads, two 64 KB stages of four k-steps each:
//   - weights were packed into fragment order at init (pack_frag),
//   - activations between layers live in HBM in B-fragment order
//     [32-candidate tile][k-step][lane][8]: the 16 features a lane holds after a
//     32 x 32 MFMA are, as they stand, its share of two k-steps of the next
//     layer (whose weights are packed in the matching order), so the epilogue
//     stores them as two coalesced 16-byte pieces and nothing is ever transposed.
// Layer 1 reads the workspace rows [e | a | c] (either layout) and takes the
// user block as the per-request bias (user fold); the last hidden layer's
// epilogue forms the ->1 dot product and writes logit and score.
#include "k_mfma.h"
#include "mfma_util.h"

namespace aif {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

struct LayerArgs {
    const char *in;             // B operand: the workspace (layer 1) or the previous layer's activations
    XLayout in_l;               // where piece p of row r lives (x_offset)
    int32_t KS;                 // k-steps of 16 (a multiple of 4)
    const char *wfrag;          // [M / 32][KS] fragments of 1 KB
    int32_t M;                  // output features (a multiple of 256)
    const float *bias;          // [M], or [n_req, M] when per_req_bias, or null
    int32_t per_req_bias;
    char *out;                  // next layer's activations in B-fragment order (unused by the last layer)
    const float *wlast;         // last hidden layer: weights of the ->1 layer [M]
    const float *blast;         // its bias or null
};

constexpr int GL_STAGE_BYTES = 64 * 1024;   // 4 k-steps x (8 A + 8 B fragments)

__device__ __forceinline__ float relu_f(float x) { return __builtin_amdgcn_fmed3f(x, 0.f, __builtin_inff()); }

template <bool LAST>
__global__ __launch_bounds__(512) void k_mlp_layer(Model m, Batch b, LayerArgs a)
{
    extern __shared__ __align__(16) char lds[];
    const int bx = blockIdx.x, by = blockIdx.y;                 // candidate block (= scheduling block), feature block
    const int r = b.blk_req[bx];
    if (r < 0) return;
    const ReqDesc rd = b.reqs[r];
    const int local0 = bx * ROW_BLOCK - rd.row_base;
    if (rd.n_cand - local0 <= 0) return;

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = lane & 31, h = lane >> 5, wm = wave & 1, wn = wave >> 1;
    const uint32_t lds0 = lds_address(lds);
    const int NS = a.KS >> 2;

    // stage st -> buffer st & 1; a wave moves 8 of the stage's 64 fragments
    auto issue = [&](int st) {
        const uint32_t dst = lds0 + (st & 1) * GL_STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int f = wave * 8 + i, ks = f >> 4, rr = f & 15, k = 4 * st + ks;
            const char *src;
            if (rr < 8)
                src = a.wfrag + ((size_t)(by * 8 + rr) * a.KS + k) * 1024 + lane * 16;
            else
                src = a.in + x_offset(a.in_l, (uint32_t)(bx * ROW_BLOCK + (rr - 8) * 32 + col), (uint32_t)(2 * k + h));
            dma16(src, dst + f * 1024);
        }
    };

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    issue(0);
    for (int st = 0; st < NS; ++st) {
        if (st + 1 < NS) {
            issue(st + 1);
            wait_vmcnt<8>();                                    // this wave's share of stage st has landed
        } else
            wait_vmcnt<0>();
        __syncthreads();                                        // ... and everybody else's
        const char *base = lds + (st & 1) * GL_STAGE_BYTES + lane * 16;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 af[4], bf[2];
#pragma unroll
            for (int i = 0; i < 4; ++i) af[i] = *(const bf16x8 *)(base + (ks * 16 + wm * 4 + i) * 1024);
#pragma unroll
            for (int j = 0; j < 2; ++j) bf[j] = *(const bf16x8 *)(base + (ks * 16 + 8 + wn * 2 + j) * 1024);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();                                        // the buffer may be refilled
    }

    const float *bias = a.bias ? a.bias + (a.per_req_bias ? (size_t)r * a.M : 0) : nullptr;
    if constexpr (!LAST) {
        const size_t tile_stride = (size_t)(a.M >> 4) * 1024;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int rt = by * 8 + wm * 4 + i;                 // row tile of the layer
            float bv[16];
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int ii = 0; ii < 4; ++ii) bv[4 * q + ii] = bias ? bias[32 * rt + 8 * q + 4 * h + ii] : 0.f;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                char *o = a.out + (size_t)(bx * 8 + wn * 2 + j) * tile_stride + (size_t)(2 * rt) * 1024 + lane * 16;
#pragma unroll
                for (int p = 0; p < 2; ++p) {                   // parts 2p, 2p + 1 of the tile -> k-step 2 rt + p
                    bf16x8 o8;
#pragma unroll
                    for (int s = 0; s < 8; ++s) o8[s] = (__bf16)relu_f(acc[i][j][8 * p + s] + bv[8 * p + s]);
                    *(bf16x8 *)(o + p * 1024) = o8;
                }
            }
        }
    } else {
        // ->1 layer: this wave's 128 features of each of its 64 candidates, then the other feature half via LDS
        float zp[2] = {0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int rt = wm * 4 + i;
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int ii = 0; ii < 4; ++ii) {
                    const int f = 32 * rt + 8 * q + 4 * h + ii;
                    const float wv = a.wlast[f], bb = bias ? bias[f] : 0.f;
#pragma unroll
                    for (int j = 0; j < 2; ++j) zp[j] += wv * relu_f(acc[i][j][4 * q + ii] + bb);
                }
        }
        float *sz = (float *)lds;                               // [256 candidates] partial of the upper feature half
#pragma unroll
        for (int j = 0; j < 2; ++j) zp[j] += __shfl_xor(zp[j], 32, 64);
        if (wm == 1 && h == 0) {
#pragma unroll
            for (int j = 0; j < 2; ++j) sz[(wn * 2 + j) * 32 + col] = zp[j];
        }
        __syncthreads();
        if (wm == 0 && h == 0) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int local = local0 + (wn * 2 + j) * 32 + col;
                if (local < rd.n_cand) {
                    float z = zp[j] + sz[(wn * 2 + j) * 32 + col] + (a.blast ? a.blast[0] : 0.f);
                    const int64_t id = rd.cand_ids[local];
                    if (id < 0 || id >= m.n_items) z = __uint_as_float(0x7FC00000u);
                    rd.logits_out[local] = z;
                    if (rd.scores_out) rd.scores_out[local] = 1.0f / (1.0f + __expf(-z));
                }
            }
        }
    }
}

// Can the layered path serve the model?  bf16, at least one hidden layer, every contraction a multiple of 64
// (four k-steps per stage), every hidden width a multiple of 256 (one block of features), the last one 256.
bool mlp_layers_ok(const Model &m)
{
    if (m.dtype != 1 || m.n_layers < 2 || m.n_layers - 1 > 3) return false;
    if (m.k1 <= 0 || m.k1 % 64) return false;
    for (int l = 1; l < m.n_layers; ++l)
        if (m.dims[l] % 256) return false;
    return m.dims[m.n_layers - 1] == 256;
}

size_t mlp_layers_buf_bytes(const Model &m, size_t x_rows, int which)
{
    // activations of hidden layer 1, 3, ... go to buffer 0, of layer 2, ... to buffer 1; the last hidden layer's are not stored
    size_t widest = 0;
    for (int l = 1; l + 1 < m.n_layers; ++l)
        if ((l - 1) % 2 == which && (size_t)m.dims[l] > widest) widest = m.dims[l];
    return x_rows * widest * 2;
}

hipError_t launch_mlp_layers(const Model &m, const Batch &b, const void *X, const MlpPack &pk, const float *bias1,
                             char *const *hbuf, hipStream_t s)
{
    if (b.n_blk == 0) return hipSuccess;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_mlp_layer<false>, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * GL_STAGE_BYTES);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_mlp_layer<true>, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * GL_STAGE_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int nh = m.n_layers - 1;
    for (int l = 0; l < nh; ++l) {
        LayerArgs a{};
        const int K = l == 0 ? m.k1 : m.dims[l];
        a.M = m.dims[l + 1];
        a.KS = K / 16;
        a.wfrag = pk.w[l];
        if (l == 0) {
            a.in = (const char *)X;
            a.in_l = x_layout(m);
            a.bias = bias1;
            a.per_req_bias = 1;
        } else {
            a.in = hbuf[(l - 1) % 2];
            a.in_l = XLayout{(uint32_t)K * 32 * 2, 16u, 16u * 32};          // fragment order: [piece][row] inside a 32-row tile
            a.bias = pk.bias[l];
            a.per_req_bias = 0;
        }
        const dim3 grid(b.n_blk, a.M / 256);
        if (l + 1 < nh) {
            a.out = hbuf[l % 2];
            hipLaunchKernelGGL(k_mlp_layer<false>, grid, dim3(512), 2 * GL_STAGE_BYTES, s, m, b, a);
        } else {
            a.wlast = pk.wlast;
            a.blast = pk.blast;
            hipLaunchKernelGGL(k_mlp_layer<true>, grid, dim3(512), 2 * GL_STAGE_BYTES, s, m, b, a);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace aif
