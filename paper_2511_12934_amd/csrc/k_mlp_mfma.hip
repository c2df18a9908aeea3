// a6-a7 on the matrix cores -- the MLP head (Sec. 1: "shallow multilayer
// perceptron") as one fused bf16 MFMA chain.
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
// Weights stream through LDS (double buffered, one 32-feature row tile per
// stage) and are shared by the waves of the block; each wave owns CT column
// tiles of 32 candidates.  The user block of layer 1 arrives as the per-request
// bias (user fold), the final ->1 layer is a dot product in the epilogue.
#include "k_mfma.h"

namespace aif {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int cmax(int a, int b) { return a > b ? a : b; }

typedef const void __attribute__((address_space(1))) *gptr_t;
typedef void __attribute__((address_space(3))) *lptr_t;

// Copy one row tile of packed weights (KS fragments of 1 KB) global -> LDS with
// the direct-to-LDS load: a wave moves whole fragments, lane i's 16 bytes land
// at fragment base + 16 i, no register staging.  The wave then has the loads
// in flight; wait_stage() + a block barrier make them visible.
template <int KS, int WAVES>
__device__ __forceinline__ void stage_tile(const char *__restrict__ src, char *dst)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int f0 = 0; f0 < KS; f0 += WAVES) {
        const int f = f0 + wave;
        if (KS % WAVES == 0 || f < KS)
            __builtin_amdgcn_global_load_lds((gptr_t)(src + f * 1024 + lane * 16), (lptr_t)(dst + f * 1024), 16, 0, 0);
    }
}
__device__ __forceinline__ void wait_stage() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ float relu(float x) { return __builtin_amdgcn_fmed3f(x, 0.f, __builtin_inff()); }

// One hidden layer for this wave's CT column tiles.  in: KIN/16 B-fragments per
// column tile.  !FINAL: out receives NOUT/16 fragments (ReLU, bf16).  FINAL:
// zpart[c] += wlast . relu(h) over the features this lane holds.  sbias / swl:
// this layer's bias and the final layer's weights, fp32 in LDS.
template <int CT, int KIN, int NOUT, bool FINAL, int WAVES, int NEXT_KS, int BUFBYTES>
__device__ __forceinline__ void mlp_layer(const bf16x8 (&in)[CT][KIN / 16], bf16x8 (&out)[CT][NOUT / 16],
                                          float (&zpart)[CT], const char *__restrict__ wsrc,
                                          const char *__restrict__ next_src, const float *sbias, const float *swl,
                                          char *lds, int &buf)
{
    constexpr int KS = KIN / 16, RT = NOUT / 32, BYTES = KIN * 64;
    const int lane = threadIdx.x & 63, h = lane >> 5;
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        __builtin_amdgcn_sched_barrier(0);
        if (r + 1 < RT)
            stage_tile<KS, WAVES>(wsrc + (size_t)(r + 1) * BYTES, lds + (buf ^ 1) * BUFBYTES);
        else if (NEXT_KS > 0)
            stage_tile<(NEXT_KS > 0 ? NEXT_KS : 1), WAVES>(next_src, lds + (buf ^ 1) * BUFBYTES);

        f32x16 acc[CT];
#pragma unroll
        for (int c = 0; c < CT; ++c)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;

        // A fragments come from LDS in groups of G, the next group in flight
        // while the current one feeds the matrix cores; the scheduling
        // barriers keep the compiler from hoisting every load of the tile
        // (which would not fit the register file next to the activations).
        const char *w = lds + buf * BUFBYTES + lane * 16;
        constexpr int G = 4, NG = KS / G;
        static_assert(KS % G == 0, "k-steps per tile");
        bf16x8 a[2][G];
#pragma unroll
        for (int t = 0; t < G; ++t) a[0][t] = *(const bf16x8 *)(w + t * 1024);
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            if (g + 1 < NG) {
#pragma unroll
                for (int t = 0; t < G; ++t) a[(g + 1) & 1][t] = *(const bf16x8 *)(w + ((g + 1) * G + t) * 1024);
            }
#pragma unroll
            for (int t = 0; t < G; ++t) {
#pragma unroll
                for (int c = 0; c < CT; ++c)
                    acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[g & 1][t], in[c][g * G + t], acc[c], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        float4 bv[4], wl[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            bv[q] = *(const float4 *)(sbias + 32 * r + 8 * q + 4 * h);
            if (FINAL) wl[q] = *(const float4 *)(swl + 32 * r + 8 * q + 4 * h);
        }
        if (FINAL) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
#pragma unroll
                for (int c = 0; c < CT; ++c) {
                    zpart[c] += wl[q].x * relu(acc[c][4 * q + 0] + bv[q].x) + wl[q].y * relu(acc[c][4 * q + 1] + bv[q].y) +
                                wl[q].z * relu(acc[c][4 * q + 2] + bv[q].z) + wl[q].w * relu(acc[c][4 * q + 3] + bv[q].w);
                }
            }
            // pin the partial sums here: left alone the compiler postpones the whole
            // dot product to the end of the kernel and spills every tile's outputs
#pragma unroll
            for (int c = 0; c < CT; ++c) asm volatile("" : "+v"(zpart[c]));
        } else {
#pragma unroll
            for (int c = 0; c < CT; ++c) {
                bf16x8 lo, hi;
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    lo[4 * q + 0] = (__bf16)relu(acc[c][4 * q + 0] + bv[q].x);
                    lo[4 * q + 1] = (__bf16)relu(acc[c][4 * q + 1] + bv[q].y);
                    lo[4 * q + 2] = (__bf16)relu(acc[c][4 * q + 2] + bv[q].z);
                    lo[4 * q + 3] = (__bf16)relu(acc[c][4 * q + 3] + bv[q].w);
                    hi[4 * q + 0] = (__bf16)relu(acc[c][8 + 4 * q + 0] + bv[2 + q].x);
                    hi[4 * q + 1] = (__bf16)relu(acc[c][8 + 4 * q + 1] + bv[2 + q].y);
                    hi[4 * q + 2] = (__bf16)relu(acc[c][8 + 4 * q + 2] + bv[2 + q].z);
                    hi[4 * q + 3] = (__bf16)relu(acc[c][8 + 4 * q + 3] + bv[2 + q].w);
                }
                asm volatile("" : "+v"(lo), "+v"(hi));       // convert now, keep 8 registers not 16
                out[c][2 * r] = lo;
                out[c][2 * r + 1] = hi;
            }
        }
        wait_stage();
        __syncthreads();
        __builtin_amdgcn_sched_barrier(0);      // nothing of the next row tile moves above this point
        buf ^= 1;
    }
}

// K1: layer-1 contraction after the user fold; H1..H3: hidden widths (0 = absent).
template <int K1, int H1, int H2, int H3, int CT, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void k_mlp_mfma(Model m, Batch b, const uint16_t *__restrict__ X,
                                                        MlpPack pk, const float *__restrict__ bias1)
{
    constexpr int THREADS = WAVES * 64, ROWS = WAVES * 32 * CT;
    constexpr int NH = H3 ? 3 : (H2 ? 2 : 1);
    constexpr int HL = NH == 1 ? H1 : (NH == 2 ? H2 : H3);          // width entering the final ->1 layer
    constexpr int KMAX = cmax(K1, cmax(NH >= 2 ? H1 : 0, NH >= 3 ? H2 : 0));
    constexpr int BUFBYTES = KMAX * 64;
    static_assert(ROW_BLOCK % ROWS == 0, "tile");
    extern __shared__ __align__(16) char lds[];
    float *sb1 = (float *)(lds + 2 * BUFBYTES), *sb2 = sb1 + H1, *sb3 = sb2 + H2, *swl = sb3 + H3;

    const int tile = blockIdx.x;
    const int r = b.blk_req[tile / (ROW_BLOCK / ROWS)];
    if (r < 0) return;
    const ReqDesc rd = b.reqs[r];
    const int row0 = tile * ROWS;
    const int local0 = row0 - rd.row_base;
    if (rd.n_cand - local0 <= 0) return;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, col = lane & 31, h = lane >> 5;
    stage_tile<K1 / 16, WAVES>(pk.w[0], lds);

    bf16x8 xin[CT][K1 / 16];
#pragma unroll
    for (int c = 0; c < CT; ++c) {
        const bf16x8 *xr = (const bf16x8 *)(X + (size_t)(row0 + (wave * CT + c) * 32 + col) * m.ldx);
#pragma unroll
        for (int j = 0; j < K1 / 16; ++j) xin[c][j] = xr[2 * j + h];
    }
    for (int i = threadIdx.x; i < H1; i += THREADS) sb1[i] = bias1[(size_t)r * H1 + i];
    if (NH >= 2)
        for (int i = threadIdx.x; i < H2; i += THREADS) sb2[i] = pk.bias[1][i];
    if (NH >= 3)
        for (int i = threadIdx.x; i < H3; i += THREADS) sb3[i] = pk.bias[2][i];
    for (int i = threadIdx.x; i < HL; i += THREADS) swl[i] = pk.wlast[i];
    wait_stage();
    __syncthreads();

    int buf = 0;
    float zpart[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c) zpart[c] = 0.f;

    if constexpr (NH == 1) {
        bf16x8 dummy[CT][H1 / 16];
        mlp_layer<CT, K1, H1, true, WAVES, 0, BUFBYTES>(xin, dummy, zpart, pk.w[0], nullptr, sb1, swl, lds, buf);
    } else if constexpr (NH == 2) {
        bf16x8 h1[CT][H1 / 16];
        mlp_layer<CT, K1, H1, false, WAVES, H1 / 16, BUFBYTES>(xin, h1, zpart, pk.w[0], pk.w[1], sb1, swl, lds, buf);
        bf16x8 dummy[CT][H2 / 16];
        mlp_layer<CT, H1, H2, true, WAVES, 0, BUFBYTES>(h1, dummy, zpart, pk.w[1], nullptr, sb2, swl, lds, buf);
    } else {
        bf16x8 h1[CT][H1 / 16];
        mlp_layer<CT, K1, H1, false, WAVES, H1 / 16, BUFBYTES>(xin, h1, zpart, pk.w[0], pk.w[1], sb1, swl, lds, buf);
        bf16x8 h2[CT][H2 / 16];
        mlp_layer<CT, H1, H2, false, WAVES, H2 / 16, BUFBYTES>(h1, h2, zpart, pk.w[1], pk.w[2], sb2, swl, lds, buf);
        bf16x8 dummy[CT][H3 / 16];
        mlp_layer<CT, H2, H3, true, WAVES, 0, BUFBYTES>(h2, dummy, zpart, pk.w[2], nullptr, sb3, swl, lds, buf);
    }

    const float bl = pk.blast ? pk.blast[0] : 0.f;
#pragma unroll
    for (int c = 0; c < CT; ++c) {
        float z = zpart[c] + __shfl_xor(zpart[c], 32, 64) + bl;
        const int local = local0 + (wave * CT + c) * 32 + col;
        if (h == 0 && local < rd.n_cand) {
            const int64_t id = rd.cand_ids[local];
            if (id < 0 || id >= m.n_items) z = __uint_as_float(0x7FC00000u);
            rd.logits_out[local] = z;
            if (rd.scores_out) rd.scores_out[local] = 1.0f / (1.0f + __expf(-z));
        }
    }
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
template <int K1, int H1, int H2, int H3, int CT, int WAVES>
static hipError_t launch_spec(const Model &m, const Batch &b, const void *X, const MlpPack &pk, const float *bias1,
                              hipStream_t s)
{
    constexpr int NH = H3 ? 3 : (H2 ? 2 : 1);
    constexpr int KMAX = cmax(K1, cmax(NH >= 2 ? H1 : 0, NH >= 3 ? H2 : 0));
    constexpr int LDS = 2 * KMAX * 64 + 4 * (H1 + H2 + H3 + (NH == 1 ? H1 : (NH == 2 ? H2 : H3)));
    constexpr int ROWS = WAVES * 32 * CT;
    auto kern = k_mlp_mfma<K1, H1, H2, H3, CT, WAVES>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(b.n_blk * (ROW_BLOCK / ROWS)), dim3(WAVES * 64), LDS, s, m, b, (const uint16_t *)X, pk,
                       bias1);
    return hipGetLastError();
}

int mlp_mfma_variant(const Model &m)
{
    if (m.dtype != 1) return -1;
    const int nh = m.n_layers - 1;
    const int k1 = m.k1, h1 = nh >= 1 ? m.dims[1] : 0, h2 = nh >= 2 ? m.dims[2] : 0, h3 = nh >= 3 ? m.dims[3] : 0;
    if (nh == 2 && k1 == 192 && h1 == 256 && h2 == 128) return 0;
    if (nh == 2 && k1 == 192 && h1 == 512 && h2 == 256) return 1;
    if (nh == 1 && k1 == 384 && h1 == 256) return 2;
    return -1;
}

hipError_t launch_mlp_variant(int variant, const Model &m, const Batch &b, const void *X, const MlpPack &pk,
                              const float *bias1, hipStream_t s)
{
    if (b.n_blk == 0) return hipSuccess;
    switch (variant) {
    case 0: return launch_spec<192, 256, 128, 0, 1, 8>(m, b, X, pk, bias1, s);
    case 1: return launch_spec<192, 512, 256, 0, 1, 8>(m, b, X, pk, bias1, s);
    case 2: return launch_spec<384, 256, 0, 0, 1, 8>(m, b, X, pk, bias1, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace aif
