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
#include "mfma_util.h"

namespace aif {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int cmax(int a, int b) { return a > b ? a : b; }


template <int N> struct IC { static constexpr int value = N; };
template <int I, int N, class F> __device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(IC<I>{});
        static_for<I + 1, N>(f);
    }
}


__device__ __forceinline__ float relu(float x) { return __builtin_amdgcn_fmed3f(x, 0.f, __builtin_inff()); }

// Static description of the chain: hidden layer l contracts KIN(l) inputs into
// NOUT(l) features; its weights are streamed in stages of U(l) row tiles
// (32 features each) chosen so that every wave moves the same number of 1 KB
// fragments per stage.
template <int K1, int H1, int H2, int H3, int WAVES> struct Chain {
    static constexpr int NH = H3 ? 3 : (H2 ? 2 : 1);
    static constexpr int kin(int l) { return l == 0 ? K1 : (l == 1 ? H1 : H2); }
    static constexpr int nout(int l) { return l == 0 ? H1 : (l == 1 ? H2 : H3); }
    static constexpr int ks(int l) { return kin(l) / 16; }                     // fragments per row tile
    static constexpr int unit(int l) { return ks(l) % WAVES == 0 ? 1 : ((2 * ks(l)) % WAVES == 0 ? 2 : 4); }
    static constexpr int nstage(int l) { return nout(l) / 32 / unit(l); }
    static constexpr int frags(int l) { return unit(l) * ks(l); }              // fragments per stage
    static constexpr int total() { return nstage(0) + (NH > 1 ? nstage(1) : 0) + (NH > 2 ? nstage(2) : 0); }
    static constexpr int layer_of(int i) { return i < nstage(0) ? 0 : (i < nstage(0) + nstage(1) ? 1 : 2); }
    static constexpr int first(int l) { return l == 0 ? 0 : (l == 1 ? nstage(0) : nstage(0) + nstage(1)); }
    static constexpr int loads(int i) { return i < total() ? frags(layer_of(i)) / WAVES : 0; }   // per wave
    static constexpr int slot_frags() { return cmax(frags(0), cmax(NH > 1 ? frags(1) : 0, NH > 2 ? frags(2) : 0)); }
    static constexpr int HL = NH == 1 ? H1 : (NH == 2 ? H2 : H3);              // width entering the ->1 layer
    static constexpr int bias_floats = H1 + H2 + H3 + HL;
    static constexpr int slots() { return (4 * slot_frags() * 1024 + 4 * bias_floats <= 160 * 1024) ? 4 : 3; }
    static constexpr int lds_bytes() { return slots() * slot_frags() * 1024 + 4 * bias_floats; }
    static_assert(nout(0) % (32 * unit(0)) == 0, "layer 1 width");
    static_assert(NH < 2 || nout(1) % (32 * unit(1)) == 0, "layer 2 width");
    static_assert(NH < 3 || nout(2) % (32 * unit(2)) == 0, "layer 3 width");
};

// Copy stage i of the weight stream global -> LDS slot: a wave moves whole 1 KB
// fragments, no register staging.
template <class C, int WAVES, int I>
__device__ __forceinline__ void issue_stage(const MlpPack &pk, char *lds)
{
    if constexpr (I < C::total()) {
        constexpr int l = C::layer_of(I), nf = C::frags(l);
        const int lane = threadIdx.x & 63;
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const char *src = pk.w[l] + (size_t)(I - C::first(l)) * nf * 1024 + lane * 16;
        const uint32_t dst = (uint32_t)(uintptr_t)(lptr_t)lds + (I % C::slots()) * C::slot_frags() * 1024;
#pragma unroll
        for (int f0 = 0; f0 < nf; f0 += WAVES) dma16(src + (f0 + wave) * 1024, dst + (f0 + wave) * 1024);
    }
}

// Epilogue of one 32-feature row tile, cut into four parts (q = 0..3: the four
// features 8q + 4h + i a lane holds): bias + ReLU, then either two bf16
// B-fragments of the next layer (lo <- q = 0, 1; hi <- q = 2, 3) or, for the
// last hidden layer, the partial dot with the ->1 layer's weights.
template <int CT, bool FINAL, int Q>
__device__ __forceinline__ void epilogue_part(const f32x16 (&acc)[CT], bf16x8 (&lo)[CT], bf16x8 (&hi)[CT],
                                              float (&zpart)[CT], const float *sbias, const float *swl, int h)
{
    const float4 bv = *(const float4 *)(sbias + 8 * Q + 4 * h);
    if constexpr (FINAL) {
        const float4 wl = *(const float4 *)(swl + 8 * Q + 4 * h);
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            zpart[c] += wl.x * relu(acc[c][4 * Q + 0] + bv.x) + wl.y * relu(acc[c][4 * Q + 1] + bv.y) +
                        wl.z * relu(acc[c][4 * Q + 2] + bv.z) + wl.w * relu(acc[c][4 * Q + 3] + bv.w);
            asm volatile("" : "+v"(zpart[c]));      // keep the partial dot here (see the convert below)
        }
    } else {
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            bf16x8 &dst = Q < 2 ? lo[c] : hi[c];
            constexpr int o = 4 * (Q & 1);
            dst[o + 0] = (__bf16)relu(acc[c][4 * Q + 0] + bv.x);
            dst[o + 1] = (__bf16)relu(acc[c][4 * Q + 1] + bv.y);
            dst[o + 2] = (__bf16)relu(acc[c][4 * Q + 2] + bv.z);
            dst[o + 3] = (__bf16)relu(acc[c][4 * Q + 3] + bv.w);
            // convert now: left alone the compiler keeps the fp32 values (twice the registers) until first use
            if constexpr ((Q & 1) == 1) asm volatile("" : "+v"(dst));
        }
    }
}

// MFMA loop of one row tile, acc = W_tile . in, with the four epilogue parts of
// the PREVIOUS row tile slipped in between the groups of MFMAs: the vector ALU
// work then runs while the matrix cores are busy instead of after them.
// A fragments come from LDS in groups of G, the next group in flight while the
// current one feeds the matrix cores; the scheduling barriers keep the compiler
// from hoisting every load of the tile (which would not fit the register file
// next to the activations).
template <int CT, int KS, class Epi>
__device__ __forceinline__ void tile_mfma(const char *w, const bf16x8 (&in)[CT][KS], f32x16 (&acc)[CT], Epi &&epi)
{
#pragma unroll
    for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
    constexpr int G = 4, NG = KS / G;
    static_assert(KS % G == 0 && NG >= 2, "k-steps per tile");
    bf16x8 a[2][G];
#pragma unroll
    for (int t = 0; t < G; ++t) a[0][t] = *(const bf16x8 *)(w + t * 1024);
    __builtin_amdgcn_sched_barrier(0);
    static_for<0, NG>([&](auto gi) {
        constexpr int g = decltype(gi)::value;
        if constexpr (g + 1 < NG) {
#pragma unroll
            for (int t = 0; t < G; ++t) a[(g + 1) & 1][t] = *(const bf16x8 *)(w + ((g + 1) * G + t) * 1024);
        }
#pragma unroll
        for (int t = 0; t < G; ++t) {
#pragma unroll
            for (int c = 0; c < CT; ++c)
                acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[g & 1][t], in[c][g * G + t], acc[c], 0, 0, 0);
        }
        // epilogue parts of the previous tile that belong to this group
        static_for<0, 4>([&](auto qi) {
            constexpr int q = decltype(qi)::value;
            // never in the last group: the first tile of a layer consumes, in its last
            // k-steps, the fragments the previous layer's last tile completes here
            constexpr int at = (q * NG) / 4 < NG - 2 ? (q * NG) / 4 : NG - 2;
            if constexpr (at == g) epi(qi);
        });
        __builtin_amdgcn_sched_barrier(0);
    });
}

// K1: layer-1 contraction after the user fold; H1..H3: hidden widths (0 = absent).
template <int K1, int H1, int H2, int H3, int CT, int WAVES>
__global__ __launch_bounds__(WAVES * 64, 2) void k_mlp_mfma(Model m, Batch b, const char *__restrict__ X, XLayout xl,
                                                           MlpPack pk, const float *__restrict__ bias1)
{
    using C = Chain<K1, H1, H2, H3, WAVES>;
    constexpr int THREADS = WAVES * 64, ROWS = WAVES * 32 * CT, NS = C::total(), D = C::slots() - 1;
    static_assert(ROW_BLOCK % ROWS == 0, "tile");
    extern __shared__ __align__(16) char lds[];                 // the weight ring, then biases and last-layer weights
    float *sb1 = (float *)(lds + C::slots() * C::slot_frags() * 1024), *sb2 = sb1 + H1, *sb3 = sb2 + H2, *swl = sb3 + H3;

    const int tile = blockIdx.x;
    const int row0 = tile * ROWS;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, col = lane & 31, h = lane >> 5;
    // The block's start is a chain of dependent memory round trips; keep it short: the weight stream
    // and the input rows do not depend on the request lookup (a padded row is still inside the
    // workspace), so they are asked for first.
    static_for<0, D>([&](auto s) { issue_stage<C, WAVES, decltype(s)::value>(pk, lds); });
    bf16x8 xin[CT][K1 / 16];
#pragma unroll
    for (int c = 0; c < CT; ++c) {
        const char *xr = X + x_offset(xl, row0 + (wave * CT + c) * 32 + col, h);
#pragma unroll
        for (int j = 0; j < K1 / 16; ++j) xin[c][j] = *(const bf16x8 *)(xr + (size_t)(2 * j) * xl.piece_stride);
    }
    const int r = b.blk_req[tile / (ROW_BLOCK / ROWS)];
    const ReqDesc rd = b.reqs[r < 0 ? 0 : r];
    const int local0 = row0 - rd.row_base;
    if (r < 0 || rd.n_cand - local0 <= 0) {         // never taken when a tile is a whole scheduling block
        wait_vmcnt<0>();                            // no load may still be heading for this block's LDS
        return;
    }
    for (int i = threadIdx.x; i < H1; i += THREADS) sb1[i] = bias1[(size_t)r * H1 + i];
    if (C::NH >= 2)
        for (int i = threadIdx.x; i < H2; i += THREADS) sb2[i] = pk.bias[1][i];
    if (C::NH >= 3)
        for (int i = threadIdx.x; i < H3; i += THREADS) sb3[i] = pk.bias[2][i];
    for (int i = threadIdx.x; i < C::HL; i += THREADS) swl[i] = pk.wlast[i];
    wait_vmcnt<0>();
    __syncthreads();

    float zpart[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c) zpart[c] = 0.f;
    bf16x8 h1[CT][C::NH >= 2 ? H1 / 16 : 1];
    bf16x8 h2[CT][C::NH >= 3 ? H2 / 16 : 1];
    f32x16 accA[CT], accB[CT];              // current / previous row tile (ping-pong)
    bf16x8 lo[CT], hi[CT];

    // epilogue part Q of row tile RT of layer L, acting on `acc`; when the tile's
    // last part is done its two fragments are filed as k-steps 2 RT, 2 RT + 1 of the next layer
    auto epi_part = [&](auto lc, auto rtc, auto qc, const f32x16(&acc)[CT]) {
        constexpr int L = decltype(lc)::value, RT = decltype(rtc)::value, Q = decltype(qc)::value;
        constexpr bool FIN = L == C::NH - 1;
        const float *sb = L == 0 ? sb1 : (L == 1 ? sb2 : sb3);
        epilogue_part<CT, FIN, Q>(acc, lo, hi, zpart, sb + 32 * RT, swl + 32 * RT, h);
        if constexpr (!FIN && Q == 3) {
#pragma unroll
            for (int c = 0; c < CT; ++c) {
                if constexpr (L == 0) {
                    h1[c][2 * RT] = lo[c];
                    h1[c][2 * RT + 1] = hi[c];
                } else {
                    h2[c][2 * RT] = lo[c];
                    h2[c][2 * RT + 1] = hi[c];
                }
            }
        }
    };

    // row tiles are numbered through all hidden layers: T -> (layer, row tile in layer)
    constexpr int RT0 = H1 / 32, RT1 = C::NH > 1 ? H2 / 32 : 0, RT2 = C::NH > 2 ? H3 / 32 : 0, NT = RT0 + RT1 + RT2;
    auto run_tile = [&](auto tc, const char *w) {
        constexpr int T = decltype(tc)::value;
        constexpr int L = T < RT0 ? 0 : (T < RT0 + RT1 ? 1 : 2);
        constexpr int RT = T - (L == 0 ? 0 : (L == 1 ? RT0 : RT0 + RT1));
        constexpr int PT = T - 1;                                       // previous tile (epilogue pending)
        constexpr int PL = PT < RT0 ? 0 : (PT < RT0 + RT1 ? 1 : 2);
        constexpr int PRT = PT - (PL == 0 ? 0 : (PL == 1 ? RT0 : RT0 + RT1));
        auto &cur = (T & 1) ? accB : accA;
        auto &prev = (T & 1) ? accA : accB;
        auto epi = [&](auto qc) {
            if constexpr (T > 0) epi_part(IC<PL>{}, IC<PRT>{}, qc, prev);
        };
        if constexpr (L == 0)
            tile_mfma<CT, K1 / 16>(w, xin, cur, epi);
        else if constexpr (L == 1)
            tile_mfma<CT, H1 / 16>(w, h1, cur, epi);
        else
            tile_mfma<CT, H2 / 16>(w, h2, cur, epi);
    };

    static_for<0, NS>([&](auto si) {
        constexpr int I = decltype(si)::value;
        constexpr int l = C::layer_of(I), U = C::unit(l), KS = C::ks(l);
        __builtin_amdgcn_sched_barrier(0);
        issue_stage<C, WAVES, I + D>(pk, lds);       // its slot was read last in stage I - 1
        const char *w0 = lds + (I % C::slots()) * C::slot_frags() * 1024 + lane * 16;
        static_for<0, U>([&](auto uc) {
            constexpr int u = decltype(uc)::value;
            constexpr int T = (l == 0 ? 0 : (l == 1 ? RT0 : RT0 + RT1)) + (I - C::first(l)) * U + u;
            run_tile(IC<T>{}, w0 + u * KS * 1024);
        });
        if constexpr (I + 1 < NS) {
            // stage I + 1 must have landed; stages I + 2 .. I + D may still be in flight
            constexpr int pend = [] { int n = 0; for (int s = I + 2; s <= I + D; ++s) n += C::loads(s); return n; }();
            wait_vmcnt<pend>();
            __syncthreads();
        }
        __builtin_amdgcn_sched_barrier(0);
    });
    {   // the last tile's epilogue has nothing left to hide behind
        constexpr int PL = C::NH - 1, PRT = (PL == 0 ? RT0 : (PL == 1 ? RT1 : RT2)) - 1;
        auto &prev = ((NT - 1) & 1) ? accB : accA;
        static_for<0, 4>([&](auto qc) { epi_part(IC<PL>{}, IC<PRT>{}, qc, prev); });
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
    using C = Chain<K1, H1, H2, H3, WAVES>;
    constexpr int LDS = C::lds_bytes();
    constexpr int ROWS = WAVES * 32 * CT;
    auto kern = k_mlp_mfma<K1, H1, H2, H3, CT, WAVES>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(b.n_blk * (ROW_BLOCK / ROWS)), dim3(WAVES * 64), LDS, s, m, b, (const char *)X, x_layout(m),
                       pk, bias1);
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
