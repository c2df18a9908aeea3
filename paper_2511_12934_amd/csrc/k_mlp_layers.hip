// a6-a7 for WIDE heads on the matrix cores -- the MLP head (Sec. 1: a light MLP
// of few layers) one layer per launch, for models whose hidden layers
// are too wide for a candidate's activations to stay in registers across the
// chain (k_mlp_mfma): e.g. 448 -> 1024 -> 512 -> 256 -> 1.
//
// Each launch is a bf16 GEMM in the transposed form of the fused chain,
// H_out^T = W H_in^T, with a 256-feature x 256-candidate tile per block: four
// waves, one per SIMD, as 2 (features) x 2 (candidates), each holding 4 x 4 MFMA
// tiles of 32 x 32 -- 256 accumulator registers per lane.  A k-step of a wave
// is 8 fragment reads from LDS for 16 MFMAs; with eight thinner waves the same
// block tile costs 6 reads per 8 MFMAs, which asks more of LDS (128 B per
// cycle and compute unit) than the matrix cores leave it time for.  Both
// operands reach LDS as ready-made 1 KB MFMA fragments by direct-to-LDS loads,
// through an eight-slot ring of k-steps (16 KB each), seven in flight:
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

constexpr int GL_STAGE_BYTES = 16 * 1024;   // one k-step: 8 A + 8 B fragments
constexpr int GL_SLOTS = 8, GL_DIST = GL_SLOTS - 1, GL_LPW = 4;      // ring, k-steps in flight, loads per wave and k-step
constexpr int GL_LDS_BYTES = GL_SLOTS * GL_STAGE_BYTES;          // the ring; the block's biases and ->1 weights follow it
constexpr int GL_LDS_TOTAL = GL_LDS_BYTES + 2 * 256 * 4;

template <int N> struct LC { static constexpr int value = N; };

__device__ __forceinline__ float relu_f(float x) { return __builtin_amdgcn_fmed3f(x, 0.f, __builtin_inff()); }

template <bool LAST>
__global__ __launch_bounds__(256) void k_mlp_layer(Model m, Batch b, LayerArgs a)
{
    extern __shared__ __align__(16) char lds[];
    // Workgroups go to the 8 XCDs in turn, each with an L2 of its own.  The feature blocks of one candidate
    // block read the same activations: give them consecutive turns of ONE XCD, so that the activations come
    // from HBM once and from that L2 for the other feature blocks.
    const int NY = a.M >> 8;
    const int xcd = blockIdx.x & 7, turn = blockIdx.x >> 3;
    const int bx = (turn / NY) * 8 + xcd, by = turn % NY;       // candidate block (= scheduling block), feature block
    if (bx >= b.n_blk) return;                                  // every scheduling block of the batch holds candidates

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = lane & 31, h = lane >> 5, wm = wave & 1, wn = wave >> 1;       // feature half, candidate half
    const uint32_t lds0 = lds_address(lds);
    const int KS = a.KS;

    // k-step k -> slot k % GL_SLOTS; a wave moves 4 of the k-step's 16 fragments: waves 0, 1 the weights'
    // (1 KB further per k-step), waves 2, 3 the candidates' (two 16-byte pieces further).  With one wave per
    // SIMD every scalar instruction of the loop is time the matrix cores stand still, so the sources are
    // pointers that advance by a constant and nothing in a k-step branches.
    const char *src[GL_LPW];
#pragma unroll
    for (int i = 0; i < GL_LPW; ++i) {
        const int rr = wave * GL_LPW + i;
        src[i] = rr < 8 ? a.wfrag + (size_t)(by * 8 + rr) * KS * 1024 + lane * 16
                        : a.in + x_offset(a.in_l, (uint32_t)(bx * ROW_BLOCK + (rr - 8) * 32 + col), (uint32_t)h);
    }
    const uint32_t src_step = wave < 2 ? 1024u : 2u * a.in_l.piece_stride;
    const uint32_t dst0 = lds0 + wave * GL_LPW * 1024;
    auto issue = [&](int k) {
        const uint32_t dst = dst0 + (k & (GL_SLOTS - 1)) * GL_STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < GL_LPW; ++i) {
            dma16(src[i], dst + i * 1024);
            src[i] += src_step;
        }
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // The block streams its operands GL_DIST k-steps ahead (a 64 KB tile pair per four k-steps would have
    // to arrive within the 1 us those MFMAs take, and does not), and the one barrier per k-step sits in the
    // MIDDLE of its MFMAs: there k-step k + 1 is confirmed (each wave waits for its own share, then the
    // barrier), k-step k + GL_DIST is sent into the slot of k-step k - 1, which every wave has long read,
    // and the fragments of k-step k + 1 are asked for, so that they arrive under the second half of k-step
    // k's MFMAs.
    bf16x8 af[2][4], bf[2][4];
    const char *fa0 = lds + lane * 16 + wm * 4 * 1024, *fb0 = lds + lane * 16 + (8 + wn * 4) * 1024;
    auto frags = [&](int k, bf16x8 *fa, bf16x8 *fb) {
        const int off = (k & (GL_SLOTS - 1)) * GL_STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < 4; ++i) fa[i] = *(const bf16x8 *)(fa0 + off + i * 1024);
#pragma unroll
        for (int j = 0; j < 4; ++j) fb[j] = *(const bf16x8 *)(fb0 + off + j * 1024);
    };
    // k-step k on fragment registers PAR; BEHIND = k-steps in flight behind k + 1 at its middle (-1: k is the last)
    auto step = [&](int k, auto par_c, auto behind_c, auto issue_c) {
        constexpr int PAR = decltype(par_c)::value, BEHIND = decltype(behind_c)::value;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[PAR][i], bf[PAR][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (BEHIND >= 0) {
            wait_vmcnt<BEHIND * GL_LPW>();
            asm volatile("s_barrier" ::: "memory");
            if constexpr (decltype(issue_c)::value) issue(k + GL_DIST);
            frags(k + 1, af[PAR ^ 1], bf[PAR ^ 1]);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 2; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[PAR][i], bf[PAR][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    };
    static_assert(GL_DIST == 7, "the tail below is written out for seven k-steps in flight");
    for (int k = 0; k < GL_DIST; ++k) issue(k);                 // KS >= GL_DIST + 1 (mlp_layers_ok)
    // A tile is 7-16 us of MFMAs, so what the block needs besides its operands is asked for only now, under
    // the operands' flight, and set down in LDS: the 256 biases of its features (per request in layer 1) and,
    // in the last hidden layer, the ->1 weights.  The request's descriptor is needed by the last layer only.
    float *sbias = (float *)(lds + GL_LDS_BYTES), *swl = sbias + 256;
    const int r = b.blk_req[bx];
    {
        const float *bias = a.bias ? a.bias + (a.per_req_bias ? (size_t)b.blk_slot[bx] * a.M : 0) + by * 256 : nullptr;
        sbias[threadIdx.x] = bias ? bias[threadIdx.x] : 0.f;
        if constexpr (LAST) swl[threadIdx.x] = a.wlast[threadIdx.x];
    }
    ReqDesc rd{};
    if constexpr (LAST) rd = b.reqs[r];
    const int local0 = bx * ROW_BLOCK - rd.row_base;
    wait_vmcnt<(GL_DIST - 1) * GL_LPW>();
    __syncthreads();
    frags(0, af[0], bf[0]);
    int k = 0;
    for (; k + 1 <= KS - 9; k += 2) {                           // KS is even: the fragment registers take turns
        step(k, LC<0>{}, LC<5>{}, LC<1>{});
        step(k + 1, LC<1>{}, LC<5>{}, LC<1>{});
    }
    step(k, LC<0>{}, LC<5>{}, LC<1>{});                         // k = KS - 8: the last k-step goes out
    step(k + 1, LC<1>{}, LC<5>{}, LC<0>{});
    step(k + 2, LC<0>{}, LC<4>{}, LC<0>{});
    step(k + 3, LC<1>{}, LC<3>{}, LC<0>{});
    step(k + 4, LC<0>{}, LC<2>{}, LC<0>{});
    step(k + 5, LC<1>{}, LC<1>{}, LC<0>{});
    step(k + 6, LC<0>{}, LC<0>{}, LC<0>{});
    step(k + 7, LC<1>{}, LC<-1>{}, LC<0>{});

    if constexpr (!LAST) {
        const size_t tile_stride = (size_t)(a.M >> 4) * 1024;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int rt = by * 8 + wm * 4 + i;                 // row tile of the layer
            float bv[16];
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int ii = 0; ii < 4; ++ii) bv[4 * q + ii] = sbias[32 * (wm * 4 + i) + 8 * q + 4 * h + ii];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                char *o = a.out + (size_t)(bx * 8 + wn * 4 + j) * tile_stride + (size_t)(2 * rt) * 1024 + lane * 16;
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
        // ->1 layer: this wave's 128 features of each of its 128 candidates, then the other feature half via LDS
        float zp[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int rt = wm * 4 + i;
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int ii = 0; ii < 4; ++ii) {
                    const int f = 32 * rt + 8 * q + 4 * h + ii;
                    const float wv = swl[f], bb = sbias[f];
#pragma unroll
                    for (int j = 0; j < 4; ++j) zp[j] += wv * relu_f(acc[i][j][4 * q + ii] + bb);
                }
        }
        __syncthreads();                                        // every wave has read its last fragments
        float *sz = (float *)lds;                               // [256 candidates] partial of the upper feature half (in the ring's place)
#pragma unroll
        for (int j = 0; j < 4; ++j) zp[j] += __shfl_xor(zp[j], 32, 64);
        if (wm == 1 && h == 0) {
#pragma unroll
            for (int j = 0; j < 4; ++j) sz[(wn * 4 + j) * 32 + col] = zp[j];
        }
        __syncthreads();
        if (wm == 0 && h == 0) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int local = local0 + (wn * 4 + j) * 32 + col;
                if (local < rd.n_cand) {
                    float z = zp[j] + sz[(wn * 4 + j) * 32 + col] + (a.blast ? a.blast[0] : 0.f);
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
// (and at least 128), every hidden width a multiple of 256 (one block of features), the last one 256.
bool mlp_layers_ok(const Model &m)
{
    if (m.dtype != 1 || m.n_layers < 2 || m.n_layers - 1 > 3) return false;
    if (m.k1 < 16 * (GL_DIST + 1) || m.k1 % 64) return false;      // at least GL_DIST + 1 k-steps per layer
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
        hipError_t e = hipFuncSetAttribute((const void *)k_mlp_layer<false>, hipFuncAttributeMaxDynamicSharedMemorySize, GL_LDS_TOTAL);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void *)k_mlp_layer<true>, hipFuncAttributeMaxDynamicSharedMemorySize, GL_LDS_TOTAL);
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
        const dim3 grid((unsigned)((b.n_blk + 7) / 8 * 8 * (a.M / 256)));      // decoded in the kernel, XCD by XCD
        if (l + 1 < nh) {
            a.out = hbuf[l % 2];
            hipLaunchKernelGGL(k_mlp_layer<false>, grid, dim3(256), GL_LDS_TOTAL, s, m, b, a);
        } else {
            a.wlast = pk.wlast;
            a.blast = pk.blast;
            hipLaunchKernelGGL(k_mlp_layer<true>, grid, dim3(256), GL_LDS_TOTAL, s, m, b, a);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace aif
