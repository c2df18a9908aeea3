// Shape-agnostic fp32-arithmetic kernels: the whole path for fp32 models and
// for any model whose sizes the MFMA kernels do not cover.  Plain, one
// candidate per wave (attention) or sixteen per block (MLP); accumulation in
// fp32 in a fixed order per candidate, so results do not depend on how a
// candidate list is sliced into requests.
#include "k_stage.h"

namespace aif {

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// ---------------------------------------------------------------------------
// a2 -- user fold.  [u|e|a|c] W1^T = u W1u^T + [e|a|c] W1rest^T: the first
// term is the same for every candidate of a request (the paper's own point:
// interaction-independent work is done once, Sec. 2), so it becomes a
// per-request bias.  One thread per output feature.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_user_fold(Model m, Batch b, const float *__restrict__ w1u,
                                                   const float *__restrict__ b1, float *__restrict__ bias1)
{
    user_fold_block<T>(blockIdx.y, blockIdx.x, m, TableReqs{b}, w1u, b1, bias1);
}

hipError_t launch_user_fold(const Model &m, const Batch &b, const float *w1u, const float *b1, float *bias1,
                            hipStream_t s)
{
    if (b.n_req == 0) return hipSuccess;
    dim3 grid((m.dims[1] + FOLD_FEATS - 1) / FOLD_FEATS, b.n_slots);      // once per distinct user of the call
    if (m.dtype == 0)
        hipLaunchKernelGGL(k_user_fold<float>, grid, dim3(256), 0, s, m, b, w1u, b1, bias1);
    else
        hipLaunchKernelGGL(k_user_fold<uint16_t>, grid, dim3(256), 0, s, m, b, w1u, b1, bias1);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// a3-a5 -- query, target attention (Eq. 3 form, query := candidate) and the
// real-time half of the cross features (Sec. 3.3).  One wave per candidate,
// ATTN_TS candidates per block, all waves step through the phases together.
// Per wave LDS: e[d_item], q[d_attn], score[max_seq_len].
// ---------------------------------------------------------------------------
constexpr int ATTN_TS = 16;

// sum_k a(k) * b(k) for k in [0, n), in order, with the loads of sixteen terms (then eight) issued before the first
// is used: a loop of load-then-multiply is waited for once per term -- a memory round trip each.
template <int U, class FA, class FB> __device__ __forceinline__ void dot_batches(int n, int &k, float &acc, FA a, FB b)
{
    for (; k + U <= n; k += U) {
        float av[U], bv[U];
#pragma unroll
        for (int j = 0; j < U; ++j) {
            av[j] = a(k + j);
            bv[j] = b(k + j);
        }
#pragma unroll
        for (int j = 0; j < U; ++j) acc += av[j] * bv[j];
    }
}
template <class FA, class FB> __device__ __forceinline__ float dot_in_order(int n, float acc, FA a, FB b)
{
    int k = 0;
    dot_batches<16>(n, k, acc, a, b);
    dot_batches<8>(n, k, acc, a, b);
    for (; k < n; ++k) acc += a(k) * b(k);
    return acc;
}

template <typename T>
__global__ __launch_bounds__(256) void k_attn_generic(Model m, Batch b, T *__restrict__ X,
                                                      const float *__restrict__ wq, int per_wave)
{
    extern __shared__ __align__(16) float smem[];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int tile = blockIdx.x;
    const int r = b.blk_req[tile / (ROW_BLOCK / ATTN_TS)];
    if (r < 0) return;
    const ReqDesc rd = b.reqs[r];
    const int row0 = tile * ATTN_TS;
    const int local0 = row0 - rd.row_base;
    int nrows = rd.n_cand - local0;
    if (nrows <= 0) return;
    if (nrows > ATTN_TS) nrows = ATTN_TS;

    float *sh_e = smem + (size_t)wave * per_wave;
    float *sh_q = sh_e + m.d_item;
    float *sh_s = sh_q + m.d_attn;
    const T *K = (const T *)rd.seq_keys;
    const T *V = (const T *)rd.seq_vals;
    const T *uc = (const T *)rd.cross_vecs;
    const int L = rd.seq_len, dh = m.d_head, da = m.d_attn;
    const float scale = 1.0f / sqrtf((float)dh);

    for (int it = 0; it < ATTN_TS / 4; ++it) {
        const int c = it * 4 + wave;
        const bool on = c < nrows;
        T *xrow = X + (size_t)(row0 + c) * m.ldx;
        if (on)
            for (int k = lane; k < m.d_item; k += 64) sh_e[k] = ld_f<T>(xrow + k);
        __syncthreads();
        if (on)
            for (int q = lane; q < da; q += 64) {
                float acc;
                if (wq) {
                    const float *wr = wq + (size_t)q * m.d_item;
                    acc = dot_in_order(m.d_item, 0.f, [&](int k) { return wr[k]; }, [&](int k) { return sh_e[k]; });
                } else
                    acc = sh_e[q];
                sh_q[q] = acc;
            }
        __syncthreads();
        for (int h = 0; h < m.n_heads; ++h) {
            const int o = h * dh;
            float mx = -INFINITY;
            if (on)
                for (int t = lane; t < L; t += 64) {
                    const T *kr = K + (size_t)t * da + o;
                    float acc = dot_in_order(dh, 0.f, [&](int k) { return sh_q[o + k]; }, [&](int k) { return ld_f<T>(kr + k); });
                    acc *= scale;
                    sh_s[t] = acc;
                    mx = fmaxf(mx, acc);
                }
            mx = wave_max(mx);
            float sum = 0.f;
            if (on)
                for (int t = lane; t < L; t += 64) {
                    const float p = expf(sh_s[t] - mx);
                    sh_s[t] = p;
                    sum += p;
                }
            sum = wave_sum(sum);
            __syncthreads();
            if (on)
                for (int k = lane; k < dh; k += 64) {
                    const float acc = dot_in_order(L, 0.f, [&](int t) { return sh_s[t]; },
                                                   [&](int t) { return ld_f<T>(V + (size_t)t * da + o + k); });
                    st_f<T>(xrow + m.d_item + o + k, L > 0 ? acc / sum : 0.f);
                }
            __syncthreads();
        }
        if (on) {
            T *xc = xrow + m.d_item + da;
            if (m.cross_in_mlp) {
                // the MLP chain forms the Hadamard products itself, or the block is folded into the user's layer-1 weights
            } else if (m.cross_mode == 1) {
                for (int k = lane; k < m.d_item; k += 64) st_f<T>(xc + k, ld_f<T>(uc + k) * sh_e[k]);
            } else if (m.cross_mode == 2) {
                const int S = m.d_item / m.d_cv;
                for (int idx = lane; idx < m.d_cross; idx += 64) {
                    const int j = idx / S, sg = idx - j * S;
                    const float acc = dot_in_order(m.d_cv, 0.f, [&](int k) { return ld_f<T>(uc + (size_t)j * m.d_cv + k); },
                                                   [&](int k) { return sh_e[sg * m.d_cv + k]; });
                    st_f<T>(xc + idx, acc);
                }
            } else if (m.cross_mode == 3) {
                // Algorithm 1 step 4: the row's trailing n_cross entries weigh the user-side vectors
                const int w0 = m.d_item - m.n_cross;
                for (int idx = lane; idx < m.d_cv; idx += 64) {
                    const float acc = dot_in_order(m.n_cross, 0.f, [&](int j) { return sh_e[w0 + j]; },
                                                   [&](int j) { return ld_f<T>(uc + (size_t)j * m.d_cv + idx); });
                    st_f<T>(xc + idx, acc);
                }
            }
        }
        __syncthreads();
    }
}

size_t attn_generic_lds_bytes(const Model &m, int max_seq_len)
{
    return (size_t)4 * (m.d_item + m.d_attn + max_seq_len) * sizeof(float);
}

hipError_t launch_attn_generic(const Model &m, const Batch &b, void *X, const float *wq, int max_seq_len,
                               hipStream_t s)
{
    if (b.n_blk == 0) return hipSuccess;
    const int per_wave = m.d_item + m.d_attn + max_seq_len;
    const size_t lds = attn_generic_lds_bytes(m, max_seq_len);
    dim3 grid(b.n_blk * (ROW_BLOCK / ATTN_TS));
    if (m.dtype == 0) {
        (void)hipFuncSetAttribute((const void *)k_attn_generic<float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        hipLaunchKernelGGL(k_attn_generic<float>, grid, dim3(256), lds, s, m, b, (float *)X, wq, per_wave);
    } else {
        (void)hipFuncSetAttribute((const void *)k_attn_generic<uint16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        hipLaunchKernelGGL(k_attn_generic<uint16_t>, grid, dim3(256), lds, s, m, b, (uint16_t *)X, wq, per_wave);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// a6-a7 -- MLP head (Sec. 1: a small MLP) over the
// virtual input [u | e | a | c]: the u block arrives as bias1 (user fold), the
// rest is the workspace row.  MLP_TS candidates per block; activations live
// in two LDS buffers laid out [feature][candidate]; thread n owns output
// feature n for all MLP_TS candidates and walks the transposed weights.
// ---------------------------------------------------------------------------
constexpr int MLP_TS = 16;

template <typename T>
__global__ __launch_bounds__(256) void k_mlp_generic(Model m, Batch b, const T *__restrict__ X,
                                                     MlpGenericWeights w, const float *__restrict__ bias1,
                                                     int buf_floats)
{
    extern __shared__ __align__(16) float smem[];
    float *bufA = smem, *bufB = smem + buf_floats;
    const int tile = blockIdx.x;
    const int r = b.blk_req[tile / (ROW_BLOCK / MLP_TS)];
    if (r < 0) return;
    const ReqDesc rd = b.reqs[r];
    const int us = rd.slot;                 // the folded layer-1 bias is kept per user slot
    const int row0 = tile * MLP_TS;
    const int local0 = row0 - rd.row_base;
    int nrows = rd.n_cand - local0;
    if (nrows <= 0) return;
    if (nrows > MLP_TS) nrows = MLP_TS;

    const int k1 = m.k1;
    for (int idx = threadIdx.x; idx < k1 * MLP_TS; idx += 256) {
        const int c = idx / k1, k = idx - c * k1;
        bufA[k * MLP_TS + c] = c < nrows ? ld_f<T>(X + (size_t)(row0 + c) * m.ldx + k) : 0.f;
    }
    __syncthreads();

    for (int l = 0; l < m.n_layers; ++l) {
        const int K = l == 0 ? k1 : m.dims[l];
        const int N = m.dims[l + 1];
        const float *wt = w.wt[l];
        const bool last = l + 1 == m.n_layers;
        for (int n = threadIdx.x; n < N; n += 256) {
            float acc[MLP_TS];
            const float b0 = l == 0 ? bias1[(size_t)us * N + n] : (w.bias[l] ? w.bias[l][n] : 0.f);
#pragma unroll
            for (int c = 0; c < MLP_TS; ++c) acc[c] = b0;
            auto term = [&](int k, float wv) {
                const float4 *xp = (const float4 *)(bufA + k * MLP_TS);
#pragma unroll
                for (int c4 = 0; c4 < MLP_TS / 4; ++c4) {
                    const float4 x = xp[c4];
                    acc[c4 * 4 + 0] += wv * x.x;
                    acc[c4 * 4 + 1] += wv * x.y;
                    acc[c4 * 4 + 2] += wv * x.z;
                    acc[c4 * 4 + 3] += wv * x.w;
                }
            };
            // sixteen weights in flight (terms still added in order of k): one at a time is a memory round trip per k
            int k = 0;
            for (; k + 16 <= K; k += 16) {
                float wv[16];
#pragma unroll
                for (int j = 0; j < 16; ++j) wv[j] = wt[(size_t)(k + j) * N + n];
#pragma unroll
                for (int j = 0; j < 16; ++j) term(k + j, wv[j]);
            }
            for (; k + 4 <= K; k += 4) {
                float wv[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) wv[j] = wt[(size_t)(k + j) * N + n];
#pragma unroll
                for (int j = 0; j < 4; ++j) term(k + j, wv[j]);
            }
            for (; k < K; ++k) term(k, wt[(size_t)k * N + n]);
#pragma unroll
            for (int c = 0; c < MLP_TS; ++c) bufB[n * MLP_TS + c] = last ? acc[c] : fmaxf(acc[c], 0.f);
        }
        __syncthreads();
        float *t = bufA; bufA = bufB; bufB = t;
    }
    if (threadIdx.x < nrows) {
        const int c = threadIdx.x;
        float z = bufA[c];
        const int64_t id = rd.cand_ids[local0 + c];
        if (id < 0 || id >= m.n_items) z = __uint_as_float(0x7FC00000u);
        rd.logits_out[local0 + c] = z;
        if (rd.scores_out) rd.scores_out[local0 + c] = 1.0f / (1.0f + expf(-z));
    }
}

static int mlp_generic_buf_floats(const Model &m)
{
    int widest = m.k1;
    for (int l = 1; l <= m.n_layers; ++l) widest = m.dims[l] > widest ? m.dims[l] : widest;
    return widest * MLP_TS;
}
size_t mlp_generic_lds_bytes(const Model &m) { return (size_t)2 * mlp_generic_buf_floats(m) * sizeof(float); }

hipError_t launch_mlp_generic(const Model &m, const Batch &b, const void *X, const MlpGenericWeights &w,
                              const float *bias1, hipStream_t s)
{
    if (b.n_blk == 0) return hipSuccess;
    const int bf = mlp_generic_buf_floats(m);
    const size_t lds = mlp_generic_lds_bytes(m);
    dim3 grid(b.n_blk * (ROW_BLOCK / MLP_TS));
    if (m.dtype == 0) {
        (void)hipFuncSetAttribute((const void *)k_mlp_generic<float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        hipLaunchKernelGGL(k_mlp_generic<float>, grid, dim3(256), lds, s, m, b, (const float *)X, w, bias1, bf);
    } else {
        (void)hipFuncSetAttribute((const void *)k_mlp_generic<uint16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        hipLaunchKernelGGL(k_mlp_generic<uint16_t>, grid, dim3(256), lds, s, m, b, (const uint16_t *)X, w, bias1, bf);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// init-time repacking
// ---------------------------------------------------------------------------
template <typename T>
__global__ void k_pack_transposed(const T *__restrict__ w, int n_out, int n_in, int col0, int ncols,
                                  float *__restrict__ wt)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)ncols * n_out) return;
    const int k = (int)(i / n_out), n = (int)(i - (size_t)k * n_out);
    wt[i] = ld_f<T>(w + (size_t)n * n_in + col0 + k);
}

hipError_t launch_pack_transposed(int dtype, const void *w, int n_out, int n_in, int col0, int ncols, float *wt,
                                  hipStream_t s)
{
    const size_t total = (size_t)ncols * n_out;
    if (!total) return hipSuccess;
    dim3 grid((unsigned)((total + 255) / 256));
    if (dtype == 0)
        hipLaunchKernelGGL(k_pack_transposed<float>, grid, dim3(256), 0, s, (const float *)w, n_out, n_in, col0, ncols, wt);
    else
        hipLaunchKernelGGL(k_pack_transposed<uint16_t>, grid, dim3(256), 0, s, (const uint16_t *)w, n_out, n_in, col0, ncols, wt);
    return hipGetLastError();
}

template <typename T>
__global__ void k_to_f32(const T *__restrict__ src, int64_t rows, int cols, int ld_src, int col0,
                         float *__restrict__ dst)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)rows * cols) return;
    const int64_t rr = (int64_t)(i / cols);
    const int cc = (int)(i - (size_t)rr * cols);
    dst[i] = ld_f<T>(src + (size_t)rr * ld_src + col0 + cc);
}

hipError_t launch_to_f32(int dtype, const void *src, int64_t rows, int cols, int ld_src, int col0, float *dst,
                         hipStream_t s)
{
    const size_t total = (size_t)rows * cols;
    if (!total) return hipSuccess;
    dim3 grid((unsigned)((total + 255) / 256));
    if (dtype == 0)
        hipLaunchKernelGGL(k_to_f32<float>, grid, dim3(256), 0, s, (const float *)src, rows, cols, ld_src, col0, dst);
    else
        hipLaunchKernelGGL(k_to_f32<uint16_t>, grid, dim3(256), 0, s, (const uint16_t *)src, rows, cols, ld_src, col0, dst);
    return hipGetLastError();
}

}  // namespace aif
