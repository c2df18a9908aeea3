// User-side network of AIF (Sec. 3.1, Eq. 1-3), the parts around the attention:
// the projections of Eq. 1, and FFN + pooling + combined vector of Eq. 2.  The
// attentions themselves (Eq. 2's self-attention over the sequence and Eq. 3's
// profile-to-sequence attention) run on the library's target-attention kernels:
// every sequence position, and the profile, is a query over the same projected
// sequence.
//
// fp32 arithmetic over the storage type, fixed summation order per output.
#include "aif_user_dev.h"

namespace aif {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// The projected profile: four adjacent lanes share an output feature, each takes a quarter of the input
// features (d_raw is a multiple of four), they meet in a fixed two-step butterfly.  All of a thread's loads are
// independent, so the row costs about one round trip to memory.
template <typename T>
__device__ __forceinline__ void project_profile(const UserWeights &w, const UserDesc &ud, T *__restrict__ X, int nthreads)
{
    const T *pr = (const T *)ud.profile;
    const int d = w.d, q = threadIdx.x & 3, chunk = w.d_raw >> 2;
    for (int n0 = 0; n0 < d; n0 += nthreads >> 2) {
        const int n = n0 + (threadIdx.x >> 2);
        float acc = 0.f;
        if (n < d) {
            const float *wr = w.wprof + (size_t)n * w.d_raw + q * chunk;
            const T *px = pr + q * chunk;
#pragma unroll 8
            for (int m = 0; m < chunk; ++m) acc = fmaf(wr[m], ld_f<T>(px + m), acc);
        }
        acc += __shfl_xor(acc, 1, 64);
        acc += __shfl_xor(acc, 2, 64);
        if (n < d && q == 0) st_f<T>(X + (size_t)(ud.row_base + ud.seq_len) * (2 * d) + n, acc);
    }
}

// ---------------------------------------------------------------------------
// Eq. 1 on the matrix cores (bf16): U^_seq^T = W_seq U_seq^T, positions as the
// columns of the B operand.  A wave owns 32 positions; lane (position c, half h)
// reads eight consecutive input features of its position per k-step straight
// from the caller's row-major sequence and receives sixteen output features of
// that position per 32-feature tile (features 8 q + 4 h + i), which it writes as
// four 8-byte pieces to the workspace row and to the user's seq_out.
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void k_user_project_mfma(UserWeights w, const UserDesc *__restrict__ users,
                                                           const int32_t *__restrict__ blk_req, uint16_t *__restrict__ X)
{
    constexpr int FT = D / 32, ROWS = 128, SUB = ROW_BLOCK / ROWS;
    const int u = blk_req[blockIdx.x / SUB];
    if (u < 0) return;
    const UserDesc ud = users[u];
    const int row0 = blockIdx.x * ROWS, local0 = row0 - ud.row_base, L = ud.seq_len;
    if (local0 > L) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, col = lane & 31, h = lane >> 5;
    const int li = local0 + wave * 32 + col;
    const int KS = w.d_raw / 16;
    if (local0 + wave * 32 < L) {                               // wave-uniform: some position of this wave exists
        const uint16_t *src = (const uint16_t *)ud.seq + (size_t)(li < L ? li : 0) * w.d_raw + 8 * h;
        const bf16x8 *wf = (const bf16x8 *)w.wseq_frag + lane;
        f32x16 acc[FT];
#pragma unroll
        for (int ft = 0; ft < FT; ++ft)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[ft][i] = 0.f;
        // all of a group's input pieces are asked for before its first MFMA: the loads are independent, and one
        // round trip to memory per group instead of one per k-step is what this short kernel's time is made of
        constexpr int G = 8;
        for (int k0 = 0; k0 < KS; k0 += G) {
            bf16x8 b[G];
#pragma unroll
            for (int j = 0; j < G; ++j)
                if (k0 + j < KS) b[j] = *(const bf16x8 *)(src + 16 * (k0 + j));
#pragma unroll
            for (int j = 0; j < G; ++j)
                if (k0 + j < KS) {
#pragma unroll
                    for (int ft = 0; ft < FT; ++ft)
                        acc[ft] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[(size_t)(ft * KS + k0 + j) * 64], b[j], acc[ft], 0, 0, 0);
                }
        }
        if (li < L) {
            uint16_t *xr = X + (size_t)(row0 + wave * 32 + col) * (2 * D), *so = (uint16_t *)ud.seq_out + (size_t)li * D;
#pragma unroll
            for (int ft = 0; ft < FT; ++ft)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    bf16x4 o4;
#pragma unroll
                    for (int i = 0; i < 4; ++i) o4[i] = (__bf16)acc[ft][4 * q + i];
                    const int f = 32 * ft + 8 * q + 4 * h;
                    *(bf16x4 *)(xr + f) = o4;
                    *(bf16x4 *)(so + f) = o4;
                }
        }
    }
    if (L >= local0 && L < local0 + ROWS) project_profile<uint16_t>(w, ud, X, 256);
}

// ---------------------------------------------------------------------------
// FFN of Eq. 2 on the matrix cores (bf16) and the pooling share of 32 positions:
// Y^T = W_ffn A^T with the accumulators preloaded with the bias, ReLU, positions
// past the end zeroed, then the sum over the wave's 32 positions (the lanes of a
// half) by a fixed butterfly.
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void k_user_ffn_mfma(UserWeights w, const UserDesc *__restrict__ users,
                                                       const int32_t *__restrict__ blk_req, const uint16_t *__restrict__ X,
                                                       float *__restrict__ part)
{
    constexpr int FT = D / 32, KS = D / 16, ROWS = 128, SUB = ROW_BLOCK / ROWS;
    const int u = blk_req[blockIdx.x / SUB];
    if (u < 0) return;
    const UserDesc ud = users[u];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, col = lane & 31, h = lane >> 5;
    const int row0 = blockIdx.x * ROWS + wave * 32, local0 = row0 - ud.row_base, L = ud.seq_len;
    if (local0 >= L) return;
    const uint16_t *src = X + (size_t)(row0 + col) * (2 * D) + D + 8 * h;      // rows past L are inside the workspace
    const bf16x8 *wf = (const bf16x8 *)w.wffn_frag + lane;
    bf16x8 b[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) b[ks] = *(const bf16x8 *)(src + 16 * ks);
    const bool live = local0 + col < L;
#pragma unroll
    for (int ft = 0; ft < FT; ++ft) {
        f32x16 acc;
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[4 * q + i] = w.b_ffn ? w.b_ffn[32 * ft + 8 * q + 4 * h + i] : 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[(size_t)(ft * KS + ks) * 64], b[ks], acc, 0, 0, 0);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            float y = live ? fmaxf(acc[v], 0.f) : 0.f;
#pragma unroll
            for (int o = 1; o < 32; o <<= 1) y += __shfl_xor(y, o, 64);
            acc[v] = y;
        }
        if (col == 0) {
            float *dst = part + (size_t)(row0 / 32) * D + 32 * ft + 4 * h;
#pragma unroll
            for (int q = 0; q < 4; ++q) *(float4 *)(dst + 8 * q) = make_float4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
        }
    }
}

// ---------------------------------------------------------------------------
// Eq. 1.  One block = USER_PROJ_ROWS rows of one user.  The rows are staged in
// LDS transposed (xs[m][row]) so that a thread reads the eight rows it owns for
// one input feature with two 16-byte reads; thread (column lane, row group) walks
// the transposed weights, one coalesced load per input feature reused for its
// eight rows.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_user_project(UserWeights w, const UserDesc *__restrict__ users,
                                                      const int32_t *__restrict__ blk_req, T *__restrict__ X)
{
    extern __shared__ __align__(16) float xs[];                 // [d_raw][USER_PROJ_ROWS]
    constexpr int RT = USER_PROJ_ROWS, SUB = ROW_BLOCK / RT;
    const int u = blk_req[blockIdx.x / SUB];
    if (u < 0) return;
    const UserDesc ud = users[u];
    const int row0 = blockIdx.x * RT;
    const int local0 = row0 - ud.row_base;
    const int L = ud.seq_len;
    if (local0 > L) return;                                     // rows 0..L (L = the profile) exist
    const int d_raw = w.d_raw, d = w.d;
    const T *seq = (const T *)ud.seq;
    for (int idx = threadIdx.x; idx < RT * d_raw; idx += 256) {
        const int r = idx / d_raw, m = idx - r * d_raw;
        const int i = local0 + r;
        xs[m * RT + r] = i < L ? ld_f<T>(seq + (size_t)i * d_raw + m) : 0.f;
    }
    __syncthreads();
    const int nl = threadIdx.x & 63, g = threadIdx.x >> 6;      // 4 row groups of 8
    T *so = (T *)ud.seq_out;
    for (int n = nl; n < d; n += 64) {
        float acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = 0.f;
        for (int m = 0; m < d_raw; ++m) {
            const float wv = w.wseq_t[(size_t)m * d + n];
            const float4 a = *(const float4 *)(xs + m * RT + g * 8), b = *(const float4 *)(xs + m * RT + g * 8 + 4);
            acc[0] = fmaf(wv, a.x, acc[0]);
            acc[1] = fmaf(wv, a.y, acc[1]);
            acc[2] = fmaf(wv, a.z, acc[2]);
            acc[3] = fmaf(wv, a.w, acc[3]);
            acc[4] = fmaf(wv, b.x, acc[4]);
            acc[5] = fmaf(wv, b.y, acc[5]);
            acc[6] = fmaf(wv, b.z, acc[6]);
            acc[7] = fmaf(wv, b.w, acc[7]);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int li = local0 + g * 8 + i;
            if (li < L) {
                st_f<T>(X + (size_t)(row0 + g * 8 + i) * (2 * d) + n, acc[i]);
                st_f<T>(so + (size_t)li * d + n, acc[i]);
            }
        }
    }
    // the profile row, if it falls into this block
    if (L >= local0 && L < local0 + RT) project_profile<T>(w, ud, X, 256);
}

size_t user_project_lds_bytes(int d_raw) { return (size_t)d_raw * USER_PROJ_ROWS * sizeof(float); }

hipError_t launch_user_project(const UserWeights &w, const UserDesc *users, const int32_t *blk_req, int n_blk, void *X,
                               hipStream_t s)
{
    if (n_blk == 0) return hipSuccess;
    if (w.wseq_frag) {
        const dim3 g(n_blk * (ROW_BLOCK / 128));
        switch (w.d) {
        case 32: hipLaunchKernelGGL(k_user_project_mfma<32>, g, dim3(256), 0, s, w, users, blk_req, (uint16_t *)X); break;
        case 64: hipLaunchKernelGGL(k_user_project_mfma<64>, g, dim3(256), 0, s, w, users, blk_req, (uint16_t *)X); break;
        case 128: hipLaunchKernelGGL(k_user_project_mfma<128>, g, dim3(256), 0, s, w, users, blk_req, (uint16_t *)X); break;
        default: return hipErrorInvalidValue;
        }
        return hipGetLastError();
    }
    const size_t lds = user_project_lds_bytes(w.d_raw);
    const dim3 grid(n_blk * (ROW_BLOCK / USER_PROJ_ROWS));
    if (w.dtype == 0) {
        (void)hipFuncSetAttribute((const void *)k_user_project<float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        hipLaunchKernelGGL(k_user_project<float>, grid, dim3(256), lds, s, w, users, blk_req, (float *)X);
    } else {
        (void)hipFuncSetAttribute((const void *)k_user_project<uint16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        hipLaunchKernelGGL(k_user_project<uint16_t>, grid, dim3(256), lds, s, w, users, blk_req, (uint16_t *)X);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// FFN of Eq. 2 (one layer with ReLU) on the attention outputs of USER_FFN_ROWS
// positions, summed over those positions in position order: the block's share
// of the pooling.  Same thread layout as the projection, sixteen rows a thread.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_user_ffn_partial(UserWeights w, const UserDesc *__restrict__ users,
                                                          const int32_t *__restrict__ blk_req, const T *__restrict__ X,
                                                          float *__restrict__ part)
{
    extern __shared__ __align__(16) float as[];                 // [d][USER_FFN_ROWS], then [4][d] group sums
    constexpr int RT = USER_FFN_ROWS, SUB = ROW_BLOCK / RT;
    const int u = blk_req[blockIdx.x / SUB];
    if (u < 0) return;
    const UserDesc ud = users[u];
    const int row0 = blockIdx.x * RT;
    const int local0 = row0 - ud.row_base;
    const int L = ud.seq_len;
    if (local0 >= L) return;
    const int d = w.d;
    float *gs = as + (size_t)d * RT;
    for (int idx = threadIdx.x; idx < RT * d; idx += 256) {
        const int r = idx / d, m = idx - r * d;
        as[m * RT + r] = local0 + r < L ? ld_f<T>(X + (size_t)(row0 + r) * (2 * d) + d + m) : 0.f;
    }
    __syncthreads();
    const int nl = threadIdx.x & 63, g = threadIdx.x >> 6;      // 4 row groups of 16
    for (int n = nl; n < d; n += 64) {
        float acc[16];
        const float b0 = w.b_ffn ? w.b_ffn[n] : 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = b0;
        for (int m = 0; m < d; ++m) {
            const float wv = w.wffn_t[(size_t)m * d + n];
            const float *ap = as + m * RT + g * 16;
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                const float4 a = *(const float4 *)(ap + 4 * i4);
                acc[4 * i4 + 0] = fmaf(wv, a.x, acc[4 * i4 + 0]);
                acc[4 * i4 + 1] = fmaf(wv, a.y, acc[4 * i4 + 1]);
                acc[4 * i4 + 2] = fmaf(wv, a.z, acc[4 * i4 + 2]);
                acc[4 * i4 + 3] = fmaf(wv, a.w, acc[4 * i4 + 3]);
            }
        }
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (local0 + g * 16 + i < L) sum += fmaxf(acc[i], 0.f);
        gs[g * d + n] = sum;
    }
    __syncthreads();
    for (int n = threadIdx.x; n < d; n += 256)
        part[(size_t)blockIdx.x * d + n] = ((gs[n] + gs[d + n]) + gs[2 * d + n]) + gs[3 * d + n];
}

size_t user_ffn_lds_bytes(int d) { return (size_t)d * (USER_FFN_ROWS + 4) * sizeof(float); }

hipError_t launch_user_ffn_partial(const UserWeights &w, const UserDesc *users, const int32_t *blk_req, int n_blk,
                                   const void *X, float *part, hipStream_t s)
{
    if (n_blk == 0) return hipSuccess;
    if (w.wffn_frag) {
        const dim3 g(n_blk * (ROW_BLOCK / 128));
        switch (w.d) {
        case 32: hipLaunchKernelGGL(k_user_ffn_mfma<32>, g, dim3(256), 0, s, w, users, blk_req, (const uint16_t *)X, part); break;
        case 64: hipLaunchKernelGGL(k_user_ffn_mfma<64>, g, dim3(256), 0, s, w, users, blk_req, (const uint16_t *)X, part); break;
        case 128: hipLaunchKernelGGL(k_user_ffn_mfma<128>, g, dim3(256), 0, s, w, users, blk_req, (const uint16_t *)X, part); break;
        default: return hipErrorInvalidValue;
        }
        return hipGetLastError();
    }
    const size_t lds = user_ffn_lds_bytes(w.d);
    const dim3 grid(n_blk * (ROW_BLOCK / USER_FFN_ROWS));
    if (w.dtype == 0) {
        (void)hipFuncSetAttribute((const void *)k_user_ffn_partial<float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        hipLaunchKernelGGL(k_user_ffn_partial<float>, grid, dim3(256), lds, s, w, users, blk_req, (const float *)X, part);
    } else {
        (void)hipFuncSetAttribute((const void *)k_user_ffn_partial<uint16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        hipLaunchKernelGGL(k_user_ffn_partial<uint16_t>, grid, dim3(256), lds, s, w, users, blk_req, (const uint16_t *)X, part);
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Pooling (mean) and the combined vector.  One block per user.
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_user_combine(UserWeights w, const UserDesc *__restrict__ users,
                                                      const T *__restrict__ X, const float *__restrict__ part)
{
    const UserDesc ud = users[blockIdx.x];
    const int d = w.d, L = ud.seq_len;
    const int nb = (L + w.part_rows - 1) / w.part_rows;
    const size_t b0 = (size_t)ud.row_base / w.part_rows;
    T *out = (T *)ud.user_vec_out;
    for (int n = threadIdx.x; n < d; n += 256) {
        float sum = 0.f;
        for (int j = 0; j < nb; ++j) sum += part[(b0 + j) * d + n];
        st_f<T>(out + n, L > 0 ? sum / (float)L : 0.f);
        out[d + n] = X[(size_t)(ud.row_base + L) * (2 * d) + d + n];       // Eq. 3: the profile row's attention
    }
}

hipError_t launch_user_combine(const UserWeights &w, const UserDesc *users, int n_users, const void *X, const float *part,
                               hipStream_t s)
{
    if (n_users == 0) return hipSuccess;
    if (w.dtype == 0)
        hipLaunchKernelGGL(k_user_combine<float>, dim3(n_users), dim3(256), 0, s, w, users, (const float *)X, part);
    else
        hipLaunchKernelGGL(k_user_combine<uint16_t>, dim3(n_users), dim3(256), 0, s, w, users, (const uint16_t *)X, part);
    return hipGetLastError();
}

}  // namespace aif
