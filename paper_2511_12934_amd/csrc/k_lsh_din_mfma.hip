// Eq. 8 on the matrix cores.
//
// DIN_i = (1 / d') sum_k A[b_ik][k] is a contraction once the candidate's bits are written one-hot: with
// X[i][(k, s)] = [b_ik == s] (2 d' columns of 0 / 1) and W[(k, s)][j] = A[s][k][j], DIN = X W / d'.  X is exact in bf16; the
// fp32 table W is not, so it is cut into three bf16 pieces, W = hi + mid + lo (hi = bf16(W), mid = bf16(W - hi), lo = the
// rest: 8 + 8 + 8 significant bits, exact), each a contraction of its own into the SAME fp32 accumulator: every lo
// product first, then every mid, then every hi, so that the d' additions at full magnitude are what they are in the
// vector-ALU kernel and the two small pieces cost rounding errors 2^-8 and 2^-16 as large.  The vector-ALU kernel reads
// its tables from LDS once per (candidate, bit, feature) -- 16 KB per candidate, which is what bound it; here a
// workgroup's 256 candidates share every fragment read.
//
// k_lsh_din_pieces writes W's pieces once per request in the order the instruction reads its column operand:
// [piece][k-step of 16 columns (k, s) = 8 bits][feature tile of 32][lane] of 16 bytes.  k_lsh_din_mfma stages them through
// LDS a run of k-steps at a time; a wave owns 64 candidates (two row tiles) and every feature tile.
#include "aif_lsh_dev.h"

namespace aif {

typedef __bf16 din_bf16x8 __attribute__((ext_vector_type(8)));
typedef float din_f32x16 __attribute__((ext_vector_type(16)));

constexpr int DIN_STAGE_KB = 48;            // fragments (1 KB each) staged in LDS at a time

__device__ __forceinline__ uint32_t bf16_rne_bits(float x)
{
    const uint32_t u = __float_as_uint(x);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;          // finite inputs (sums of embeddings)
}

// lane = (feature of the tile, which 8 of the k-step's 16 columns); column K = (bit k = K / 2, value s = K % 2)
__global__ __launch_bounds__(256) void k_lsh_din_pieces(LshModel m, const float *__restrict__ A, uint4 *__restrict__ out, size_t req_stride)
{
    const int ft_n = m.d_out / 32, ks_n = m.d_bits / 8;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= ks_n * ft_n * 64) return;
    const int lane = idx & 63, ft = (idx >> 6) % ft_n, ks = idx / (64 * ft_n);
    const int j = ft * 32 + (lane & 31), h = lane >> 5;
    const float *Ar = A + (size_t)blockIdx.y * 2 * m.d_bits * m.d_out;
    uint32_t piece[3][4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        uint32_t half[3][2];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const float w = Ar[((size_t)s * m.d_bits + ks * 8 + 4 * h + u) * m.d_out + j];
            const uint32_t hi = bf16_rne_bits(w);
            const float r1 = w - __uint_as_float(hi << 16);
            const uint32_t mid = bf16_rne_bits(r1);
            const float r2 = r1 - __uint_as_float(mid << 16);
            half[0][s] = bf16_rne_bits(r2);                 // accumulated first
            half[1][s] = mid;
            half[2][s] = hi;
        }
#pragma unroll
        for (int p = 0; p < 3; ++p) piece[p][u] = half[p][0] | (half[p][1] << 16);
    }
    uint4 *o = out + (size_t)blockIdx.y * req_stride;
#pragma unroll
    for (int p = 0; p < 3; ++p)
        o[((size_t)(p * ks_n + ks) * ft_n + ft) * 64 + lane] = make_uint4(piece[p][0], piece[p][1], piece[p][2], piece[p][3]);
}

// FT: feature tiles (d = 32 FT).  ksp: k-steps per staging; divides d' / 8.
template <int FT>
__global__ __launch_bounds__(256) void k_lsh_din_mfma(LshModel m, LshBatch b, const uint8_t *__restrict__ sig_table,
                                                      const uint4 *__restrict__ pieces, size_t req_stride, int ksp,
                                                      int32_t *__restrict__ bad)
{
    extern __shared__ __align__(16) char lds[];
    uint4 *sw = (uint4 *)lds;                                   // [ksp][FT][64]
    int blk = blockIdx.x;                                       // a contiguous run of blocks per XCD: a user's pieces in one L2
    {
        const int per_xcd = b.n_blk >> 3;
        if (blk < 8 * per_xcd) blk = (blk & 7) * per_xcd + (blk >> 3);
    }
    const int r = b.blk_req[blk];
    if (r < 0) return;
    const LshReqDesc rd = b.reqs[r];
    const int local0 = blk * LSH_BLOCK - rd.cand_base;
    const int nrows = min(LSH_BLOCK, rd.n_cand - local0);
    if (nrows <= 0) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, col = lane & 31, h = lane >> 5;
    const int nw = m.d_bits / 32, ks_n = m.d_bits / 8;

    // this lane's candidate in each of the wave's two row tiles: its signature, whether it exists, whether its id is valid
    uint32_t sig[2][8];
    uint32_t live_mask[2], ok_mask[2];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
        const int cand = wave * 64 + rt * 32 + col;
        const bool live = cand < nrows;
        int64_t id = live ? rd.cand_ids[local0 + cand] : 0;
        const bool ok = id >= 0 && id < m.n_items;
        if (!ok) id = 0;
        const uint32_t *p = (const uint32_t *)(sig_table + (size_t)id * (nw * 4));
#pragma unroll
        for (int w = 0; w < 8; ++w) sig[rt][w] = w < nw ? p[w] : 0u;
        live_mask[rt] = (uint32_t)__ballot(live);               // lanes 0..31: one bit per candidate of the row tile
        ok_mask[rt] = (uint32_t)__ballot(ok);
    }
    din_f32x16 acc[2][FT];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int ft = 0; ft < FT; ++ft)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[rt][ft][i] = 0.f;

    const uint4 *src = pieces + (size_t)r * req_stride;
    const int stage_frags = ksp * FT * 64;                      // 16-byte pieces per staging
    for (int p = 0; p < 3; ++p) {
        for (int ks0 = 0; ks0 < ks_n; ks0 += ksp) {
            __syncthreads();
            const uint4 *from = src + (size_t)(p * ks_n + ks0) * FT * 64;
            for (int i = threadIdx.x; i < stage_frags; i += 256) sw[i] = from[i];
            __syncthreads();
            for (int ksl = 0; ksl < ksp; ++ksl) {
                const int ks = ks0 + ksl;                       // byte ks of the signature, its high nibble for the first half
                din_bf16x8 x[2];
#pragma unroll
                for (int rt = 0; rt < 2; ++rt) {
                    uint32_t word = sig[rt][0];
#pragma unroll
                    for (int w = 1; w < 8; ++w) word = (ks >> 2) == w ? sig[rt][w] : word;
                    const uint32_t byte = (word >> (8 * (ks & 3))) & 0xFFu, nib = h ? (byte & 15u) : (byte >> 4);
                    uint32_t xw[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) xw[u] = (nib >> (3 - u)) & 1u ? 0x3F800000u : 0x00003F80u;     // (s = 0, s = 1): one of them 1.0
                    x[rt] = __builtin_bit_cast(din_bf16x8, make_uint4(xw[0], xw[1], xw[2], xw[3]));
                }
#pragma unroll
                for (int ft = 0; ft < FT; ++ft) {
                    const din_bf16x8 w = __builtin_bit_cast(din_bf16x8, sw[(ksl * FT + ft) * 64 + lane]);
#pragma unroll
                    for (int rt = 0; rt < 2; ++rt) acc[rt][ft] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x[rt], w, acc[rt][ft], 0, 0, 0);
                }
            }
        }
    }

    // cell v of a lane: candidate 8 (v / 4) + 4 h + v % 4 of the row tile, feature `col` of the feature tile
    const float inv = 1.0f / (float)m.d_bits, nanv = __uint_as_float(0x7FC00000u);
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int c = 8 * (v / 4) + 4 * h + (v % 4);
            if (!((live_mask[rt] >> c) & 1u)) continue;
            const bool ok = (ok_mask[rt] >> c) & 1u;
            float *o = rd.din_out + (size_t)(local0 + wave * 64 + rt * 32 + c) * m.d_out + col;
#pragma unroll
            for (int ft = 0; ft < FT; ++ft) o[ft * 32] = ok ? acc[rt][ft][v] * inv : nanv;
        }
        if (lane == 0) {
            const int n_bad = __builtin_popcount(live_mask[rt] & ~ok_mask[rt]);
            if (n_bad) atomicAdd(bad, n_bad);
        }
    }
}

bool lsh_din_on_mfma(const LshModel &m) { return m.d_out % 32 == 0 && m.d_out <= 128 && m.d_bits <= 256; }

size_t lsh_din_pieces_stride(const LshModel &m)                // 16-byte pieces per request
{
    return (size_t)3 * (m.d_bits / 8) * (m.d_out / 32) * 64;
}

hipError_t launch_lsh_din_mfma(const LshModel &m, const LshBatch &b, const uint8_t *sig_table, const float *A, void *pieces,
                               int32_t *bad, hipStream_t s)
{
    if (b.n_blk == 0) return hipSuccess;
    if (!lsh_din_on_mfma(m) || !pieces) return hipErrorInvalidValue;
    const int ft = m.d_out / 32, ks_n = m.d_bits / 8;
    const size_t stride = lsh_din_pieces_stride(m);
    hipLaunchKernelGGL(k_lsh_din_pieces, dim3((ks_n * ft * 64 + 255) / 256, b.n_req), dim3(256), 0, s, m, A, (uint4 *)pieces, stride);
    int ksp = ks_n;                                             // the largest run of k-steps that divides them and fits the staging
    while (ksp * ft > DIN_STAGE_KB || ks_n % ksp) --ksp;
    const size_t lds = (size_t)ksp * ft * 1024;
    const dim3 grid(b.n_blk), blk(256);
    switch (ft) {
    case 1: hipLaunchKernelGGL(k_lsh_din_mfma<1>, grid, blk, lds, s, m, b, sig_table, (const uint4 *)pieces, stride, ksp, bad); break;
    case 2: hipLaunchKernelGGL(k_lsh_din_mfma<2>, grid, blk, lds, s, m, b, sig_table, (const uint4 *)pieces, stride, ksp, bad); break;
    case 3: hipLaunchKernelGGL(k_lsh_din_mfma<3>, grid, blk, lds, s, m, b, sig_table, (const uint4 *)pieces, stride, ksp, bad); break;
    default: hipLaunchKernelGGL(k_lsh_din_mfma<4>, grid, blk, lds, s, m, b, sig_table, (const uint4 *)pieces, stride, ksp, bad); break;
    }
    return hipGetLastError();
}

}  // namespace aif
