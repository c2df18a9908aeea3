// LSH-based long-sequence behaviour modelling (Sec. 4.3): signature similarity
// by XNOR + population count (Eq. 6, 7), LSH-DIN (Eq. 8) and SimTier (Eq. 9).
//
// SimTier needs every (candidate, history item) similarity, so its kernel walks
// the b x l pairs: a lane owns one candidate, the history signatures are the
// same for all lanes and arrive through scalar loads, a pair costs two XNORs,
// two population counts and a handful of integer instructions that bump one
// byte of a packed 64-bit histogram (eight tiers, flushed before a byte can
// overflow).  Plain integer work, bound by the vector ALU.
//
// LSH-DIN does NOT need the pairs.  Eq. 8 has no softmax: the weight of
// history item t is (number of equal bits) / d' = (1/d') sum_k [b_ik == b_tk],
// so
//     DIN_i = (1/d') sum_k A[b_ik][k],   A[s][k] = sum over t with b_tk == s of U~_t,
// and the 2 d' vectors A[s][k] belong to the user alone.  They are formed once
// per request (a2 of this path: user-side staging, in chunks of the history
// summed in a fixed order), after which a candidate costs d' additions per
// output feature instead of l multiply-adds.  Same value as Eq. 8 up to the
// order of the fp32 additions.
#include "aif_lsh_dev.h"

#include <cstdlib>

namespace aif {

__device__ __forceinline__ float lsh_ld(const void *p, int dtype, size_t i)
{
    return dtype == 0 ? ((const float *)p)[i] : __uint_as_float(((uint32_t)((const uint16_t *)p)[i]) << 16);
}

// ---------------------------------------------------------------------------
// user side, partial sums.  Block (chunk, request); a work item is (bit k, group of 16 features).
// ---------------------------------------------------------------------------
constexpr int LSH_TSUB = 128;           // history items staged in LDS at a time

__global__ __launch_bounds__(256) void k_lsh_user_partial(LshModel m, LshBatch b, int max_chunks, float *__restrict__ part)
{
    extern __shared__ __align__(16) char lds[];
    const int r = blockIdx.y, chunk = blockIdx.x;
    const LshReqDesc rd = b.reqs[r];
    const int chunk_len = lsh_chunk_len(rd.seq_len);
    const int t_lo = chunk * chunk_len;
    if (t_lo >= rd.seq_len) return;
    const int t_hi = min(rd.seq_len, t_lo + chunk_len);
    const int d = m.d_out, nb = m.d_bits / 8, jg = d / 16, items = m.d_bits * jg;
    float *su = (float *)lds;                               // [LSH_TSUB][d]
    uint8_t *ss = (uint8_t *)(su + LSH_TSUB * d);           // [LSH_TSUB][nb]
    float *out = part + ((size_t)r * max_chunks + chunk) * 2 * m.d_bits * d;

    for (int item0 = 0; item0 < items; item0 += 256) {
        const int item = item0 + threadIdx.x;
        const bool work = item < items;
        const int k = work ? item / jg : 0, j0 = work ? (item - k * jg) * 16 : 0;
        float a0[16], a1[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) a0[i] = a1[i] = 0.f;
        for (int ts = t_lo; ts < t_hi; ts += LSH_TSUB) {
            const int nt = min(LSH_TSUB, t_hi - ts);
            __syncthreads();
            for (int i = threadIdx.x; i < nt * d; i += 256) su[i] = lsh_ld(rd.seq_emb, m.dtype, (size_t)ts * d + i);
            for (int i = threadIdx.x; i < nt * nb; i += 256) ss[i] = rd.seq_sigs[(size_t)ts * nb + i];
            __syncthreads();
            if (work) {
                // sums of the staged items first, then into the chunk's sums: short chains of additions
                float s0[16], s1[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) s0[i] = s1[i] = 0.f;
                for (int t = 0; t < nt; ++t) {
                    // bit k of a signature: byte k / 8, first bit most significant
                    const float bit = (float)((ss[t * nb + (k >> 3)] >> (7 - (k & 7))) & 1);
                    const float4 *u4 = (const float4 *)(su + t * d + j0);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float4 u = u4[q];
                        s1[4 * q + 0] = fmaf(bit, u.x, s1[4 * q + 0]);
                        s1[4 * q + 1] = fmaf(bit, u.y, s1[4 * q + 1]);
                        s1[4 * q + 2] = fmaf(bit, u.z, s1[4 * q + 2]);
                        s1[4 * q + 3] = fmaf(bit, u.w, s1[4 * q + 3]);
                        s0[4 * q + 0] = fmaf(1.f - bit, u.x, s0[4 * q + 0]);
                        s0[4 * q + 1] = fmaf(1.f - bit, u.y, s0[4 * q + 1]);
                        s0[4 * q + 2] = fmaf(1.f - bit, u.z, s0[4 * q + 2]);
                        s0[4 * q + 3] = fmaf(1.f - bit, u.w, s0[4 * q + 3]);
                    }
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    a0[i] += s0[i];
                    a1[i] += s1[i];
                }
            }
        }
        if (work) {
            float4 *o0 = (float4 *)(out + (size_t)k * d + j0);
            float4 *o1 = (float4 *)(out + (size_t)(m.d_bits + k) * d + j0);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                o0[q] = make_float4(a0[4 * q], a0[4 * q + 1], a0[4 * q + 2], a0[4 * q + 3]);
                o1[q] = make_float4(a1[4 * q], a1[4 * q + 1], a1[4 * q + 2], a1[4 * q + 3]);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// The same partial sums on the matrix cores, for bf16 embeddings.  part[s][k][j] = sum_t [b_tk == s] U~[t][j] is a
// contraction over the history: (bits as 0/1, inverted for s = 0) [2 d' x l] times U~ [l x d].  0, 1 and the
// embeddings are exact in bf16 and the MFMA accumulates in fp32, so the values are those of the loop above up to the
// order of the additions.  The contraction index t is the slow axis of both inputs as the caller stores them, so
// both pass through LDS: 64 history items at a time, the embeddings set down transposed ([j][t]: a lane's eight
// consecutive t are one 16-byte read), the signatures turned into bit planes over t by wave ballots (lane = t), from
// which an A fragment -- eight consecutive t of one bit position -- is one byte, expanded to eight bf16 through a
// 256-entry table in LDS.  Block = (chunk of lsh_chunk_len items, request), four waves; the 2 d' / 32 x d / 32 result
// tiles are dealt round the waves, TPW each.
// ---------------------------------------------------------------------------
typedef __bf16 lsh_bf16x8 __attribute__((ext_vector_type(8)));
typedef float lsh_f32x16 __attribute__((ext_vector_type(16)));
constexpr int LSH_TS = 64;              // history items per trip through LDS: four MFMA k-steps

template <int TPW>
__global__ __launch_bounds__(256) void k_lsh_user_partial_mfma(LshModel m, LshBatch b, int max_chunks, float *__restrict__ part)
{
    extern __shared__ __align__(16) char lds[];
    const int r = blockIdx.y, chunk = blockIdx.x;
    const LshReqDesc rd = b.reqs[r];
    const int chunk_len = lsh_chunk_len(rd.seq_len);
    const int t_lo = chunk * chunk_len;
    if (t_lo >= rd.seq_len) return;
    const int t_hi = min(rd.seq_len, t_lo + chunk_len);
    const int d = m.d_out, db = m.d_bits, nb = db / 8, CT = d / 32;
    constexpr int USTR = LSH_TS * 2 + 16;                        // bytes per transposed embedding row (64 t + padding)
    uint4 *lut = (uint4 *)lds;                                   // [256] byte -> eight bf16 of 0 / 1, first bit = first slot
    char *su = lds + 4096;                                       // [d][USTR]: U~ of the trip, transposed
    uint32_t *bp = (uint32_t *)(su + (size_t)d * USTR);          // [d'][2]: bit k of the trip's 64 signatures, lane t = bit t
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, col = lane & 31, h = lane >> 5;
    {
        const uint32_t v = threadIdx.x;                          // slot s of the fragment = bit s of the byte (t0 + s)
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = ((v >> (2 * i)) & 1u) * 0x3F80u + ((v >> (2 * i + 1)) & 1u) * 0x3F800000u;
        lut[threadIdx.x] = make_uint4(w[0], w[1], w[2], w[3]);
    }
    lsh_f32x16 acc[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    const uint16_t *emb = (const uint16_t *)rd.seq_emb;

    for (int ts = t_lo; ts < t_hi; ts += LSH_TS) {
        __syncthreads();                                         // the last trip's fragments have been read
        // embeddings: 16-byte pieces (eight features of one item) read in row order, written transposed
        for (int pc = threadIdx.x; pc < LSH_TS * d / 8; pc += 256) {
            const int t = pc / (d / 8), j0 = (pc - t * (d / 8)) * 8;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (ts + t < t_hi) v = *(const uint4 *)(emb + (size_t)(ts + t) * d + j0);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 8; ++i)
                *(uint16_t *)(su + (size_t)(j0 + i) * USTR + 2 * t) = (uint16_t)(w[i >> 1] >> (16 * (i & 1)));
        }
        // signatures: lane = history item; bit k of all 64 items by one ballot; the waves share the bit positions
        {
            const int t = ts + lane;
            const uint8_t *sg = rd.seq_sigs + (size_t)t * nb;
            for (int k = wave; k < db; k += 4) {
                const uint32_t byte = t < t_hi ? sg[k >> 3] : 0u;            // first bit most significant
                const unsigned long long mask = __ballot((byte >> (7 - (k & 7))) & 1u);
                if (lane == 0) {
                    bp[2 * k] = (uint32_t)mask;
                    bp[2 * k + 1] = (uint32_t)(mask >> 32);
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < LSH_TS / 16; ++ks) {
            const int tb = 16 * ks + 8 * h;                      // this lane's eight items of the k-step
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                const int idx = wave + 4 * i, rt = idx / CT, ct = idx - rt * CT;
                const int row = 32 * rt + col, sbit = row / db, k = row - sbit * db;        // row = s d' + k
                uint32_t byte = (bp[2 * k + (tb >> 5)] >> (tb & 31)) & 0xFFu;
                if (sbit == 0) byte ^= 0xFFu;                    // the items whose bit is 0
                const lsh_bf16x8 A = __builtin_bit_cast(lsh_bf16x8, lut[byte]);
                const lsh_bf16x8 B = *(const lsh_bf16x8 *)(su + (size_t)(32 * ct + col) * USTR + 2 * tb);
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, B, acc[i], 0, 0, 0);
            }
        }
    }
    float *out = part + ((size_t)r * max_chunks + chunk) * 2 * db * d;
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        const int idx = wave + 4 * i, rt = idx / CT, ct = idx - rt * CT;
#pragma unroll
        for (int e = 0; e < 16; ++e) out[(size_t)(32 * rt + 8 * (e >> 2) + 4 * h + (e & 3)) * d + 32 * ct + col] = acc[i][e];
    }
}

// bf16 embeddings, whole 32-tiles, a number of result tiles the four waves share evenly: the matrix-core form
static int lsh_user_mfma_tpw(const LshModel &m)
{
    if (m.dtype != 1 || m.d_out % 32 || m.d_bits % 32) return 0;
    const int nt = (2 * m.d_bits / 32) * (m.d_out / 32);
    return (nt == 8 || nt == 16 || nt == 32) ? nt / 4 : 0;
}

hipError_t launch_lsh_user_partial(const LshModel &m, const LshBatch &b, int grid_chunks, int max_chunks, float *part,
                                   hipStream_t s)
{
    if (b.n_req == 0 || grid_chunks == 0) return hipSuccess;
    if (const int tpw = lsh_user_mfma_tpw(m)) {
        const char *off = getenv("AIF_LSH_USER_VALU");           // testing: the vector-ALU form on a shape the matrix cores serve
        if (!(off && off[0] == '1')) {
            const size_t bytes = 4096 + (size_t)m.d_out * (LSH_TS * 2 + 16) + (size_t)m.d_bits * 8;
            const dim3 grid(grid_chunks, b.n_req), block(256);
            if (tpw == 2) hipLaunchKernelGGL(k_lsh_user_partial_mfma<2>, grid, block, bytes, s, m, b, max_chunks, part);
            else if (tpw == 4) hipLaunchKernelGGL(k_lsh_user_partial_mfma<4>, grid, block, bytes, s, m, b, max_chunks, part);
            else hipLaunchKernelGGL(k_lsh_user_partial_mfma<8>, grid, block, bytes, s, m, b, max_chunks, part);
            return hipGetLastError();
        }
    }
    const size_t lds = (size_t)LSH_TSUB * (m.d_out * 4 + m.d_bits / 8);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_lsh_user_partial, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(k_lsh_user_partial, dim3(grid_chunks, b.n_req), dim3(256), lds, s, m, b, max_chunks, part);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void k_lsh_user_reduce(LshModel m, LshBatch b, int max_chunks, const float *__restrict__ part,
                                                         float *__restrict__ A)
{
    const int r = blockIdx.y;
    const size_t n = (size_t)2 * m.d_bits * m.d_out;
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int L = b.reqs[r].seq_len;
    const int chunks = lsh_chunks(L);
    float acc = 0.f;
    for (int c = 0; c < chunks; ++c) acc += part[((size_t)r * max_chunks + c) * n + i];
    A[(size_t)r * n + i] = acc;
}

hipError_t launch_lsh_user_reduce(const LshModel &m, const LshBatch &b, int max_chunks, const float *part, float *A,
                                  hipStream_t s)
{
    if (b.n_req == 0) return hipSuccess;
    const size_t n = (size_t)2 * m.d_bits * m.d_out;
    hipLaunchKernelGGL(k_lsh_user_reduce, dim3((unsigned)((n + 255) / 256), b.n_req), dim3(256), 0, s, m, b, max_chunks, part, A);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Eq. 8.  Block = LSH_BLOCK candidates of one request; d / 16 threads per candidate, 16 features each.
// The user's table A[2][d'][d] is staged in LDS in slices of KC bits.
// ---------------------------------------------------------------------------
constexpr int LSH_DIN_LDS = 64 * 1024;

__global__ __launch_bounds__(256) void k_lsh_din(LshModel m, LshBatch b, const uint8_t *__restrict__ sig_table,
                                                 const float *__restrict__ A, int32_t *__restrict__ bad)
{
    extern __shared__ __align__(16) char lds[];
    float *sa = (float *)lds;                                   // [2][kc][d]
    int blk = blockIdx.x;                                       // a contiguous run of blocks per XCD, as in k_lsh_simtier: a user's table in one L2
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
    const int d = m.d_out, jg = d / 16, nb = m.d_bits / 8;
    const int per_round = 256 / jg;                             // candidates served at once
    const int kc = min(m.d_bits, LSH_DIN_LDS / (2 * d * 4)) & ~7;   // bits per slice, whole bytes
    const float *Ar = A + (size_t)r * 2 * m.d_bits * d;
    const int sub = threadIdx.x / jg, j0 = (threadIdx.x - sub * jg) * 16;
    const float inv = 1.0f / (float)m.d_bits;
    int n_bad = 0;

    for (int c0 = 0; c0 < nrows; c0 += per_round) {
        const int cand = c0 + sub;
        const bool live = sub < per_round && cand < nrows;
        int64_t id = live ? rd.cand_ids[local0 + cand] : 0;
        const bool ok = id >= 0 && id < m.n_items;
        if (!ok) {
            id = 0;
            if (live && j0 == 0) ++n_bad;
        }
        const uint8_t *sig = sig_table + (size_t)id * nb;
        float acc[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
        for (int k0 = 0; k0 < m.d_bits; k0 += kc) {
            const int kn = min(kc, m.d_bits - k0);
            __syncthreads();
            if (c0 == 0 || kc < m.d_bits) {                     // the whole table fits: staged once
                for (int i = threadIdx.x; i < 2 * kn * d / 4; i += 256) {
                    const int s = i / (kn * d / 4), rem = i - s * (kn * d / 4);
                    ((float4 *)sa)[i] = ((const float4 *)(Ar + ((size_t)s * m.d_bits + k0) * d))[rem];
                }
            }
            __syncthreads();
            if (live) {
                for (int kb = 0; kb < kn; kb += 8) {
                    const uint32_t byte = sig[(k0 + kb) >> 3];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int bit = (byte >> (7 - u)) & 1;
                        const float4 *a4 = (const float4 *)(sa + ((size_t)bit * kn + kb + u) * d + j0);
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const float4 v = a4[q];
                            acc[4 * q + 0] += v.x;
                            acc[4 * q + 1] += v.y;
                            acc[4 * q + 2] += v.z;
                            acc[4 * q + 3] += v.w;
                        }
                    }
                }
            }
        }
        if (live) {
            float4 *o = (float4 *)(rd.din_out + (size_t)(local0 + cand) * d + j0);
            const float nanv = __uint_as_float(0x7FC00000u);
#pragma unroll
            for (int q = 0; q < 4; ++q)
                o[q] = ok ? make_float4(acc[4 * q] * inv, acc[4 * q + 1] * inv, acc[4 * q + 2] * inv, acc[4 * q + 3] * inv)
                          : make_float4(nanv, nanv, nanv, nanv);
        }
    }
    if (n_bad) atomicAdd(bad, n_bad);
}

hipError_t launch_lsh_din(const LshModel &m, const LshBatch &b, const uint8_t *sig_table, const float *A, int32_t *bad,
                          hipStream_t s)
{
    if (b.n_blk == 0) return hipSuccess;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_lsh_din, hipFuncAttributeMaxDynamicSharedMemorySize, LSH_DIN_LDS);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(k_lsh_din, dim3(b.n_blk), dim3(256), LSH_DIN_LDS, s, m, b, sig_table, A, bad);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Eq. 6, 7, 9.  A lane owns one candidate and walks the whole history.
// DW = signature width in 32-bit words.
// ---------------------------------------------------------------------------
template <int DW>
__global__ __launch_bounds__(256) void k_lsh_simtier(LshModel m, LshBatch b, const uint8_t *__restrict__ sig_table)
{
    // Workgroups go to the 8 XCDs in turn, each with an L2 of its own.  Every XCD takes a contiguous run of the
    // blocks, so that the blocks of one user -- which all walk that user's history signatures -- share an L2 instead
    // of all eight fetching them.
    int blk = blockIdx.x;
    {
        const int per_xcd = b.n_blk >> 3;
        if (blk < 8 * per_xcd) blk = (blk & 7) * per_xcd + (blk >> 3);
    }
    const int r = b.blk_req[blk];
    if (r < 0) return;
    const LshReqDesc rd = b.reqs[r];
    const int local = blk * LSH_BLOCK - rd.cand_base + threadIdx.x;
    const bool live = local < rd.n_cand;
    int64_t id = live ? rd.cand_ids[local] : 0;
    const bool ok = id >= 0 && id < m.n_items;
    if (!ok) id = 0;
    uint32_t sig[DW];
    {
        const uint32_t *p = (const uint32_t *)(sig_table + (size_t)id * (DW * 4));
#pragma unroll
        for (int w = 0; w < DW; ++w) sig[w] = p[w];
    }
    const uint32_t *__restrict__ hs = (const uint32_t *)rd.seq_sigs;    // the same for every lane: scalar loads
    const int L = rd.seq_len;
    // 8 * tier = min(8 (N - 1), ((equal * N * tier_mul) >> 17) & ~7); equal <= 256 and N * tier_mul < 2^19 fit a
    // 24-bit multiply, and the multiply-shift is exact for equal N <= 2048, d' <= 256
    const uint32_t scale = (uint32_t)m.n_tiers * (uint32_t)m.tier_mul, top8 = 8u * (uint32_t)(m.n_tiers - 1);
    uint32_t total[LSH_MAX_TIERS];
#pragma unroll
    for (int j = 0; j < LSH_MAX_TIERS; ++j) total[j] = 0;
    unsigned long long packed = 0;                          // eight byte-wide tier counters

    auto visit = [&](const uint32_t *h) {
        uint32_t equal = 0;
#pragma unroll
        for (int w = 0; w < DW; ++w) equal += __builtin_popcount(~(sig[w] ^ h[w]));
        uint32_t tier8 = (__umul24(equal, scale) >> 17) & ~7u;
        tier8 = tier8 < top8 ? tier8 : top8;
        packed += 1ull << tier8;
    };
    auto flush = [&]() {
#pragma unroll
        for (int j = 0; j < LSH_MAX_TIERS; ++j) total[j] += (uint32_t)(packed >> (8 * j)) & 255u;
        packed = 0;
    };
    constexpr int UNROLL = 16, PER_FLUSH = 15;              // 240 increments at most between flushes
    int t = 0;
    while (t + UNROLL <= L) {
        const int stop = min(L - UNROLL + 1, t + UNROLL * PER_FLUSH);
        for (; t < stop; t += UNROLL) {
            uint32_t h[UNROLL * DW];
#pragma unroll
            for (int u = 0; u < UNROLL * DW; ++u) h[u] = hs[(size_t)t * DW + u];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) visit(h + u * DW);
        }
        flush();
    }
    for (; t < L; ++t) {
        uint32_t h[DW];
#pragma unroll
        for (int w = 0; w < DW; ++w) h[w] = hs[(size_t)t * DW + w];
        visit(h);
    }
    flush();
    if (live) {
        int32_t *o = rd.tier_out + (size_t)local * m.n_tiers;
        for (int j = 0; j < m.n_tiers; ++j) o[j] = ok ? (int32_t)total[j] : -1;
    }
}

hipError_t launch_lsh_simtier(const LshModel &m, const LshBatch &b, const uint8_t *sig_table, hipStream_t s)
{
    if (b.n_blk == 0) return hipSuccess;
    const dim3 grid(b.n_blk), block(256);
    switch (m.d_bits / 32) {
    case 1: hipLaunchKernelGGL(k_lsh_simtier<1>, grid, block, 0, s, m, b, sig_table); break;
    case 2: hipLaunchKernelGGL(k_lsh_simtier<2>, grid, block, 0, s, m, b, sig_table); break;
    case 3: hipLaunchKernelGGL(k_lsh_simtier<3>, grid, block, 0, s, m, b, sig_table); break;
    case 4: hipLaunchKernelGGL(k_lsh_simtier<4>, grid, block, 0, s, m, b, sig_table); break;
    case 5: hipLaunchKernelGGL(k_lsh_simtier<5>, grid, block, 0, s, m, b, sig_table); break;
    case 6: hipLaunchKernelGGL(k_lsh_simtier<6>, grid, block, 0, s, m, b, sig_table); break;
    case 7: hipLaunchKernelGGL(k_lsh_simtier<7>, grid, block, 0, s, m, b, sig_table); break;
    case 8: hipLaunchKernelGGL(k_lsh_simtier<8>, grid, block, 0, s, m, b, sig_table); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace aif
