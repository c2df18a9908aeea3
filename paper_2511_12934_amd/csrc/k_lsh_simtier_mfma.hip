// Eq. 6, 7, 9 with the similarity on the matrix cores.
//
// The number of equal bits of two d'-bit signatures is a contraction: with the bits written as +1 / -1 their dot
// product is (equal - unequal), so 2 * equal = d' + dot.  One v_mfma_i32_32x32x32_i8 forms 32 x 32 of those dots over
// 32 bits; started from an accumulator of d' it leaves 2 * equal in every cell.  The candidates are the columns (a
// lane owns one candidate and holds 16 history items' values of it), the history items the rows: their +1 / -1 bytes
// are written once per request by k_lsh_expand in the order the instruction reads them, and every wave streams them
// from there.  Only the product over ALL bits matters, so any assignment of bits to the instruction's k index serves,
// as long as rows and columns use the same one.
//
// What is left per (candidate, history item) is Eq. 9's count into tiers, and the vector ALU is what binds, so it is
// done on four values at a time.  N divides 2 d' to a power of two here, so tier = (2 * equal) >> SH; the candidates'
// bytes are +-2^(8 - SH) instead of +-1, which puts the tier into the SECOND BYTE of the 32-bit cell.  Two byte permutes
// and an OR bring the tiers of four cells into one word, a third permute (a table of eight bytes) turns them into
// four one-hot bytes, and the words of one-hot bytes are summed bit position by bit position in a network of
// carry-save adders (two 3-input bit operations each) whose planes hold the counts in binary.  The planes are read
// out with population counts at the end (or every 960 words).  About 1.7 vector instructions per value instead of 10.
// Two corrections at the end: the rows past the history's end are zero vectors, which count as d' / 2 equal bits and
// are taken off that tier again; a signature equal to the candidate's in every bit gives tier index N, whose one-hot
// byte is empty -- the last tier's count is the history length less all the others.
#include "aif_lsh_dev.h"

namespace aif {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int SMT_PART_BLOCKS = 2048; // a batch of fewer blocks than this has its histories cut into parts, a block each
constexpr int SMT_MAX_PARTS = 16;
constexpr int SMT_GROUP = 4;         // row tiles (32 history items each) per pass of the adder network
constexpr int SMT_PLANES = 6;        // planes of weight 16 .. 512 above the network's ones, twos, fours, eights
constexpr int SMT_FLUSH = 60;        // passes between read-outs: 60 * 16 words (+ 12 of a ragged end) <= 1023, what ten planes count

// sixteen signature bits -> sixteen bytes of +scale (bit set) or -scale, bit j in byte j
__device__ __forceinline__ v4i signed_bytes(uint32_t bits16, uint32_t scale)
{
    const uint32_t minus = (0x100u - scale) * 0x01010101u, flip = scale ^ (0x100u - scale);
    v4i r;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t x = (((bits16 >> (4 * q)) & 15u) * 0x00204081u) & 0x01010101u;      // bit i of the four in byte i
        r[q] = (int)(minus ^ (x * flip));                                                   // 1 -> scale, 0 -> 256 - scale
    }
    return r;
}

// The history of every request as the instruction's row operand: [row tile][k-step][lane] of 16 bytes; lane = (row of
// the tile, which half of the k-step's 32 bits).  Rows past the end are zero vectors.
template <int KS>
__global__ __launch_bounds__(256) void k_lsh_expand(LshBatch b, v4i *__restrict__ out, size_t req_stride)
{
    const LshReqDesc rd = b.reqs[blockIdx.y];
    const int nrt = (rd.seq_len + 31) / 32;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= nrt * KS * 64) return;
    const int lane = idx & 63, s = (idx >> 6) % KS, rt = idx / (64 * KS);
    const int row = rt * 32 + (lane & 31), h = lane >> 5;
    v4i v = {0, 0, 0, 0};
    if (row < rd.seq_len) {
        const uint32_t w = ((const uint32_t *)rd.seq_sigs)[(size_t)row * KS + s];
        v = signed_bytes((w >> (16 * h)) & 0xFFFFu, 1u);
    }
    out[(size_t)blockIdx.y * req_stride + idx] = v;
}

__device__ __forceinline__ void csa(uint32_t &sum, uint32_t &carry, uint32_t a, uint32_t b, uint32_t c)
{
    sum = __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);          // a ^ b ^ c
    carry = __builtin_amdgcn_bitop3_b32(a, b, c, 0xE8);        // majority
}

// The counts of one candidate as they come out of the planes -> Eq. 9's tiers.  Two corrections: the rows past the
// history's end were zero vectors and counted as d' / 2 equal bits; the last tier is the history less all the others.
__device__ __forceinline__ void simtier_store(const LshModel &m, const LshReqDesc &rd, int local, int sh, const int32_t (&n)[LSH_MAX_TIERS])
{
    const int64_t id = rd.cand_ids[local];
    int32_t *o = rd.tier_out + (size_t)local * m.n_tiers;
    if (id < 0 || id >= m.n_items) {
        for (int t = 0; t < m.n_tiers; ++t) o[t] = -1;
        return;
    }
    const int pad_tier = m.d_bits >> sh, pad = (rd.seq_len + 31) / 32 * 32 - rd.seq_len;
    int32_t below = 0;
#pragma unroll
    for (int t = 0; t < LSH_MAX_TIERS; ++t) {
        if (t < m.n_tiers - 1) {
            const int32_t v = n[t] - (t == pad_tier ? pad : 0);
            o[t] = v;
            below += v;
        }
    }
    o[m.n_tiers - 1] = rd.seq_len - below;
}

// KS: k-steps of 32 bits (d' = 32 KS); COLS: column tiles of 32 candidates a wave keeps (its candidates' operands stay in
// registers: 4 COLS KS of them).  The block's 256 candidates are 8 / COLS groups of columns; where that leaves waves over
// (COLS = 4) two waves share a group and halve the history.  gridDim.y > 1: the history is cut into that many parts as
// well, a block each, and the counts go to `parts` [part][candidate slot][tier] for k_lsh_simtier_finish -- for batches
// too small to fill the chip otherwise (a handful of users with long histories).
// Every wave reads its row tiles from L2 itself: with 128-bit signatures (4 KB a tile) that stream, not the vector ALU,
// is what binds, and four column tiles a wave (a tile's bytes serve 128 candidates, two tiles in flight) is what the
// registers allow.
template <int KS, int COLS>
__global__ __launch_bounds__(256, 2) void k_lsh_simtier_mfma(LshModel m, LshBatch b, const uint8_t *__restrict__ sig_table,
                                                             const v4i *__restrict__ hist, size_t req_stride, int sh,
                                                             int32_t *__restrict__ parts)
{
    constexpr int SMT_COLS = COLS, GROUPS = 8 / COLS, SHARE = 4 / GROUPS;      // waves that share a group of columns
    static_assert(COLS == 2 || COLS == 4, "column tiles per wave");
    __shared__ int32_t cnt[LSH_MAX_TIERS][LSH_BLOCK];
    // as in the vector-ALU kernel: the blocks of one user go to one XCD, whose L2 then holds that user's history
    int blk = blockIdx.x;
    {
        const int per_xcd = b.n_blk >> 3;
        if (blk < 8 * per_xcd) blk = (blk & 7) * per_xcd + (blk >> 3);
    }
    const int r = b.blk_req[blk];
    if (r < 0) return;
    const LshReqDesc rd = b.reqs[r];
    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, h = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);             // the same in every lane: the loop's bounds are scalars
    const int cg = wave % GROUPS, hh = wave / GROUPS;   // which candidates of the block, which share of the history
    const int first = blk * LSH_BLOCK - rd.cand_base;

    // column operand: this lane's half of each k-step's 32 bits, for its candidate in each of the column tiles
    v4i bf[SMT_COLS][KS];
#pragma unroll
    for (int ct = 0; ct < SMT_COLS; ++ct) {
        const int local = first + cg * (SMT_COLS * 32) + ct * 32 + col;
        int64_t id = local < rd.n_cand ? rd.cand_ids[local] : 0;
        if (id < 0 || id >= m.n_items) id = 0;
        const uint32_t *p = (const uint32_t *)(sig_table + (size_t)id * (KS * 4));
#pragma unroll
        for (int s = 0; s < KS; ++s) bf[ct][s] = signed_bytes((p[s] >> (16 * h)) & 0xFFFFu, 1u << (8 - sh));
    }
#pragma unroll
    for (int t = 0; t < LSH_MAX_TIERS; ++t) cnt[t][tid] = 0;
    __syncthreads();

    const int nrt = (rd.seq_len + 31) / 32;
    const int per_part = (nrt + (int)gridDim.y - 1) / (int)gridDim.y;          // row tiles of this block ...
    const int part_begin = min(nrt, (int)blockIdx.y * per_part), part_end = min(nrt, part_begin + per_part);
    const int per_wave = (part_end - part_begin + SHARE - 1) / SHARE;           // ... and of this wave
    const int rt_begin = min(part_end, part_begin + hh * per_wave), rt_end = min(part_end, rt_begin + per_wave);
    const v4i *__restrict__ hrow = hist + (size_t)r * req_stride + lane;

    // one-hot byte of tier t: bit t; the permute's selectors 0..3 take the second operand's bytes, 4..7 the first's
    constexpr uint32_t HOT_LO = 0x08040201u, HOT_HI = 0x80402010u;
    uint32_t ones[SMT_COLS], twos[SMT_COLS], fours[SMT_COLS], eights[SMT_COLS], plane[SMT_COLS][SMT_PLANES];
#pragma unroll
    for (int ct = 0; ct < SMT_COLS; ++ct) {
        ones[ct] = twos[ct] = fours[ct] = eights[ct] = 0;
#pragma unroll
        for (int j = 0; j < SMT_PLANES; ++j) plane[ct][j] = 0;
    }
    auto read_out = [&]() {
#pragma unroll
        for (int ct = 0; ct < SMT_COLS; ++ct) {
            const int cand = cg * (SMT_COLS * 32) + ct * 32 + col;
#pragma unroll
            for (int t = 0; t < LSH_MAX_TIERS; ++t) {
                const uint32_t mask = 0x01010101u << t;
                uint32_t n = __builtin_popcount(ones[ct] & mask) + 2 * __builtin_popcount(twos[ct] & mask) +
                             4 * __builtin_popcount(fours[ct] & mask) + 8 * __builtin_popcount(eights[ct] & mask);
#pragma unroll
                for (int j = 0; j < SMT_PLANES; ++j) n += (uint32_t)__builtin_popcount(plane[ct][j] & mask) << (4 + j);
                if (n) atomicAdd(&cnt[t][cand], (int32_t)n);
            }
            ones[ct] = twos[ct] = fours[ct] = eights[ct] = 0;
#pragma unroll
            for (int j = 0; j < SMT_PLANES; ++j) plane[ct][j] = 0;
        }
    };

    // The one-hot words of one row tile against column tile ct.  The cells start from d' * 2^(8 - SH) and end as
    // (2 * equal) << (8 - SH): their second byte is the tier.  The start value is kept in registers of its own (it is
    // no inline constant; formed anew it would cost an instruction per cell).
    v16i start;
#pragma unroll
    for (int i = 0; i < 16; ++i) start[i] = (32 * KS) << (8 - sh);
#pragma unroll
    for (int i = 0; i < 16; ++i) asm volatile("" : "+v"(start[i]));
    auto tile_words = [&](const v4i(&af)[KS], int ct, uint32_t(&w)[4]) {
        v16i acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[0], bf[ct][0], start, 0, 0, 0);
#pragma unroll
        for (int s = 1; s < KS; ++s) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[s], bf[ct][s], acc, 0, 0, 0);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            // second bytes of cells 4q, 4q + 1 into bytes 0, 1 and of 4q + 2, 4q + 3 into bytes 2, 3 (selector 12: a zero byte)
            const uint32_t lo = __builtin_amdgcn_perm((uint32_t)acc[4 * q + 1], (uint32_t)acc[4 * q], 0x0C0C0501u);
            const uint32_t hi = __builtin_amdgcn_perm((uint32_t)acc[4 * q + 3], (uint32_t)acc[4 * q + 2], 0x05010C0Cu);
            w[q] = __builtin_amdgcn_perm(HOT_HI, HOT_LO, lo | hi);
        }
    };
    auto load_rows = [&](int rt, v4i(&af)[KS]) {
#pragma unroll
        for (int s = 0; s < KS; ++s) af[s] = hrow[(size_t)(rt * KS + s) * 64];
    };

    int passes = 0, rt0 = rt_begin;
    // a row tile is asked for AHEAD tiles before its turn, into the registers of the tile just read (past the last
    // whole pass the last tile is asked for again)
    constexpr int AHEAD = KS * COLS > 8 ? 2 : SMT_GROUP;        // the registers a long signature's operands leave
    static_assert(SMT_GROUP % AHEAD == 0, "a tile's registers are the same in every pass");
    v4i rows[AHEAD][KS];
    const int rt_last = rt_begin + (rt_end - rt_begin) / SMT_GROUP * SMT_GROUP - 1;      // of the whole passes
    if (rt0 + SMT_GROUP <= rt_end)
#pragma unroll
        for (int u = 0; u < AHEAD; ++u) load_rows(rt0 + u, rows[u]);
    for (; rt0 + SMT_GROUP <= rt_end; rt0 += SMT_GROUP) {
        uint32_t f[SMT_COLS], e[SMT_COLS];                      // carries of weight 4 and 8 waiting for their partner
#pragma unroll
        for (int u = 0; u < SMT_GROUP; ++u) {
            uint32_t w[SMT_COLS][4];
#pragma unroll
            for (int ct = 0; ct < SMT_COLS; ++ct) tile_words(rows[u % AHEAD], ct, w[ct]);
            load_rows(min(rt0 + u + AHEAD, rt_last), rows[u % AHEAD]);
#pragma unroll
            for (int ct = 0; ct < SMT_COLS; ++ct) {
                uint32_t ca, cb, fu;
                csa(ones[ct], ca, ones[ct], w[ct][0], w[ct][1]);
                csa(ones[ct], cb, ones[ct], w[ct][2], w[ct][3]);
                csa(twos[ct], fu, twos[ct], ca, cb);
                if (u % 2 == 0)
                    f[ct] = fu;
                else {
                    uint32_t eu;
                    csa(fours[ct], eu, fours[ct], f[ct], fu);
                    if (u == 1)
                        e[ct] = eu;
                    else {
                        uint32_t up;                            // weight 16: rippled into the planes
                        csa(eights[ct], up, eights[ct], e[ct], eu);
#pragma unroll
                        for (int j = 0; j < SMT_PLANES; ++j) {
                            const uint32_t next = plane[ct][j] & up;
                            plane[ct][j] ^= up;
                            up = next;
                        }
                    }
                }
            }
        }
        if (++passes == SMT_FLUSH) {
            read_out();
            passes = 0;
        }
    }
    // the last one to three row tiles: every word rippled through all the planes (16 more words: still within what they count)
    for (; rt0 < rt_end; ++rt0) {
        v4i af[KS];
        load_rows(rt0, af);
#pragma unroll
        for (int ct = 0; ct < SMT_COLS; ++ct) {
            uint32_t w[4];
            tile_words(af, ct, w);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint32_t up = w[q], next;
                next = ones[ct] & up, ones[ct] ^= up, up = next;
                next = twos[ct] & up, twos[ct] ^= up, up = next;
                next = fours[ct] & up, fours[ct] ^= up, up = next;
                next = eights[ct] & up, eights[ct] ^= up, up = next;
#pragma unroll
                for (int j = 0; j < SMT_PLANES; ++j) {
                    next = plane[ct][j] & up;
                    plane[ct][j] ^= up;
                    up = next;
                }
            }
        }
    }
    read_out();
    __syncthreads();

    const int local = first + tid;
    if (gridDim.y > 1) {            // raw counts; the slot exists whether or not a candidate sits in it
        int32_t *o = parts + ((size_t)blockIdx.y * b.n_blk * LSH_BLOCK + (size_t)blk * LSH_BLOCK + tid) * LSH_MAX_TIERS;
#pragma unroll
        for (int t = 0; t < LSH_MAX_TIERS; ++t) o[t] = cnt[t][tid];
        return;
    }
    if (local >= rd.n_cand) return;
    int32_t n[LSH_MAX_TIERS];
#pragma unroll
    for (int t = 0; t < LSH_MAX_TIERS; ++t) n[t] = cnt[t][tid];
    simtier_store(m, rd, local, sh, n);
}

__global__ __launch_bounds__(256) void k_lsh_simtier_finish(LshModel m, LshBatch b, int sh, const int32_t *__restrict__ parts, int n_parts)
{
    const int blk = blockIdx.x, r = b.blk_req[blk];
    if (r < 0) return;
    const LshReqDesc rd = b.reqs[r];
    const int local = blk * LSH_BLOCK - rd.cand_base + (int)threadIdx.x;
    if (local >= rd.n_cand) return;
    int32_t n[LSH_MAX_TIERS];
#pragma unroll
    for (int t = 0; t < LSH_MAX_TIERS; ++t) n[t] = 0;
    for (int p = 0; p < n_parts; ++p) {
        const int4 *q = (const int4 *)(parts + ((size_t)p * b.n_blk * LSH_BLOCK + (size_t)blk * LSH_BLOCK + threadIdx.x) * LSH_MAX_TIERS);
        const int4 lo = q[0], hi = q[1];
        n[0] += lo.x, n[1] += lo.y, n[2] += lo.z, n[3] += lo.w;
        n[4] += hi.x, n[5] += hi.y, n[6] += hi.z, n[7] += hi.w;
    }
    simtier_store(m, rd, local, sh, n);
}

static int simtier_shift(const LshModel &m)                     // 2 d' / N = 2^shift, or -1
{
    int sh = 0;
    while (sh < 9 && (1 << sh) * m.n_tiers < 2 * m.d_bits) ++sh;
    return (1 << sh) * m.n_tiers == 2 * m.d_bits ? sh : -1;
}

bool lsh_simtier_on_mfma(const LshModel &m)
{
    static_assert(LSH_MAX_TIERS == 8, "eight one-hot bits a byte, eight counts a slot");
    const int sh = simtier_shift(m);
    // the candidates' bytes are +-2^(8 - shift): at least 1
    return (m.d_bits == 32 || m.d_bits == 64 || m.d_bits == 128) && sh >= 0 && sh <= 8;
}

size_t lsh_hist_stride(const LshModel &m, int max_seq_len)      // 16-byte pieces per request
{
    return (size_t)((max_seq_len + 31) / 32) * (m.d_bits / 32) * 64;
}

size_t lsh_simtier_parts_bytes() { return (size_t)(SMT_PART_BLOCKS + SMT_MAX_PARTS) * LSH_BLOCK * LSH_MAX_TIERS * 4; }

hipError_t launch_lsh_simtier_mfma(const LshModel &m, const LshBatch &b, const uint8_t *sig_table, void *hist, size_t req_stride,
                                   int longest, void *parts, hipStream_t s)
{
    if (b.n_blk == 0) return hipSuccess;
    if (!lsh_simtier_on_mfma(m) || !hist || !parts) return hipErrorInvalidValue;
    const int sh = simtier_shift(m);
    const int ks = m.d_bits / 32;
    const int nrt = (longest + 31) / 32, pieces = nrt * ks * 64;
    if (pieces > 0) {
        const dim3 grid((pieces + 255) / 256, b.n_req);
        switch (ks) {
        case 1: hipLaunchKernelGGL(k_lsh_expand<1>, grid, dim3(256), 0, s, b, (v4i *)hist, req_stride); break;
        case 2: hipLaunchKernelGGL(k_lsh_expand<2>, grid, dim3(256), 0, s, b, (v4i *)hist, req_stride); break;
        default: hipLaunchKernelGGL(k_lsh_expand<4>, grid, dim3(256), 0, s, b, (v4i *)hist, req_stride); break;
        }
    }
    // parts: enough blocks to fill the chip a few times over, each with at least two passes of the adder network per wave
    int n_parts = SMT_PART_BLOCKS / b.n_blk;
    n_parts = n_parts < nrt / (4 * SMT_GROUP) ? n_parts : nrt / (4 * SMT_GROUP);
    n_parts = n_parts > SMT_MAX_PARTS ? SMT_MAX_PARTS : n_parts < 1 ? 1 : n_parts;
    const dim3 grid(b.n_blk, n_parts);
    int32_t *pp = (int32_t *)parts;
    switch (ks) {
    case 1: hipLaunchKernelGGL((k_lsh_simtier_mfma<1, 4>), grid, dim3(256), 0, s, m, b, sig_table, (const v4i *)hist, req_stride, sh, pp); break;
    case 2: hipLaunchKernelGGL((k_lsh_simtier_mfma<2, 4>), grid, dim3(256), 0, s, m, b, sig_table, (const v4i *)hist, req_stride, sh, pp); break;
    default: hipLaunchKernelGGL((k_lsh_simtier_mfma<4, 4>), grid, dim3(256), 0, s, m, b, sig_table, (const v4i *)hist, req_stride, sh, pp); break;
    }
    if (n_parts > 1) hipLaunchKernelGGL(k_lsh_simtier_finish, dim3(b.n_blk), dim3(256), 0, s, m, b, sh, (const int32_t *)pp, n_parts);
    return hipGetLastError();
}

}  // namespace aif
