// a3-a5 on the matrix cores for models with a query projection and 16-wide
// heads -- q = W_q e (the reading of Eq. 1's projection for the candidate
// side), target attention of every candidate over the request's behaviour
// sequence, Softmax(q K^T / sqrt(d_h)) V per head (operator of Eq. 3 with the
// candidate as the query), and the real-time half of the cross features
// (Sec. 3.3): Hadamard, or the dot products of the request's cross vectors
// with the segments of the item vector.
//
// As in k_attn_mfma everything is formed transposed so that a lane owns ONE
// candidate (column c = lane % 32, half h = lane / 32):
//   Q^T = W_q E^T      A = 32 query features x 16 item features, B = the row's 16-byte pieces
//   S^T = K q^T        A = 32 keys x 16 (one head), B = the head's query
//   O^T = V^T P^T      A = [16 features of the head ; a row of ones ; zeros] x 16 keys, B = the probabilities
// A 32x32 result leaves rows 8 (i / 4) + 4 h + i % 4 in register i of lane (c, h).
// The contraction index of a product may be assigned to (half, slot) in any
// way as long as both operands agree, so
//   - registers 8 (hd % 2) .. + 7 of feature tile hd / 2 of Q^T are, as they
//     stand, the B operand of head hd's score product (K is packed with its
//     16 dimensions in that order),
//   - the sixteen probabilities of a key tile are two k-steps of the B operand
//     of the second product (V packed in that key order), as in k_attn_mfma.
// With 16-wide heads the vector ALU (one exponential per score) is what binds,
// not the matrix cores, so the matrix cores take everything they can:
//   - the query is scaled by log2(e) / sqrt(d_h) before it is rounded to bf16,
//     and the score product accumulates onto -bound, so the product's result
//     is the exponent itself (no multiply-add per score);
//   - the sixteen empty rows of the second product's A operand hold a row of
//     ones: row 16 of O^T is the softmax denominator (no add per score), and
//     it is the sum of the ROUNDED probabilities, the weights that multiply V;
//   - ones and V are zero for keys past the end of the sequence: no masking.
// What is left per score is one v_exp_f32 and half a bf16 conversion.
//
// bound = |q'| max_t |k_t| >= every score (Cauchy-Schwarz) replaces the running
// maximum; when it is large enough to risk underflow the wave takes the true
// maximum in an extra pass over K.  Both are the exact softmax up to rounding.
//
// K/V packed per request (k_pack_kv16) stream through a three-slot ring in
// LDS, eight 32-key tiles (24 KB) per stage, by direct-to-LDS loads.
#include <cstdlib>
#include "k_mfma.h"
#include "k_stage.h"
#include "mfma_util.h"

namespace aif {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2p __attribute__((ext_vector_type(2)));

namespace {

constexpr float P_LOG2E = 1.4426950408889634f;
constexpr float P_BOUND_LIMIT = 57.f;        // in log2 units: exponents stay within [-114, 0]
constexpr int P_NT = 8;                      // key tiles per stage
constexpr int P_STAGE_FRAGS = 3 * P_NT;      // K, V of keys 0-15, V of keys 16-31 per tile
constexpr int P_STAGE_BYTES = P_STAGE_FRAGS * 1024;
constexpr int P_SLOTS = 3, P_DIST = P_SLOTS - 1;
constexpr int P_MAX_HEADS = 32;
constexpr int P_MAX_CROSS_FRAGS = 4;         // d_cross_vec <= 64
constexpr int P_LDS_BYTES = P_SLOTS * P_STAGE_BYTES + P_MAX_HEADS * 4 + P_MAX_CROSS_FRAGS * 1024;

__device__ __forceinline__ void store_stream4(void *p, bf16x4 v)
{
    __builtin_nontemporal_store(__builtin_bit_cast(u32x2p, v), (u32x2p *)p);
}

// ---------------------------------------------------------------------------
// a2 -- K and V of request r, head hd, stage st (P_NT key tiles) into fragment order, and the largest
// key norm of the stage.  Per request: chunk(head, key tile kt) = 3 fragments of 1 KB at
// ((head * nktp + kt) * 3) KB, with o = 16 head:
//   K:      [lane][s] = K[32 kt + lane % 32][o + 8 (s / 4) + 4 (lane / 32) + s % 4]
//   V, jj:  [lane][s] = row lane % 32 of [V^T ; 1 ; 0] at key 32 kt + 16 jj + 8 (s / 4) + 4 (lane / 32) + s % 4
// Keys >= seq_len read as zero in all rows, the row of ones included; a stage is written whole, so the
// tiles between the end of the sequence and the end of its last stage are zero and add nothing.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void pack_kv16_block(int st, int hd, int r, const Model &m, const Batch &b, char *__restrict__ kvpack,
                                                size_t pack_stride, float *__restrict__ kmax, int nktp)
{
    __shared__ float red[4];
    // r: the user slot (one pack per distinct user of the call)
    const ReqDesc *rd = b.reqs + slot_request(b, r);
    const int L = rd->seq_len, nkt = (L + 31) >> 5;
    if (P_NT * st >= nkt) return;
    const uint16_t *K = (const uint16_t *)rd->seq_keys, *V = (const uint16_t *)rd->seq_vals;
    const int da = m.d_attn, o = hd * 16;
    uint4 *dst = (uint4 *)(kvpack + (size_t)r * pack_stride + ((size_t)(hd * nktp + P_NT * st) * 3) * 1024);
    // V is needed transposed (a lane holds eight keys of ONE feature), which read straight from memory is eight 2-byte
    // loads at the row stride per piece.  Instead a thread brings its key's 32-byte slice of V into LDS (thread = key of
    // the stage; a key past the sequence's end re-reads the last key and is zeroed on the way out) and the pieces are
    // put together from there.  K's pieces are 16 contiguous bytes of a row each: all asked for before the barrier too,
    // none under a condition of its own, so the block makes one trip to memory.
    __shared__ __align__(16) uint16_t sv[32 * P_NT][16];
    const int Lm = L - 1;                                   // L >= 1 here (the stage has a key tile)
    constexpr int TRIPS = P_STAGE_FRAGS * 64 / 256;
    static_assert(P_STAGE_FRAGS * 64 % 256 == 0 && 32 * P_NT == 256, "whole trips; a key per thread");
    {
        const uint4 *vr = (const uint4 *)(V + (size_t)min(32 * P_NT * st + (int)threadIdx.x, Lm) * da + o);
        const uint4 v0 = vr[0], v1 = vr[1];
        *(uint4 *)&sv[threadIdx.x][0] = v0;
        *(uint4 *)&sv[threadIdx.x][8] = v1;
    }
    uint2 klo[TRIPS], khi[TRIPS];
#pragma unroll
    for (int it = 0; it < TRIPS; ++it) {
        const int pc = threadIdx.x + 256 * it;
        const int tl = pc / 192, rem = pc - tl * 192, lane = rem & 63;
        const int kt = P_NT * st + tl, hh = lane >> 5, row = lane & 31;
        const uint16_t *kr = K + (size_t)min(32 * kt + row, Lm) * da + o;     // (asked for by the V pieces' lanes too: no condition)
        klo[it] = *(const uint2 *)(kr + 4 * hh);
        khi[it] = *(const uint2 *)(kr + 8 + 4 * hh);
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < TRIPS; ++it) {
        const int pc = threadIdx.x + 256 * it;
        const int tl = pc / 192, rem = pc - tl * 192, frag = rem >> 6, lane = rem & 63;
        const int kt = P_NT * st + tl, hh = lane >> 5, row = lane & 31;
        uint4 out = make_uint4(0, 0, 0, 0);
        if (frag == 0) {
            if (32 * kt + row < L) out = make_uint4(klo[it].x, klo[it].y, khi[it].x, khi[it].y);
        } else if (row <= 16) {
            const int t0 = 32 * kt + 16 * (frag - 1) + 4 * hh, s0 = t0 - 32 * P_NT * st, f = min(row, 15);
            uint32_t w[4];
#pragma unroll
            for (int p2 = 0; p2 < 4; ++p2) {                // slots 2 p2 and 2 p2 + 1 <-> keys t0 + 8 (p2 / 2) + 2 (p2 % 2) and the next
                const int d = 8 * (p2 >> 1) + 2 * (p2 & 1), ta = t0 + d, tb = ta + 1;
                const uint32_t lo = ta < L ? (row < 16 ? (uint32_t)sv[s0 + d][f] : 0x3F80u) : 0u;
                const uint32_t hi = tb < L ? (row < 16 ? (uint32_t)sv[s0 + d + 1][f] : 0x3F80u) : 0u;
                w[p2] = lo | (hi << 16);
            }
            out = make_uint4(w[0], w[1], w[2], w[3]);
        }
        dst[pc] = out;
    }
    // largest key norm among this stage's 256 keys
    {
        const int t = 32 * P_NT * st + threadIdx.x;
        float ss = 0.f;
        if (t < L) {
            const uint4 *kr = (const uint4 *)(K + (size_t)t * da + o);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const uint4 q = kr[i];
                const uint32_t ws[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float a0 = __uint_as_float(ws[j] << 16), a1 = __uint_as_float(ws[j] & 0xFFFF0000u);
                    ss += a0 * a0 + a1 * a1;
                }
            }
        }
        float nrm = sqrtf(ss);
#pragma unroll
        for (int off = 32; off; off >>= 1) nrm = fmaxf(nrm, __shfl_xor(nrm, off, 64));
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = nrm;
        __syncthreads();
        // rounded up a little: the bound must dominate the fp32-accumulated score
        if (threadIdx.x == 0)
            kmax[((size_t)r * m.n_heads + hd) * (nktp / P_NT) + st] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])) * 1.001f;
    }
}

__global__ __launch_bounds__(256) void k_pack_kv16(Model m, Batch b, char *__restrict__ kvpack, size_t pack_stride,
                                                   float *__restrict__ kmax, int nktp)
{
    pack_kv16_block(blockIdx.x, blockIdx.y, blockIdx.z, m, b, kvpack, pack_stride, kmax, nktp);
}

// The user-side staging of a call as ONE launch: K/V packing, user fold and (Model::cross_in_mlp == 2) the users'
// layer-1 weights are independent of one another and small -- one after the other they are three launches' worth
// of latency in front of the attention kernel.
struct StageProjArgs {
    Model m;
    Batch b;
    char *kvpack;
    size_t pack_stride;
    float *kmax;
    int32_t nktp, stages;
    const float *w1u, *b1;
    float *bias1;
    int32_t quads;
    int32_t n_pack, n_fold, n_w0;       // blocks of the three jobs
    FoldW0 w0;
};
__global__ __launch_bounds__(256) void k_stage_proj(StageProjArgs a)
{
    int idx = blockIdx.x;
    if (idx < a.n_pack) {
        const int st = idx % a.stages, rest = idx / a.stages;
        pack_kv16_block(st, rest % a.m.n_heads, rest / a.m.n_heads, a.m, a.b, a.kvpack, a.pack_stride, a.kmax, a.nktp);
        return;
    }
    idx -= a.n_pack;
    if (idx < a.n_fold) {
        user_fold_block<uint16_t>(idx / a.quads, idx % a.quads, a.m, TableReqs{a.b}, a.w1u, a.b1, a.bias1);
        return;
    }
    idx -= a.n_fold;
    if (idx < a.n_w0) fold_w0_block(idx / a.w0.blocks_per_slot, idx % a.w0.blocks_per_slot, a.m, TableReqs{a.b}, a.w0);
}

// ---------------------------------------------------------------------------
// projection + attention + cross.  One wave = 32 candidates, all heads in turn.
// NFT = d_attn / 32 feature tiles of the query = n_heads / 2.
// ---------------------------------------------------------------------------
// GATHER: the kernel is also a1 (Sec. 3.2): a lane takes the pieces of its candidate's item vector from the table
// row its id names instead of the workspace, and sets them down in the workspace for the MLP after the projection
// has read them.  An id outside the table reads row 0 and is counted, as in the gather kernel.
template <int NFT, int WAVES, bool GATHER>
__global__ __launch_bounds__(WAVES * 64, 4) void k_attn_proj(Model m, Batch b, char *__restrict__ X, XLayout xl,
                                                         const char *__restrict__ wq_pack,
                                                         const char *__restrict__ kvpack, size_t pack_stride,
                                                         const float *__restrict__ kmax, int nktp,
                                                         const char *__restrict__ table, int32_t *__restrict__ bad)
{
    constexpr int ROWS = WAVES * 32, H = 2 * NFT;
    static_assert(ROW_BLOCK % ROWS == 0, "tile");
    static_assert(P_STAGE_FRAGS % WAVES == 0, "every wave issues the same number of loads");
    static_assert(P_DIST == 2, "the ring is primed with two stages, one before and one after the cross block");
    extern __shared__ __align__(16) char lds[];
    float *skm = (float *)(lds + P_SLOTS * P_STAGE_BYTES);         // [H] max |k_t|
    bf16x8 *sa = (bf16x8 *)(skm + P_MAX_HEADS);                    // cross vectors as A fragments

    // every XCD (own L2) takes a contiguous run of tiles, so the blocks that stream one request's K/V share an L2
    const int per_xcd = gridDim.x >> 3;
    const int bid = blockIdx.x;
    const int tile = bid < 8 * per_xcd ? (bid & 7) * per_xcd + (bid >> 3) : bid;
    const int row0 = tile * ROWS;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), col = lane & 31, h = lane >> 5;
    char *xrow = X + x_offset(xl, row0 + wave * 32 + col, 0);
    auto piece = [&](int p) { return (bf16x8 *)(xrow + (size_t)p * xl.piece_stride); };

    const int r = b.blk_req[tile / (ROW_BLOCK / ROWS)];
    if (r < 0) return;
    const ReqDesc rd = b.reqs[r];
    const int local0 = row0 - rd.row_base;
    if (rd.n_cand - local0 <= 0) return;

    const int L = rd.seq_len;
    const int nkt = (L + 31) >> 5, nst = (nkt + P_NT - 1) / P_NT, total = H * nst, nstp = nktp / P_NT;
    const int us = rd.slot;                       // K/V and key norms are kept per user, not per slice
    const char *pk = kvpack + (size_t)us * pack_stride;
    const bool live = local0 + wave * 32 + col < rd.n_cand;
    const char *trow = nullptr;                   // GATHER: this lane's row of the table (row 0 past the request's end)
    if constexpr (GATHER) {
        int id = live ? rd.cand_ids[local0 + wave * 32 + col] : 0;
        if (id < 0 || (int64_t)id >= m.n_items) {
            if (h == 0) atomicAdd(bad, 1);
            id = 0;
        }
        trow = table + (size_t)id * (size_t)(m.d_item * 2);
    }
    // piece p < d_item / 8 of the lane's item vector
    auto item_piece = [&](int p) -> bf16x8 {
        if constexpr (GATHER) return *(const bf16x8 *)(trow + p * 16);
        else return *piece(p);
    };
    const uint32_t ring = lds_address(lds);
    auto stage_src = [&](int i) {
        const int sh = i / nst, ss = i - sh * nst;
        return pk + ((size_t)(sh * nktp + P_NT * ss) * 3) * 1024;
    };
    auto stage_load = [&](int i) {
        const char *src = stage_src(i) + lane * 16;
        const uint32_t dst = __builtin_amdgcn_readfirstlane(ring + (i % P_SLOTS) * P_STAGE_BYTES);     // (the stage count is the same in every lane)
#pragma unroll
        for (int f0 = 0; f0 < P_STAGE_FRAGS; f0 += WAVES) dma16(src + (f0 + wave) * 1024, dst + (f0 + wave) * 1024);
    };

    // ---- block set-up: W_q into the LDS the ring will take later (its fragments are read by all waves),
    // key-norm bounds, the cross vectors as A fragments -------------------------------------------------
    const int KS = m.d_item / 16;                 // a multiple of 4
    for (int f = wave; f < NFT * KS; f += WAVES) dma16(wq_pack + (size_t)f * 1024 + lane * 16, ring + f * 1024);
    for (int hd = wave; hd < H; hd += WAVES) {
        float km = 0.f;
        for (int i = lane; i < nst; i += 64) km = fmaxf(km, kmax[((size_t)us * H + hd) * nstp + i]);
#pragma unroll
        for (int off = 32; off; off >>= 1) km = fmaxf(km, __shfl_xor(km, off, 64));
        if (lane == 0) skm[hd] = km;
    }
    const int ksc = m.d_cv / 16;                  // SEGDOT: k-steps per segment of the item vector
    const bool segdot = m.cross_mode == 2 && !m.cross_in_mlp;      // else the block is folded into the user's layer-1 weights
    if (segdot) {
        // fragment kk: [lane][s] = Vc[lane % 32][16 kk + 8 (lane / 32) + s], rows >= n_cross zero
        const uint16_t *Vc = (const uint16_t *)rd.cross_vecs;
        uint16_t *sa16 = (uint16_t *)sa;
        for (int i = threadIdx.x; i < ksc * 512; i += WAVES * 64) {
            const int sl = i & 7, ln = (i >> 3) & 63, kk = i >> 9, row = ln & 31;
            sa16[i] = row < m.n_cross ? Vc[(size_t)row * m.d_cv + 16 * kk + 8 * (ln >> 5) + sl] : (uint16_t)0;
        }
    }
    wait_vmcnt<0>();
    __syncthreads();

    // ---- query projection Q^T = W_q E^T; queries of all heads scaled so that the score product yields
    // the exponent to base 2 -------------------------------------------------------------------------
    const int pc_cross = (m.d_item + m.d_attn) / 8;
    bf16x8 q[H];
    {
        f32x16 Q[NFT];
#pragma unroll
        for (int ft = 0; ft < NFT; ++ft)
#pragma unroll
            for (int i = 0; i < 16; ++i) Q[ft][i] = 0.f;
        const bf16x8 *wq = (const bf16x8 *)lds + lane;
        for (int j0 = 0; j0 < KS; j0 += 4) {
            bf16x8 e[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) e[u] = item_piece(2 * (j0 + u) + h);
            if constexpr (GATHER) {
                if (live) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) *piece(2 * (j0 + u) + h) = e[u];
                }
            }
#pragma unroll
            for (int ft = 0; ft < NFT; ++ft)
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    Q[ft] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wq[(ft * KS + j0 + u) * 64], e[u], Q[ft], 0, 0, 0);
        }
        const float cs = P_LOG2E * 0.25f;         // log2(e) / sqrt(16)
#pragma unroll
        for (int hd = 0; hd < H; ++hd)
#pragma unroll
            for (int s = 0; s < 8; ++s) q[hd][s] = (__bf16)(Q[hd >> 1][8 * (hd & 1) + s] * cs);
    }
    __syncthreads();                              // every wave has read W_q: the ring may take its place
    if (total > 0) stage_load(0);

    // ---- the cross block, from the same row pieces (a second pass over them, under the ring's first load) ----
    if (m.cross_mode == 1 && !m.cross_in_mlp && live) {      // unless the MLP chain forms the Hadamard products itself
        const bf16x8 *uc = (const bf16x8 *)rd.cross_vecs;
        for (int pc = h; pc < m.d_item / 8; pc += 2) {
            const bf16x8 e = item_piece(pc), uv = uc[pc];
            bf16x8 o8;
#pragma unroll
            for (int sl = 0; sl < 8; ++sl) o8[sl] = (__bf16)((float)e[sl] * (float)uv[sl]);
            *piece(pc_cross + pc) = o8;
        }
    }
    if (segdot) {
        // A lane ends up with single features of its candidate, 2 bytes each and far apart in the row: they
        // are gathered in LDS (a private strip of the ring's last two slots per wave, rows padded by 16
        // bytes) and leave as whole 16-byte pieces.
        const int nseg = m.d_item / m.d_cv, sstr = m.d_cross * 2 + 16;
        char *scr = lds + P_STAGE_BYTES + wave * (2 * P_STAGE_BYTES / WAVES);
        for (int seg = 0; seg < nseg; ++seg) {
            f32x16 Cc;
#pragma unroll
            for (int i = 0; i < 16; ++i) Cc[i] = 0.f;
            for (int kk0 = 0; kk0 < ksc; kk0 += 4) {
                bf16x8 e[4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (kk0 + u < ksc) e[u] = item_piece(2 * (seg * ksc + kk0 + u) + h);
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (kk0 + u < ksc) Cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sa[(kk0 + u) * 64 + lane], e[u], Cc, 0, 0, 0);
            }
            // cross feature (vector row, segment) sits at column row * nseg + seg of the cross block
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int row = 8 * (i >> 2) + 4 * h + (i & 3);
                if (row < m.n_cross) *(__bf16 *)(scr + col * sstr + (row * nseg + seg) * 2) = (__bf16)Cc[i];
            }
        }
        const int npc = m.d_cross / 8;
        for (int idx = lane; idx < 32 * npc; idx += 64) {
            const int cand = idx & 31, pc = idx >> 5;
            if (local0 + wave * 32 + cand < rd.n_cand)
                *(bf16x8 *)(X + x_offset(xl, row0 + wave * 32 + cand, pc_cross + pc)) = *(const bf16x8 *)(scr + cand * sstr + pc * 16);
        }
    }
    __syncthreads();                              // the strips have been read: the ring's second slot may fill
    if (total > 1) stage_load(1);
    wait_vmcnt<0>();
    __syncthreads();

    const char *kv0 = lds + lane * 16;
    int it = 0;
    // a wave whose 32 rows lie past the request's end (the last block of a request) computes nothing: it only keeps
    // its place in the ring -- its share of every stage's loads and the stage's barrier
    const bool idle = __builtin_amdgcn_readfirstlane((int)(local0 + wave * 32 >= rd.n_cand)) != 0;     // the same in every lane
    if (idle) {
        for (int i = 0; i < total; ++i) {
            wait_vmcnt<0>();
            asm volatile("s_barrier" ::: "memory");
            if (i + P_DIST < total) stage_load(i + P_DIST);
        }
        return;
    }
#pragma unroll
    for (int hd = 0; hd < H; ++hd) {
        float ss = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s) ss += (float)q[hd][s] * (float)q[hd][s];
        ss += __shfl_xor(ss, 32, 64);
        float mc = sqrtf(ss) * 1.001f * skm[hd];
        // per candidate: its bits do not depend on which candidates share its wave
        const bool need_max = live && mc > P_BOUND_LIMIT;
        if (__any(need_max)) {
            // rare: the true maximum, by an extra pass over K read straight from memory
            float mx = -INFINITY;
            for (int kt = 0; kt < nkt; ++kt) {
                f32x16 S;
#pragma unroll
                for (int i = 0; i < 16; ++i) S[i] = 0.f;
                S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(pk + ((size_t)(hd * nktp + kt) * 3) * 1024 + lane * 16),
                                                            q[hd], S, 0, 0, 0);
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int t = 32 * kt + 8 * (v >> 2) + 4 * h + (v & 3);
                    if (t < L) mx = fmaxf(mx, S[v]);
                }
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            if (need_max) mc = mx;
        }
        f32x16 NEG;
#pragma unroll
        for (int i = 0; i < 16; ++i) NEG[i] = -mc;

        f32x16 O;
#pragma unroll
        for (int i = 0; i < 16; ++i) O[i] = 0.f;

        // The head's key tiles are one stream: the score product of tile t + 1 (its K fragment read from
        // LDS a tile ahead) is issued as soon as the last exponential of tile t has read the accumulator,
        // between the two halves of tile t's second product, and runs under them -- across stage
        // boundaries too, because the block's one barrier per stage sits in the MIDDLE of a stage: there
        // stage it + 1 is confirmed (every wave waits for its own share of the loads, then the barrier), and
        // stage it + 2 is sent into the slot of stage it - 1, which every wave has left.  After the last
        // tile of the head the product computed ahead belongs to no one and is dropped.
        bf16x8 Kf = *(const bf16x8 *)(kv0 + (it % P_SLOTS) * P_STAGE_BYTES);
        f32x16 S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Kf, q[hd], NEG, 0, 0, 0);
        for (int st = 0; st < nst; ++st) {
            const char *sb = kv0 + (it % P_SLOTS) * P_STAGE_BYTES;
            const char *sbn = kv0 + ((it + 1) % P_SLOTS) * P_STAGE_BYTES;
#pragma unroll
            for (int tl = 0; tl < P_NT; ++tl) {
                const bf16x8 V0 = *(const bf16x8 *)(sb + tl * 3072 + 1024);
                const bf16x8 V1 = *(const bf16x8 *)(sb + tl * 3072 + 2048);
                Kf = *(const bf16x8 *)(tl + 1 < P_NT ? sb + (tl + 1) * 3072 : sbn);
                bf16x8 P0, P1;
#pragma unroll
                for (int v = 0; v < 8; ++v) P0[v] = (__bf16)__builtin_amdgcn_exp2f(S[v]);
                O = __builtin_amdgcn_mfma_f32_32x32x16_bf16(V0, P0, O, 0, 0, 0);
#pragma unroll
                for (int v = 0; v < 8; ++v) P1[v] = (__bf16)__builtin_amdgcn_exp2f(S[8 + v]);
                S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Kf, q[hd], NEG, 0, 0, 0);
                O = __builtin_amdgcn_mfma_f32_32x32x16_bf16(V1, P1, O, 0, 0, 0);
                if (tl == P_NT / 2 - 1) {
                    wait_vmcnt<0>();
                    asm volatile("s_barrier" ::: "memory");
                    if (it + P_DIST < total) stage_load(it + P_DIST);
                }
            }
            ++it;
        }

        // row 16 of O^T (register 8 of half 0; half 1 holds row 20, zeros) is the sum of the probabilities
        float l = O[8];
        l += __shfl_xor(l, 32, 64);
        const float inv = L > 0 ? 1.0f / l : 0.f;
        if (live) {
            bf16x4 o0, o1;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                o0[i] = (__bf16)(O[i] * inv);
                o1[i] = (__bf16)(O[4 + i] * inv);
            }
            // features 4 h + i and 8 + 4 h + i of head hd: half h of two consecutive pieces
            const int p0 = (m.d_item + hd * 16) / 8;
            store_stream4((bf16x4 *)piece(p0) + h, o0);
            store_stream4((bf16x4 *)piece(p0 + 1) + h, o1);
        }
    }
}

template <int NFT, int WAVES, bool GATHER>
hipError_t launch_proj_spec(const Model &m, const Batch &b, void *X, const MfmaPlan &plan, const void *table, int32_t *bad,
                            hipStream_t s)
{
    constexpr int ROWS = WAVES * 32;
    auto kern = k_attn_proj<NFT, WAVES, GATHER>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, P_LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(b.n_blk * (ROW_BLOCK / ROWS)), dim3(WAVES * 64), P_LDS_BYTES, s, m, b, (char *)X,
                       x_layout(m), (const char *)plan.wq_pack, (const char *)plan.kvpack, plan.pack_stride,
                       (const float *)plan.kmax, plan.nktp, (const char *)table, bad);
    return hipGetLastError();
}

template <int NFT, int WAVES>
hipError_t launch_proj_gather(const Model &m, const Batch &b, void *X, const MfmaPlan &plan, const void *table, int32_t *bad,
                              hipStream_t s)
{
    if (table) return bad ? launch_proj_spec<NFT, WAVES, true>(m, b, X, plan, table, bad, s) : hipErrorInvalidValue;
    return launch_proj_spec<NFT, WAVES, false>(m, b, X, plan, nullptr, nullptr, s);
}

}  // namespace

// Shapes the kernel serves: bf16, W_q present, 16-wide heads (2, 4 or 8 of them), item vectors a multiple of
// 64 wide and W_q small enough for LDS (72 KB); cross NONE, HADAMARD, or SEGDOT with at most 32 vectors of a width that is a multiple of 16 up to 64.
bool attn_proj_ok(const Model &m, bool has_wq)
{
    if (m.dtype != 1 || !has_wq || m.d_head != 16 || m.d_item % 64) return false;
    if ((size_t)m.d_attn * m.d_item * 2 > (size_t)P_SLOTS * P_STAGE_BYTES) return false;     // W_q is staged in the ring's LDS
    if (m.n_heads != 2 && m.n_heads != 4 && m.n_heads != 8) return false;
    if (m.cross_mode == 2)      // the cross block of 32 candidates passes through a 6 KB strip of LDS
        return m.n_cross <= 32 && m.d_cv % 16 == 0 && m.d_cv <= 16 * P_MAX_CROSS_FRAGS && m.d_cross * 2 + 16 <= 2 * P_STAGE_BYTES / 8 / 32;
    return m.cross_mode == 0 || m.cross_mode == 1;
}

size_t attn_proj_pack_stride(const Model &m, int max_seq_len, int *nktp_out)
{
    const int nktp = (((max_seq_len + 31) >> 5) + P_NT - 1) / P_NT * P_NT;
    if (nktp_out) *nktp_out = nktp;
    return (size_t)m.n_heads * nktp * 3 * 1024;
}

bool stage_proj_fusable(const Model &m, const MfmaPlan &plan)
{
    return m.dtype == 1 && plan.attn && plan.attn_variant == ATTN_VARIANT_PROJ;
}

hipError_t launch_stage_proj(const Model &m, const Batch &b, const float *w1u, const float *b1, float *bias1,
                             const MfmaPlan &plan, hipStream_t s)
{
    if (b.n_req == 0) return hipSuccess;
    StageProjArgs a{};
    a.m = m;
    a.b = b;
    a.kvpack = plan.kvpack;
    a.pack_stride = plan.pack_stride;
    a.kmax = plan.kmax;
    a.nktp = plan.nktp;
    a.stages = plan.nktp / P_NT;
    a.w1u = w1u;
    a.b1 = b1;
    a.bias1 = bias1;
    a.quads = (m.dims[1] + FOLD_FEATS - 1) / FOLD_FEATS;
    a.n_pack = b.n_slots * m.n_heads * a.stages;
    a.n_fold = b.n_slots * a.quads;
    if (m.cross_in_mlp == 2) {
        const hipError_t e = fold_w0_args(m, plan, a.w0);
        if (e != hipSuccess) return e;
        a.n_w0 = b.n_slots * a.w0.blocks_per_slot;
    }
    hipLaunchKernelGGL(k_stage_proj, dim3(a.n_pack + a.n_fold + a.n_w0), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_attn_proj(const Model &m, const Batch &b, void *X, const MfmaPlan &plan, bool small, bool kv_packed,
                            hipStream_t s, const void *gather_table, int32_t *bad)
{
    if (plan.nktp > 0 && !kv_packed)
        hipLaunchKernelGGL(k_pack_kv16, dim3(plan.nktp / P_NT, m.n_heads, b.n_slots), dim3(256), 0, s, m, b, plan.kvpack,
                           plan.pack_stride, plan.kmax, plan.nktp);
    switch (m.n_heads) {
    case 2: return small ? launch_proj_gather<1, 2>(m, b, X, plan, gather_table, bad, s) : launch_proj_gather<1, 8>(m, b, X, plan, gather_table, bad, s);
    case 4: return small ? launch_proj_gather<2, 2>(m, b, X, plan, gather_table, bad, s) : launch_proj_gather<2, 8>(m, b, X, plan, gather_table, bad, s);
    case 8: return small ? launch_proj_gather<4, 2>(m, b, X, plan, gather_table, bad, s) : launch_proj_gather<4, 8>(m, b, X, plan, gather_table, bad, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace aif
