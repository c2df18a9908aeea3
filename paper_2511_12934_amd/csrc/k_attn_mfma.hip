// a3-a5 on the matrix cores -- target attention of every candidate over the
// request's behaviour sequence, Softmax(q K^T / sqrt(d_h)) V (operator of
// Eq. 3 with the candidate as the query), plus the real-time half of the
// cross features (Sec. 3.3).
//
// Everything is formed transposed so that a lane owns ONE candidate:
//   S^T = K q^T   (A = 32 keys x d_h, B = candidates as columns)
//   O^T = V^T P^T (A = 32 features x 32 keys, B = the probabilities)
// A 32x32 MFMA result leaves, in lane (candidate c, half h), the scores of keys
// 8q + 4h + i of that candidate.  The softmax reduction over keys is therefore
// in-lane plus one exchange between the two halves, and the sixteen
// probabilities a lane holds are, as they stand, two k-steps of the B operand
// of the second product -- V is stored once per request in the matching key
// order (k_pack_kv), so P never moves between lanes or through LDS.
//
// The request's K and V (shared by all its candidates and mini-batches,
// Sec. 3.1) are packed once per call into MFMA fragment order and streamed
// through a four-slot ring in LDS, two 32-key tiles per stage, three stages in
// flight, with direct-to-LDS loads; all waves of a block share them.
//
// The keys are packed times log2(e) / sqrt(d_h) (pack_kv_block), so the first
// product is the weight's exponent in base 2 and a weight costs one
// exponential.  Softmax is shift invariant: no running maximum (and none of
// the rescaling of O it forces).  Every exponent is bounded in size by
// |q| max_t |k'_t| (Cauchy-Schwarz, k' the packed key); while that bound is
// small enough for fp32 (2^+-40) the exponents are used as they are, and if it
// is not, the wave first takes the candidate's true maximum in an extra pass
// over K and subtracts it (under a scalar branch, or in a plain loop beside
// the pipelined one: it is rare).
// Both are the exact softmax up to rounding.
#include <cstdlib>
#include <type_traits>

#include "k_mfma.h"
#include "k_stage.h"
#include "mfma_util.h"

namespace aif {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Streaming stores for the attention and cross blocks: they are written once and read by the next
// kernel, and lines left dirty in the eight L2s would have to be written back when the kernel ends.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void store_stream(bf16x8 *p, bf16x8 v) { __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v), (u32x4 *)p); }
__device__ __forceinline__ void store_stream(bf16x4 *p, bf16x4 v) { __builtin_nontemporal_store(__builtin_bit_cast(u32x2, v), (u32x2 *)p); }


// Loads the compiler does not track: completion is waited for by hand (wait_vmcnt), so that the wait can name how many
// YOUNGER memory operations may still be in flight.  The compiler's own wait at the head of the item loop is whole
// (the first pass's loads and the later passes' meet there, and a load through a pointer of unknown address space is
// waited for together with everything else): every item then began by waiting for the previous item's stores.
// The price: the compiler believes the destination final at once.  A value loaded this way must have ONE load site per
// loop (a second site gets registers of its own and is "copied" into place before anything has arrived) and must not be
// read, copied or carried into another variable before the hand-placed wait; the item block that the gather tests
// compare bit for bit is made of exactly these registers, so a violation shows there at once.
__device__ __forceinline__ void load16_untracked(bf16x8 &dst, const char *p)
{
    asm volatile("global_load_dwordx4 %0, %1, off" : "=&v"(dst) : "v"(p) : "memory");
}
__device__ __forceinline__ void load4_untracked(int &dst, const void *p)
{
    asm volatile("global_load_dword %0, %1, off" : "=&v"(dst) : "v"(p) : "memory");
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
// acc + a[2i] b[2i] + a[2i + 1] b[2i + 1], i = 0..3, as four two-term dot products (one instruction each)
__device__ __forceinline__ float dot8(const bf16x8 &a, const bf16x8 &b, float acc)
{
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a, a, 0, 1), __builtin_shufflevector(b, b, 0, 1), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a, a, 2, 3), __builtin_shufflevector(b, b, 2, 3), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a, a, 4, 5), __builtin_shufflevector(b, b, 4, 5), acc, false);
    acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(a, a, 6, 7), __builtin_shufflevector(b, b, 6, 7), acc, false);
    return acc;
}
// BEA cross block (Sec. 4.1, Algorithm 1 step 4) on the matrix cores: C^T = V^T w^T with the
// candidates as columns.  The contraction runs over the row's last 16 * ksb entries (the "window",
// ksb = ceil(n_cross / 16) k-steps); window entries in front of the n_cross bridge weights meet
// zero rows of V.  The A operand of k-step ks and feature tile ft is the fragment
//   [lane][s] = Vpad[16 ks + 8 (lane / 32) + s][32 ft + lane % 32],  Vpad[w] = V[w - pad] or 0, pad = 16 ksb - n_cross
// and the B operand of a lane (candidate c, half h) is piece d_item / 8 - 2 ksb + 2 ks + h of its row.
struct BeaGeom {
    int ksb, ftc, pad, piece0;
};
__host__ __device__ inline BeaGeom bea_geom(const Model &m)
{
    const int ksb = (m.n_cross + 15) / 16;
    return BeaGeom{ksb, m.d_cv / 32, 16 * ksb - m.n_cross, m.d_item / 8 - 2 * ksb};
}
constexpr int BEA_MAX_FRAGS = 4;             // ksb * ftc fragments of 1 KB the kernels keep
__device__ __forceinline__ uint16_t bea_a_element(const uint16_t *V, const Model &m, const BeaGeom &g, int ks, int ft, int lane, int s)
{
    const int w = 16 * ks + 8 * (lane >> 5) + s - g.pad;
    return w >= 0 ? V[(size_t)w * m.d_cv + 32 * ft + (lane & 31)] : (uint16_t)0;
}
// The first product is the weight's exponent in base 2.  Its size is bounded by |q| times the largest packed key norm;
// within this limit the exponent is used as it is -- weights between 2^-40 and 2^40, their sums far inside fp32, and the
// common factor cancels in the division -- beyond it the candidate's true maximum is found and subtracted.
constexpr float BOUND_LIMIT = 40.f;

// The streaming kernels sum a candidate's keys in KEY_PARTS runs of whole 64-key stages, run q = stages
// [q nst / KEY_PARTS, (q + 1) nst / KEY_PARTS), each run from zero, and add the runs' sums in the order of q.
// One wave walking all runs in turn (k_attn_mfma) and one wave per run (k_attn_split, for batches too small
// to fill the chip with a wave per 32 candidates) therefore give the same bits.
constexpr int KEY_PARTS = 8;
__host__ __device__ inline int key_part_begin(int q, int nst) { return q * nst / KEY_PARTS; }

// Whether a request's packed K/V of all heads fit in the LDS the resident kernel keeps them in.  A request is
// served by the resident kernel exactly when this holds (and the model has a resident kernel at all: the batch
// then has tile groups), whatever else is in the batch -- its bits do not depend on the company.
constexpr int RES_LDS_FRAGS = 152;            // 1 KB fragments of K/V that may stay resident
__host__ __device__ inline bool res_fits(const Model &m, int seq_len)
{
    const int nkt2 = ((((seq_len + 31) >> 5) + 1) & ~1);
    return (long)m.n_heads * nkt2 * (m.d_head / 8) <= RES_LDS_FRAGS;
}

// Copy NFRAG fragments of 1 KB global -> LDS; every wave moves NFRAG / WAVES of them.
template <int NFRAG, int WAVES>
__device__ __forceinline__ void stage_frags(const char *__restrict__ src, uint32_t lds_dst)
{
    static_assert(NFRAG % WAVES == 0, "every wave issues the same number of loads");
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
#pragma unroll
    for (int f0 = 0; f0 < NFRAG; f0 += WAVES) dma16(src + (f0 + wave) * 1024 + lane * 16, lds_dst + (f0 + wave) * 1024);
}

// ---------------------------------------------------------------------------
// a2 -- per request: K and V into fragment order, and max |k_t| per head and 64-key stage
// (body and layout: pack_kv_block).
// ---------------------------------------------------------------------------
template <int DH>
__global__ __launch_bounds__(256) void k_pack_kv(Model m, Batch b, char *__restrict__ kvpack, size_t pack_stride,
                                                 float *__restrict__ kmax_part, int nktp)
{
    pack_kv_block<DH>(blockIdx.z, blockIdx.y, blockIdx.x, m, TableReqs{b}, kvpack, pack_stride, kmax_part, nktp);
}

// ---------------------------------------------------------------------------
// attention + Hadamard cross.  One wave = 32 candidates, all heads in turn.
// ---------------------------------------------------------------------------
template <int DH, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void k_attn_mfma(Model m, Batch b, char *__restrict__ X, XLayout xl,
                                                         const char *__restrict__ kvpack, size_t pack_stride,
                                                         const float *__restrict__ kmax, int nktp)
{
    constexpr int FR = DH / 8, JS = DH / 16, FT = DH / 32, STAGE_BYTES = 2 * FR * 1024, ROWS = WAVES * 32;
    static_assert(ROW_BLOCK % ROWS == 0, "tile");
    extern __shared__ __align__(16) char lds[];

    // Workgroups go to the 8 XCDs in turn, each with an L2 of its own.  Give every XCD a contiguous
    // run of tiles, so the blocks that stream one request's K/V share an L2 instead of all eight
    // fetching it.
    const int per_xcd = gridDim.x >> 3;
    const int bid = blockIdx.x;
    const int tile = bid < 8 * per_xcd ? (bid & 7) * per_xcd + (bid >> 3) : bid;
    const int row0 = tile * ROWS;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, col = lane & 31, h = lane >> 5;
    // this lane's candidate: piece p of its row is at xrow + p * xl.piece_stride
    char *xrow = X + x_offset(xl, row0 + wave * 32 + col, 0);
    auto piece = [&](int p) { return (bf16x8 *)(xrow + (size_t)p * xl.piece_stride); };
    // The block's start is a chain of dependent memory round trips; keep it short.  The query rows
    // do not depend on the request lookup (a padded row is still inside the workspace): ask first.
    bf16x8 q[JS];
#pragma unroll
    for (int j = 0; j < JS; ++j) q[j] = *piece(2 * j + h);

    const int r = b.blk_req[tile / (ROW_BLOCK / ROWS)];
    if (r < 0) return;
    const ReqDesc rd = b.reqs[r];
    const int local0 = row0 - rd.row_base;
    if (rd.n_cand - local0 <= 0) return;
    if (b.n_groups > 0 && res_fits(m, rd.seq_len)) return;      // the resident kernel's

    const int L = rd.seq_len, H = m.n_heads;
    const int nkt = (L + 31) >> 5, nst = (nkt + 1) >> 1, total = H * nst;
    const int us = rd.slot;                         // K/V and key norms are kept per user, not per slice
    const char *pk = kvpack + (size_t)us * pack_stride;
    const int local = local0 + wave * 32 + col;
    const bool live = local < rd.n_cand;

    constexpr int SLOTS = 4, DIST = SLOTS - 1, LPW = 2 * FR / WAVES;      // ring, prefetch distance, loads per wave and stage
    const uint32_t ring = lds_address(lds);
    auto stage_src = [&](int i) {
        const int sh = i / nst, ss = i - sh * nst;
        return pk + ((size_t)(sh * nktp + 2 * ss) * FR) * 1024;
    };
    auto load_kmax = [&](int hd) {
        float km = 0.f;
        for (int i = lane; i < nst; i += 64) km = fmaxf(km, kmax[((size_t)us * H + hd) * (nktp / 2) + i]);
        return km;
    };
    // The compiler does not know of the hand-issued loads: wherever it waits for a load of its own it
    // waits for all of them.  So the first head's key-norm bounds are asked for before the ring is
    // primed, and everything is waited for once.
    float km = load_kmax(0);
    for (int i = 0; i < DIST && i < total; ++i) stage_frags<2 * FR, WAVES>(stage_src(i), ring + i * STAGE_BYTES);
    wait_vmcnt<0>();
    __syncthreads();

    int it = 0;
    for (int hd = 0; hd < H; ++hd) {
        if (hd > 0) {
#pragma unroll
            for (int j = 0; j < JS; ++j) q[j] = *piece(hd * (DH / 8) + 2 * j + h);
            km = load_kmax(hd);
        }
        float ss = 0.f;                     // |q|^2 of this half's pieces, two terms an instruction
#pragma unroll
        for (int j = 0; j < JS; ++j) ss = dot8(q[j], q[j], ss);
        ss += __shfl_xor(ss, 32, 64);
#pragma unroll
        for (int off = 32; off; off >>= 1) km = fmaxf(km, __shfl_xor(km, off, 64));
        float mc = sqrtf(ss) * 1.001f * km;
        // A candidate's choice between the bound and the true maximum depends on its own row only
        // (rows past the end of the request hold whatever the workspace held before and take no part),
        // so its bits do not depend on which candidates share its wave.
        const bool need_max = live && mc > BOUND_LIMIT;
        const bool shifted = __any(need_max);                // the same in every lane: a scalar branch
        if (shifted) {
            // rare: take the true maximum with an extra pass over K (read straight from memory)
            float mx = -INFINITY;
            for (int kt = 0; kt < nkt; ++kt) {
                const char *src = pk + ((size_t)(hd * nktp + kt) * FR) * 1024 + lane * 16;
                f32x16 S;
#pragma unroll
                for (int i = 0; i < 16; ++i) S[i] = 0.f;
#pragma unroll
                for (int j = 0; j < JS; ++j)
                    S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(src + j * 1024), q[j], S, 0, 0, 0);
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int t = 32 * kt + 8 * (v >> 2) + 4 * h + (v & 3);
                    if (t < L) mx = fmaxf(mx, S[v]);
                }
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            mc = need_max ? mx : 0.f;       // a candidate within the limit keeps its exponents as they are: x - 0 = x
        }

        // O, l: the current run of key tiles; Ot, lt: the runs before it (KEY_PARTS)
        f32x16 O[FT], Ot[FT];
#pragma unroll
        for (int ft = 0; ft < FT; ++ft)
#pragma unroll
            for (int i = 0; i < 16; ++i) O[ft][i] = Ot[ft][i] = 0.f;
        float l4[4] = {0.f, 0.f, 0.f, 0.f}, lt = 0.f;      // the run's denominator: weight v of every key tile into partial sum v % 4
        int qn = 1, bnd = key_part_begin(1, nst);          // the next run and its first stage
        auto fold = [&]() {
#pragma unroll
            for (int ft = 0; ft < FT; ++ft)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    Ot[ft][i] += O[ft][i];
                    O[ft][i] = 0.f;
                }
            lt += (l4[0] + l4[1]) + (l4[2] + l4[3]);
            l4[0] = l4[1] = l4[2] = l4[3] = 0.f;
        };

        for (int st = 0; st < nst; ++st) {
            // stage it + DIST goes into the slot stage it - 1 was read from
            if (it + DIST < total) stage_frags<2 * FR, WAVES>(stage_src(it + DIST), ring + ((it + DIST) % SLOTS) * STAGE_BYTES);
            const int buf = it % SLOTS;
            while (st == bnd) {                             // a run ends here (empty runs: several)
                fold();
                bnd = key_part_begin(++qn, nst);
            }
#pragma unroll
            for (int k2 = 0; k2 < 2; ++k2) {
                const int kt = 2 * st + k2;
                const char *base = lds + buf * STAGE_BYTES + k2 * FR * 1024 + lane * 16;
                f32x16 S;
#pragma unroll
                for (int i = 0; i < 16; ++i) S[i] = 0.f;
#pragma unroll
                for (int j = 0; j < JS; ++j)
                    S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(base + j * 1024), q[j], S, 0, 0, 0);
                float p[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) p[v] = S[v];
                if (shifted)
#pragma unroll
                    for (int v = 0; v < 16; ++v) p[v] -= mc;
#pragma unroll
                for (int v = 0; v < 16; ++v) p[v] = __builtin_amdgcn_exp2f(p[v]);
                if (32 * kt + 32 > L) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int t = 32 * kt + 8 * (v >> 2) + 4 * h + (v & 3);
                        if (t >= L) p[v] = 0.f;
                    }
                }
                // the softmax denominator is the fp32 sum of the weights as they leave the exponential; the second
                // product takes them rounded to bf16
                bf16x8 P0, P1;
#pragma unroll
                for (int v = 0; v < 8; ++v) {
                    P0[v] = (__bf16)p[v];
                    P1[v] = (__bf16)p[8 + v];
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) l4[v & 3] += p[v];
#pragma unroll
                for (int ft = 0; ft < FT; ++ft) {
                    O[ft] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(base + (JS + ft) * 1024), P0, O[ft], 0, 0, 0);
                    O[ft] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(base + (JS + FT + ft) * 1024), P1, O[ft], 0, 0, 0);
                }
            }
            // stage it + 1 must have landed; the later ones (as far as they exist) may stay in flight
            {
                const int later = total - 2 - it;
                if (later >= 2)
                    wait_vmcnt<2 * LPW>();
                else if (later == 1)
                    wait_vmcnt<LPW>();
                else
                    wait_vmcnt<0>();
            }
            __syncthreads();
            ++it;
        }
        for (; qn <= KEY_PARTS; ++qn) fold();               // the last run, and the empty ones before it

        lt += __shfl_xor(lt, 32, 64);
        const float inv = L > 0 ? 1.0f / lt : 0.f;
        if (live) {
#pragma unroll
            for (int ft = 0; ft < FT; ++ft)
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) {
                    bf16x4 o4;
#pragma unroll
                    for (int i = 0; i < 4; ++i) o4[i] = (__bf16)(Ot[ft][4 * qd + i] * inv);
                    // features 8 qd + 4 h + i of this tile: half h of one piece
                    store_stream((bf16x4 *)piece((m.d_item + hd * DH) / 8 + 4 * ft + qd) + h, o4);
                }
        }
    }

    if (m.cross_mode == 1 && !m.cross_in_mlp && live) {      // unless the MLP chain forms the Hadamard products itself
        const bf16x8 *uc = (const bf16x8 *)rd.cross_vecs;
        const int pc0 = (m.d_item + m.d_attn) / 8;
        for (int pc = h; pc < m.d_item / 8; pc += 2) {
            const bf16x8 e = *piece(pc), u = uc[pc];
            bf16x8 o8;
#pragma unroll
            for (int s = 0; s < 8; ++s) o8[s] = (__bf16)((float)e[s] * (float)u[s]);
            store_stream(piece(pc0 + pc), o8);
        }
    }
    if (m.cross_mode == 3 && !m.cross_in_mlp) {      // unless the block is folded into the user's layer-1 weights
        const BeaGeom g = bea_geom(m);
        const uint16_t *Vu = (const uint16_t *)rd.cross_vecs;
        const int pc0 = (m.d_item + m.d_attn) / 8;
        for (int ft = 0; ft < g.ftc; ++ft) {
            f32x16 Cc;
#pragma unroll
            for (int i = 0; i < 16; ++i) Cc[i] = 0.f;
            for (int ks = 0; ks < g.ksb; ++ks) {
                uint16_t a8[8];
#pragma unroll
                for (int sl = 0; sl < 8; ++sl) a8[sl] = bea_a_element(Vu, m, g, ks, ft, lane, sl);
                bf16x8 A;
                __builtin_memcpy(&A, a8, 16);
                Cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, *piece(g.piece0 + 2 * ks + h), Cc, 0, 0, 0);
            }
            if (live) {
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) {
                    bf16x4 o4;
#pragma unroll
                    for (int i = 0; i < 4; ++i) o4[i] = (__bf16)Cc[4 * qd + i];
                    store_stream((bf16x4 *)piece(pc0 + 4 * ft + qd) + h, o4);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// The streaming computation for a batch too small to give every SIMD a wave at 32 candidates a wave (one
// request of 10^4 candidates is 313 such waves for 1,024 SIMDs, each walking the whole sequence: a chain of
// a few hundred cycles per key tile with nobody to share the SIMD).  Here a workgroup is ONE 32-candidate
// tile and its waves take a run of 64-key stages each (the runs of k_attn_mfma; two runs each when the tiles
// outnumber the compute units), so the chain is an eighth (a quarter) as long; the runs' sums meet in LDS and are added in the order of the runs -- the order in which
// k_attn_mfma adds them, so the bits are the same.  A lone wave shares its K/V with nobody: fragments come
// straight from memory (the L2s: every workgroup reads the same pack) into registers, three tiles in
// rotation, two in flight.  Inside a tile the S product of the next tile alternates with this tile's
// exponentials in the instruction stream, as in the resident kernel.
// ---------------------------------------------------------------------------
template <int DH> constexpr int split_lds_bytes() { return KEY_PARTS * (DH / 32 * 16 + 1) * 64 * 4; }

template <int DH, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void k_attn_split(Model m, Batch b, char *__restrict__ X, XLayout xl,
                                                          const char *__restrict__ kvpack, size_t pack_stride,
                                                          const float *__restrict__ kmax, int nktp)
{
    // WAVES = KEY_PARTS: a run a wave.  WAVES = KEY_PARTS / 2: two consecutive runs a wave, for the batches whose
    // tiles outnumber the compute units -- a workgroup of eight waves takes a compute unit's registers alone, and
    // the tiles beyond the first 256 would wait for a second round.
    constexpr int FR = DH / 8, JS = DH / 16, FT = DH / 32, NREG = FT * 16, NQ = KEY_PARTS, RPW = KEY_PARTS / WAVES;
    static_assert(KEY_PARTS % WAVES == 0, "whole runs per wave");
    extern __shared__ __align__(16) char lds[];
    float *part = (float *)lds;                        // [run][register (NREG of O, then l)][lane]

    const int tile = blockIdx.x, row0 = tile * 32;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), col = lane & 31, h = lane >> 5;
    char *xrow = X + x_offset(xl, row0 + col, 0);
    auto piece = [&](int p) { return (bf16x8 *)(xrow + (size_t)p * xl.piece_stride); };
    bf16x8 q[JS];                                      // asked for before the request is looked up, as in k_attn_mfma
#pragma unroll
    for (int j = 0; j < JS; ++j) q[j] = *piece(2 * j + h);

    const int r = b.blk_req[row0 / ROW_BLOCK];
    if (r < 0) return;
    const ReqDesc rd = b.reqs[r];
    const int local0 = row0 - rd.row_base;
    if (rd.n_cand - local0 <= 0) return;
    if (b.n_groups > 0 && res_fits(m, rd.seq_len)) return;      // the resident kernel's

    const int L = rd.seq_len, H = m.n_heads;
    const int nkt = (L + 31) >> 5, nst = (nkt + 1) >> 1;
    const int us = rd.slot;
    const char *pk = kvpack + (size_t)us * pack_stride + lane * 16;
    const bool live = local0 + col < rd.n_cand;
    // this wave's runs, in tiles: whole stages of two (the last one of an odd sequence ends in the pack's empty tile)
    const int kt0 = 2 * key_part_begin(RPW * wave, nst), kt1 = 2 * key_part_begin(RPW * (wave + 1), nst);

    for (int hd = 0; hd < H; ++hd) {
        if (hd > 0) {
#pragma unroll
            for (int j = 0; j < JS; ++j) q[j] = *piece(hd * (DH / 8) + 2 * j + h);
        }
        const char *kvh = pk + (size_t)hd * nktp * FR * 1024;           // fragment i of tile t: kvh + (t FR + i) KB
        // the key-norm bounds are asked for first and looked at after the fragments have been asked for: a lane
        // takes stage `lane` (an index past the end re-reads the last stage: no condition, no wait on the spot)
        const float *kmh = kmax + ((size_t)us * H + hd) * (nktp / 2);
        float km = nst > 0 ? kmh[lane < nst ? lane : nst - 1] : 0.f;
        // two sets of K fragments and two of V fragments take turns: while tile t's V and tile t + 1's K are in use,
        // tile t + 1's V and tile t + 2's K are in flight.  A tile index past the run re-reads the run's last tile
        // (fetched, not used), so the loop body has no conditions.
        const int ktl = kt1 > kt0 ? kt1 - 1 : 0;
        auto tile_src = [&](int kt) { return kvh + (size_t)(kt < ktl ? kt : ktl) * FR * 1024; };
        auto fetch_k = [&](bf16x8(&f)[JS], int kt) {
            const char *src = tile_src(kt);
#pragma unroll
            for (int i = 0; i < JS; ++i) f[i] = *(const bf16x8 *)(src + i * 1024);
        };
        auto fetch_v = [&](bf16x8(&f)[2 * FT], int kt) {
            const char *src = tile_src(kt) + JS * 1024;
#pragma unroll
            for (int i = 0; i < 2 * FT; ++i) f[i] = *(const bf16x8 *)(src + i * 1024);
        };
        // (the run's first K has a set of its own: a set that is both used and refilled ahead of the loop reaches the
        // loop through a register copy, and a copy of a register that a load is still filling waits for that load)
        bf16x8 k0[JS], ka[JS], kb[JS], va[2 * FT], vb[2 * FT];
        if (nkt > 0) {
            fetch_k(k0, kt0);
            fetch_k(kb, kt0 + 1);
            fetch_v(va, kt0);
            fetch_k(ka, kt0 + 2);
            fetch_v(vb, kt0 + 1);
        }
        for (int i = lane + 64; i < nst; i += 64) km = fmaxf(km, kmh[i]);       // sequences beyond 4096 keys

        float ss = 0.f;
#pragma unroll
        for (int j = 0; j < JS; ++j) ss = dot8(q[j], q[j], ss);
        ss += __shfl_xor(ss, 32, 64);
#pragma unroll
        for (int off = 32; off; off >>= 1) km = fmaxf(km, __shfl_xor(km, off, 64));
        float mc = sqrtf(ss) * 1.001f * km;
        const bool need_max = live && mc > BOUND_LIMIT;      // per candidate, as in k_attn_mfma
        const bool shifted = __any(need_max);                // the same in every lane: a scalar branch
        if (shifted) {
            // rare: the true maximum, by an extra pass over all of K in every wave (the maximum has no order)
            float mx = -INFINITY;
            for (int kt = 0; kt < nkt; ++kt) {
                const char *src = kvh + (size_t)kt * FR * 1024;
                f32x16 S;
#pragma unroll
                for (int i = 0; i < 16; ++i) S[i] = 0.f;
#pragma unroll
                for (int j = 0; j < JS; ++j)
                    S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(src + j * 1024), q[j], S, 0, 0, 0);
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int t = 32 * kt + 8 * (v >> 2) + 4 * h + (v & 3);
                    if (t < L) mx = fmaxf(mx, S[v]);
                }
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            mc = need_max ? mx : 0.f;       // a candidate within the limit keeps its exponents as they are: x - 0 = x
        }

        f32x16 O[FT];
#pragma unroll
        for (int ft = 0; ft < FT; ++ft)
#pragma unroll
            for (int i = 0; i < 16; ++i) O[ft][i] = 0.f;
        float l4[4] = {0.f, 0.f, 0.f, 0.f};                 // as in k_attn_mfma
        // a finished run's sums go to LDS and the next run starts from zero
        if (hd > 0) __syncthreads();                        // the previous head's sums have been read
        int qn = RPW * wave;
        auto flush = [&]() {
            float *mine = part + (size_t)qn * (NREG + 1) * 64 + lane;
#pragma unroll
            for (int ft = 0; ft < FT; ++ft)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    mine[(ft * 16 + i) * 64] = O[ft][i];
                    O[ft][i] = 0.f;
                }
            mine[NREG * 64] = (l4[0] + l4[1]) + (l4[2] + l4[3]);
            l4[0] = l4[1] = l4[2] = l4[3] = 0.f;
            ++qn;
        };
        if (kt1 > kt0) {
            f32x16 S;
#pragma unroll
            for (int i = 0; i < 16; ++i) S[i] = 0.f;
#pragma unroll
            for (int j = 0; j < JS; ++j) S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0[j], q[j], S, 0, 0, 0);
            // tile kt: exponentials of S (its scores), second product with vc (its V); meanwhile the S product of tile
            // kt + 1 from kn (after the run's last tile: of that tile again, unused); both sets are refilled, two tiles on
            auto body = [&](bf16x8(&vc)[2 * FT], bf16x8(&kn)[JS], int kt) {
                f32x16 Sn;
                float p[16];
                if (shifted) {              // rare: the candidate's maximum comes off every exponent (a scalar branch)
#pragma unroll
                    for (int v = 0; v < 16; ++v) S[v] -= mc;
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < JS; ++j) {
                    if (j == 0) {
                        f32x16 Z;
#pragma unroll
                        for (int i = 0; i < 16; ++i) Z[i] = 0.f;
                        Sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kn[0], q[0], Z, 0, 0, 0);
                    } else
                        Sn = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kn[j], q[j], Sn, 0, 0, 0);
#pragma unroll
                    for (int v = 16 / JS * j; v < 16 / JS * (j + 1); ++v) {
                        p[v] = __builtin_amdgcn_exp2f(S[v]);
                        asm volatile("" : "+v"(p[v]));      // computed HERE: a value with no side effect would sink to its first use
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                fetch_k(kn, kt + 3);
                if (32 * kt + 32 > L) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int t = 32 * kt + 8 * (v >> 2) + 4 * h + (v & 3);
                        if (t >= L) p[v] = 0.f;
                    }
                }
                bf16x8 P0, P1;
#pragma unroll
                for (int v = 0; v < 8; ++v) {
                    P0[v] = (__bf16)p[v];
                    P1[v] = (__bf16)p[8 + v];
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) l4[v & 3] += p[v];
#pragma unroll
                for (int ft = 0; ft < FT; ++ft) {
                    O[ft] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vc[ft], P0, O[ft], 0, 0, 0);
                    O[ft] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vc[FT + ft], P1, O[ft], 0, 0, 0);
                }
                // the refill stays BEHIND the last use of the set (a load moved above it would need registers of its
                // own, and the copy back at the loop's end would wait for every load in flight)
                __builtin_amdgcn_sched_barrier(0);
                fetch_v(vc, kt + 2);
                __builtin_amdgcn_sched_barrier(0);
                S = Sn;
            };
            int bnd = 2 * key_part_begin(qn + 1, nst);      // first tile of the next run
            for (int kt = kt0; kt < kt1; kt += 2) {
                if constexpr (RPW > 1) {
                    while (kt == bnd) {                     // a run ends here (empty runs: several)
                        flush();
                        bnd = 2 * key_part_begin(qn + 1, nst);
                    }
                }
                body(va, kb, kt);
                body(vb, ka, kt + 1);
            }
        }
        while (qn < RPW * (wave + 1)) flush();              // the last run, and the empty ones around it

        // the runs' sums meet in LDS ...
        __syncthreads();
        // ... and are added in the order of the runs, from zero; wave w normalises and stores quads w, w + WAVES, ...
        float lt = 0.f;
#pragma unroll
        for (int qn = 0; qn < NQ; ++qn) lt += part[((size_t)qn * (NREG + 1) + NREG) * 64 + lane];
        lt += __shfl_xor(lt, 32, 64);
        const float inv = L > 0 ? 1.0f / lt : 0.f;
        for (int g = wave; g < FT * 4; g += WAVES) {
            float t[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int qn = 0; qn < NQ; ++qn)
#pragma unroll
                for (int i = 0; i < 4; ++i) t[i] += part[((size_t)qn * (NREG + 1) + 4 * g + i) * 64 + lane];
            if (live) {
                bf16x4 o4;
#pragma unroll
                for (int i = 0; i < 4; ++i) o4[i] = (__bf16)(t[i] * inv);
                // register 4 g + i = feature tile g / 4, quad g % 4: features 8 (g % 4) + 4 h + i of that tile
                store_stream((bf16x4 *)piece((m.d_item + hd * DH) / 8 + g) + h, o4);
            }
        }
    }

    // the real-time half of the cross features, as in k_attn_mfma; the waves share the pieces / feature tiles
    if (m.cross_mode == 1 && !m.cross_in_mlp && live) {
        const bf16x8 *uc = (const bf16x8 *)rd.cross_vecs;
        const int pc0 = (m.d_item + m.d_attn) / 8;
        for (int pc = 2 * wave + h; pc < m.d_item / 8; pc += 2 * WAVES) {
            const bf16x8 e = *piece(pc), u = uc[pc];
            bf16x8 o8;
#pragma unroll
            for (int s = 0; s < 8; ++s) o8[s] = (__bf16)((float)e[s] * (float)u[s]);
            store_stream(piece(pc0 + pc), o8);
        }
    }
    if (m.cross_mode == 3 && !m.cross_in_mlp) {      // unless the block is folded into the user's layer-1 weights
        const BeaGeom g = bea_geom(m);
        const uint16_t *Vu = (const uint16_t *)rd.cross_vecs;
        const int pc0 = (m.d_item + m.d_attn) / 8;
        for (int ft = wave; ft < g.ftc; ft += WAVES) {
            f32x16 Cc;
#pragma unroll
            for (int i = 0; i < 16; ++i) Cc[i] = 0.f;
            for (int ks = 0; ks < g.ksb; ++ks) {
                uint16_t a8[8];
#pragma unroll
                for (int sl = 0; sl < 8; ++sl) a8[sl] = bea_a_element(Vu, m, g, ks, ft, lane, sl);
                bf16x8 A;
                __builtin_memcpy(&A, a8, 16);
                Cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, *piece(g.piece0 + 2 * ks + h), Cc, 0, 0, 0);
            }
            if (live) {
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) {
                    bf16x4 o4;
#pragma unroll
                    for (int i = 0; i < 4; ++i) o4[i] = (__bf16)Cc[4 * qd + i];
                    store_stream((bf16x4 *)piece(pc0 + 4 * ft + qd) + h, o4);
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------
// The same computation with the request's K/V RESIDENT in LDS.  All candidates of
// a request share its behaviour sequence (Sec. 3.1), so when the packed K/V of all
// heads fit in one CU's LDS a workgroup loads them once and then serves a whole
// group of 32-candidate tiles of that request: after the one barrier that follows
// the load its 16 waves run free of each other, one tile at a time each, and the
// four waves of a SIMD fill one another's waits.  Inside a tile the S product of
// key tile t + 1 is issued before the exponentials of key tile t, so the matrix
// cores work under the vector ALU.  Per candidate the arithmetic, and its order,
// is that of k_attn_mfma: the two kernels give the same bits.
//
// GATHER: the kernel is also a1 (Sec. 3.2, the index into the table of item vectors).  Without W_q the query
// pieces a lane needs ARE pieces of its candidate's item vector, so it takes them straight from the table
// row its id names -- asked for a whole item ahead, like the workspace rows otherwise -- and sets them down in
// the workspace for the MLP on the way.  The separate gather launch, its write of the item block and this
// kernel's read of it fall away.  An id outside the table reads row 0 and is counted, as in the gather kernel.
// ---------------------------------------------------------------------------
constexpr int RES_WAVES = 12;
constexpr int RES_MAX_HEADS = 64;
constexpr int RES_MAX_ITEM_PIECES = 256;      // d_item / 8 the Hadamard operand may have to stay in LDS
constexpr int RES_LDS_BYTES = RES_LDS_FRAGS * 1024 + RES_MAX_HEADS * 4 + RES_MAX_ITEM_PIECES * 16 + 16;

template <int DH, bool GATHER>
__global__ __launch_bounds__(RES_WAVES * 64) void k_attn_res(Model m, Batch b, char *__restrict__ X, XLayout xl,
                                                             const char *__restrict__ kvpack, size_t pack_stride,
                                                             const float *__restrict__ kmax, int nktp,
                                                             const char *__restrict__ table, int32_t *__restrict__ bad)
{
    constexpr int FR = DH / 8, JS = DH / 16, FT = DH / 32;
    extern __shared__ __align__(16) char lds[];
    float *skm = (float *)(lds + RES_LDS_FRAGS * 1024);         // [n_heads] max |k_t|
    bf16x8 *su = (bf16x8 *)(skm + RES_MAX_HEADS);               // the request's Hadamard operand
    int *s_next = (int *)(su + RES_MAX_ITEM_PIECES);            // next item of the group nobody has taken yet

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), col = lane & 31, h = lane >> 5;
    const AttnGroup g = b.groups[blockIdx.x];
    const int r = g.r;
    const ReqDesc rd = b.reqs[r];
    const int L = rd.seq_len, H = m.n_heads;
    const int nkt = (L + 31) >> 5, nkt2 = (nkt + 1) & ~1, head_frags = nkt2 * FR;
    const int us = rd.slot;                         // K/V and key norms are kept per user, not per slice
    const char *pk = kvpack + (size_t)us * pack_stride;

    const int n_tiles = g.t1 - g.t0;
    auto row_of = [&](int tile) { return X + x_offset(xl, rd.row_base + (g.t0 + tile) * 32 + col, 0); };
    // GATHER: the id of this lane's candidate in a tile as the request gives it (0 past the request's end), and
    // the table row it names
    auto raw_id = [&](int t) {
        const int lc = (g.t0 + t) * 32 + col;
        return lc < rd.n_cand ? rd.cand_ids[lc] : 0;
    };
    // the same as an untracked load (a lane past the request's end reads the request's first id and drops it)
    auto raw_id_untracked = [&](int &dst, int t) {
        const int lc = (g.t0 + t) * 32 + col;
        load4_untracked(dst, rd.cand_ids + (lc < rd.n_cand ? lc : 0));
    };
    auto in_request = [&](int t) { return (g.t0 + t) * 32 + col < rd.n_cand; };
    auto checked = [&](int raw, bool count) {           // count: once per candidate (by the item of its first head)
        if (raw < 0 || (int64_t)raw >= m.n_items) {
            if (h == 0 && count) atomicAdd(bad, 1);
            raw = 0;
        }
        return raw;
    };
    auto table_row = [&](int id) { return table + (size_t)id * (size_t)(m.d_item * 2); };

    // The whole pack -> LDS, heads back to back (in the pack a head takes nktp key tiles).  The wave's first query
    // rides along: its id is asked for ahead of the first half of the pack and its row pieces between the halves, so
    // that id -> row (two trips to memory) pass under the pack's flight instead of after the barrier.  (A wave with
    // no tile in the group reads the group's last tile's: no condition around the loads.)
    // A wave's unit of work is an item = (tile, head), item i = tile i / H, head i % H: with several heads a group's
    // items divide over the waves far more evenly than its tiles would.
    const int n_items = n_tiles * H;
    const float inv_h = 1.0f / (float)H;
    auto tile_of = [&](int item) {                      // item / H (exact: the estimate is off by one at most)
        if (H == 1) return item;
        int t = (int)((float)item * inv_h);
        const int rem = item - t * H;
        t += rem >= H ? 1 : (rem < 0 ? -1 : 0);
        return t;
    };
    bf16x8 q[JS];
    int id = 0;                             // GATHER: row of the table the current item's candidate has
    const int item_first = wave < n_items ? wave : n_items - 1;
    const int tile_first = tile_of(item_first), hd_first = item_first - tile_first * H;
    int raw_first = 0;
    if constexpr (GATHER) raw_first = raw_id(tile_first);
    const uint32_t ring = lds_address(lds);
    const int nfrag = H * head_frags, nhalf = nfrag / 2;
    auto pack_to_lds = [&](int f0, int f1) {
        for (int f = f0 + wave; f < f1; f += RES_WAVES) {
            const int hd = f / head_frags, rem = f - hd * head_frags;
            dma16(pk + ((size_t)hd * nktp * FR + rem) * 1024 + lane * 16, ring + f * 1024);
        }
    };
    pack_to_lds(0, nhalf);
    if constexpr (GATHER) {
        id = checked(wave < n_items ? raw_first : 0, hd_first == 0);     // (a stand-in id is not the request's: never counted as bad)
        const char *tr = table_row(id);
#pragma unroll
        for (int j = 0; j < JS; ++j) load16_untracked(q[j], tr + (hd_first * (DH / 8) + 2 * j + h) * 16);
    } else {
        const char *xr = row_of(tile_first);
#pragma unroll
        for (int j = 0; j < JS; ++j) load16_untracked(q[j], xr + (size_t)(hd_first * (DH / 8) + 2 * j + h) * xl.piece_stride);
    }
    pack_to_lds(nhalf, nfrag);
    for (int hd = wave; hd < H; hd += RES_WAVES) {
        float km = 0.f;
        for (int i = lane; i < nkt2 / 2; i += 64) km = fmaxf(km, kmax[((size_t)us * H + hd) * (nktp / 2) + i]);
#pragma unroll
        for (int off = 32; off; off >>= 1) km = fmaxf(km, __shfl_xor(km, off, 64));
        if (lane == 0) skm[hd] = km;
    }
    const bool hadamard = m.cross_mode == 1 && !m.cross_in_mlp;      // else the MLP chain forms the Hadamard products itself
    if (hadamard)
        for (int i = threadIdx.x; i < m.d_item / 8; i += RES_WAVES * 64) su[i] = ((const bf16x8 *)rd.cross_vecs)[i];
    const bool bea = m.cross_mode == 3 && !m.cross_in_mlp;           // else it is folded into the user's layer-1 weights
    const BeaGeom bg = bea_geom(m);
    if (bea) {
        // the request's user-side vectors as A fragments (k-step major), in the LDS the Hadamard operand would take
        uint16_t *sa = (uint16_t *)su;
        const uint16_t *Vu = (const uint16_t *)rd.cross_vecs;
        for (int i = threadIdx.x; i < bg.ksb * bg.ftc * 512; i += RES_WAVES * 64) {
            const int sl = i & 7, ln = (i >> 3) & 63, f = i >> 9;
            sa[i] = bea_a_element(Vu, m, bg, f / bg.ftc, f % bg.ftc, ln, sl);
        }
    }
    if (threadIdx.x == 0) *s_next = RES_WAVES;
    wait_vmcnt<0>();
    __syncthreads();

    const char *kv0 = lds + lane * 16;
    const int pc_cross = (m.d_item + m.d_attn) / 8;             // first piece of the cross block

    // A wave's work is a sequence of (tile, head) items, handed out on demand -- the SIMD
    // favours its older waves, so with a fixed share per wave the young ones would finish the kernel
    // alone.  The only global reads an item needs are its query pieces; they are asked for as soon as
    // the previous item has issued its last S product (the registers are free from then on), so their
    // latency passes under that item's last exponentials, second product and stores.
    auto take_item = [&]() {
        int t = 0;
        if (lane == 0) t = atomicAdd(s_next, 1);
        return __builtin_amdgcn_readfirstlane(t);
    };
    int item = wave, tile = tile_first, hd = hd_first;
    while (item < n_items) {
        // the item's query: asked for when the previous item had issued its last S product; younger than those loads
        // are only that item's 4 FT output stores (before the first item the kernel's opening wait has covered them)
        wait_vmcnt<4 * FT>();
#pragma unroll
        for (int j = 0; j < JS; ++j) asm volatile("" : "+v"(q[j]));
        const int next_item = take_item();
        const int next_tile = tile_of(next_item), next_hd = next_item - next_tile * H;
        // the next item's id is asked for now and looked at only when this item's last S product has been issued
        int next_raw = 0;
        if constexpr (GATHER)
            if (next_item < n_items) raw_id_untracked(next_raw, next_tile);
        const int local = (g.t0 + tile) * 32 + col;
        const bool live = local < rd.n_cand;
        char *xrow = row_of(tile);
        auto piece = [&](int p) { return (bf16x8 *)(xrow + (size_t)p * xl.piece_stride); };
        if constexpr (GATHER) {
            // a1: this head's slice of the item vector goes into the workspace
            if (live) {
#pragma unroll
                for (int j = 0; j < JS; ++j) *piece(hd * (DH / 8) + 2 * j + h) = q[j];
            }
        }

        // real-time half of the cross features: the query pieces ARE item-vector pieces (no W_q here),
        // so the ones this lane holds are multiplied in place; the stores drain under the attention loop
        if (hadamard && live) {
#pragma unroll
            for (int j = 0; j < JS; ++j) {
                const int pc = hd * (DH / 8) + 2 * j + h;
                if (pc < m.d_item / 8) {
                    const bf16x8 u = su[pc];
                    bf16x8 o8;
#pragma unroll
                    for (int s = 0; s < 8; ++s) o8[s] = (__bf16)((float)q[j][s] * (float)u[s]);
                    store_stream(piece(pc_cross + pc), o8);
                }
            }
        }
        // item-vector pieces beyond the attention width (d_item > d_attn)
        if ((hadamard || GATHER) && live && hd == H - 1)
            for (int pc = m.d_attn / 8 + h; pc < m.d_item / 8; pc += 2) {
                bf16x8 e;
                if constexpr (GATHER) {
                    e = *(const bf16x8 *)(table_row(id) + pc * 16);
                    store_stream(piece(pc), e);
                } else {
                    e = *piece(pc);
                }
                if (hadamard) {
                    const bf16x8 u = su[pc];
                    bf16x8 o8;
#pragma unroll
                    for (int s = 0; s < 8; ++s) o8[s] = (__bf16)((float)e[s] * (float)u[s]);
                    store_stream(piece(pc_cross + pc), o8);
                }
            }

        // Algorithm 1 step 4, once per tile: the row's bridge weights against the user-side vectors
        if (bea && hd == 0) {
            for (int ft = 0; ft < bg.ftc; ++ft) {
                f32x16 Cc;
#pragma unroll
                for (int i = 0; i < 16; ++i) Cc[i] = 0.f;
                for (int ks = 0; ks < bg.ksb; ++ks) {
                    // the row's bridge weights: from the workspace, or (GATHER: the row is not there yet) from the table
                    bf16x8 wrow;
                    if constexpr (GATHER) wrow = *(const bf16x8 *)(table_row(id) + (bg.piece0 + 2 * ks + h) * 16);
                    else wrow = *piece(bg.piece0 + 2 * ks + h);
                    Cc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(su[(ks * bg.ftc + ft) * 64 + lane], wrow, Cc, 0, 0, 0);
                }
                if (live) {
#pragma unroll
                    for (int qd = 0; qd < 4; ++qd) {
                        bf16x4 o4;
#pragma unroll
                        for (int i = 0; i < 4; ++i) o4[i] = (__bf16)Cc[4 * qd + i];
                        store_stream((bf16x4 *)piece(pc_cross + 4 * ft + qd) + h, o4);
                    }
                }
            }
        }

        float ss = 0.f;                     // |q|^2 of this half's pieces, two terms an instruction
#pragma unroll
        for (int j = 0; j < JS; ++j) ss = dot8(q[j], q[j], ss);
        ss += __shfl_xor(ss, 32, 64);
        const char *kvh = kv0 + (size_t)hd * head_frags * 1024;
        auto s_tile = [&](int kt) {
            const char *base = kvh + kt * FR * 1024;
            f32x16 S;
#pragma unroll
            for (int i = 0; i < 16; ++i) S[i] = 0.f;
#pragma unroll
            for (int j = 0; j < JS; ++j)
                S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(base + j * 1024), q[j], S, 0, 0, 0);
            return S;
        };
        float mc = sqrtf(ss) * 1.001f * skm[hd];
        const bool need_max = live && mc > BOUND_LIMIT;      // per candidate, as in k_attn_mfma
        const bool shifted = __any(need_max);                // the same in every lane: a scalar branch
        if (shifted) {
            // rare: take the true maximum with an extra pass over K
            float mx = -INFINITY;
            for (int kt = 0; kt < nkt; ++kt) {
                const f32x16 S = s_tile(kt);
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int t = 32 * kt + 8 * (v >> 2) + 4 * h + (v & 3);
                    if (t < L) mx = fmaxf(mx, S[v]);
                }
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            mc = need_max ? mx : 0.f;       // a candidate within the limit keeps its exponents as they are: x - 0 = x
        }

        f32x16 O[FT];
#pragma unroll
        for (int ft = 0; ft < FT; ++ft)
#pragma unroll
            for (int i = 0; i < 16; ++i) O[ft][i] = 0.f;
        // the softmax denominator: the weights as they leave the exponential (fp32; the second product takes them
        // rounded to bf16), weight v of every key tile into partial sum v % 4
        float l4[4] = {0.f, 0.f, 0.f, 0.f};
        // ---- the key-tile loop, software-pipelined inside the wave ------------------------------------------
        // A wave issues in order, so what must overlap has to alternate in its instruction stream.  Per key tile t:
        //   - the S product of tile t + 1 is a chain of JS MFMAs, each waiting for the one before: one link per
        //     slot, and in the same slot the exponents and exponentials of 16 / JS scores of tile t (about as many
        //     issue cycles as the MFMA takes), so neither the matrix cores nor the vector ALU wait for the other;
        //   - the K fragment a link has just consumed is refilled from LDS with tile t + 2's (a whole tile of lead),
        //     V fragments of tile t are asked for at the top of the tile;
        //   - the second product's MFMAs (feature tiles alternating, so consecutive ones are independent) carry the
        //     adds of the row sums (the softmax denominator) between them.
        // Scheduling barriers pin the slots; within a slot the compiler is free.  Per candidate the arithmetic and
        // its order are unchanged.
        const char *kbase = kvh;                                       // K fragment j of tile t: kbase + (t FR + j) KB
        bf16x8 kf[JS], vf[2 * FT];
        f32x16 S, S1;
        // tile kt: exponentials of Sin, second product; with NEXT also the S product of tile kt + 1 into Sout
        auto step = [&](int kt, const f32x16 &Sin, f32x16 &Sout, auto next_c, bool ragged) {
            constexpr bool NEXT = decltype(next_c)::value;
            const char *vbase = kbase + (kt * FR + JS) * 1024;
#pragma unroll
            for (int i = 0; i < 2 * FT; ++i) vf[i] = *(const bf16x8 *)(vbase + i * 1024);
            const int kn = kt + 2 < nkt ? kt + 2 : nkt - 1;         // refill: the tile after next (clamped: read, not used)
            __builtin_amdgcn_sched_barrier(0);
            float p[16];
#pragma unroll
            for (int j = 0; j < JS; ++j) {
                if constexpr (NEXT) {
                    if (j == 0) {
                        f32x16 Z;
#pragma unroll
                        for (int i = 0; i < 16; ++i) Z[i] = 0.f;
                        Sout = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[0], q[0], Z, 0, 0, 0);
                    } else
                        Sout = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[j], q[j], Sout, 0, 0, 0);
                    kf[j] = *(const bf16x8 *)(kbase + (kn * FR + j) * 1024);
                }
#pragma unroll
                for (int v = 16 / JS * j; v < 16 / JS * (j + 1); ++v) {
                    p[v] = __builtin_amdgcn_exp2f(Sin[v]);
                    asm volatile("" : "+v"(p[v]));      // computed HERE: a value with no side effect would sink to its first use
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (ragged) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int t = 32 * kt + 8 * (v >> 2) + 4 * h + (v & 3);
                    if (t >= L) p[v] = 0.f;
                }
            }
            bf16x8 P0, P1;
#pragma unroll
            for (int v = 0; v < 8; ++v) {
                P0[v] = (__bf16)p[v];
                P1[v] = (__bf16)p[8 + v];
            }
            __builtin_amdgcn_sched_barrier(0);
            // per feature tile the P0 step, then the P1 step; issued feature tile by feature tile within a step; the
            // row sums ride between the MFMAs
#pragma unroll
            for (int i = 0; i < 2 * FT; ++i) {
                const int ft = i % FT;
                O[ft] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i], i < FT ? P0 : P1, O[ft], 0, 0, 0);
                // the denominator's share of this slot: plain fp32 adds run beside the MFMAs, the two-term dot products
                // that summed the rounded weights and the MFMAs exclude each other
#pragma unroll
                for (int v = 16 / (2 * FT) * i; v < 16 / (2 * FT) * (i + 1); ++v) l4[v & 3] += p[v];
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        using Yes = std::true_type;
        using No = std::false_type;
        if (shifted) {
            // rare: the candidate's maximum is subtracted from every exponent.  A plain loop over the key tiles, the
            // arithmetic and its order those of the pipelined steps.
            for (int kt = 0; kt < nkt; ++kt) {
                const f32x16 Sk = s_tile(kt);
                const char *vbase = kbase + (kt * FR + JS) * 1024;
                float p[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int t = 32 * kt + 8 * (v >> 2) + 4 * h + (v & 3);
                    p[v] = t < L ? __builtin_amdgcn_exp2f(Sk[v] - mc) : 0.f;
                }
                bf16x8 P0, P1;
#pragma unroll
                for (int v = 0; v < 8; ++v) {
                    P0[v] = (__bf16)p[v];
                    P1[v] = (__bf16)p[8 + v];
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) l4[v & 3] += p[v];
#pragma unroll
                for (int i = 0; i < 2 * FT; ++i)
                    O[i % FT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)(vbase + i * 1024), i < FT ? P0 : P1, O[i % FT], 0, 0, 0);
            }
        } else if (nkt > 0) {
#pragma unroll
            for (int j = 0; j < JS; ++j) kf[j] = *(const bf16x8 *)(kbase + j * 1024);
#pragma unroll
            for (int i = 0; i < 16; ++i) S[i] = 0.f;
#pragma unroll
            for (int j = 0; j < JS; ++j) S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[j], q[j], S, 0, 0, 0);
            {
                const int k1 = nkt > 1 ? 1 : 0;
#pragma unroll
                for (int j = 0; j < JS; ++j) kf[j] = *(const bf16x8 *)(kbase + (k1 * FR + j) * 1024);
            }
            __builtin_amdgcn_sched_barrier(0);
            int kt = 0;
            for (; kt + 2 < nkt; kt += 2) {
                step(kt, S, S1, Yes{}, false);
                step(kt + 1, S1, S, Yes{}, false);
            }
            if (kt + 1 < nkt) {
                step(kt, S, S1, Yes{}, false);
                S = S1;
            }
        }
        // The last S product of this item has been issued: the next item's query may take the registers.  (One site for
        // both the ordinary and the empty sequence: a second copy of these loads on another path into this point makes
        // the compiler wait, at the key-tile loop's first MFMA, for every memory operation in flight -- the item's
        // stores included.)
        if (next_item < n_items) {
            if constexpr (GATHER) {
                // the id asked for at the item's start: younger than it are at least this item's JS stores of the item block
                if (__any(live)) wait_vmcnt<JS>();
                else wait_vmcnt<0>();
                asm volatile("" : "+v"(next_raw));
                id = checked(in_request(next_tile) ? next_raw : 0, next_hd == 0);
                const char *tr = table_row(id);
#pragma unroll
                for (int j = 0; j < JS; ++j) load16_untracked(q[j], tr + (next_hd * (DH / 8) + 2 * j + h) * 16);
            } else {
                const char *xr = row_of(next_tile);
#pragma unroll
                for (int j = 0; j < JS; ++j) load16_untracked(q[j], xr + (size_t)(next_hd * (DH / 8) + 2 * j + h) * xl.piece_stride);
            }
        }
        if (!shifted && nkt > 0) step(nkt - 1, S, S1, No{}, 32 * nkt > L);
        // The next item waits for these loads with this item's 4 FT output stores still in flight (they are younger).  A
        // tile always has a candidate; should none of its lanes be live the stores are skipped, and the wait is whole.
        if (!__any(live)) wait_vmcnt<0>();

        float l = (l4[0] + l4[1]) + (l4[2] + l4[3]);
        l += __shfl_xor(l, 32, 64);
        const float inv = L > 0 ? 1.0f / l : 0.f;
        if (live) {
#pragma unroll
            for (int ft = 0; ft < FT; ++ft)
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) {
                    bf16x4 o4;
#pragma unroll
                    for (int i = 0; i < 4; ++i) o4[i] = (__bf16)(O[ft][4 * qd + i] * inv);
                    store_stream((bf16x4 *)piece((m.d_item + hd * DH) / 8 + 4 * ft + qd) + h, o4);
                }
        }
        item = next_item;
        tile = next_tile;
        hd = next_hd;
    }
}

// Host: groups of tiles for k_attn_res -- of the requests whose K/V fit; *n_streamed = the requests left to the
// streaming kernels (those that do not fit; all, when the model has no resident kernel).
size_t attn_max_groups(size_t x_rows, int max_users) { return x_rows / (32 * RES_WAVES) + (size_t)max_users + 1; }

int attn_plan_groups(const Model &m, const ReqDesc *reqs, int n_req, int n_cu, AttnGroup *out, int *n_streamed, AttnPlanInfo *info)
{
    if (info) *info = AttnPlanInfo{RES_WAVES, 0u};
    *n_streamed = 0;
    for (int r = 0; r < n_req; ++r) *n_streamed += reqs[r].n_cand > 0;
    if (m.n_heads > RES_MAX_HEADS || m.d_item / 8 > RES_MAX_ITEM_PIECES) return 0;
    if (m.d_head != 64 && m.d_head != 32) return 0;       // the resident kernel has these two head widths
    long total = 0;
    for (int r = 0; r < n_req; ++r)
        if (res_fits(m, reqs[r].seq_len)) total += (reqs[r].n_cand + 31) / 32;
    if (total == 0) return 0;
    // about one group per CU (its waves take the (tile, head) items one at a time, so a group need not be whole rounds)
    long per = (total + n_cu - 1) / n_cu;
    if (per < RES_WAVES) per = RES_WAVES;
    if (info) info->per = (int32_t)per;
    int n = 0;
    for (int r = 0; r < n_req; ++r) {
        const int tiles = (reqs[r].n_cand + 31) / 32;
        if (tiles == 0 || !res_fits(m, reqs[r].seq_len)) continue;
        --*n_streamed;
        if (info && r < 32) info->resident |= 1u << r;
        const int ng = (int)((tiles + per - 1) / per);
        for (int i = 0; i < ng; ++i)          // even split: sizes differ by at most one tile
            out[n++] = AttnGroup{r, (int)((long)tiles * i / ng), (int)((long)tiles * (i + 1) / ng), 0};
    }
    return n;
}

// ---- dispatch -----------------------------------------------------------------
int attn_mfma_variant(const Model &m, bool has_wq)
{
    if (attn_proj_ok(m, has_wq)) return ATTN_VARIANT_PROJ;
    if (m.dtype != 1 || has_wq) return -1;
    if (m.cross_mode == 3) {
        // BEA on the matrix cores: whole 32-feature tiles, the window inside the row, fragments within budget
        const BeaGeom g = bea_geom(m);
        if (m.d_cv % 32 || g.piece0 < 0 || g.ksb * g.ftc > BEA_MAX_FRAGS) return -1;
    } else if (m.cross_mode != 0 && m.cross_mode != 1)
        return -1;
    if (m.d_head == 64) return 0;
    if (m.d_head == 32) return 1;
    return -1;
}

size_t attn_pack_stride(const Model &m, int max_seq_len, int *nktp_out)
{
    if (m.d_head == 16) return attn_proj_pack_stride(m, max_seq_len, nktp_out);
    const int nktp = ((((max_seq_len + 31) >> 5) + 1) & ~1);
    if (nktp_out) *nktp_out = nktp;
    return (size_t)m.n_heads * nktp * (m.d_head / 8) * 1024;
}

static int n_compute_units()
{
    static int n_cu = 0;
    if (!n_cu) {
        int dev = 0;
        hipDeviceProp_t prop;
        n_cu = (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
                   ? prop.multiProcessorCount : 256;
    }
    return n_cu;
}

// Up to this many 32-candidate tiles in the batch the key-split kernel serves the streamed requests
// (eight waves a tile: beyond two tiles per compute unit the SIMDs are full without it).
static int split_max_tiles()
{
    static int n = -1;
    if (n < 0) {
        const char *e = getenv("AIF_SPLIT_TILES");      // measurement: where the key-split kernel stops paying
        n = e ? atoi(e) : 2 * n_compute_units();
    }
    return n;
}

// A batch too small to give every compute unit an eight-wave block of the streaming kernels (a single
// 10^4-candidate request is 40 of them) is cut finer: same arithmetic per candidate, more compute units at work.
static bool small_batch(const Batch &b) { return b.n_blk < n_compute_units(); }

template <int DH, int WAVES>
static void launch_streaming(const Model &m, const Batch &b, void *X, char *kvpack, size_t stride, float *kmax, int nktp, hipStream_t s)
{
    constexpr int LDS = 4 * 2 * (DH / 8) * 1024, ROWS = WAVES * 32;
    hipLaunchKernelGGL((k_attn_mfma<DH, WAVES>), dim3(b.n_blk * (ROW_BLOCK / ROWS)), dim3(WAVES * 64), LDS, s, m, b,
                       (char *)X, x_layout(m), (const char *)kvpack, stride, (const float *)kmax, nktp);
}

template <int DH>
static hipError_t launch_attn_spec(const Model &m, const Batch &b, void *X, char *kvpack, size_t stride, float *kmax,
                                   int nktp, bool kv_packed, const void *gather_table, int32_t *bad, hipStream_t s)
{
    if (nktp > 0 && !kv_packed)
        hipLaunchKernelGGL(k_pack_kv<DH>, dim3(nktp / 2, m.n_heads, b.n_slots), dim3(256), 0, s, m, b, kvpack, stride, kmax, nktp);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_attn_res<DH, false>, hipFuncAttributeMaxDynamicSharedMemorySize, RES_LDS_BYTES);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)k_attn_res<DH, true>, hipFuncAttributeMaxDynamicSharedMemorySize, RES_LDS_BYTES);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)k_attn_split<DH, KEY_PARTS>, hipFuncAttributeMaxDynamicSharedMemorySize, split_lds_bytes<DH>());
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)k_attn_split<DH, KEY_PARTS / 2>, hipFuncAttributeMaxDynamicSharedMemorySize, split_lds_bytes<DH>());
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    // the requests whose K/V fit in LDS: the resident kernel
    if (b.n_groups > 0) {
        if (gather_table)
            hipLaunchKernelGGL((k_attn_res<DH, true>), dim3(b.n_groups), dim3(RES_WAVES * 64), RES_LDS_BYTES, s, m, b, (char *)X,
                               x_layout(m), (const char *)kvpack, stride, (const float *)kmax, nktp,
                               (const char *)gather_table, bad);
        else
            hipLaunchKernelGGL((k_attn_res<DH, false>), dim3(b.n_groups), dim3(RES_WAVES * 64), RES_LDS_BYTES, s, m, b, (char *)X,
                               x_layout(m), (const char *)kvpack, stride, (const float *)kmax, nktp, (const char *)nullptr,
                               (int32_t *)nullptr);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess || b.n_streamed == 0) return e;
    }
    // the others: the streaming kernels (their blocks leave the resident kernel's requests alone)
    if (gather_table) return hipErrorInvalidValue;      // only the resident kernel gathers: the caller asked attn_gathers()
    const int tiles = b.n_blk * (ROW_BLOCK / 32);
    if (tiles <= n_compute_units() && tiles <= split_max_tiles())
        hipLaunchKernelGGL((k_attn_split<DH, KEY_PARTS>), dim3(tiles), dim3(KEY_PARTS * 64), split_lds_bytes<DH>(), s, m, b, (char *)X,
                           x_layout(m), (const char *)kvpack, stride, (const float *)kmax, nktp);
    else if (tiles <= split_max_tiles())
        hipLaunchKernelGGL((k_attn_split<DH, KEY_PARTS / 2>), dim3(tiles), dim3(KEY_PARTS / 2 * 64), split_lds_bytes<DH>(), s, m, b,
                           (char *)X, x_layout(m), (const char *)kvpack, stride, (const float *)kmax, nktp);
    else if (small_batch(b))
        launch_streaming<DH, 2>(m, b, X, kvpack, stride, kmax, nktp, s);
    else
        launch_streaming<DH, 8>(m, b, X, kvpack, stride, kmax, nktp, s);
    return hipGetLastError();
}

// Whether the attention launch of this batch also indexes the item table: k_attn_res with GATHER (no W_q, the
// plan's variants 0 and 1) when K/V are resident (the batch has tile groups), k_attn_proj with GATHER always.
bool attn_gathers(const Model &m, const Batch &b, const MfmaPlan &plan)
{
    if (m.dtype != 1 || !plan.attn || b.n_blk == 0) return false;
    if (plan.attn_variant == ATTN_VARIANT_PROJ) return true;
    return (plan.attn_variant == 0 || plan.attn_variant == 1) && b.n_groups > 0 && b.n_streamed == 0;
}

hipError_t launch_attn_variant(const Model &m, const Batch &b, void *X, const MfmaPlan &plan, bool kv_packed,
                               const void *gather_table, int32_t *bad, hipStream_t s)
{
    if (b.n_blk == 0) return hipSuccess;
    char *kvpack = plan.kvpack;
    float *kmax = plan.kmax;
    const size_t stride = plan.pack_stride;
    const int nktp = plan.nktp;
    switch (plan.attn_variant) {
    case ATTN_VARIANT_PROJ: return launch_attn_proj(m, b, X, plan, small_batch(b), kv_packed, s, gather_table, bad);
    case 0: return launch_attn_spec<64>(m, b, X, kvpack, stride, kmax, nktp, kv_packed, gather_table, bad, s);
    case 1: return launch_attn_spec<32>(m, b, X, kvpack, stride, kmax, nktp, kv_packed, gather_table, bad, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace aif
