// a6-a7 on the matrix cores -- the MLP head (Sec. 1: a light MLP of few
// layers) as one fused bf16 MFMA chain.
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
// Weights stream through a ring in LDS, shared by the waves of the block; each
// wave owns one column tile of 32 candidates.  The user block of layer 1
// arrives as the per-request bias (user fold), the final ->1 layer is a dot
// product in the epilogue.
//
// This header holds the kernel template and its launcher; each chain shape is instantiated in a translation unit
// of its own (k_mlp_chain_*.hip) so that they compile side by side.
#pragma once
#include <utility>

#include "k_mfma.h"
#include "mfma_util.h"

namespace aif {


typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef const f32x4 __attribute__((address_space(3))) *lds_f32x4_t;


template <int N> struct IC { static constexpr int value = N; };
template <int I0, class F, int... Is> __device__ __forceinline__ void static_for_seq(F &&f, std::integer_sequence<int, Is...>)
{
    (f(IC<I0 + Is>{}), ...);
}
// f(IC<I>{}), ..., f(IC<N - 1>{}): runs of at most 256 steps as one fold expression each -- the widest chain is a
// straight line of 2,176 steps, more than the compiler's limits on template recursion or on the terms of one fold
template <int I, int N, class F> __device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        constexpr int n = N - I < 256 ? N - I : 256;
        static_for_seq<I>(f, std::make_integer_sequence<int, n>{});
        static_for<I + n, N>(f);
    }
}


__device__ __forceinline__ float relu(float x) { return __builtin_amdgcn_fmed3f(x, 0.f, __builtin_inff()); }

// Static description of the chain.  The weights of all hidden layers form ONE
// stream of 1 KB fragments (fragment = the A operand of one MFMA: 32 output
// features x 16 contraction indices), in the order the MFMAs consume them:
// layer by layer, row tile by row tile, k-step by k-step.  The stream is cut
// into stages of SF fragments that travel through a ring of SLOTS slots in LDS.
template <int K1, int H1, int H2, int H3, int WAVES, int SF, int SLOTS> struct Chain {
    static constexpr int NH = H3 ? 3 : (H2 ? 2 : 1);
    static constexpr int kin(int l) { return l == 0 ? K1 : (l == 1 ? H1 : H2); }
    static constexpr int nout(int l) { return l == 0 ? H1 : (l == 1 ? H2 : H3); }
    static constexpr int ks(int l) { return kin(l) / 16; }                     // k-steps (fragments) per row tile
    static constexpr int nfl(int l) { return l < NH ? nout(l) / 32 * ks(l) : 0; }   // fragments of layer l
    static constexpr int fbase(int l) { int n = 0; for (int i = 0; i < l; ++i) n += nfl(i); return n; }
    static constexpr int nf() { return fbase(3); }
    static constexpr int ns() { return nf() / SF; }
    static constexpr int tbase(int l) { int n = 0; for (int i = 0; i < l && i < NH; ++i) n += nout(i) / 32; return n; }
    static constexpr int nt() { return tbase(3); }
    // fragment F of the stream -> layer, global row tile, k-step, byte offset in the ring
    static constexpr int flayer(int F) { return F < fbase(1) ? 0 : (F < fbase(2) ? 1 : 2); }
    static constexpr int ftile(int F) { return tbase(flayer(F)) + (F - fbase(flayer(F))) / ks(flayer(F)); }
    static constexpr int fk(int F) { return (F - fbase(flayer(F))) % ks(flayer(F)); }
    // a block runs the stream twice (two tiles): pass P continues the ring where pass P - 1 left it
    static constexpr int slot(int I, int P) { return (I + P * ns()) % SLOTS; }
    static constexpr int foff(int F, int P) { return slot(F / SF, P) * SF * 1024 + (F % SF) * 1024; }
    static constexpr int tlayer(int T) { return T < tbase(1) ? 0 : (T < tbase(2) ? 1 : 2); }
    static constexpr int trt(int T) { return T - tbase(tlayer(T)); }
    // The epilogue of row tile T - 1 runs in four parts at k-steps epos(0..3) of row tile T, and at
    // k-step kinit the accumulator of row tile T + 1 is preloaded with its biases.
    static constexpr int estep(int KS) { return (KS - 8) / 4 < 1 ? 1 : (KS - 8) / 4; }
    static constexpr int epos(int q, int KS) { return 1 + q * estep(KS); }
    static constexpr int kinit(int KS) { return epos(3, KS) + 1; }
    static constexpr int LPW = SF / WAVES;                                      // loads per wave and stage
    static constexpr int HL = NH == 1 ? H1 : (NH == 2 ? H2 : H3);              // width entering the ->1 layer
    static constexpr int bias_floats = 2 * H1 + H2 + H3 + HL + 1;              // layer-1 biases (per request): one set per tile of the pair; the ->1 layer's bias last
    static constexpr int ring_bytes = SLOTS * SF * 1024;
    static constexpr int lds_bytes = ring_bytes + 4 * bias_floats;
    static_assert(SF % WAVES == 0, "every wave moves the same number of fragments per stage");
    static_assert(nfl(0) % SF == 0 && nfl(1) % SF == 0 && nfl(2) % SF == 0, "a stage lies inside one layer");
    static_assert(SLOTS >= 3, "a stage is confirmed half a stage before its first read");
    static_assert(lds_bytes <= 160 * 1024, "LDS");
};

// Copy stage I of the weight stream global -> LDS slot: a wave moves whole 1 KB
// fragments, no register staging.
// w0: layer 1's fragments when they are the tile's user's own (UW), else null: the model's (pk.w[0])
template <class C, int WAVES, int SF, int SLOTS, int I, int P = 0>
__device__ __forceinline__ void issue_stage(const MlpPack &pk, char *lds, const char *w0 = nullptr)
{
    if constexpr (I < C::ns()) {
        constexpr int l = C::flayer(I * SF);
        const int lane = threadIdx.x & 63;
        const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        const char *base = pk.w[l];
        if constexpr (l == 0)
            if (w0) base = w0;
        const char *src = base + (size_t)(I * SF - C::fbase(l)) * 1024 + wave * 1024;     // wave-uniform
        const uint32_t dst = lds_address(lds) + C::slot(I, P) * SF * 1024 + wave * 1024;
#pragma unroll
        for (int f0 = 0; f0 < SF; f0 += WAVES) dma16_s(src + f0 * 1024, lane * 16, dst + f0 * 1024);
    }
}

// K1: layer-1 contraction after the user fold; H1..H3: hidden widths (0 = absent).
// One wave = 32 candidates; a block = WAVES waves sharing the weight ring (four waves in every shape that is built).
// PER_CU blocks share a compute unit: two, out of phase with each other, where a candidate's activations of two
// consecutive layers fit in half the registers of a SIMD lane (256); one, with all 512 (the accumulation-register half
// holds the activations the matrix cores read), for the widest head: 448 -> 1024 -> 512 -> 256, whose 1024-wide
// hidden layer alone is 256 registers per lane -- still less than the trip through HBM a launch per layer costs.
//
// The body is one straight line of nf() steps, one MFMA each.  Step F
//   - asks LDS for the fragment of step F + RING - 1 (a ring of RING fragment registers keeps the
//     matrix cores fed across row tiles and stages without a bubble at their boundaries),
//   - issues its MFMA,
//   - may carry a part of the previous row tile's epilogue (ReLU, conversion to the next layer's
//     B fragments, or the partial dot with the ->1 layer) so the vector ALU works under the MFMAs,
//   - may preload the next row tile's accumulator with its biases (the bias add costs nothing then),
//   - in the middle of stage I: waits for its own share of stage I + 1, meets the other waves at
//     the block barrier (after which stage I + 1 is complete in LDS and stage I - 1 is no longer
//     read by anyone) and refills the slot of stage I - 1 with stage I + SLOTS - 1.
// The barrier is hand-issued: the compiler's own would first drain the LDS reads in flight.
//
// A block takes TWO tiles of WAVES * 32 candidates, 2 g and 2 g + 1, and runs the body twice.  What a block has to
// wait for in a row before its first MFMA -- request lookup, then its biases, then the first weights: 12,000
// cycles against the 36,000 of a tile's stream on the 256 -> 512 -> 256 head -- is paid once per pair: the
// second tile's weight stream, fragment registers and bias preload are the first tile's running on (pass 1
// finds every stage in the ring slot where pass 0's count leaves it), its request's descriptor comes by
// scalar loads at the block's start and its layer-1 biases by a direct-to-LDS load into a second buffer.
// Only its input rows cannot come early (no register is free before the first tile's last MFMA): they are
// asked for at the first tile's end and the second tile's first MFMAs wait for them.
// EH > 0: the last EH k-steps of layer 1 are the Hadamard cross block c = u (.) e (Sec. 3.3) of the first EH k-steps (the
// item block): formed here, in registers, from the item fragments and the request's operand u (kept in LDS), rounded to
// bf16 as the attention kernel would have stored it -- the workspace's cross block is then neither written nor read.
// UW: layer 1's weights are the tile's USER's own (MlpPack::w0_user, one set per user slot, made by the staging launch):
// the Hadamard cross block's share of layer 1, sum_k W1c[n, k] u_k e_k, is linear in the item vector, so it is folded
// into the item block's weights once per user, W'[n, k] = W1e[n, k] + u_k W1c[n, k] (Sec. 2: what does not depend on the
// candidate is done once) -- layer 1 then contracts over [item | attention] only.  The first stages of the stream
// then wait for the tile -> slot lookup.
template <int K1, int H1, int H2, int H3, int WAVES, int SF, int SLOTS, int PER_CU, int EH, int UW>
__global__ __launch_bounds__(WAVES * 64, PER_CU) void k_mlp_mfma(int64_t n_items, const ReqDesc *__restrict__ reqs,
                                                           const int32_t *__restrict__ blk_req,
                                                           const int32_t *__restrict__ blk_slot, const char *__restrict__ X,
                                                           XLayout xl, MlpPack pk, const float *__restrict__ bias1, int n_pairs)
{
    using C = Chain<K1, H1, H2, H3, WAVES, SF, SLOTS>;
    constexpr int THREADS = WAVES * 64, ROWS = WAVES * 32, NF = C::nf(), NS = C::ns(), NT = C::nt(), D = SLOTS - 1;
    constexpr int RING = 4;
    // The second tile's biases are first read at step FB of the first tile.  Sent at the first step of stage IB they
    // are older than every stage sent from there on, so the wait and barrier in the middle of stage IB + D - 1
    // (which leave only the D - 2 youngest stages in flight) confirm them.
    constexpr int FB = NF - C::ks(C::NH - 1) + C::kinit(C::ks(C::NH - 1));
    constexpr int IB = (FB - SF / 2 - 1) / SF - (D - 1);
    static_assert(ROW_BLOCK % ROWS == 0, "tile");
    static_assert(SF / 2 >= RING, "fragment prefetch never runs past a confirmed stage");
    static_assert(NF % RING == 0 && NT % 2 == 0, "fragment registers and accumulators carry over into the second tile");
    static_assert(IB >= 1 && IB + D <= NS && (IB + D - 1) * SF + SF / 2 < FB, "the second tile's biases are confirmed before their first read");
    static_assert(H1 * 4 % 1024 == 0 && H1 * 4 / 1024 <= WAVES, "the second tile's biases: one 1 KB load per wave");
    extern __shared__ __align__(16) char lds[];                 // the weight ring, then biases and last-layer weights
    float *sb1 = (float *)(lds + C::ring_bytes), *sb2 = sb1 + 2 * H1, *sb3 = sb2 + H2, *swl = sb3 + H3;
    constexpr int KX = K1 / 16 - EH;                            // k-steps of layer 1 read from the workspace
    uint32_t *su = (uint32_t *)(lds + C::ring_bytes + (4 * C::bias_floats + 15) / 16 * 16);    // Hadamard operands of both tiles, EH * 8 words each
    // what the end of a tile needs of its request (two whole descriptors would not fit the scalar registers)
    struct Out {
        const int32_t *cand_ids;
        float *logits_out, *scores_out;
        int32_t n_cand, row_base;
    };
    auto out_of = [&](int r) {
        const ReqDesc *q = reqs + r;
        return Out{q->cand_ids, q->logits_out, q->scores_out, q->n_cand, q->row_base};
    };
    auto cross_of = [&](int r) { return (const uint32_t *)reqs[r].cross_vecs; };

    // blocks 0 .. n_pairs - 1 take two tiles each, the blocks after them the remaining tiles one by one
    const bool has_next = (int)blockIdx.x < n_pairs;
    // UW: workgroups go to the 8 XCDs in turn, each with an L2 of its own; every XCD takes a contiguous run of the pairs,
    // so that the tiles that stream one user's layer-1 weights share an L2 instead of all eight fetching them
    int pair = (int)blockIdx.x;
    if constexpr (UW) {
        const int per_xcd = n_pairs >> 3;
        if (pair < 8 * per_xcd) pair = (pair & 7) * per_xcd + (pair >> 3);
    }
    const int tile0 = has_next ? 2 * pair : (int)blockIdx.x + n_pairs;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, col = lane & 31, h = lane >> 5;
    const int wave_u = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // The block's start is a chain of dependent memory round trips; keep it short: the weight stream
    // and the input rows do not depend on the request lookup, so they are asked for first.
    if constexpr (!UW) static_for<0, D>([&](auto s) { issue_stage<C, WAVES, SF, SLOTS, decltype(s)::value>(pk, lds); });
    bf16x8 xin[K1 / 16];
    auto load_xin = [&](int t) {
        const char *xr = X + x_offset(xl, t * ROWS + wave * 32 + col, h);
#pragma unroll
        for (int j = 0; j < KX; ++j) xin[j] = *(const bf16x8 *)(xr + (size_t)(2 * j) * xl.piece_stride);
    };
    load_xin(tile0);
    // ... and so are the layers' own biases and the ->1 weights (into registers; LDS gets them below)
    constexpr int N1 = (H1 + THREADS - 1) / THREADS, N2 = (H2 + THREADS - 1) / THREADS, N3 = (H3 + THREADS - 1) / THREADS,
                  NL = (C::HL + THREADS - 1) / THREADS;
    float g2[N2 ? N2 : 1], g3[N3 ? N3 : 1], gl[NL], gb = pk.blast[0];
    auto at = [&](const float *p, int n, int i) { return p[i < n ? i : n - 1]; };       // a thread past the end re-reads the last word
    if (C::NH >= 2)
#pragma unroll
        for (int j = 0; j < N2; ++j) g2[j] = at(pk.bias[1], H2, threadIdx.x + j * THREADS);
    if (C::NH >= 3)
#pragma unroll
        for (int j = 0; j < N3; ++j) g3[j] = at(pk.bias[2], H3, threadIdx.x + j * THREADS);
#pragma unroll
    for (int j = 0; j < NL; ++j) gl[j] = at(pk.wlast, C::HL, threadIdx.x + j * THREADS);
    // The request lookup: tile -> request (both tiles' at once) -> descriptors (both at once) -> layer-1 biases and
    // candidate ids (all at once).  Three round trips in a row, none of them behind a load it does not depend on.
    const int t1 = has_next ? tile0 + 1 : tile0;
    const int r0 = blk_req[tile0 / (ROW_BLOCK / ROWS)], r1 = blk_req[t1 / (ROW_BLOCK / ROWS)];
    // the folded layer-1 biases are kept per user slot (the slices of one candidate list share them): same round trip
    const int s0 = blk_slot[tile0 / (ROW_BLOCK / ROWS)], s1 = blk_slot[t1 / (ROW_BLOCK / ROWS)];
    const char *w0a = nullptr, *w0b = nullptr;                  // UW: the two tiles' users' layer-1 fragments
    if constexpr (UW) {
        w0a = pk.w0_user + (size_t)s0 * pk.w0_stride;
        w0b = pk.w0_user + (size_t)s1 * pk.w0_stride;
        static_for<0, D>([&](auto s) { issue_stage<C, WAVES, SF, SLOTS, decltype(s)::value>(pk, lds, w0a); });
    }
    const Out rd0 = out_of(r0), rd1 = out_of(r1);
    float g1[N1];
#pragma unroll
    for (int j = 0; j < N1; ++j) g1[j] = at(bias1 + (size_t)s0 * H1, H1, threadIdx.x + j * THREADS);
    // Which lanes will store a result, and which of them carry an id outside the table, is settled here, as two
    // wave masks per tile: the tile's end then has no load to wait for before its stores.
    // (position 0 stands in for a lane with no candidate)
    const int lc0 = tile0 * ROWS - rd0.row_base + wave * 32 + col, lc1 = t1 * ROWS - rd1.row_base + wave * 32 + col;
    const bool lv0 = h == 0 && lc0 < rd0.n_cand, lv1 = h == 0 && lc1 < rd1.n_cand;
    const int64_t id0 = rd0.cand_ids[lv0 ? lc0 : 0], id1 = rd1.cand_ids[lv1 ? lc1 : 0];
    // the two tiles' Hadamard operands, two bf16 a word (a thread past the end re-reads the last word)
    uint32_t gu0 = 0, gu1 = 0;
    if constexpr (EH > 0) {
        const int w = (int)threadIdx.x < EH * 8 ? (int)threadIdx.x : EH * 8 - 1;
        gu0 = cross_of(r0)[w];
        gu1 = cross_of(r1)[w];
    }
    // Everything asked for above is pinned here, the ids still in flight: left alone the compiler moves a load down
    // into the condition its value is stored under, behind the wait of whatever comes before it.
#pragma unroll
    for (int j = 0; j < N1; ++j) asm volatile("" : "+v"(g1[j])::"memory");
    if (C::NH >= 2)
#pragma unroll
        for (int j = 0; j < N2; ++j) asm volatile("" : "+v"(g2[j])::"memory");
    if (C::NH >= 3)
#pragma unroll
        for (int j = 0; j < N3; ++j) asm volatile("" : "+v"(g3[j])::"memory");
#pragma unroll
    for (int j = 0; j < NL; ++j) asm volatile("" : "+v"(gl[j])::"memory");
    asm volatile("" : "+v"(gb)::"memory");
    const uint64_t live0 = __ballot(lv0), live1 = __ballot(lv1);
    const uint64_t bad0 = __ballot(lv0 && (id0 < 0 || id0 >= n_items)), bad1 = __ballot(lv1 && (id1 < 0 || id1 >= n_items));
    if (threadIdx.x == 0) swl[C::HL] = gb;
    if constexpr (EH > 0) {
        if ((int)threadIdx.x < EH * 8) {
            su[threadIdx.x] = gu0;
            su[EH * 8 + threadIdx.x] = gu1;
        }
    }
#pragma unroll
    for (int j = 0; j < N1; ++j)
        if ((int)threadIdx.x + j * THREADS < H1) sb1[threadIdx.x + j * THREADS] = g1[j];
    if (C::NH >= 2)
#pragma unroll
        for (int j = 0; j < N2; ++j)
            if ((int)threadIdx.x + j * THREADS < H2) sb2[threadIdx.x + j * THREADS] = g2[j];
    if (C::NH >= 3)
#pragma unroll
        for (int j = 0; j < N3; ++j)
            if ((int)threadIdx.x + j * THREADS < H3) sb3[threadIdx.x + j * THREADS] = g3[j];
#pragma unroll
    for (int j = 0; j < NL; ++j)
        if ((int)threadIdx.x + j * THREADS < C::HL) swl[threadIdx.x + j * THREADS] = gl[j];
    wait_vmcnt<0>();
    __syncthreads();

    float zpart = 0.f;
    bf16x8 h1[C::NH >= 2 ? H1 / 16 : 1];
    bf16x8 h2[C::NH >= 3 ? H2 / 16 : 1];
    f32x16 acc[2];                          // row tiles T and T - 1 (ping-pong)
    bf16x8 areg[RING];
    f32x4 wlv[4];                           // the ->1 layer's weights for the row tile in flight

    const char *wl0 = lds + lane * 16;
    // Biases and ->1 weights are read as (one opaque per-lane base) + (immediate offset): left to itself the
    // compiler forms every such address in a register of its own, keeps the first tile's for the second and
    // spills them, and each reload waits for the whole weight ring in flight.
    uint32_t bb = lds_address(sb1) + 16 * h;
    asm volatile("" : "+v"(bb));
    constexpr int OB2 = 2 * H1, OB3 = OB2 + H2, OWL = OB3 + H3;         // float offsets of sb2, sb3, swl from sb1
    auto lds4 = [&](int float_off) -> f32x4 { return *(lds_f32x4_t)(uintptr_t)(bb + 4 * float_off); };
    auto preload_from = [&](int float_off, f32x16 &a) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x4 bv = lds4(float_off + 8 * q);
            a[4 * q + 0] = bv.x;
            a[4 * q + 1] = bv.y;
            a[4 * q + 2] = bv.z;
            a[4 * q + 3] = bv.w;
        }
    };
    // part Q of the epilogue of row tile T: the four features 8 Q + 4 h + i of this lane's candidate
    auto epi_part = [&](auto tc, auto qc) {
        constexpr int T = decltype(tc)::value, Q = decltype(qc)::value, L = C::tlayer(T), RT = C::trt(T);
        const f32x16 &a = acc[T & 1];
        if constexpr (L == C::NH - 1) {
            zpart += wlv[Q].x * relu(a[4 * Q + 0]) + wlv[Q].y * relu(a[4 * Q + 1]) + wlv[Q].z * relu(a[4 * Q + 2]) +
                     wlv[Q].w * relu(a[4 * Q + 3]);
            asm volatile("" : "+v"(zpart));         // keep the partial dot here
        } else {
            // slot s of half h <-> feature 16 j + 8 (s / 4) + 4 h + s % 4: parts 0, 1 fill k-step 2 RT, parts 2, 3 k-step 2 RT + 1
            bf16x8 &dst = [&]() -> bf16x8 & {
                if constexpr (L == 0)
                    return h1[2 * RT + (Q >> 1)];
                else
                    return h2[2 * RT + (Q >> 1)];
            }();
            constexpr int o = 4 * (Q & 1);
            dst[o + 0] = (__bf16)relu(a[4 * Q + 0]);
            dst[o + 1] = (__bf16)relu(a[4 * Q + 1]);
            dst[o + 2] = (__bf16)relu(a[4 * Q + 2]);
            dst[o + 3] = (__bf16)relu(a[4 * Q + 3]);
            // convert now: left alone the compiler keeps the fp32 values (twice the registers) until first use
            if constexpr ((Q & 1) == 1) asm volatile("" : "+v"(dst));
        }
    };
    // k-step KX + j of layer 1 of pass P: the Hadamard products of item k-step j with the request's operand, whose
    // element 16 j + 8 h + s meets slot s of this lane
    auto make_cross = [&](auto pc, auto jc) {
        constexpr int P = decltype(pc)::value, J = decltype(jc)::value;
        const bf16x8 uf = *(const bf16x8 *)((const char *)su + P * EH * 32 + J * 32 + 16 * h);
        bf16x8 cx;
#pragma unroll
        for (int s = 0; s < 8; ++s) cx[s] = (__bf16)((float)xin[J][s] * (float)uf[s]);
        xin[KX + J] = cx;
    };
    auto finish = [&](int tile, const Out &rd, uint64_t live, uint64_t bad) {      // the tile's logits and scores
        float z = zpart + __shfl_xor(zpart, 32, 64) + swl[C::HL];
        const int local = tile * ROWS - rd.row_base + wave * 32 + col;
        if ((live >> lane) & 1) {
            if ((bad >> lane) & 1) z = __uint_as_float(0x7FC00000u);
            // (stores through pointers known to be global memory: behind a store whose address space the compiler does
            // not know, the second tile's wait for its input rows becomes a wait for every memory operation in flight)
            typedef float __attribute__((address_space(1))) *gfloat_t;
            ((gfloat_t)rd.logits_out)[local] = z;
            if (rd.scores_out) ((gfloat_t)rd.scores_out)[local] = 1.0f / (1.0f + __expf(-z));
        }
    };

    preload_from(0, acc[0]);
    static_for<0, RING - 1>([&](auto fc) {
        constexpr int F = decltype(fc)::value;
        areg[F] = *(const bf16x8 *)(wl0 + C::foff(F, 0));
    });
    __builtin_amdgcn_sched_barrier(0);

    // pass P of the body; `more`: another pass follows (pass 0 of a complete pair)
    auto pass = [&](auto pc, bool more) {
        constexpr int P = decltype(pc)::value;
        static_for<0, NF>([&](auto fc) {
            constexpr int F = decltype(fc)::value;
            constexpr int L = C::flayer(F), T = C::ftile(F), K = C::fk(F), KS = C::ks(L), I = F / SF;
            if constexpr (P == 0 && F == IB * SF) {
                // the second tile's layer-1 biases travel to the second buffer (waves 0 .. H1 / 256 - 1, 1 KB each).
                // They are older than the stages sent from here on, so D stages later they have landed, like a stage.
                if (more && wave_u < H1 * 4 / 1024)
                    dma16_s((const char *)(bias1 + (size_t)s1 * H1) + wave_u * 1024, lane_off16_now(),
                            lds_address(sb1 + H1) + wave_u * 1024);
            }
            if constexpr (F % SF == SF / 2) {
                if constexpr (I + D < NS) {
                    // stage I + 1 must have landed; the D - 2 stages after it may stay in flight
                    wait_vmcnt<(D - 2) * C::LPW>();
                    asm volatile("s_barrier" ::: "memory");
                    issue_stage<C, WAVES, SF, SLOTS, I + D, P>(pk, lds, P == 0 ? w0a : w0b);
                } else {
                    bool on = false;
                    if constexpr (P == 0) on = more;
                    if (on) {
                        // the stream runs on into the second tile: stage I + D is its stage I + D - NS
                        wait_vmcnt<(D - 2) * C::LPW>();
                        asm volatile("s_barrier" ::: "memory");
                        issue_stage<C, WAVES, SF, SLOTS, I + D - NS, 1>(pk, lds, w0b);
                    } else if constexpr (I + 1 < NS) {
                        // the block's last tile: nothing more is sent; stages I + 2 .. NS - 1 may stay in flight
                        wait_vmcnt<(NS - 1 - (I + 1)) * C::LPW>();
                        asm volatile("s_barrier" ::: "memory");
                    }
                }
            }
            // the cross block's k-steps are first used at step KX of the first row tile: formed one per step before it
            if constexpr (EH > 0 && T == 0 && K < EH) make_cross(pc, IC<K>{});
            if constexpr (F + RING - 1 < NF)
                areg[(F + RING - 1) % RING] = *(const bf16x8 *)(wl0 + C::foff(F + RING - 1, P));
            else if constexpr (P == 0)      // the second tile's first fragments (read, and never used, when there is none:
                                            // an assignment under a condition would keep the old registers alive all along)
                areg[(F + RING - 1) % RING] = *(const bf16x8 *)(wl0 + C::foff(F + RING - 1 - NF, 1));
            if constexpr (L == 0)
                acc[T & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(areg[F % RING], xin[K], acc[T & 1], 0, 0, 0);
            else if constexpr (L == 1)
                acc[T & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(areg[F % RING], h1[K], acc[T & 1], 0, 0, 0);
            else
                acc[T & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(areg[F % RING], h2[K], acc[T & 1], 0, 0, 0);
            if constexpr (T > 0) {
                static_for<0, 4>([&](auto qc) {
                    if constexpr (K == C::epos(decltype(qc)::value, KS)) epi_part(IC<T - 1>{}, qc);
                });
            }
            if constexpr (K == C::kinit(KS)) {
                if constexpr (T + 1 < NT) {                       // acc of row tile T + 1 <- its biases
                    constexpr int L1 = C::tlayer(T + 1);
                    preload_from((L1 == 0 ? P * H1 : (L1 == 1 ? OB2 : OB3)) + 32 * C::trt(T + 1), acc[(T + 1) & 1]);
                } else if constexpr (P == 0)                      // the second tile's first row tile (NT is even)
                    preload_from(H1, acc[0]);
                if constexpr (L == C::NH - 1) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) wlv[q] = lds4(OWL + 32 * C::trt(T) + 8 * q);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        });
        // every register is free again: the second tile's input rows (the first's once more if there is no
        // second: unconditional, or the old rows' registers would have to stay alive through the whole tile)
        if constexpr (P == 0) load_xin(more ? tile0 + 1 : tile0);
        // the last row tile's epilogue has nothing left to hide behind
        static_for<0, 4>([&](auto qc) { epi_part(IC<NT - 1>{}, qc); });
    };

    pass(IC<0>{}, has_next);
    finish(tile0, rd0, live0, bad0);
    if (!has_next) return;
    zpart = 0.f;
    pass(IC<1>{}, false);
    finish(tile0 + 1, rd1, live1, bad1);
}

// ---- dispatch -----------------------------------------------------------------
static inline int n_cu()
{
    static int n = 0;
    if (!n) {
        int dev = 0;
        hipDeviceProp_t prop;
        n = (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
                ? prop.multiProcessorCount : 256;
    }
    return n;
}

template <int K1, int H1, int H2, int H3, int WAVES, int SF, int SLOTS, int PER_CU = 2, int EH = 0, int UW = 0>
static hipError_t launch_spec(const Model &m, const Batch &b, const void *X, const MlpPack &pk, const float *bias1,
                              hipStream_t s)
{
    using C = Chain<K1, H1, H2, H3, WAVES, SF, SLOTS>;
    constexpr int LDS = (C::lds_bytes + 15) / 16 * 16 + 2 * EH * 32;
    constexpr int ROWS = WAVES * 32;
    auto kern = k_mlp_mfma<K1, H1, H2, H3, WAVES, SF, SLOTS, PER_CU, EH, UW>;
    if (UW && !pk.w0_user) return hipErrorInvalidValue;
    static_assert(PER_CU * LDS <= 160 * 1024, "the blocks of a compute unit share its LDS");
    static_assert(EH * 8 <= WAVES * 64 && 2 * EH < K1 / 16, "Hadamard operand: one word per thread; item and cross blocks inside layer 1");
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    // Two tiles per block where there are tiles to spare: the last tile of every block a compute unit holds at a time
    // goes one per block, after the pairs, so that the launch ends evenly (a pair on a unit while others idle would
    // cost more than the pairs save), and a batch of up to that many tiles keeps every unit it can reach busy.
    const int n_tiles = b.n_blk * (ROW_BLOCK / ROWS);
    const int per_cu = PER_CU;                        // blocks a unit holds at a time
    int n_single = n_tiles < per_cu * n_cu() ? n_tiles : per_cu * n_cu();
    if ((n_tiles - n_single) & 1) ++n_single;
    const int n_pairs = (n_tiles - n_single) / 2;
    hipLaunchKernelGGL(kern, dim3(n_pairs + n_single), dim3(WAVES * 64), LDS, s, m.n_items, b.reqs, b.blk_req, b.blk_slot, (const char *)X,
                       x_layout(m), pk, bias1, n_pairs);
    return hipGetLastError();
}


}  // namespace aif
