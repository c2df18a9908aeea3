// a8 -- keep the best k of a request's candidates (Sec. 1: pre-ranking cuts
// about 10^4 candidates to about 10^2).  One 1024-thread block per request.
//
// Logits map to order-preserving 32-bit keys (NaN -> 0, the lowest; -0 -> +0).
// Four 8-bit radix passes over LDS histograms find the exact key T of the
// k-th best and how many candidates with key == T are needed (the keys of up to
// the first 20 K candidates stay in registers between the passes; logits of one
// request crowd into a few bins of the leading byte, so each wave first counts
// its lanes per bin by ballot and adds once per bin); a gather pass
// takes every key > T plus the first ties in position order (block-wide
// prefix count over contiguous position chunks), and a bitonic sort of the
// <= 4096 selected (key, ~position) pairs in LDS orders them: key descending,
// lower position first.  The result is a pure function of the logits.
//
// Before that, a shortcut that usually settles the request in one counting pass
// (requests of at most 20 K candidates): the logits are counted into 2048 bins
// that are equal intervals of [min, max] of the request's finite logits -- a
// monotone map, so every candidate of a higher bin beats every candidate of a
// lower one and equal logits share a bin.  The bin b* that holds the k-th best
// is read off the suffix sums; the candidates of the bins >= b* (k plus a
// handful when the logits are spread out) are laid out bin by bin, the highest
// bin first (the suffix sums say where each bin starts), and each finds its rank
// as its bin's start plus how many of its own bin beat it, on the same
// (key, ~position) pairs as the sort.  When
// those bins hold more than 1024 candidates (logits piled on one value) or the
// request has no two distinct finite logits, the radix passes take over.  Both
// routes give the same result: the exact top k in the order stated above.
#include "aif_dev.h"

namespace aif {

constexpr int TK_THREADS = 1024;
constexpr int TK_MAX_SLOTS = 20;           // logits per thread kept in registers at most (20 K candidates: the largest configured request)

// hist[bin] += 1 for every active lane.  Up to TK_AGG distinct bins of the wave are added with one
// atomic each (lanes counted by ballot); lanes left after that add on their own.
constexpr int TK_AGG = 3;
__device__ __forceinline__ void hist_add(uint32_t *hist, bool active, uint32_t bin)
{
    unsigned long long todo = __ballot(active);
#pragma unroll
    for (int round = 0; round < TK_AGG; ++round) {
        if (!todo) return;
        const int leader = __ffsll((long long)todo) - 1;
        const uint32_t lb = (uint32_t)__builtin_amdgcn_readlane((int)bin, leader);      // leader is wave-uniform
        const unsigned long long same = __ballot(active && bin == lb);
        if ((int)(threadIdx.x & 63) == leader) atomicAdd(&hist[lb], (uint32_t)__popcll(same));
        if (bin == lb) active = false;
        todo &= ~same;
    }
    if (active) atomicAdd(&hist[bin], 1u);
}

__device__ __forceinline__ uint32_t logit_key(float z)
{
    uint32_t u = __float_as_uint(z);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0u;        // NaN below everything
    if (u == 0x80000000u) u = 0u;                          // -0 ties with +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float key_logit(uint32_t key)      // inverse of logit_key (key 0 gives a NaN)
{
    return __uint_as_float((key & 0x80000000u) ? (key ^ 0x80000000u) : ~key);
}

// Wave-wide reductions on the data-parallel-primitive lanes of the vector ALU (a permute through the LDS path costs a
// round trip per step, and the steps depend on one another).  Every lane must be active.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t x)        // the lane CTRL names; 0 where it names none or the row is masked
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, ROW_MASK, 0xF, false);
}
template <bool MAX, int CTRL>
__device__ __forceinline__ float min_max_with(float x)
{
    const float y = __uint_as_float(dpp_or_zero<CTRL>(__float_as_uint(x)));
    return MAX ? fmaxf(x, y) : fminf(x, y);
}
__device__ __forceinline__ float lane_value(float x, int lane)
{
    return __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(x), lane));
}
template <bool MAX>
__device__ __forceinline__ float wave_min_max(float x)
{
    x = min_max_with<MAX, 0xB1>(x);             // quad_perm [1,0,3,2]: the neighbour
    x = min_max_with<MAX, 0x4E>(x);             // quad_perm [2,3,0,1]: the other pair of the quad
    x = min_max_with<MAX, 0x141>(x);            // row_half_mirror: the other quad of the eight
    x = min_max_with<MAX, 0x140>(x);            // row_mirror: the other eight of the row of 16
    const float r0 = lane_value(x, 0), r1 = lane_value(x, 16), r2 = lane_value(x, 32), r3 = lane_value(x, 48);
    return MAX ? fmaxf(fmaxf(r0, r1), fmaxf(r2, r3)) : fminf(fminf(r0, r1), fminf(r2, r3));
}
__device__ __forceinline__ uint32_t wave_prefix_sum(uint32_t x)     // inclusive, over the lanes 0 .. own
{
    x += dpp_or_zero<0x111>(x);                 // row_shr:1, 2, 4, 8: the prefix inside each row of 16
    x += dpp_or_zero<0x112>(x);
    x += dpp_or_zero<0x114>(x);
    x += dpp_or_zero<0x118>(x);
    x += dpp_or_zero<0x142, 0xA>(x);            // row_bcast:15 into rows 1 and 3: the row before
    x += dpp_or_zero<0x143, 0xC>(x);            // row_bcast:31 into rows 2 and 3: the first two rows
    return x;
}

constexpr int TKF_BINS = 2048;              // two per thread
constexpr int TKF_SELMAX = 1024;            // candidates the shortcut may have to rank

// NaN and -inf: the lowest bin, +inf: the highest (the key orders them inside it)
__device__ __forceinline__ int value_bin(float v, float lo, float scale)
{
    const float f = fminf(fmaxf((v - lo) * scale, 0.f), (float)(TKF_BINS - 1));       // fmaxf(NaN, 0) = 0
    return (int)f;
}

// FEW: the descriptors of at most TK_FEW lists arrive in the kernel's arguments (a call that has them on the host
// needs no upload then); every index into the argument array is a constant after unrolling.
// SLOTS: logits per thread kept in registers between the passes.  The block's work per pass grows with SLOTS whether
// the slots are filled or not (one compute unit does all of it), so the launch picks the smallest that holds the
// longest list; a longer list still works (its tail is re-read from memory in every radix pass).
constexpr int TK_FEW = TOPK_FEW;
struct TopkFew {
    TopkDesc d[TK_FEW];
};
template <bool FEW, int SLOTS>
__global__ __launch_bounds__(TK_THREADS) void k_topk(const TopkDesc *__restrict__ descs, TopkFew few, int k, int kpad,
                                                     int32_t *__restrict__ idx_out, float *__restrict__ val_out)
{
    extern __shared__ __align__(16) unsigned long long sel[];   // [kpad]
    __shared__ uint32_t hist[256];
    __shared__ uint32_t wave_cnt[TK_THREADS / 64];
    __shared__ uint32_t s_prefix[2], s_remaining[2], s_ngreater, s_key_count;   // [pass parity]
    __shared__ uint32_t fhist[TKF_BINS], fabove[TKF_BINS], ftaken[TKF_BINS];
    __shared__ float s_lo[TK_THREADS / 64], s_hi[TK_THREADS / 64];
    __shared__ uint32_t s_bstar, s_total;

    const int r = blockIdx.x;
    TopkDesc desc;
    if constexpr (FEW) {
        desc = few.d[0];
#pragma unroll
        for (int i = 1; i < TK_FEW; ++i)
            if (r == i) desc = few.d[i];
    } else
        desc = descs[r];
    const float *z = desc.logits;
    const int n = desc.n;
    const int tid = threadIdx.x;
    const int kk = k < n ? k : n;
    int32_t *idx_o = idx_out + (size_t)r * k;
    float *val_o = val_out + (size_t)r * k;

    for (int j = tid + kk; j < k; j += TK_THREADS) {
        idx_o[j] = -1;
        val_o[j] = -INFINITY;
    }
    if (kk == 0) return;

    if (tid == 0) {
        s_prefix[0] = 0;
        s_remaining[0] = (uint32_t)kk;
    }
    if (tid < 256) hist[tid] = 0;
    // every load is issued before the first is looked at: in the last slot in use the positions past the end re-read
    // the last logit (a load under a lane's own condition would be waited for on the spot, a round trip per slot);
    // the slots past that one are skipped by the whole block
    float zv[SLOTS];
#pragma unroll
    for (int j = 0; j < SLOTS; ++j) {
        const int i = tid + j * TK_THREADS;
        zv[j] = 0.f;
        if (j * TK_THREADS < n) zv[j] = z[i < n ? i : n - 1];
    }
    // ---- shortcut: one counting pass over value bins -------------------------------------------------
    if (n <= SLOTS * TK_THREADS) {
        // the range of the finite logits (the re-read last logit changes neither end; a NaN is passed over by fminf / fmaxf)
        float lo = INFINITY, hi = -INFINITY;
#pragma unroll
        for (int j = 0; j < SLOTS; ++j) {
            if (j * TK_THREADS < n) {
                lo = fminf(lo, zv[j]);
                hi = fmaxf(hi, zv[j]);
            }
        }
        if (__any(!(lo > -INFINITY) || !(hi < INFINITY))) {             // an infinity among them: leave those out
            lo = INFINITY;
            hi = -INFINITY;
#pragma unroll
            for (int j = 0; j < SLOTS; ++j) {
                if (j * TK_THREADS < n && fabsf(zv[j]) < INFINITY) {
                    lo = fminf(lo, zv[j]);
                    hi = fmaxf(hi, zv[j]);
                }
            }
        }
        lo = wave_min_max<false>(lo);
        hi = wave_min_max<true>(hi);
        if ((tid & 63) == 0) {
            s_lo[tid >> 6] = lo;
            s_hi[tid >> 6] = hi;
        }
        fhist[tid] = 0;
        fhist[tid + TK_THREADS] = 0;
        ftaken[tid] = 0;
        ftaken[tid + TK_THREADS] = 0;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < TK_THREADS / 64; ++w) {
            lo = fminf(lo, s_lo[w]);
            hi = fmaxf(hi, s_hi[w]);
        }
        const float scale = (float)TKF_BINS / (hi - lo);
        if (hi > lo && scale < INFINITY) {                              // the same decision in every thread
            int bin[SLOTS];                                             // kept for the collection below (-1: no candidate)
#pragma unroll
            for (int j = 0; j < SLOTS; ++j) {
                bin[j] = -1;
                if (j * TK_THREADS < n) {
                    const int b = value_bin(zv[j], lo, scale);
                    if (tid + j * TK_THREADS < n) {
                        bin[j] = b;
                        atomicAdd(&fhist[b], 1u);
                    }
                }
            }
            __syncthreads();
            // suffix sums over the bins, S[b] = candidates in bins >= b.  A thread has two bins, the higher threads the
            // lower bins, so that the sums run up the lanes.
            const int b_even = TKF_BINS - 2 - 2 * tid;
            const uint32_t h0 = fhist[b_even], h1 = fhist[b_even + 1];
            const uint32_t pfx = wave_prefix_sum(h0 + h1);
            if ((tid & 63) == 63) wave_cnt[tid >> 6] = pfx;
            __syncthreads();
            uint32_t s_even = pfx;                                      // S[b_even]
            for (int w = 0; w < (tid >> 6); ++w) s_even += wave_cnt[w];
            const uint32_t s_odd = s_even - h0;                         // S[b_even + 1]
            fabove[b_even] = s_odd;                                     // candidates in the bins above this one
            fabove[b_even + 1] = s_odd - h1;
            if (s_even >= (uint32_t)kk && s_odd < (uint32_t)kk) {
                s_bstar = b_even;
                s_total = s_even;
            }
            if (s_odd >= (uint32_t)kk && s_odd - h1 < (uint32_t)kk) {
                s_bstar = b_even + 1;
                s_total = s_odd;
            }
            __syncthreads();
            if (s_total <= (uint32_t)TKF_SELMAX) {
                // a counting sort by bin: the candidates of bin b take the slots [above[b], above[b] + count[b]) in
                // any order, so a higher bin's come first and a candidate's rank is above[b] plus how many of its own
                // bin beat it -- a look at the few that share its bin (one or two where the logits are spread out).
                // A thread seldom holds more than one or two of them: it takes them one at a time, every wave as many
                // turns as its busiest lane needs (a branch per register slot would cost every wave a turn per slot).
                const int bstar = (int)s_bstar;
                uint32_t mine_slots = 0;
#pragma unroll
                for (int j = 0; j < SLOTS; ++j) mine_slots |= bin[j] >= bstar ? 1u << j : 0u;
                while (__any(mine_slots != 0u)) {
                    const bool have = mine_slots != 0u;
                    const int j = __ffs((int)mine_slots) - 1;
                    mine_slots &= mine_slots - 1u;
                    float v = 0.f;
#pragma unroll
                    for (int jj = 0; jj < SLOTS; ++jj) v = jj == j ? zv[jj] : v;
                    if (have) {
                        const int b = value_bin(v, lo, scale);          // the bin it was counted in
                        sel[fabove[b] + atomicAdd(&ftaken[b], 1u)] =
                            ((unsigned long long)logit_key(v) << 32) | (0xFFFFFFFFu - (uint32_t)(tid + j * TK_THREADS));
                    }
                }
                __syncthreads();
                if ((uint32_t)tid < s_total) {
                    const unsigned long long mine = sel[tid];
                    const uint32_t key = (uint32_t)(mine >> 32), i = 0xFFFFFFFFu - (uint32_t)(mine & 0xFFFFFFFFull);
                    // its bin again, from the key: the key gives the logit back bit for bit, except where it merges
                    // values (NaNs, the two zeros), and those it merges share a bin
                    const int b = value_bin(key_logit(key), lo, scale);
                    const uint32_t first = fabove[b], count = fhist[b];
                    uint32_t rank = first;                              // the pairs are distinct: the ranks are a permutation
                    for (uint32_t t = 0; t < count; ++t) rank += sel[first + t] > mine ? 1u : 0u;
                    if (rank < (uint32_t)kk) {
                        idx_o[rank] = (int32_t)i;
                        val_o[rank] = key == 0u || key == 0x80000000u ? z[i] : key_logit(key);
                    }
                }
                return;
            }
        }
    }

    uint32_t kreg[SLOTS];
#pragma unroll
    for (int j = 0; j < SLOTS; ++j) kreg[j] = tid + j * TK_THREADS < n ? logit_key(zv[j]) : 0u;
    // ---- radix select -----------------------------------------------------------------------------------
    __syncthreads();
    uint32_t mask = 0;
    int par = 0;
    for (int shift = 24; shift >= 0; shift -= 8, par ^= 1) {
        const uint32_t prefix = s_prefix[par];
#pragma unroll
        for (int j = 0; j < SLOTS; ++j) {
            const int i = tid + j * TK_THREADS;
            if (j * TK_THREADS < n)                                 // uniform over the block
                hist_add(hist, i < n && (kreg[j] & mask) == prefix, (kreg[j] >> shift) & 255u);
        }
        for (int i0 = SLOTS * TK_THREADS; i0 < n; i0 += TK_THREADS) {
            const int i = i0 + tid;
            const uint32_t key = i < n ? logit_key(z[i]) : 0u;
            hist_add(hist, i < n && (key & mask) == prefix, (key >> shift) & 255u);
        }
        __syncthreads();
        // bin holding the rem-th best: suffix sums S[b] = sum_{b' >= b} hist[b'] over the 256 bins
        // (four waves, one bin per thread); the bin b with S[b] >= rem > S[b + 1] is unique
        uint32_t hv = 0, sfx = 0;
        if (tid < 256) {
            hv = hist[tid];
            hist[tid] = 0;                                  // ready for the next pass
            sfx = hv;                                       // inclusive suffix sum within the wave
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const uint32_t v = __shfl_down(sfx, o, 64);
                if ((tid & 63) + o < 64) sfx += v;
            }
            if ((tid & 63) == 0) wave_cnt[tid >> 6] = sfx;
        }
        __syncthreads();
        if (tid < 256) {
            uint32_t above = 0;                             // bins of the higher waves
            for (int w = (tid >> 6) + 1; w < 4; ++w) above += wave_cnt[w];
            const uint32_t incl = sfx + above, excl = incl - hv;
            const uint32_t rem = s_remaining[par];
            if (incl >= rem && excl < rem) {
                s_prefix[par ^ 1] = prefix | ((uint32_t)tid << shift);
                s_remaining[par ^ 1] = rem - excl;
                s_key_count = hv;                           // after the last pass: candidates with key == T
            }
        }
        mask |= 255u << shift;
        __syncthreads();
    }
    const uint32_t T = s_prefix[par];
    const uint32_t n_ties = s_remaining[par];             // >= 1 ties with key == T are taken
    const uint32_t n_greater = (uint32_t)kk - n_ties;
    const bool all_ties = s_key_count == n_ties;          // every candidate with key == T is selected

    // candidates strictly better than T: any slot in [0, n_greater)
    if (tid == 0) s_ngreater = 0;
    for (int j = tid; j < kpad; j += TK_THREADS) sel[j] = 0ull;
    __syncthreads();

    if (all_ties) {
        // the usual case (no duplicates straddling the cut): everything with key >= T, any slot order
#pragma unroll
        for (int j = 0; j < SLOTS; ++j) {
            const int i = tid + j * TK_THREADS;
            if (i < n && kreg[j] >= T) {
                const uint32_t slot = atomicAdd(&s_ngreater, 1u);
                sel[slot] = ((unsigned long long)kreg[j] << 32) | (0xFFFFFFFFu - (uint32_t)i);
            }
        }
        for (int i = SLOTS * TK_THREADS + tid; i < n; i += TK_THREADS) {
            const uint32_t key = logit_key(z[i]);
            if (key >= T) {
                const uint32_t slot = atomicAdd(&s_ngreater, 1u);
                sel[slot] = ((unsigned long long)key << 32) | (0xFFFFFFFFu - (uint32_t)i);
            }
        }
    } else {
        // ties in position order: thread t owns positions [t*chunk, (t+1)*chunk)
        const int chunk = (n + TK_THREADS - 1) / TK_THREADS;
        const int lo = tid * chunk;
        const int hi = lo + chunk < n ? lo + chunk : n;
        uint32_t my_ties = 0;
        for (int i = lo; i < hi; ++i) {
            const uint32_t key = logit_key(z[i]);
            if (key > T) {
                const uint32_t slot = atomicAdd(&s_ngreater, 1u);
                sel[slot] = ((unsigned long long)key << 32) | (0xFFFFFFFFu - (uint32_t)i);
            } else if (key == T)
                ++my_ties;
        }
        // exclusive prefix of my_ties over the block
        uint32_t incl = my_ties;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t v = __shfl_up(incl, o, 64);
            if ((tid & 63) >= o) incl += v;
        }
        if ((tid & 63) == 63) wave_cnt[tid >> 6] = incl;
        __syncthreads();
        uint32_t before = incl - my_ties;
        for (int w = 0; w < (tid >> 6); ++w) before += wave_cnt[w];
        if (my_ties && before < n_ties) {
            uint32_t rank = before;
            for (int i = lo; i < hi && rank < n_ties; ++i) {
                if (logit_key(z[i]) == T) {
                    sel[n_greater + rank] = ((unsigned long long)T << 32) | (0xFFFFFFFFu - (uint32_t)i);
                    ++rank;
                }
            }
        }
    }
    __syncthreads();

    // bitonic sort, descending, kpad a power of two; pads (0) sink to the end
    if (kpad <= 128) {
        // one wave does it alone: its LDS accesses complete in order, no block barrier per step
        if (tid < 64) {
            for (int size = 2; size <= kpad; size <<= 1) {
                for (int stride = size >> 1; stride > 0; stride >>= 1) {
                    if (tid < kpad / 2) {
                        const int a = 2 * tid - (tid & (stride - 1));
                        const int bq = a + stride;
                        const bool desc = (a & size) == 0;
                        const unsigned long long va = sel[a], vb = sel[bq];
                        if ((va < vb) == desc) {
                            sel[a] = vb;
                            sel[bq] = va;
                        }
                    }
                    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                }
            }
        }
        __syncthreads();
    } else {
        for (int size = 2; size <= kpad; size <<= 1) {
            for (int stride = size >> 1; stride > 0; stride >>= 1) {
                for (int j = tid; j < kpad / 2; j += TK_THREADS) {
                    const int a = 2 * j - (j & (stride - 1));
                    const int bq = a + stride;
                    const bool desc = (a & size) == 0;
                    const unsigned long long va = sel[a], vb = sel[bq];
                    if ((va < vb) == desc) {
                        sel[a] = vb;
                        sel[bq] = va;
                    }
                }
                __syncthreads();
            }
        }
    }
    for (int j = tid; j < kk; j += TK_THREADS) {
        const uint32_t i = 0xFFFFFFFFu - (uint32_t)(sel[j] & 0xFFFFFFFFull);
        idx_o[j] = (int32_t)i;
        val_o[j] = z[i];
    }
}

template <bool FEW>
static void launch_topk_slots(int n_max, dim3 grid, size_t lds, hipStream_t s, const TopkDesc *descs, const TopkFew &few, int k,
                              int kpad, int32_t *idx_out, float *val_out)
{
    const dim3 blk(TK_THREADS);
    if (n_max <= 1 * TK_THREADS)
        hipLaunchKernelGGL((k_topk<FEW, 1>), grid, blk, lds, s, descs, few, k, kpad, idx_out, val_out);
    else if (n_max <= 2 * TK_THREADS)
        hipLaunchKernelGGL((k_topk<FEW, 2>), grid, blk, lds, s, descs, few, k, kpad, idx_out, val_out);
    else if (n_max <= 5 * TK_THREADS)
        hipLaunchKernelGGL((k_topk<FEW, 5>), grid, blk, lds, s, descs, few, k, kpad, idx_out, val_out);
    else if (n_max <= 10 * TK_THREADS)
        hipLaunchKernelGGL((k_topk<FEW, 10>), grid, blk, lds, s, descs, few, k, kpad, idx_out, val_out);
    else
        hipLaunchKernelGGL((k_topk<FEW, TK_MAX_SLOTS>), grid, blk, lds, s, descs, few, k, kpad, idx_out, val_out);
}

hipError_t launch_topk(const TopkDesc *descs, int n_req, int n_max, int k, int32_t *idx_out, float *val_out, hipStream_t s)
{
    if (n_req == 0) return hipSuccess;
    int kpad = 2;
    while (kpad < k) kpad <<= 1;
    const int sel_slots = kpad > TKF_SELMAX ? kpad : TKF_SELMAX;
    launch_topk_slots<false>(n_max, dim3(n_req), (size_t)sel_slots * 8, s, descs, TopkFew{}, k, kpad, idx_out, val_out);
    return hipGetLastError();
}

hipError_t launch_topk_few(const TopkDesc *descs_host, int n_req, int k, int32_t *idx_out, float *val_out, hipStream_t s)
{
    if (n_req == 0) return hipSuccess;
    if (n_req > TK_FEW) return hipErrorInvalidValue;
    TopkFew few{};
    int n_max = 0;
    for (int r = 0; r < n_req; ++r) {
        few.d[r] = descs_host[r];
        n_max = descs_host[r].n > n_max ? descs_host[r].n : n_max;
    }
    int kpad = 2;
    while (kpad < k) kpad <<= 1;
    const int sel_slots = kpad > TKF_SELMAX ? kpad : TKF_SELMAX;
    launch_topk_slots<true>(n_max, dim3(n_req), (size_t)sel_slots * 8, s, nullptr, few, k, kpad, idx_out, val_out);
    return hipGetLastError();
}

}  // namespace aif
