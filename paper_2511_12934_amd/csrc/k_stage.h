// Bodies of the three kernels that stage a batch before the attention kernel
// -- a1 gather, a2 user fold, a2 K/V packing -- as device functions of a
// 256-thread block, so that each can be launched alone or all three as one
// grid (k_stage): they are independent of one another, the gather is bound by
// HBM and the other two by latency, so one launch hides the small ones under
// the gather and saves two launches.
#pragma once
#include "aif_dev.h"

namespace aif {

constexpr int GATHER_UNROLL = 4;

// Where a staging block finds its request: in the batch's device tables, or -- a batch of few requests -- in the
// kernel's own arguments (the tables are then still on their way: the same launch writes them, few_fill).
struct TableReqs {
    const Batch &b;
    __device__ __forceinline__ int block_request(int blk) const { return b.blk_req[blk]; }
    __device__ __forceinline__ ReqDesc request(int r) const { return b.reqs[r]; }
    __device__ __forceinline__ ReqDesc slot_desc(int slot) const { return b.reqs[slot_request(b, slot)]; }
};

// Descriptor tables of a batch of at most FEW_MAX requests -- the latency cases: one request, or one request cut into
// mini-batches (Sec. 5.3) -- written by the device itself from kernel arguments (no pinned staging, no copy command,
// nothing to wait for on the host): the requests, block -> request and block -> user slot, slot -> request, the
// attention groups (as attn_plan_groups cuts them) and the top-k descriptors.  Every index into the argument arrays
// is a constant after unrolling: an argument array indexed by a variable would be copied to scratch memory first.
constexpr int FEW_MAX = 16;
struct FewFill {
    ReqDesc rd[FEW_MAX];
    TopkDesc td[FEW_MAX];
    int32_t slot_req[FEW_MAX];  // slot -> a request that brings the slot's user tensors
    ReqDesc *reqs;
    int32_t *blk_req, *blk_slot, *slot_req_dev;
    AttnGroup *groups;
    TopkDesc *topk;             // null: the call selects nothing
    int32_t n_req, n_slots, n_blk, n_groups;
    int32_t per;                // tiles per attention group at most (attn_plan_groups)
    uint32_t resident;          // bit r: request r is the resident attention kernel's (it has groups)
};
// N: how many entries of the argument arrays the code looks at (1: the single request; FEW_MAX otherwise)
template <int N> __device__ __forceinline__ ReqDesc few_request(const FewFill &f, int r)
{
    ReqDesc out = f.rd[0];
#pragma unroll
    for (int i = 1; i < N; ++i)
        if (r == i) out = f.rd[i];
    return out;
}
template <int N> __device__ __forceinline__ int few_block_request(const FewFill &f, int blk)
{
    int r = -1;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const int b0 = f.rd[i].row_base / ROW_BLOCK, nb = (f.rd[i].n_cand + ROW_BLOCK - 1) / ROW_BLOCK;
        if (i < f.n_req && blk >= b0 && blk < b0 + nb) r = i;
    }
    return r;
}
template <int N> struct FewReqs {
    const FewFill &f;
    __device__ __forceinline__ int block_request(int blk) const { return few_block_request<N>(f, blk); }
    __device__ __forceinline__ ReqDesc request(int r) const { return few_request<N>(f, r); }
    __device__ __forceinline__ ReqDesc slot_desc(int slot) const
    {
        int r = f.slot_req[0];
#pragma unroll
        for (int i = 1; i < N; ++i)
            if (slot == i) r = f.slot_req[i];
        return few_request<N>(f, r);
    }
};
template <int N> __device__ __forceinline__ void few_fill(const FewFill &f, int i)
{
#pragma unroll
    for (int r = 0; r < N; ++r) {
        if (i == r && r < f.n_req) {
            f.reqs[r] = f.rd[r];
            if (f.topk) f.topk[r] = f.td[r];
        }
        if (i == r && r < f.n_slots) f.slot_req_dev[r] = f.slot_req[r];
    }
    if (i < f.n_blk) {
        const int r = few_block_request<N>(f, i);
        f.blk_req[i] = r;
        f.blk_slot[i] = r < 0 ? 0 : few_request<N>(f, r).slot;
    }
    if (i < f.n_groups) {
        // group i: the requests in order, each resident one cut evenly into ceil(tiles / per) groups
        int acc = 0;
        AttnGroup g{0, 0, 0, 0};
#pragma unroll
        for (int r = 0; r < N; ++r) {
            const int tiles = (f.rd[r].n_cand + 31) / 32;
            if (r < f.n_req && ((f.resident >> r) & 1u) && tiles > 0) {
                const int ng = (tiles + f.per - 1) / f.per;
                if (i >= acc && i < acc + ng)
                    g = AttnGroup{r, (int)((long)tiles * (i - acc) / ng), (int)((long)tiles * (i - acc + 1) / ng), 0};
                acc += ng;
            }
        }
        f.groups[i] = g;
    }
}
__host__ __device__ inline int few_fill_items(const FewFill &f)
{
    int n = f.n_blk > f.n_groups ? f.n_blk : f.n_groups;
    return n > FEW_MAX ? n : FEW_MAX;
}

// a1 -- one ROW_BLOCK of the workspace: X[row, 0:d_item] = table[id].
// LOG_RV >= 0: a row is 2^LOG_RV pieces of 16 bytes (shift instead of divide); LOG_RV < 0: any count.
template <int LOG_RV, class Reqs>
__device__ __forceinline__ void gather_block(int blk, const uint4 *__restrict__ table, int64_t n_items, int row_vec,
                                             const Reqs &src, char *__restrict__ X, const XLayout &xl,
                                             int32_t *__restrict__ bad)
{
    const int r = src.block_request(blk);
    if (r < 0) return;
    const ReqDesc rdv = src.request(r), *rd = &rdv;
    const int row_base = rd->row_base;
    const int local0 = blk * ROW_BLOCK - row_base;
    int nrows = rd->n_cand - local0;
    if (nrows <= 0) return;
    if (nrows > ROW_BLOCK) nrows = ROW_BLOCK;
    const int32_t *ids = rd->cand_ids + local0;
    char *out = X + (size_t)((row_base + local0) / X_TILE) * xl.tile_bytes;     // blocks start on tile boundaries
    if (LOG_RV >= 0) row_vec = 1 << LOG_RV;
    const int total = nrows * row_vec;
    int n_bad = 0;
    for (int base = threadIdx.x; base < total; base += 256 * GATHER_UNROLL) {
        uint4 v[GATHER_UNROLL];
        int row[GATHER_UNROLL], piece[GATHER_UNROLL];
        int64_t id[GATHER_UNROLL];
#pragma unroll
        for (int j = 0; j < GATHER_UNROLL; ++j) {
            const int idx = base + j * 256;
            row[j] = LOG_RV >= 0 ? idx >> LOG_RV : idx / row_vec;
            piece[j] = idx - row[j] * row_vec;
            id[j] = idx < total ? ids[row[j]] : 0;
        }
#pragma unroll
        for (int j = 0; j < GATHER_UNROLL; ++j) {
            if (id[j] < 0 || id[j] >= n_items) {
                id[j] = 0;
                if (piece[j] == 0) ++n_bad;
            }
            if (base + j * 256 < total) v[j] = table[(size_t)id[j] * row_vec + piece[j]];
        }
#pragma unroll
        for (int j = 0; j < GATHER_UNROLL; ++j) {
            const int idx = base + j * 256;
            if (idx < total) {
                // streaming stores: measured 1.5x faster than plain ones here (the rows are written once,
                // at a stride, and the reads that follow come from another kernel)
                uint4 *p = (uint4 *)(out + x_offset(xl, row[j], piece[j]));
                __builtin_nontemporal_store(v[j].x, &p->x);
                __builtin_nontemporal_store(v[j].y, &p->y);
                __builtin_nontemporal_store(v[j].z, &p->z);
                __builtin_nontemporal_store(v[j].w, &p->w);
            }
        }
    }
    if (n_bad) atomicAdd(bad, n_bad);
}

// a1 for the workspace in fragment order -- the same copy through LDS.  In that layout a 32-row tile keeps
// its 16-byte pieces as [piece][row], so rows written piece by piece land 512 bytes apart, 16 bytes at a
// time.  Here the block instead reads 1024 pieces per trip as whole rows (every byte of a touched row,
// four independent loads per thread), sets them down in LDS in tile order, and writes the tiles' item
// blocks as contiguous 16 KB-per-32-piece runs; the next trip's rows are already in flight during the
// exchange, and the two LDS buffers take turns so one barrier per trip is enough.
template <int LOG_RV, class Reqs>
__device__ __forceinline__ void gather_block_tiled(int blk, const uint4 *__restrict__ table, int64_t n_items,
                                                   const Reqs &src, char *__restrict__ X, const XLayout &xl,
                                                   int32_t *__restrict__ bad)
{
    constexpr int RV = 1 << LOG_RV;                      // pieces per row: 8, 16 or 32
    constexpr int NV = LOG_RV == 3 ? 8 : 4;              // 16-byte loads in flight per thread (128-byte rows: the block's 256 rows in one trip)
    constexpr int ROWS = (256 * NV) >> LOG_RV;           // rows per trip
    constexpr int PSTR = LOG_RV == 3 ? 544 : 528;        // LDS bytes per 32-row run of one piece: no bank conflicts either way
    constexpr int BUF = 8 * NV * PSTR;                   // 8 NV runs per trip
    constexpr int NBUF = ROW_BLOCK / ROWS > 1 ? 2 : 1;   // a single trip needs no second buffer
    static_assert(LOG_RV >= 3 && LOG_RV <= 5 && ROW_BLOCK % ROWS == 0, "row widths of 128, 256, 512 bytes");
    __shared__ __align__(16) char buf[NBUF * BUF];
    __shared__ int32_t sid[ROW_BLOCK];

    const int r = src.block_request(blk);
    if (r < 0) return;
    const ReqDesc rdv = src.request(r), *rd = &rdv;
    const int row_base = rd->row_base;
    const int local0 = blk * ROW_BLOCK - row_base;
    int nrows = rd->n_cand - local0;
    if (nrows <= 0) return;
    if (nrows > ROW_BLOCK) nrows = ROW_BLOCK;
    char *out = X + (size_t)((row_base + local0) / X_TILE) * xl.tile_bytes;
    {
        int64_t id = 0;
        if ((int)threadIdx.x < nrows) {
            id = rd->cand_ids[local0 + threadIdx.x];
            if (id < 0 || id >= n_items) {
                id = 0;
                atomicAdd(bad, 1);
            }
        }
        sid[threadIdx.x] = (int32_t)id;
    }
    __syncthreads();

    uint4 v[NV];
    auto fetch = [&](int trip) {
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int idx = threadIdx.x + 256 * j, row = trip * ROWS + (idx >> LOG_RV), piece = idx & (RV - 1);
            v[j] = row < nrows ? table[(size_t)sid[row] * RV + piece] : make_uint4(0, 0, 0, 0);
        }
    };
    const int ntrip = (nrows + ROWS - 1) / ROWS;
    fetch(0);
    for (int trip = 0; trip < ntrip; ++trip) {
        char *lb = buf + (trip & (NBUF - 1)) * BUF;
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int idx = threadIdx.x + 256 * j, row = idx >> LOG_RV, piece = idx & (RV - 1);
            *(uint4 *)(lb + ((row >> 5) * RV + piece) * PSTR + (row & 31) * 16) = v[j];
        }
        if (trip + 1 < ntrip) fetch(trip + 1);
        __syncthreads();
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int idx = threadIdx.x + 256 * j, run = idx >> 5, row = idx & 31;      // run = (tile of the trip, piece)
            const int tt = run >> LOG_RV, piece = run & (RV - 1);
            if (trip * ROWS + tt * 32 + row < nrows) {
                const uint4 w = *(const uint4 *)(lb + run * PSTR + row * 16);
                uint4 *p = (uint4 *)(out + (size_t)(trip * (ROWS / 32) + tt) * xl.tile_bytes + (size_t)piece * xl.piece_stride + row * 16);
                __builtin_nontemporal_store(w.x, &p->x);
                __builtin_nontemporal_store(w.y, &p->y);
                __builtin_nontemporal_store(w.z, &p->z);
                __builtin_nontemporal_store(w.w, &p->w);
            }
        }
    }
}

// a2 -- user fold: FOLD_FEATS consecutive layer-1 features n = FOLD_FEATS * part + thread % 64 of user slot s,
// bias1[s, n] = b1[n] + sum_k W1[n, k] u[k] over the user columns (w1ut = those columns transposed,
// [d_user, H1], so that the threads of a wave read consecutive words).  The job is a chain of dependent
// loads, so the columns are cut into four runs, one per wave of the 256-thread block, eight loads in flight
// each; the four partial sums are added in run order (a fixed order: the same bits in every call).
constexpr int FOLD_FEATS = 64;
template <typename T, class Reqs>
__device__ __forceinline__ void user_fold_block(int slot, int part, const Model &m, const Reqs &src,
                                                const float *__restrict__ w1ut, const float *__restrict__ b1,
                                                float *__restrict__ bias1)
{
    __shared__ float part_sum[3][FOLD_FEATS];
    const int lane = threadIdx.x & 63, run = threadIdx.x >> 6;
    const int n = part * FOLD_FEATS + lane;
    const int h1 = m.dims[1];
    const bool on = n < h1;
    const ReqDesc rdv = src.slot_desc(slot);
    const T *u = (const T *)rdv.user_vec;
    const int per = (m.d_user + 3) / 4, k0 = run * per, k1 = min(m.d_user, k0 + per);
    float acc = 0.f;
    if (on) {
        int k = k0;
        for (; k + 8 <= k1; k += 8) {
            float w[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) w[j] = w1ut[(size_t)(k + j) * h1 + n];
#pragma unroll
            for (int j = 0; j < 8; ++j) acc = fmaf(w[j], ld_f<T>(u + k + j), acc);
        }
        for (; k < k1; ++k) acc = fmaf(w1ut[(size_t)k * h1 + n], ld_f<T>(u + k), acc);
    }
    if (run > 0) part_sum[run - 1][lane] = acc;
    __syncthreads();
    if (run == 0 && on) bias1[(size_t)slot * h1 + n] = (((b1 ? b1[n] : 0.f) + acc) + part_sum[0][lane]) + (part_sum[1][lane] + part_sum[2][lane]);
}

// a2 -- layer 1's weights of user slot `slot` with the cross block folded in (Model::cross_in_mlp == 2).
// Hadamard (Sec. 3.3): the block's share of a layer-1 pre-activation, sum_k W1c[n, k] u_k e_k, is linear in the item
// vector e, so
//   W'[n, k] = bf16(W1e[n, k] + u_k W1c[n, k])        (the product is exact in fp32, the sum rounded once)
// takes its place and layer 1 contracts over [item | attention] only.
// BEA (Sec. 4.1, Algorithm 1 step 4): the block is v^ = w^ V with the bridge weights w^ = the item row's last n_cross
// entries, so its share is sum_j e[d_item - n_cross + j] M[n, j] with M = W1c V^T, a matrix of the user alone:
//   W'[n, d_item - n_cross + j] = bf16(W1e[n, .] + sum_f W1c[n, f] V[j, f])   (fp32 sums in the order of f).
// Segment dots (Sec. 3.3; c[j S + s] = <Vc_j, e_s> over the S = d_item / d_cv segments e_s of the item vector): the
// share is sum_s sum_k e[s d_cv + k] sum_j W1c[n, j S + s] Vc[j, k], so
//   W'[n, s d_cv + k] = bf16(W1e[n, .] + sum_j W1c[n, j S + s] Vc[j, k])      (fp32 sums in the order of j).  Source and result are in the MLP chain's
// fragment order (k_mlp_mfma.hip): fragment (row tile rt, k-step j) = 64 lanes x 8 values, lane (n = 32 rt + lane % 32,
// h = lane / 32) holding k = 16 j + 8 h + s; the source has K1 / 16 k-steps [item | attention | cross] per row tile,
// the result (d_item + d_attn) / 16; the attention block's fragments are copied.  One 16-byte piece a thread.
constexpr int FOLD_PIECES = 4;              // 16-byte pieces of the result a thread makes
constexpr int FOLD_BEA_V = 2048;            // BEA: n_cross * d_cv values of the user's vectors a block keeps in LDS
constexpr int FOLD_BEA_DCV = 64;            // ... and the widest vector
constexpr int FOLD_SEG_CHUNK = 16;          // segment dots: vectors taken at a time
struct FoldW0 {
    const uint4 *src;           // the model's layer-1 fragments, [H1 / 32][K1 / 16][64] pieces
    uint4 *dst;                 // [slot][H1 / 32][(d_item + d_attn) / 16][64] pieces
    size_t stride;              // bytes per slot
    int32_t blocks_per_slot;
};
__device__ __forceinline__ uint32_t fold_pair(uint32_t we, uint32_t wc, uint32_t u)
{
    auto lo = [](uint32_t v) { return __uint_as_float(v << 16); };
    auto hi = [](uint32_t v) { return __uint_as_float(v & 0xFFFF0000u); };
    auto bf = [](float f) {                          // round to nearest even; the operands are finite
        const uint32_t b = __float_as_uint(f);
        return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
    };
    return bf(fmaf(lo(u), lo(wc), lo(we))) | (bf(fmaf(hi(u), hi(wc), hi(we))) << 16);
}
template <class Reqs>
__device__ __forceinline__ void fold_w0_block(int slot, int part, const Model &m, const Reqs &src, const FoldW0 &f)
{
    const int ks_e = m.d_item / 16, ks_new = (m.d_item + m.d_attn) / 16, ks_old = m.k1 / 16;
    const int n_piece = m.dims[1] / 32 * ks_new * 64;
    // BEA: the user's vectors (at most FOLD_BEA_V values) once per block, widened to fp32, in LDS: every lane of a
    // wave reads the same entry at a time
    __shared__ float4 sV[FOLD_BEA_V / 4];
    if (m.cross_mode == 3 || m.cross_mode == 2) {
        const uint2 *Vg = (const uint2 *)src.slot_desc(slot).cross_vecs;            // [n_cross, d_cv], four values a step
        for (int i = threadIdx.x; i < m.n_cross * m.d_cv / 4; i += 256) {
            const uint2 v = Vg[i];
            sV[i] = make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xFFFF0000u), __uint_as_float(v.y << 16),
                                __uint_as_float(v.y & 0xFFFF0000u));
        }
        __syncthreads();
    }
    if (m.cross_mode == 2) {
        // Segment dots: a thread takes one k-step (two 16-byte pieces) of one (row n, segment sg) of the user's weights --
        // entries W'[n, sg d_cv + 16 qk ..], which use the n_cross weights W1c[n, jv S + sg] -- and its share of the
        // attention block's pieces (copies).
        const int S = m.d_item / m.d_cv, H1 = m.dims[1], ksc = m.d_cv / 16;
        const int t = part * 256 + (int)threadIdx.x;                    // row-minor: a wave's lanes are consecutive rows
        if (t >= H1 * S * ksc) return;
        const int qk = t / (H1 * S), sg = (t / H1) % S, n = t % H1, rt = n >> 5, ln = n & 31;
        auto lo = [](uint32_t v) { return __uint_as_float(v << 16); };
        auto hi = [](uint32_t v) { return __uint_as_float(v & 0xFFFF0000u); };
        auto bf = [](float v) {
            const uint32_t b = __float_as_uint(v);
            return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
        };
        // entry c of row n of W1c is slot c % 8 of lane n % 32 + 32 ((c % 16) / 8) of cross k-step c / 16; a vector past
        // the last re-reads the last and counts for nothing
        const uint16_t *src16 = (const uint16_t *)f.src;
        uint4 *dslot = f.dst + (size_t)slot * (f.stride / 16);
        // the two halves of k-step sg ksc + qk; both asked for before the first is looked at
        const int j = sg * ksc + qk;
        const uint4 wes[2] = {f.src[(size_t)(rt * ks_old + j) * 64 + ln], f.src[(size_t)(rt * ks_old + j) * 64 + ln + 32]};
        float acc[2][8];
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[h][i] = 0.f;
        // the vectors in the order of jv, FOLD_SEG_CHUNK at a time (no exit inside a chunk: a vector past the last
        // re-reads the last and counts for nothing)
        for (int jv0 = 0; jv0 < m.n_cross; jv0 += FOLD_SEG_CHUNK) {
            float wj[FOLD_SEG_CHUNK];
#pragma unroll
            for (int u = 0; u < FOLD_SEG_CHUNK; ++u) {
                const int jv = jv0 + u, c = (jv < m.n_cross ? jv : m.n_cross - 1) * S + sg;
                const uint16_t w = src16[((size_t)(rt * ks_old + ks_new + (c >> 4)) * 64 + ln + 32 * ((c >> 3) & 1)) * 8 + (c & 7)];
                wj[u] = jv < m.n_cross ? __uint_as_float((uint32_t)w << 16) : 0.f;
            }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int kk0 = 16 * qk + 8 * h;
#pragma unroll
                for (int u = 0; u < FOLD_SEG_CHUNK; ++u) {
                    const int jv = jv0 + u, row = jv < m.n_cross ? jv : m.n_cross - 1;
                    const float4 va = sV[(row * m.d_cv + kk0) / 4], vb = sV[(row * m.d_cv + kk0) / 4 + 1];
                    acc[h][0] = fmaf(wj[u], va.x, acc[h][0]);
                    acc[h][1] = fmaf(wj[u], va.y, acc[h][1]);
                    acc[h][2] = fmaf(wj[u], va.z, acc[h][2]);
                    acc[h][3] = fmaf(wj[u], va.w, acc[h][3]);
                    acc[h][4] = fmaf(wj[u], vb.x, acc[h][4]);
                    acc[h][5] = fmaf(wj[u], vb.y, acc[h][5]);
                    acc[h][6] = fmaf(wj[u], vb.z, acc[h][6]);
                    acc[h][7] = fmaf(wj[u], vb.w, acc[h][7]);
                }
            }
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            uint32_t ow[4] = {wes[h].x, wes[h].y, wes[h].z, wes[h].w};
#pragma unroll
            for (int i = 0; i < 4; ++i) ow[i] = bf(lo(ow[i]) + acc[h][2 * i]) | (bf(hi(ow[i]) + acc[h][2 * i + 1]) << 16);
            dslot[(size_t)(rt * ks_new + j) * 64 + ln + 32 * h] = make_uint4(ow[0], ow[1], ow[2], ow[3]);
        }
        // the attention block's fragments, copied: piece (row tile, k-step ks_e + ja, lane)
        const int ks_a = ks_new - ks_e, n_copy = H1 / 32 * ks_a * 64;
        for (int i = t; i < n_copy; i += H1 * S * ksc) {
            const int lane = i & 63, ja = (i >> 6) % ks_a, rt2 = (i >> 6) / ks_a;
            dslot[(size_t)(rt2 * ks_new + ks_e + ja) * 64 + lane] = f.src[(size_t)(rt2 * ks_old + ks_e + ja) * 64 + lane];
        }
        return;
    }
    // FOLD_PIECES pieces a thread (few, fat blocks: the launch's blocks all carry the gather's LDS, and a second round of
    // them would cost more than the pieces do)
#pragma unroll
    for (int it = 0; it < FOLD_PIECES; ++it) {
    const int p = min((part * FOLD_PIECES + it) * 256 + (int)threadIdx.x, n_piece - 1);     // piece of the slot's result (past the end: the last again)
    const int lane = p & 63, j = (p >> 6) % ks_new, rt = (p >> 6) / ks_new, h = lane >> 5;
    uint4 out = f.src[(size_t)(rt * ks_old + j) * 64 + lane];
    if (m.cross_mode == 3) {
        const int w0 = m.d_item - m.n_cross, k0 = 16 * j + 8 * h;       // this piece holds k0 .. k0 + 7 of row n
        if (j < ks_e && k0 + 8 > w0) {
            auto lo = [](uint32_t v) { return __uint_as_float(v << 16); };
            auto hi = [](uint32_t v) { return __uint_as_float(v & 0xFFFF0000u); };
            // row n of W1c, eight entries a piece (a piece index past the row re-reads the last: no load under a condition)
            const int nf8 = m.d_cv / 8;
            uint4 wc[FOLD_BEA_DCV / 8];
#pragma unroll
            for (int f8 = 0; f8 < FOLD_BEA_DCV / 8; ++f8) {
                const int g = f8 < nf8 ? f8 : nf8 - 1;
                wc[f8] = f.src[(size_t)(rt * ks_old + ks_new + (g >> 1)) * 64 + (lane & 31) + 32 * (g & 1)];
            }
            float wf[FOLD_BEA_DCV];                                     // ... widened once
#pragma unroll
            for (int f8 = 0; f8 < FOLD_BEA_DCV / 8; ++f8) {
                const uint32_t ww[4] = {wc[f8].x, wc[f8].y, wc[f8].z, wc[f8].w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {                           // (entries past the row's end: zero, they add nothing)
                    wf[8 * f8 + 2 * i] = f8 < nf8 ? lo(ww[i]) : 0.f;
                    wf[8 * f8 + 2 * i + 1] = f8 < nf8 ? hi(ww[i]) : 0.f;
                }
            }
            float acc[8];
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                acc[s] = 0.f;
                const int jb = k0 + s - w0;
                if (jb < 0) continue;
#pragma unroll
                for (int f4 = 0; f4 < FOLD_BEA_DCV / 4; ++f4) {         // in the order of f; no exit inside: the indices stay constants
                    const float4 vv = sV[jb * 2 * nf8 + (f4 < 2 * nf8 ? f4 : 2 * nf8 - 1)];
                    acc[s] = fmaf(wf[4 * f4 + 0], vv.x, acc[s]);
                    acc[s] = fmaf(wf[4 * f4 + 1], vv.y, acc[s]);
                    acc[s] = fmaf(wf[4 * f4 + 2], vv.z, acc[s]);
                    acc[s] = fmaf(wf[4 * f4 + 3], vv.w, acc[s]);
                }
            }
            auto bf = [](float v) {
                const uint32_t b = __float_as_uint(v);
                return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
            };
            uint32_t ow[4] = {out.x, out.y, out.z, out.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t a = k0 + 2 * i >= w0 ? bf(lo(ow[i]) + acc[2 * i]) : (ow[i] & 0xFFFFu);
                const uint32_t b2 = k0 + 2 * i + 1 >= w0 ? bf(hi(ow[i]) + acc[2 * i + 1]) : (ow[i] >> 16);
                ow[i] = a | (b2 << 16);
            }
            out = make_uint4(ow[0], ow[1], ow[2], ow[3]);
        }
    } else if (j < ks_e) {
        const uint4 wc = f.src[(size_t)(rt * ks_old + ks_new + j) * 64 + lane];
        const uint4 u = ((const uint4 *)src.slot_desc(slot).cross_vecs)[2 * j + h];
        out.x = fold_pair(out.x, wc.x, u.x);
        out.y = fold_pair(out.y, wc.y, u.y);
        out.z = fold_pair(out.z, wc.z, u.z);
        out.w = fold_pair(out.w, wc.w, u.w);
    }
    f.dst[(size_t)slot * (f.stride / 16) + p] = out;
    }
}

// a2 -- K and V of user slot `slot` (the tensors of the request that stands for it), head hd, 64-key stage st into MFMA fragment order, and max |k_t| of the stage.
// Layout per slot: chunk(head, key tile kt) = FR fragments of 1 KB at
// ((head * nktp + kt) * FR) KB:  JS K-fragments  [lane][s] = K[32kt + lane%32][o + 16j + 8(lane/32) + s]
// then 2*FT V-fragments (jj, ft): [lane][s] = V[32kt + 16jj + 8(s/4) + 4(lane/32) + s%4][o + 32ft + lane%32]
// with o = head * DH; keys >= seq_len read as zero.
// Eight keys' elements of one piece, each times `scale` and rounded to bf16 again (nearest even: the hardware's
// conversion, two values an instruction).
__device__ __forceinline__ uint4 scaled_bf16x8(uint4 v, float scale)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        bf16x2_t r;
        r[0] = (__bf16)(__uint_as_float(w[j] << 16) * scale);
        r[1] = (__bf16)(__uint_as_float(w[j] & 0xFFFF0000u) * scale);
        w[j] = __builtin_bit_cast(uint32_t, r);
    }
    return make_uint4(w[0], w[1], w[2], w[3]);
}

// The keys are packed times log2(e) / sqrt(d_head): the first product of the attention kernels then IS the exponent of
// the softmax weight in base 2 (Sec. 3.3's scaled dot product, the scale and the change of base done once per user and
// key instead of once per candidate and key; one more rounding of the key to bf16).
constexpr float ATTN_LOG2E = 1.4426950408889634f;
template <int DH, class Reqs>
__device__ __forceinline__ void pack_kv_block(int slot, int hd, int st, const Model &m, const Reqs &src,
                                              char *__restrict__ kvpack, size_t pack_stride,
                                              float *__restrict__ kmax_part, int nktp)
{
    constexpr int FR = DH / 8, JS = DH / 16, FT = DH / 32;
    const ReqDesc rdv = src.slot_desc(slot), *rd = &rdv;
    const int L = rd->seq_len;
    const int nkt2 = (((L + 31) >> 5) + 1) & ~1;
    if (2 * st >= nkt2) return;
    const float kscale = ATTN_LOG2E / sqrtf((float)DH);
    const uint16_t *K = (const uint16_t *)rd->seq_keys, *V = (const uint16_t *)rd->seq_vals;
    const int da = m.d_attn, o = hd * DH;
    uint4 *dst = (uint4 *)(kvpack + (size_t)slot * pack_stride + ((size_t)(hd * nktp + 2 * st) * FR) * 1024);
    // One 16-byte piece (a lane's share of a fragment) per thread and step.  Every load is issued before the first
    // is looked at: keys past the sequence's end re-read its last key and are zeroed afterwards (a load under a
    // condition of its own is waited for on the spot -- eight round trips in a row for a piece of V).
    constexpr int STEPS = 2 * FR * 64 / 256;
    uint4 kpiece[STEPS];
    uint32_t ve[STEPS][8];
#pragma unroll
    for (int it = 0; it < STEPS; ++it) {
        const int pc = threadIdx.x + 256 * it;
        const int k2 = pc / (FR * 64), rem = pc - k2 * (FR * 64);
        const int frag = rem >> 6, lane = rem & 63;
        const int kt = 2 * st + k2, hh = lane >> 5;
        if (frag < JS) {                                        // the same for a whole wave
            const int t = 32 * kt + (lane & 31);
            kpiece[it] = *(const uint4 *)(K + (size_t)(t < L ? t : L - 1) * da + o + 16 * frag + 8 * hh);
        } else {
            const int fv = frag - JS, jj = fv / FT, ft = fv - jj * FT;
            const int f = o + 32 * ft + (lane & 31), t0 = 32 * kt + 16 * jj + 4 * hh;
#pragma unroll
            for (int sl = 0; sl < 8; ++sl) {                   // slot sl <-> key t0 + 8 (sl / 4) + sl % 4
                const int t = t0 + 8 * (sl >> 2) + (sl & 3);
                ve[it][sl] = V[(size_t)(t < L ? t : L - 1) * da + f];
            }
        }
    }
#pragma unroll
    for (int it = 0; it < STEPS; ++it) {
        const int pc = threadIdx.x + 256 * it;
        const int k2 = pc / (FR * 64), rem = pc - k2 * (FR * 64);
        const int frag = rem >> 6, lane = rem & 63;
        const int kt = 2 * st + k2, hh = lane >> 5;
        uint4 out;
        if (frag < JS) {
            out = 32 * kt + (lane & 31) < L ? scaled_bf16x8(kpiece[it], kscale) : make_uint4(0, 0, 0, 0);
        } else {
            const int jj = (frag - JS) / FT, t0 = 32 * kt + 16 * jj + 4 * hh;
            uint32_t w[4];
#pragma unroll
            for (int p2 = 0; p2 < 4; ++p2) {                 // slots 2 p2 and 2 p2 + 1
                const int ta = t0 + 8 * ((2 * p2) >> 2) + ((2 * p2) & 3), tb = ta + 1;
                const uint32_t lo = ta < L ? ve[it][2 * p2] : 0u;
                const uint32_t hi = tb < L ? ve[it][2 * p2 + 1] : 0u;
                w[p2] = lo | (hi << 16);
            }
            out = make_uint4(w[0], w[1], w[2], w[3]);
        }
        dst[pc] = out;
    }
    // largest key norm among this stage's 64 keys
    if (threadIdx.x < 64) {
        const int t = 64 * st + threadIdx.x;
        float ss = 0.f;
        if (t < L) {
            const uint4 *kr = (const uint4 *)(K + (size_t)t * da + o);
#pragma unroll
            for (int i = 0; i < DH / 8; ++i) {
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
        // the packed key is the key times kscale, rounded (each element at most 1 + 2^-8 times as large); the bound is
        // rounded up a little more: it must dominate the fp32-accumulated first product
        if (threadIdx.x == 0) kmax_part[((size_t)slot * m.n_heads + hd) * (nktp / 2) + st] = nrm * kscale * (1.f + 1.f / 256.f) * 1.001f;
    }
}

}  // namespace aif
