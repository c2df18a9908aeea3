// a1 -- index the nearline item-vector table by candidate id (Sec. 3.2: the
// vectors of all items are "stored in an indexing table"; at pre-ranking they
// are combined with the user vectors).  Pure data movement: HBM-bound.
//
// Rows are moved as 16-byte pieces.  A row of R bytes is handled by R/16
// neighbouring lanes, so a wave reads 64*16 B spread over 1024/R rows with
// every byte of each touched row used, and writes whole 128 B runs of the
// workspace in either of its layouts (x_offset).  Each thread first fetches
// UNROLL ids, then has UNROLL independent row loads in flight before its first
// store.
#include "aif_dev.h"

namespace aif {

constexpr int GATHER_UNROLL = 4;

// LOG_RV >= 0: a row is 2^LOG_RV pieces of 16 bytes (shift instead of divide); LOG_RV < 0: any count.
template <int LOG_RV>
__global__ __launch_bounds__(256) void k_gather(const uint4 *__restrict__ table, int64_t n_items, int row_vec,
                                                Batch b, char *__restrict__ X, XLayout xl,
                                                int32_t *__restrict__ bad)
{
    const int blk = blockIdx.x;
    const int r = b.blk_req[blk];
    if (r < 0) return;
    const ReqDesc *rd = b.reqs + r;
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

hipError_t launch_gather(const Model &m, const Batch &b, const void *table, void *X, int32_t *bad,
                         hipStream_t s)
{
    if (b.n_blk == 0) return hipSuccess;
    const int esz = m.dtype == 0 ? 4 : 2;
    const int row_vec = m.d_item * esz / 16;
    const XLayout xl = x_layout(m);
    auto go = [&](auto kern) {
        hipLaunchKernelGGL(kern, dim3(b.n_blk), dim3(256), 0, s, (const uint4 *)table, m.n_items, row_vec, b, (char *)X,
                           xl, bad);
    };
    switch (row_vec) {
    case 8: go(k_gather<3>); break;
    case 16: go(k_gather<4>); break;
    case 32: go(k_gather<5>); break;
    default: go(k_gather<-1>); break;
    }
    return hipGetLastError();
}

}  // namespace aif
