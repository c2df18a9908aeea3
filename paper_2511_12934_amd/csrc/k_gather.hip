// a1 -- index the nearline item-vector table by candidate id (Sec. 3.2: the
// vectors of all items are "stored in an indexing table"; at pre-ranking they
// are combined with the user vectors).  Pure data movement: HBM-bound.
//
// Rows are moved as 16-byte pieces.  A row of R bytes is handled by R/16
// neighbouring lanes, so a wave reads 64*16 B spread over 1024/R rows with
// every byte of each touched row used, and writes one contiguous run of the
// workspace (rows of one request are consecutive, row stride ldx).  Each
// thread keeps UNROLL independent row loads in flight before its first store.
#include "aif_dev.h"

namespace aif {

constexpr int GATHER_UNROLL = 4;

__global__ __launch_bounds__(256) void k_gather(const uint4 *__restrict__ table, int64_t n_items,
                                                int row_vec, Batch b, uint4 *__restrict__ X,
                                                int ldx_vec, int32_t *__restrict__ bad)
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
    uint4 *out = X + (size_t)(row_base + local0) * ldx_vec;
    const int total = nrows * row_vec;
    int n_bad = 0;
    for (int base = threadIdx.x; base < total; base += 256 * GATHER_UNROLL) {
        uint4 v[GATHER_UNROLL];
        int row[GATHER_UNROLL], piece[GATHER_UNROLL];
#pragma unroll
        for (int j = 0; j < GATHER_UNROLL; ++j) {
            const int idx = base + j * 256;
            row[j] = idx / row_vec;
            piece[j] = idx - row[j] * row_vec;
            if (idx < total) {
                int64_t id = ids[row[j]];
                if (id < 0 || id >= n_items) {
                    id = 0;
                    if (piece[j] == 0) ++n_bad;
                }
                v[j] = table[(size_t)id * row_vec + piece[j]];
            }
        }
#pragma unroll
        for (int j = 0; j < GATHER_UNROLL; ++j) {
            const int idx = base + j * 256;
            if (idx < total) out[(size_t)row[j] * ldx_vec + piece[j]] = v[j];
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
    const int ldx_vec = m.ldx * esz / 16;
    hipLaunchKernelGGL(k_gather, dim3(b.n_blk), dim3(256), 0, s, (const uint4 *)table, m.n_items, row_vec, b,
                       (uint4 *)X, ldx_vec, bad);
    return hipGetLastError();
}

}  // namespace aif
