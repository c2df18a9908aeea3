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
#include "k_stage.h"

namespace aif {

// LOG_RV >= 0: a row is 2^LOG_RV pieces of 16 bytes (shift instead of divide); LOG_RV < 0: any count.
template <int LOG_RV>
__global__ __launch_bounds__(256) void k_gather(const uint4 *__restrict__ table, int64_t n_items, int row_vec,
                                                Batch b, char *__restrict__ X, XLayout xl,
                                                int32_t *__restrict__ bad)
{
    gather_block<LOG_RV>(blockIdx.x, table, n_items, row_vec, b, X, xl, bad);
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
