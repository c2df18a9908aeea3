// a1 -- index the nearline item-vector table by candidate id (Sec. 3.2: the
// vectors of all items are kept in an index table; at pre-ranking they
// meet the user vectors).  Pure data movement: HBM-bound.
//
// Rows are moved as 16-byte pieces.  A row of R bytes is handled by R/16
// neighbouring lanes, so a wave reads 64*16 B spread over 1024/R rows with
// every byte of each touched row used, and writes whole 128 B runs of the
// workspace in either of its layouts (x_offset).  Each thread first fetches
// UNROLL ids, then has UNROLL independent row loads in flight before its first
// store.
#include "k_stage.h"
#include <cstdlib>

namespace aif {

// LOG_RV >= 0: a row is 2^LOG_RV pieces of 16 bytes (shift instead of divide); LOG_RV < 0: any count.
template <int LOG_RV>
__global__ __launch_bounds__(256) void k_gather(const uint4 *__restrict__ table, int64_t n_items, int row_vec,
                                                Batch b, char *__restrict__ X, XLayout xl,
                                                int32_t *__restrict__ bad)
{
    gather_block<LOG_RV>(blockIdx.x, table, n_items, row_vec, TableReqs{b}, X, xl, bad);
}

// the workspace in fragment order: through LDS (gather_block_tiled)
template <int LOG_RV>
__global__ __launch_bounds__(256) void k_gather_tiled(const uint4 *__restrict__ table, int64_t n_items, Batch b,
                                                      char *__restrict__ X, XLayout xl, int32_t *__restrict__ bad)
{
    gather_block_tiled<LOG_RV>(blockIdx.x, table, n_items, TableReqs{b}, X, xl, bad);
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
    if (m.x_tiled && (row_vec == 8 || row_vec == 16 || row_vec == 32)) {
        auto got = [&](auto kern) {
            hipLaunchKernelGGL(kern, dim3(b.n_blk), dim3(256), 0, s, (const uint4 *)table, m.n_items, b, (char *)X, xl, bad);
        };
        if (row_vec == 8) got(k_gather_tiled<3>);
        if (row_vec == 16) got(k_gather_tiled<4>);
        if (row_vec == 32) got(k_gather_tiled<5>);
        return hipGetLastError();
    }
    switch (row_vec) {
    case 8: go(k_gather<3>); break;
    case 16: go(k_gather<4>); break;
    case 32: go(k_gather<5>); break;
    default: go(k_gather<-1>); break;
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Incremental update of the table (Sec. 3.4): the gather run backwards -- rows arrive contiguous and leave
// for random rows of the table.  Same piece-per-lane layout, four pieces in flight per thread.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_update_rows(uint4 *__restrict__ table, int64_t n_items, int row_vec,
                                                     const int32_t *__restrict__ ids, const uint4 *__restrict__ rows,
                                                     int n, int32_t *__restrict__ bad)
{
    constexpr int U = 4;
    const size_t total = (size_t)n * row_vec;
    const size_t base = ((size_t)blockIdx.x * U) * 256 + threadIdx.x;
    uint4 v[U];
    int64_t id[U];
    int piece[U];
    int n_bad = 0;
#pragma unroll
    for (int j = 0; j < U; ++j) {
        const size_t idx = base + (size_t)j * 256;
        const size_t row = idx / row_vec;
        piece[j] = (int)(idx - row * row_vec);
        id[j] = -1;
        if (idx < total) {
            id[j] = ids[row];
            {
                typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
                const u32x4 w = __builtin_nontemporal_load((const u32x4 *)(rows + idx));      // read once
                v[j] = make_uint4(w.x, w.y, w.z, w.w);
            }
            if (id[j] < 0 || id[j] >= n_items) {
                id[j] = -1;
                if (piece[j] == 0) ++n_bad;
            }
        }
    }
#pragma unroll
    for (int j = 0; j < U; ++j)
        if (id[j] >= 0) {
            // streaming stores: whole rows written once, for kernels that come later (plain stores measured 10 % slower)
            uint4 *p = table + (size_t)id[j] * row_vec + piece[j];
            __builtin_nontemporal_store(v[j].x, &p->x);
            __builtin_nontemporal_store(v[j].y, &p->y);
            __builtin_nontemporal_store(v[j].z, &p->z);
            __builtin_nontemporal_store(v[j].w, &p->w);
        }
    if (n_bad) atomicAdd(bad, n_bad);
}

hipError_t launch_update_rows(const Model &m, void *table, const int32_t *ids, const void *rows, int n, int32_t *bad,
                              hipStream_t s)
{
    if (n == 0) return hipSuccess;
    const int row_vec = m.d_item * (m.dtype == 0 ? 4 : 2) / 16;
    const size_t total = (size_t)n * row_vec;
    hipLaunchKernelGGL(k_update_rows, dim3((unsigned)((total + 1023) / 1024)), dim3(256), 0, s, (uint4 *)table, m.n_items,
                       row_vec, ids, (const uint4 *)rows, n, bad);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// The per-call descriptor tables, pinned host memory -> device: a few KB.  As a kernel that reads the host
// buffer through its device mapping the copy is one more launch on the caller's stream; as a copy command it
// goes to a copy engine and back, which kept the stream idle for some 20 us between two calls.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_upload(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int n16)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n16) dst[i] = src[i];
}

hipError_t launch_upload(const void *src_mapped, void *dst, size_t bytes, hipStream_t s)
{
    const int n16 = (int)((bytes + 15) / 16);
    if (n16 == 0) return hipSuccess;
    hipLaunchKernelGGL(k_upload, dim3((n16 + 255) / 256), dim3(256), 0, s, (const uint4 *)src_mapped, (uint4 *)dst, n16);
    return hipGetLastError();
}

hipError_t staging_alloc(size_t bytes, char **host, char **mapped)
{
    *host = *mapped = nullptr;
    const char *copy = getenv("AIF_STAGING_COPY");        // testing: the route taken where the mapping is refused
    const bool try_mapped = !(copy && copy[0] == '1');
    if (try_mapped && hipHostMalloc((void **)host, bytes, hipHostMallocCoherent | hipHostMallocMapped) == hipSuccess) {
        void *dev = nullptr;
        if (hipHostGetDevicePointer(&dev, *host, 0) == hipSuccess) *mapped = (char *)dev;
        else (void)hipGetLastError();
        return hipSuccess;
    }
    if (try_mapped) (void)hipGetLastError();
    *host = nullptr;
    return hipHostMalloc((void **)host, bytes, hipHostMallocDefault);
}

hipError_t staging_upload(const char *host, const char *mapped, size_t off, void *dst, size_t bytes, hipStream_t s)
{
    if (mapped) return launch_upload(mapped + off, dst, bytes, s);
    return hipMemcpyAsync(dst, host + off, bytes, hipMemcpyHostToDevice, s);
}

}  // namespace aif
