// Internal device-side types and launcher prototypes of libaif (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aif {

// Rows of the workspace handled by one scheduling block.  Every request's
// rows start on a multiple of ROW_BLOCK, so a block never straddles requests.
constexpr int ROW_BLOCK = 256;
constexpr int MAX_LAYERS = 8;
constexpr int TOPK_MAX = 4096;

struct ReqDesc {
    const void *user_vec;
    const void *cross_vecs;     // never null when cross_mode != NONE (host substitutes user_vec)
    const void *seq_keys;
    const void *seq_vals;
    const int32_t *cand_ids;
    float *logits_out;
    float *scores_out;          // may be null
    int32_t seq_len;
    int32_t n_cand;
    int32_t row_base;           // first workspace row of this request (multiple of ROW_BLOCK)
    int32_t index;              // position in the batch
    int32_t slot;               // user slot: requests of one call that bring the same user tensors (the mini-batch
                                // slices of one candidate list, Sec. 3.1) share one folded bias, one packed K/V
    int32_t pad_;
};

// A run of 32-candidate tiles of ONE request, the unit of work of the attention kernel that keeps
// the request's K/V resident in LDS: tiles [t0, t1), numbered within the request.
struct AttnGroup {
    int32_t r, t0, t1, pad;
};

// What one call hands to its kernels.
struct Batch {
    const ReqDesc *reqs;        // device, [n_req]
    const int32_t *blk_req;     // device, [n_blk]: request owning each ROW_BLOCK of the workspace
    const AttnGroup *groups;    // device, [n_groups]; n_groups = 0: the batch does not use them
    const int32_t *blk_slot;    // device, [n_blk]: user slot of the request owning each ROW_BLOCK (= reqs[blk_req[i]].slot)
    const int32_t *slot_req;    // device, [n_slots]: a request that brings slot s's user tensors; null: slot s = request s
    int32_t n_req;
    int32_t n_blk;
    int32_t n_groups;
    int32_t n_streamed;         // requests left to the streaming attention kernels (K/V too long for the resident one)
    int32_t n_slots;            // distinct users of the call: the user-side staging (fold, K/V packing) runs once per slot
};
__device__ __forceinline__ int slot_request(const Batch &b, int slot) { return b.slot_req ? b.slot_req[slot] : slot; }

struct Model {
    int32_t dtype;              // 0 fp32, 1 bf16
    int64_t n_items;
    int32_t d_item, d_user, d_attn, n_heads, d_head;
    int32_t cross_mode, n_cross, d_cv, d_cross;
    int32_t ldx;                // width of the workspace matrix [e | a | c], in elements
    int32_t x_tiled;            // layout of the workspace inside each tile of X_TILE rows, see x_offset
    int32_t n_layers;
    int32_t dims[MAX_LAYERS + 1];   // dims[0] = D_in
    int32_t k1;                 // D_in - d_user: layer-1 contraction left per candidate after the user fold
    int32_t cross_in_mlp;       // Hadamard cross only: the MLP chain forms c = u (.) e itself from the item block it reads anyway
                                // (same products, same rounding); the attention kernel then leaves the cross block of the
                                // workspace unwritten -- a third of its stores, and of the MLP's loads
};

// Where the workspace keeps 16-byte piece `piece` of row `row` (byte offset).  Rows are grouped in
// tiles of X_TILE = 32 (one MFMA column tile).  Row-major inside the tile, or -- when both consumers
// are the MFMA kernels -- "tiled": pieces ordered [piece][row], so that the 32 rows' copies of one
// piece are one contiguous 512 B run and a wave's B-fragment load (pieces 2j and 2j + 1 of 32 rows)
// is one contiguous 1 KB instead of 64 strided 16 B accesses.  A tile takes the same bytes either way.
constexpr int X_TILE = 32;
struct XLayout {
    uint32_t tile_bytes, row_stride, piece_stride;
};
__host__ __device__ inline XLayout x_layout(const Model &m)
{
    const uint32_t row_bytes = (uint32_t)m.ldx * (m.dtype == 0 ? 4u : 2u);
    return m.x_tiled ? XLayout{row_bytes * X_TILE, 16u, 16u * X_TILE} : XLayout{row_bytes * X_TILE, row_bytes, 16u};
}
__host__ __device__ inline size_t x_offset(const XLayout &l, uint32_t row, uint32_t piece)
{
    return (size_t)(row / X_TILE) * l.tile_bytes + (size_t)(row % X_TILE) * l.row_stride + (size_t)piece * l.piece_stride;
}

// bf16 <-> fp32 on raw bit patterns (round to nearest even).
__device__ __forceinline__ float bf2f(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t f2bf(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
template <typename T> __device__ __forceinline__ float ld_f(const T *p);
template <> __device__ __forceinline__ float ld_f<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float ld_f<uint16_t>(const uint16_t *p) { return bf2f(*p); }
template <typename T> __device__ __forceinline__ void st_f(T *p, float v);
template <> __device__ __forceinline__ void st_f<float>(float *p, float v) { *p = v; }
template <> __device__ __forceinline__ void st_f<uint16_t>(uint16_t *p, float v) { *p = f2bf(v); }

// ---- launchers (each enqueues on `s` and returns the launch status) -------

// a1: X[row, 0:d_item] = table[id].  Bad ids read row 0 and bump *bad.
hipError_t launch_gather(const Model &m, const Batch &b, const void *table, void *X, int32_t *bad,
                         hipStream_t s);

// Sec. 3.4, incremental update: table[ids[i]] = rows[i] in 16-byte pieces; bad ids write nothing and bump *bad.
// src_mapped: the device mapping of a pinned host buffer (hipHostGetDevicePointer); bytes are rounded up to 16,
// both buffers must hold the rounded size
hipError_t launch_upload(const void *src_mapped, void *dst, size_t bytes, hipStream_t s);
// Pinned host memory for the per-call descriptor tables: coherent and mapped, so that a kernel may read it
// (*mapped = its device address); where that is refused plain pinned memory, *mapped = null.  Freed with hipHostFree.
hipError_t staging_alloc(size_t bytes, char **host, char **mapped);
// bytes [off, off + bytes) of such a buffer -> dst, on stream s: launch_upload if mapped, else a copy command
hipError_t staging_upload(const char *host, const char *mapped, size_t off, void *dst, size_t bytes, hipStream_t s);
hipError_t launch_update_rows(const Model &m, void *table, const int32_t *ids, const void *rows, int n, int32_t *bad,
                              hipStream_t s);

// a2: per user slot s, bias1[s, n] = b1[n] + sum_m W1[n, m] u[m] over the user columns (w1u: those columns
// transposed, fp32 [d_user, H1]).
hipError_t launch_user_fold(const Model &m, const Batch &b, const float *w1u, const float *b1,
                            float *bias1, hipStream_t s);

// a3-a5, any shape, fp32 arithmetic: X[row, d_item:] = [attention | cross].
hipError_t launch_attn_generic(const Model &m, const Batch &b, void *X, const float *wq, int max_seq_len,
                               hipStream_t s);
size_t attn_generic_lds_bytes(const Model &m, int max_seq_len);

// a6-a7, any shape, fp32 arithmetic.  wt[l] = transposed fp32 weights [K_l, N_l].
struct MlpGenericWeights {
    const float *wt[MAX_LAYERS];
    const float *bias[MAX_LAYERS];      // bias[0] unused (folded into bias1)
};
hipError_t launch_mlp_generic(const Model &m, const Batch &b, const void *X, const MlpGenericWeights &w,
                              const float *bias1, hipStream_t s);
size_t mlp_generic_lds_bytes(const Model &m);

// a8: per-request radix select + sort.
struct TopkDesc {
    const float *logits;
    int32_t n;
};
// n_max: the longest list (the kernel keeps that many logits in registers; a longer list is still selected from, slower)
hipError_t launch_topk(const TopkDesc *descs /*device*/, int n_req, int n_max, int k, int32_t *idx_out, float *val_out,
                       hipStream_t s);
// at most TOPK_FEW lists whose descriptors are on the HOST: they travel in the kernel's arguments, nothing is uploaded
constexpr int TOPK_FEW = 16;
hipError_t launch_topk_few(const TopkDesc *descs /*host*/, int n_req, int k, int32_t *idx_out, float *val_out,
                           hipStream_t s);

// init-time repacking (device -> device, any storage type -> fp32)
hipError_t launch_pack_transposed(int dtype, const void *w, int n_out, int n_in, int col0, int ncols,
                                  float *wt /*[ncols, n_out]*/, hipStream_t s);
hipError_t launch_to_f32(int dtype, const void *src, int64_t rows, int cols, int ld_src, int col0,
                         float *dst /*[rows, cols]*/, hipStream_t s);

}  // namespace aif
