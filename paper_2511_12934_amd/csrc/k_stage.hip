// a1 + a2 in one launch for the bf16 MFMA path: the blocks of one grid take the
// three staging jobs of a batch -- K/V packing, user fold, gather -- by block
// index.  The jobs do not depend on one another; all are read by the attention
// kernel that follows.  The small, latency-bound jobs come first in the grid so
// that they run under the HBM-bound gather instead of before or after it.
// When the attention kernel that follows indexes the item table itself (k_attn_res with
// GATHER) the grid has no gather blocks; its first blocks may then carry the call's descriptor
// tables from pinned host memory to the device, which saves the upload its own launch.
// A batch of few requests (the latency cases: Sec. 5.3 measures a single request, alone or cut into mini-batches)
// needs neither: the requests' descriptors arrive in the kernel's arguments, every block reads them there, and the
// first blocks write the device tables the later kernels read.
#include "k_mfma.h"
#include "k_stage.h"

namespace aif {

struct StageArgs {
    Model m;
    Batch b;
    const uint4 *table;
    char *X;
    XLayout xl;
    int32_t *bad;
    const float *w1u, *b1;
    float *bias1;
    char *kvpack;
    size_t pack_stride;
    float *kmax;
    int32_t nktp, row_vec;
    int32_t n_pack, n_fold;         // blocks of the first two jobs
    int32_t n_w0;                   // blocks that fold the Hadamard cross block into the slots' layer-1 weights (0: not this model)
    FoldW0 w0;
    int32_t stages, quads;          // 64-key stages per head (nktp / 2); blocks of FOLD_FEATS layer-1 features
    const uint4 *up_src;            // descriptor tables to copy (mapped host memory -> device), 16 bytes a thread
    uint4 *up_dst;
    int32_t up_n16, n_up;           // 16-byte pieces; blocks of this job (0: the tables are on the device already)
};
struct StageFewArgs {
    StageArgs a;                    // a.n_up = blocks that write the tables (few_fill), a.up_* unused
    FewFill fill;
};

// LOG_RV = STAGE_NO_GATHER: the launch has no gather blocks (the attention kernel indexes the table itself) -- built
// without the gather's LDS buffers, which would otherwise limit how many of the small blocks a compute unit holds
constexpr int STAGE_NO_GATHER = -2;
template <int LOG_RV, int DH, class Reqs>
__device__ __forceinline__ void stage_block(const StageArgs &a, const Reqs &src, int idx)
{
    if (idx < a.n_pack) {
        const int st = idx % a.stages, rest = idx / a.stages;
        pack_kv_block<DH>(rest / a.m.n_heads, rest % a.m.n_heads, st, a.m, src, a.kvpack, a.pack_stride, a.kmax, a.nktp);
        return;
    }
    idx -= a.n_pack;
    if (idx < a.n_fold) {
        user_fold_block<uint16_t>(idx / a.quads, idx % a.quads, a.m, src, a.w1u, a.b1, a.bias1);
        return;
    }
    idx -= a.n_fold;
    if (idx < a.n_w0) {
        fold_w0_block(idx / a.w0.blocks_per_slot, idx % a.w0.blocks_per_slot, a.m, src, a.w0);
        return;
    }
    idx -= a.n_w0;
    if constexpr (LOG_RV == STAGE_NO_GATHER) return;
    if constexpr (LOG_RV >= 3 && LOG_RV <= 5) {
        if (a.m.x_tiled) {
            gather_block_tiled<LOG_RV>(idx, a.table, a.m.n_items, src, a.X, a.xl, a.bad);
            return;
        }
    }
    gather_block<LOG_RV>(idx, a.table, a.m.n_items, a.row_vec, src, a.X, a.xl, a.bad);
}

template <int LOG_RV, int DH>
__global__ __launch_bounds__(256) void k_stage(StageArgs a)
{
    const int idx = blockIdx.x;
    if (idx < a.n_up) {
        const int i = idx * 256 + (int)threadIdx.x;
        if (i < a.up_n16) a.up_dst[i] = a.up_src[i];
        return;
    }
    stage_block<LOG_RV, DH>(a, TableReqs{a.b}, idx - a.n_up);
}

template <int LOG_RV, int DH, int N>
__global__ __launch_bounds__(256) void k_stage_few(StageFewArgs o)
{
    const int idx = blockIdx.x;
    if (idx < o.a.n_up) {
        few_fill<N>(o.fill, idx * 256 + (int)threadIdx.x);
        return;
    }
    stage_block<LOG_RV, DH>(o.a, FewReqs<N>{o.fill}, idx - o.a.n_up);
}

template <int LOG_RV, int DH>
static void launch_stage_few(const StageFewArgs &o, dim3 grid, hipStream_t s)
{
    if (o.fill.n_req == 1 && o.fill.n_slots == 1)
        hipLaunchKernelGGL((k_stage_few<LOG_RV, DH, 1>), grid, dim3(256), 0, s, o);
    else
        hipLaunchKernelGGL((k_stage_few<LOG_RV, DH, FEW_MAX>), grid, dim3(256), 0, s, o);
}

template <int DH>
static hipError_t launch_stage_dh(const StageArgs &a, int n_gather, const FewFill *one, hipStream_t s)
{
    const dim3 grid(a.n_up + a.n_pack + a.n_fold + a.n_w0 + n_gather);
    if (one) {
        const StageFewArgs o{a, *one};
        switch (n_gather ? a.row_vec : STAGE_NO_GATHER) {
        case STAGE_NO_GATHER: launch_stage_few<STAGE_NO_GATHER, DH>(o, grid, s); break;
        case 8: launch_stage_few<3, DH>(o, grid, s); break;
        case 16: launch_stage_few<4, DH>(o, grid, s); break;
        case 32: launch_stage_few<5, DH>(o, grid, s); break;
        default: launch_stage_few<-1, DH>(o, grid, s); break;
        }
        return hipGetLastError();
    }
    switch (n_gather ? a.row_vec : STAGE_NO_GATHER) {
    case STAGE_NO_GATHER: hipLaunchKernelGGL((k_stage<STAGE_NO_GATHER, DH>), grid, dim3(256), 0, s, a); break;
    case 8: hipLaunchKernelGGL((k_stage<3, DH>), grid, dim3(256), 0, s, a); break;
    case 16: hipLaunchKernelGGL((k_stage<4, DH>), grid, dim3(256), 0, s, a); break;
    case 32: hipLaunchKernelGGL((k_stage<5, DH>), grid, dim3(256), 0, s, a); break;
    default: hipLaunchKernelGGL((k_stage<-1, DH>), grid, dim3(256), 0, s, a); break;
    }
    return hipGetLastError();
}

// the fold of the cross block into the users' layer-1 weights as a launch of its own (models whose staging is not k_stage)
__global__ __launch_bounds__(256) void k_fold_w0(Model m, Batch b, FoldW0 f)
{
    fold_w0_block(blockIdx.x / f.blocks_per_slot, blockIdx.x % f.blocks_per_slot, m, TableReqs{b}, f);
}

hipError_t fold_w0_args(const Model &m, const MfmaPlan &plan, FoldW0 &f)
{
    if (!plan.w0_user || !plan.wpack[0]) return hipErrorInvalidValue;
    f.src = (const uint4 *)plan.wpack[0];
    f.dst = (uint4 *)plan.w0_user;
    f.stride = plan.w0_stride;
    f.blocks_per_slot = m.cross_mode == 2 ? (m.dims[1] * (m.d_item / 16) + 255) / 256             // a thread per (row, item k-step)
                                          : (m.dims[1] / 32 * ((m.d_item + m.d_attn) / 16) * 64 + 256 * FOLD_PIECES - 1) / (256 * FOLD_PIECES);
    return hipSuccess;
}

hipError_t launch_fold_w0(const Model &m, const Batch &b, const MfmaPlan &plan, hipStream_t s)
{
    if (m.cross_in_mlp != 2 || b.n_slots == 0) return hipSuccess;
    FoldW0 f{};
    const hipError_t e = fold_w0_args(m, plan, f);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_fold_w0, dim3(b.n_slots * f.blocks_per_slot), dim3(256), 0, s, m, b, f);
    return hipGetLastError();
}

bool stage_fusable(const Model &m, const MfmaPlan &plan)
{
    return m.dtype == 1 && plan.attn && (m.d_head == 64 || m.d_head == 32);
}

hipError_t launch_stage(const Model &m, const Batch &b, const void *table, void *X, int32_t *bad, const float *w1u,
                        const float *b1, float *bias1, const MfmaPlan &plan, bool gather, hipStream_t s,
                        const StageUpload *up, const FewFill *one)
{
    if (b.n_req == 0) return hipSuccess;
    if (up && gather) return hipErrorInvalidValue;      // the gather's many blocks read the device copy
    if (one && (up || b.n_req > FEW_MAX || b.n_req != one->n_req || b.n_slots != one->n_slots)) return hipErrorInvalidValue;
    StageArgs a;
    a.m = m;
    a.b = b;
    a.up_src = nullptr;
    a.up_dst = nullptr;
    a.up_n16 = a.n_up = 0;
    if (up) {
        a.b.reqs = up->reqs_mapped;
        a.b.slot_req = up->slot_req_mapped;
        a.up_src = (const uint4 *)up->src_mapped;
        a.up_dst = (uint4 *)up->dst;
        a.up_n16 = (int32_t)((up->bytes + 15) / 16);
        a.n_up = (a.up_n16 + 255) / 256;
    }
    if (one) a.n_up = (few_fill_items(*one) + 255) / 256;
    a.table = (const uint4 *)table;
    a.X = (char *)X;
    a.xl = x_layout(m);
    a.bad = bad;
    a.w1u = w1u;
    a.b1 = b1;
    a.bias1 = bias1;
    a.kvpack = plan.kvpack;
    a.pack_stride = plan.pack_stride;
    a.kmax = plan.kmax;
    a.nktp = plan.nktp;
    a.row_vec = m.d_item * 2 / 16;
    a.stages = plan.nktp / 2;
    a.quads = (m.dims[1] + FOLD_FEATS - 1) / FOLD_FEATS;
    a.n_pack = b.n_slots * m.n_heads * a.stages;     // once per distinct user of the call, not per slice (Sec. 3.1)
    a.n_fold = b.n_slots * a.quads;
    a.n_w0 = 0;
    a.w0 = FoldW0{};
    if (m.cross_in_mlp == 2) {
        const hipError_t e = fold_w0_args(m, plan, a.w0);
        if (e != hipSuccess) return e;
        a.n_w0 = b.n_slots * a.w0.blocks_per_slot;
    }
    const int n_gather = gather ? b.n_blk : 0;      // none when the attention kernel indexes the table itself
    return m.d_head == 64 ? launch_stage_dh<64>(a, n_gather, one, s) : launch_stage_dh<32>(a, n_gather, one, s);
}

}  // namespace aif
