// Host side of libaif: the C ABI of include/aif.h.  Validates, sizes the
// workspace, repacks weights once, and per call stages the request table and
// enqueues  gather -> user fold -> attention + cross -> MLP  (and top-k) on
// the caller's stream.
#include "../../include/aif.h"
#include "aif_dev.h"
#include "k_mfma.h"
#include "k_stage.h"

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <tuple>
#include <string>
#include <vector>

using namespace aif;

// The per-call workspace of aif_score_topk_static (the entry point for callers that cannot allocate): every GPU the
// library runs on holds its own copy of this array, at its own address, until the process ends.  In host code the
// name is only a handle: the device address comes from hipGetSymbolAddress, once per device (scratch_of).
static __device__ __align__(256) unsigned char scratch[AIF_STATIC_SCRATCH_BYTES];

namespace {

constexpr int NSLOT = 8;
constexpr int MAX_DEVICES = 64;
constexpr int STATIC_MAX_GROUPS = 1024;
std::mutex g_scratch_mutex;
unsigned char *g_scratch_ptr[MAX_DEVICES] = {};      // device address of `scratch` on each device, set at the first init there

// The device address of `scratch` on the CURRENT device `dev`; resolved once per device.
hipError_t scratch_of(int dev, unsigned char **out)
{
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[dev] = (unsigned char *)p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

// The descriptor tables of a one-request batch written as a launch of its own (one_fill): for the models whose
// staging is not the fused launch, which would carry them.
__global__ __launch_bounds__(256) void k_static_fill(FewFill f) { few_fill<1>(f, blockIdx.x * 256 + threadIdx.x); }

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
thread_local std::string g_init_error = "";

struct DevBuf {
    void *p = nullptr;
    hipError_t alloc(size_t bytes)
    {
        if (bytes == 0) bytes = 16;
        return hipMalloc(&p, bytes);
    }
    void release()
    {
        if (p) (void)hipFree(p);
        p = nullptr;
    }
};

}  // namespace

struct aif_ctx {
    Model m{};
    int device = 0;
    int max_seq_len = 0, max_candidates = 0, max_users = 0;
    const void *table = nullptr;

    // repacked weights (owned)
    DevBuf w1u;                       // fp32 [d_user, H1]: user columns of layer 1, transposed
    DevBuf wq;                        // fp32 [d_attn, d_item] (generic attention)
    DevBuf wt[MAX_LAYERS];            // fp32 transposed [K_l, N_l] (generic MLP)
    DevBuf bias[MAX_LAYERS];          // fp32 [N_l]
    bool has_bias[MAX_LAYERS] = {};
    bool has_wq = false;
    MfmaPlan mfma{};                  // MFMA kernels' packed weights and eligibility

    // workspace (owned)
    DevBuf X;                         // [x_rows, ldx] storage type
    DevBuf bias1;                     // fp32 [max_users, H1]
    DevBuf bad;                       // int32 counter
    size_t x_rows = 0;
    int n_cu = 256;                   // compute units of the device (sizes the attention groups)
    bool attn_indexed = false;        // the last scoring call's attention kernel read the item table itself
    int last_slots = 0;               // distinct users (user slots) of the last scoring call
    unsigned char *scratch_dev = nullptr;   // this device's copy of the file-scope scratch array (aif_score_topk_static)
    bool separate_gather = false;     // testing (AIF_SEPARATE_GATHER=1): the gather always as blocks or a launch of its own

    // descriptor staging ring
    char *h_stage = nullptr;          // pinned
    char *h_stage_dev = nullptr;      // its device mapping (null: none, uploads go through hipMemcpyAsync)
    DevBuf d_stage;
    size_t slot_bytes = 0;
    hipEvent_t ev[NSLOT] = {};
    bool ev_live[NSLOT] = {};
    int next_slot = 0;

    std::vector<int32_t> row_base;    // host copy for aif_peek_features
    std::vector<const void *> peek_cross;   // per request of the last batch: its Hadamard operand (device), for aif_peek_features
    std::string err;

    // optional per-kernel event timing
    bool prof_on = false;
    int prof_max = 0, prof_batch_calls = 0, prof_topk_calls = 0;
    uint32_t prof_mask = 0;               // bit per AIF_STAGE_*: the stages whose bounding events are recorded
    int prof_every = 1, prof_seen_batch = 0, prof_seen_topk = 0;   // only every prof_every-th call is recorded
    std::vector<hipEvent_t> prof_batch;   // 5 events per recorded aif_score_batch
    std::vector<hipEvent_t> prof_topk;    // 2 events per recorded aif_topk
};

namespace {

aif_status fail(aif_ctx *c, aif_status st, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (c)
        c->err = buf;
    else
        g_init_error = buf;
    return st;
}

#define HIP_TRY(ctxp, expr)                                                                         \
    do {                                                                                            \
        hipError_t e_ = (expr);                                                                     \
        if (e_ != hipSuccess)                                                                       \
            return fail(ctxp, e_ == hipErrorOutOfMemory ? AIF_ENOMEM : AIF_EDEVICE, "%s: %s", #expr, \
                        hipGetErrorString(e_));                                                     \
    } while (0)

int round_up(int v, int a) { return (v + a - 1) / a * a; }

void destroy(aif_ctx *c)
{
    if (!c) return;
    c->w1u.release();
    c->wq.release();
    for (auto &b : c->wt) b.release();
    for (auto &b : c->bias) b.release();
    mfma_release(c->mfma);
    c->X.release();
    c->bias1.release();
    c->bad.release();
    c->d_stage.release();
    if (c->h_stage) (void)hipHostFree(c->h_stage);
    for (int i = 0; i < NSLOT; ++i)
        if (c->ev[i]) (void)hipEventDestroy(c->ev[i]);
    for (auto e : c->prof_batch) (void)hipEventDestroy(e);
    for (auto e : c->prof_topk) (void)hipEventDestroy(e);
    delete c;
}

// The first `bytes` of a staging slot, host -> device, on the caller's stream: by a kernel that reads the pinned
// buffer through its device mapping (coherent host memory: never cached on the device), else by a copy command.
static hipError_t upload(aif_ctx *c, int slot, size_t bytes, hipStream_t s)
{
    const size_t off = (size_t)slot * c->slot_bytes;
    return staging_upload(c->h_stage, c->h_stage_dev, off, (char *)c->d_stage.p + off, bytes, s);
}

// Take the next staging slot, waiting (normally not at all) for the call that
// last used it.
aif_status take_slot(aif_ctx *c, int *slot)
{
    const int s = c->next_slot;
    c->next_slot = (s + 1) % NSLOT;
    if (c->ev_live[s]) HIP_TRY(c, hipEventSynchronize(c->ev[s]));
    *slot = s;
    return AIF_OK;
}

aif_status check_device(aif_ctx *c)
{
    int cur = -1;
    HIP_TRY(c, hipGetDevice(&cur));
    if (cur != c->device) return fail(c, AIF_EDEVICE, "context belongs to device %d, current device is %d", c->device, cur);
    return AIF_OK;
}

aif_status init_impl(const aif_config *cfg, const aif_weights *wts, aif_ctx *c)
{
    if (cfg->dtype != AIF_F32 && cfg->dtype != AIF_BF16) return fail(nullptr, AIF_EINVAL, "unknown dtype %d", (int)cfg->dtype);
    if (cfg->flags != 0) return fail(nullptr, AIF_EINVAL, "flags must be 0");
    if (cfg->n_items <= 0 || cfg->d_item <= 0 || cfg->d_user < 0 || cfg->d_attn <= 0 || cfg->n_heads <= 0 ||
        cfg->max_seq_len < 0 || cfg->n_layers <= 0 || cfg->max_candidates <= 0 || cfg->max_users <= 0)
        return fail(nullptr, AIF_EINVAL, "non-positive size in aif_config");
    if (cfg->n_layers > MAX_LAYERS) return fail(nullptr, AIF_ESHAPE, "at most %d MLP layers", MAX_LAYERS);
    if (!cfg->layer_dims || !wts->item_table || !wts->w) return fail(nullptr, AIF_EINVAL, "NULL layer_dims, item_table or w");
    if (cfg->d_attn % cfg->n_heads) return fail(nullptr, AIF_ESHAPE, "d_attn %d is not a multiple of n_heads %d", cfg->d_attn, cfg->n_heads);
    if (!wts->w_q && cfg->d_attn > cfg->d_item) return fail(nullptr, AIF_ESHAPE, "without w_q, d_attn must not exceed d_item");

    Model &m = c->m;
    m.dtype = (int)cfg->dtype;
    m.n_items = cfg->n_items;
    m.d_item = cfg->d_item;
    m.d_user = cfg->d_user;
    m.d_attn = cfg->d_attn;
    m.n_heads = cfg->n_heads;
    m.d_head = cfg->d_attn / cfg->n_heads;
    m.cross_mode = (int)cfg->cross_mode;
    m.n_cross = cfg->n_cross;
    m.d_cv = cfg->d_cross_vec;
    switch (cfg->cross_mode) {
    case AIF_CROSS_NONE: m.d_cross = 0; break;
    case AIF_CROSS_HADAMARD: m.d_cross = cfg->d_item; break;
    case AIF_CROSS_SEGDOT:
        if (cfg->n_cross <= 0 || cfg->d_cross_vec <= 0 || cfg->d_item % cfg->d_cross_vec)
            return fail(nullptr, AIF_ESHAPE, "SEGDOT needs n_cross > 0 and d_cross_vec dividing d_item");
        m.d_cross = cfg->n_cross * (cfg->d_item / cfg->d_cross_vec);
        break;
    case AIF_CROSS_BEA:
        if (cfg->n_cross <= 0 || cfg->n_cross > cfg->d_item || cfg->d_cross_vec <= 0)
            return fail(nullptr, AIF_ESHAPE, "BEA needs 0 < n_cross <= d_item and d_cross_vec > 0");
        m.d_cross = cfg->d_cross_vec;
        break;
    default: return fail(nullptr, AIF_EINVAL, "unknown cross_mode %d", (int)cfg->cross_mode);
    }
    const int esz = m.dtype == 0 ? 4 : 2, vec = 16 / esz;
    if (m.d_item % vec || m.d_attn % vec || m.d_cross % vec)
        return fail(nullptr, AIF_ESHAPE, "d_item, d_attn and the cross width must be multiples of %d elements", vec);
    m.ldx = m.d_item + m.d_attn + m.d_cross;
    m.n_layers = cfg->n_layers;
    for (int l = 0; l <= cfg->n_layers; ++l) {
        m.dims[l] = cfg->layer_dims[l];
        if (m.dims[l] <= 0) return fail(nullptr, AIF_EINVAL, "layer_dims[%d] <= 0", l);
    }
    if (m.dims[0] != m.d_user + m.ldx)
        return fail(nullptr, AIF_ESHAPE, "layer_dims[0] = %d but d_user + d_item + d_attn + d_cross = %d", m.dims[0], m.d_user + m.ldx);
    if (m.dims[m.n_layers] != 1) return fail(nullptr, AIF_ESHAPE, "the last layer must have one output");
    m.k1 = m.dims[0] - m.d_user;
    for (int l = 0; l < m.n_layers; ++l)
        if (!wts->w[l]) return fail(nullptr, AIF_EINVAL, "w[%d] is NULL", l);
    if ((uintptr_t)wts->item_table % 16) return fail(nullptr, AIF_EINVAL, "item_table must be 16-byte aligned");

    c->max_seq_len = cfg->max_seq_len;
    c->max_candidates = cfg->max_candidates;
    c->max_users = cfg->max_users;
    c->table = wts->item_table;
    HIP_TRY(nullptr, hipGetDevice(&c->device));
    HIP_TRY(nullptr, scratch_of(c->device, &c->scratch_dev));

    // ---- weight copies ---------------------------------------------------
    hipStream_t s = nullptr;
    const int H1 = m.dims[1];
    HIP_TRY(nullptr, c->w1u.alloc((size_t)H1 * m.d_user * 4));
    HIP_TRY(nullptr, launch_pack_transposed(m.dtype, wts->w[0], H1, m.dims[0], 0, m.d_user, (float *)c->w1u.p, s));
    for (int l = 0; l < m.n_layers; ++l) {
        const int n_in = m.dims[l], n_out = m.dims[l + 1];
        const int col0 = l == 0 ? m.d_user : 0, ncols = n_in - col0;
        HIP_TRY(nullptr, c->wt[l].alloc((size_t)ncols * n_out * 4));
        HIP_TRY(nullptr, launch_pack_transposed(m.dtype, wts->w[l], n_out, n_in, col0, ncols, (float *)c->wt[l].p, s));
        const void *bl = wts->b ? wts->b[l] : nullptr;
        c->has_bias[l] = bl != nullptr;
        if (bl) {
            HIP_TRY(nullptr, c->bias[l].alloc((size_t)n_out * 4));
            HIP_TRY(nullptr, launch_to_f32(m.dtype, bl, 1, n_out, n_out, 0, (float *)c->bias[l].p, s));
        }
    }
    c->has_wq = wts->w_q != nullptr;
    if (c->has_wq) {
        HIP_TRY(nullptr, c->wq.alloc((size_t)m.d_attn * m.d_item * 4));
        HIP_TRY(nullptr, launch_to_f32(m.dtype, wts->w_q, m.d_attn, m.d_item, m.d_item, 0, (float *)c->wq.p, s));
    }
    c->x_rows = (size_t)c->max_users * round_up(c->max_candidates, ROW_BLOCK);
    HIP_TRY(nullptr, mfma_plan(m, c->max_seq_len, c->max_users, c->x_rows, wts->w_q, wts->w, c->mfma, s));
    // both consumers of the workspace read MFMA fragments: keep it in fragment order (x_offset)
    {
        const char *rm = getenv("AIF_X_ROW_MAJOR");      // testing: the MFMA kernels on the row-major layout
        m.x_tiled = (c->mfma.attn && c->mfma.mlp && !(rm && rm[0] == '1')) ? 1 : 0;
        const char *sg = getenv("AIF_SEPARATE_GATHER");  // testing: both gather routes must give the same bits
        c->separate_gather = sg && sg[0] == '1';
        const char *cm = getenv("AIF_CROSS_MATERIALIZED");   // testing: the Hadamard cross block written to the workspace even where the MLP chain could form it
        m.cross_in_mlp = (c->mfma.mlp && mlp_chain_forms_cross(c->mfma.mlp_variant, m) && !(cm && cm[0] == '1')) ? 1 : 0;
        // ... and where the staging launch can do it, the cross block is folded into each user's layer-1 weights instead
        const char *cf = getenv("AIF_CROSS_FOLD");           // testing and measurement: "0" keeps the products in the chain
        const bool foldable = c->mfma.mlp && mlp_chain_folds_cross(c->mfma.mlp_variant, m) && !(cm && cm[0] == '1');
        if (foldable && !(cf && cf[0] == '0')) {
            c->mfma.w0_stride = mlp_w0_user_bytes(m);
            HIP_TRY(nullptr, hipMalloc((void **)&c->mfma.w0_user, c->mfma.w0_stride * (size_t)c->max_users));
            m.cross_in_mlp = 2;
        }
    }

    const bool attn_ok = c->mfma.attn || attn_generic_lds_bytes(m, c->max_seq_len) <= 160 * 1024;
    const bool mlp_ok = c->mfma.mlp || mlp_generic_lds_bytes(m) <= 160 * 1024;
    if (!attn_ok) return fail(nullptr, AIF_ESHAPE, "max_seq_len %d needs more LDS than a compute unit has", c->max_seq_len);
    if (!mlp_ok) return fail(nullptr, AIF_ESHAPE, "MLP layers wider than the LDS budget of the generic kernel");
    // a bf16 model outside the matrix-core kernels' shapes still runs, much more slowly: say so where the caller can read it
    if (m.dtype == 1 && !(c->mfma.attn && c->mfma.mlp)) {
        const char *force = getenv("AIF_FORCE_GENERIC");
        char note[256];
        snprintf(note, sizeof note, "note: bf16 model served by the shape-agnostic fp32 kernels for%s%s%s (%s)",
                 c->mfma.attn ? "" : " attention", !c->mfma.attn && !c->mfma.mlp ? " and" : "", c->mfma.mlp ? "" : " the MLP head",
                 force && force[0] == '1' ? "AIF_FORCE_GENERIC=1" : "no matrix-core kernel for these widths");
        c->err = note;
    }

    // ---- workspace ---------------------------------------------------------
    c->x_rows = (size_t)c->max_users * round_up(c->max_candidates, ROW_BLOCK);
    HIP_TRY(nullptr, c->X.alloc(c->x_rows * m.ldx * esz));
    HIP_TRY(nullptr, c->bias1.alloc((size_t)c->max_users * H1 * 4));
    HIP_TRY(nullptr, c->bad.alloc(4));
    HIP_TRY(nullptr, hipMemsetAsync(c->bad.p, 0, 4, s));

    const size_t n_blk_max = c->x_rows / ROW_BLOCK;
    size_t sb = (size_t)c->max_users * sizeof(ReqDesc) + 2 * (n_blk_max + 4) * sizeof(int32_t) +
                (size_t)c->max_users * sizeof(int32_t) + 16 + attn_max_groups(c->x_rows, c->max_users) * sizeof(AttnGroup);
    {
        int dev = 0;
        hipDeviceProp_t prop;
        HIP_TRY(nullptr, hipGetDevice(&dev));
        HIP_TRY(nullptr, hipGetDeviceProperties(&prop, dev));
        c->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    }
    sb += (size_t)c->max_users * sizeof(TopkDesc) + 16;     // aif_score_topk stages both tables in one slot
    c->slot_bytes = (sb + 255) / 256 * 256;
    HIP_TRY(nullptr, staging_alloc(c->slot_bytes * NSLOT, &c->h_stage, &c->h_stage_dev));
    HIP_TRY(nullptr, c->d_stage.alloc(c->slot_bytes * NSLOT));
    for (int i = 0; i < NSLOT; ++i) HIP_TRY(nullptr, hipEventCreateWithFlags(&c->ev[i], hipEventDisableTiming | hipEventDisableSystemFence));
    HIP_TRY(nullptr, hipStreamSynchronize(s));
    return AIF_OK;
}

}  // namespace

extern "C" {

aif_status aif_score_init(const aif_config *cfg, const aif_weights *weights, aif_ctx **out)
{
    if (!cfg || !weights || !out) return fail(nullptr, AIF_EINVAL, "NULL argument");
    aif_ctx *c = new (std::nothrow) aif_ctx();
    if (!c) return fail(nullptr, AIF_ENOMEM, "out of host memory");
    const aif_status st = init_impl(cfg, weights, c);
    if (st != AIF_OK) {
        destroy(c);
        return st;
    }
    *out = c;
    return AIF_OK;
}

void aif_score_destroy(aif_ctx *ctx) { destroy(ctx); }

const char *aif_last_error(const aif_ctx *ctx) { return ctx ? ctx->err.c_str() : g_init_error.c_str(); }

// Score n_req requests; with k > 0 also select each request's k best (one staging copy, one more launch).
static aif_status score_impl(aif_ctx *c, const aif_request *reqs, int32_t n_req, int32_t k, int32_t *idx_out,
                             float *val_out, void *hip_stream)
{
    if (!c) return AIF_EINVAL;
    if (n_req < 0 || (n_req > 0 && !reqs)) return fail(c, AIF_EINVAL, "NULL request array or negative n_req");
    if (k > 0 && n_req > 0 && (!idx_out || !val_out)) return fail(c, AIF_EINVAL, "NULL idx_out or val_out");
    if (k > TOPK_MAX) return fail(c, AIF_ERANGE, "k %d exceeds %d", k, TOPK_MAX);
    if (n_req > c->max_users) return fail(c, AIF_ERANGE, "n_req %d exceeds max_users %d", n_req, c->max_users);
    const Model &m = c->m;
    for (int r = 0; r < n_req; ++r) {
        const aif_request &q = reqs[r];
        if (q.n_cand < 0 || q.seq_len < 0) return fail(c, AIF_EINVAL, "request %d: negative n_cand or seq_len", r);
        if (q.n_cand > c->max_candidates) return fail(c, AIF_ERANGE, "request %d: n_cand %d exceeds max_candidates %d", r, q.n_cand, c->max_candidates);
        if (q.seq_len > c->max_seq_len) return fail(c, AIF_ERANGE, "request %d: seq_len %d exceeds max_seq_len %d", r, q.seq_len, c->max_seq_len);
        if ((m.d_user > 0 && !q.user_vec) || (q.seq_len > 0 && (!q.seq_keys || !q.seq_vals)) ||
            (q.n_cand > 0 && (!q.cand_ids || !q.logits_out)))
            return fail(c, AIF_EINVAL, "request %d: NULL tensor pointer", r);
        if (((uintptr_t)q.user_vec | (uintptr_t)q.cross_vecs | (uintptr_t)q.seq_keys | (uintptr_t)q.seq_vals) % 16)
            return fail(c, AIF_EINVAL, "request %d: user tensors must be 16-byte aligned", r);
        if ((m.cross_mode == AIF_CROSS_SEGDOT || m.cross_mode == AIF_CROSS_BEA) && !q.cross_vecs)
            return fail(c, AIF_EINVAL, "request %d: SEGDOT and BEA need cross_vecs", r);
        if (m.cross_mode == AIF_CROSS_HADAMARD && !q.cross_vecs && m.d_user != m.d_item)
            return fail(c, AIF_ESHAPE, "request %d: HADAMARD without cross_vecs needs d_user == d_item", r);
    }
    aif_status st = check_device(c);
    if (st != AIF_OK) return st;
    if (n_req == 0) return AIF_OK;
    hipStream_t s = (hipStream_t)hip_stream;

    int slot;
    st = take_slot(c, &slot);
    if (st != AIF_OK) return st;
    char *h = c->h_stage + (size_t)slot * c->slot_bytes;
    char *d = (char *)c->d_stage.p + (size_t)slot * c->slot_bytes;
    ReqDesc *hd = (ReqDesc *)h;
    c->row_base.assign(n_req, 0);
    c->peek_cross.assign(n_req, nullptr);
    // Rows per request first (the tables that follow the descriptors are sized by the block count), and the user
    // slots: requests that bring the same user tensors -- the mini-batch slices of one candidate list -- share one
    // slot, so that the user-side staging runs once per user and not once per slice (Sec. 3.1).
    int n_blk_total = 0;
    for (int r = 0; r < n_req; ++r) n_blk_total += round_up(reqs[r].n_cand, ROW_BLOCK) / ROW_BLOCK;
    int32_t *hb = (int32_t *)(h + (size_t)n_req * sizeof(ReqDesc));       // blk_req [n_blk]
    int32_t *hs = hb + n_blk_total;                                        // blk_slot [n_blk]
    int32_t *hq = hs + n_blk_total;                                        // slot_req [n_slots]
    int n_slots = 0;
    {
        typedef std::tuple<const void *, const void *, const void *, const void *, int32_t> UserKey;
        std::map<UserKey, int> seen;
        for (int r = 0; r < n_req; ++r) {
            const aif_request &q = reqs[r];
            const UserKey key(q.user_vec, q.cross_vecs, q.seq_keys, q.seq_vals, q.seq_len);
            auto it = n_req > 1 ? seen.find(key) : seen.end();
            if (it == seen.end()) {
                if (n_req > 1) seen.emplace(key, n_slots);
                hq[n_slots] = r;
                hd[r].slot = n_slots++;
            } else
                hd[r].slot = it->second;
        }
    }
    c->last_slots = n_slots;
    int rows = 0;
    for (int r = 0; r < n_req; ++r) {
        const aif_request &q = reqs[r];
        ReqDesc &e = hd[r];
        e.pad_ = 0;
        e.user_vec = q.user_vec;
        e.cross_vecs = q.cross_vecs ? q.cross_vecs : q.user_vec;
        e.seq_keys = q.seq_keys;
        e.seq_vals = q.seq_vals;
        e.cand_ids = q.cand_ids;
        e.logits_out = q.logits_out;
        e.scores_out = q.scores_out;
        e.seq_len = q.seq_len;
        e.n_cand = q.n_cand;
        e.row_base = rows;
        e.index = r;
        c->row_base[r] = rows;
        c->peek_cross[r] = e.cross_vecs;
        const int nb = round_up(q.n_cand, ROW_BLOCK) / ROW_BLOCK;
        for (int j = 0; j < nb; ++j) {
            hb[rows / ROW_BLOCK + j] = r;
            hs[rows / ROW_BLOCK + j] = e.slot;
        }
        rows += nb * ROW_BLOCK;
    }
    Batch b;
    b.reqs = (const ReqDesc *)d;
    b.blk_req = (const int32_t *)(d + ((char *)hb - h));
    b.blk_slot = (const int32_t *)(d + ((char *)hs - h));
    b.slot_req = (const int32_t *)(d + ((char *)hq - h));
    b.n_req = n_req;
    b.n_blk = rows / ROW_BLOCK;
    b.n_slots = n_slots;
    // groups of tiles for the attention kernel that keeps K/V resident, 16-byte aligned after the three tables
    const size_t goff = ((size_t)((char *)(hq + n_slots) - h) + 15) / 16 * 16;
    b.n_streamed = 0;
    AttnPlanInfo plan_info{};
    b.n_groups = c->mfma.attn ? attn_plan_groups(m, hd, n_req, c->n_cu, (AttnGroup *)(h + goff), &b.n_streamed, &plan_info) : 0;
    b.groups = (const AttnGroup *)(d + goff);
    size_t bytes = goff + (size_t)b.n_groups * sizeof(AttnGroup);
    const size_t toff = (bytes + 15) / 16 * 16;
    if (k > 0) {
        TopkDesc *ht = (TopkDesc *)(h + toff);
        for (int r = 0; r < n_req; ++r) {
            ht[r].logits = reqs[r].logits_out;
            ht[r].n = reqs[r].n_cand;
        }
        bytes = toff + (size_t)n_req * sizeof(TopkDesc);
    }
    const bool fused = stage_fusable(m, c->mfma);
    const bool staged_proj = !fused && stage_proj_fusable(m, c->mfma);
    // where it can, the attention kernel takes the item vectors from the table itself
    const bool attn_indexes = c->mfma.attn && !c->separate_gather && attn_gathers(m, b, c->mfma);
    c->attn_indexed = attn_indexes;
    // A few requests (the latency cases: one request, or one cut into mini-batches) send their descriptors in the
    // staging launch's arguments and that launch writes the tables on the device: nothing is uploaded.  Otherwise, when
    // the staging launch has few blocks (no gather blocks) it carries the tables to the device itself.
    const bool stage_fills = fused && n_req <= FEW_MAX;
    const bool stage_uploads = fused && !stage_fills && attn_indexes && c->h_stage_dev;
    FewFill fill{};
    if (stage_fills) {
        for (int r = 0; r < n_req; ++r) {
            fill.rd[r] = hd[r];
            fill.td[r] = TopkDesc{reqs[r].logits_out, reqs[r].n_cand};
        }
        for (int sl = 0; sl < n_slots; ++sl) fill.slot_req[sl] = hq[sl];
        fill.reqs = (ReqDesc *)d;
        fill.blk_req = (int32_t *)(d + ((char *)hb - h));
        fill.blk_slot = (int32_t *)(d + ((char *)hs - h));
        fill.slot_req_dev = (int32_t *)(d + ((char *)hq - h));
        fill.groups = (AttnGroup *)(d + goff);
        fill.topk = k > 0 ? (TopkDesc *)(d + toff) : nullptr;
        fill.n_req = n_req;
        fill.n_slots = n_slots;
        fill.n_blk = b.n_blk;
        fill.n_groups = b.n_groups;
        fill.per = plan_info.per;
        fill.resident = plan_info.resident;
    }
    if (!stage_uploads && !stage_fills) HIP_TRY(c, upload(c, slot, bytes, s));

    hipEvent_t *pe = nullptr;
    if (c->prof_on && c->prof_batch_calls < c->prof_max && c->prof_seen_batch++ % c->prof_every == 0)
        pe = &c->prof_batch[(size_t)5 * c->prof_batch_calls++];
    // event i stands before stage i of {gather, user fold, attention, MLP} and after stage i - 1
    auto mark = [&](int i) -> hipError_t {
        const uint32_t need = (i < 4 ? 1u << i : 0u) | (i > 0 ? 1u << (i - 1) : 0u);
        return pe && (c->prof_mask & need) ? hipEventRecord(pe[i], s) : hipSuccess;
    };
    HIP_TRY(c, mark(0));
    if (fused) {
        // gather (unless the attention kernel does it), user fold and K/V packing as one launch; timed as the gather stage
        StageUpload up{};
        if (stage_uploads) {
            const char *mapped = c->h_stage_dev + (size_t)slot * c->slot_bytes;
            up = {mapped, d, bytes, (const ReqDesc *)mapped, (const int32_t *)(mapped + ((char *)hq - h))};
        }
        HIP_TRY(c, launch_stage(m, b, c->table, c->X.p, (int32_t *)c->bad.p, (const float *)c->w1u.p,
                                c->has_bias[0] ? (const float *)c->bias[0].p : nullptr, (float *)c->bias1.p, c->mfma,
                                !attn_indexes, s, stage_uploads ? &up : nullptr, stage_fills ? &fill : nullptr));
        HIP_TRY(c, mark(1));
    } else {
        if (!attn_indexes) HIP_TRY(c, launch_gather(m, b, c->table, c->X.p, (int32_t *)c->bad.p, s));
        HIP_TRY(c, mark(1));
        if (staged_proj) {      // K/V packing, user fold and the users' layer-1 weights as one launch
            HIP_TRY(c, launch_stage_proj(m, b, (const float *)c->w1u.p, c->has_bias[0] ? (const float *)c->bias[0].p : nullptr,
                                         (float *)c->bias1.p, c->mfma, s));
        } else {
            HIP_TRY(c, launch_user_fold(m, b, (const float *)c->w1u.p, c->has_bias[0] ? (const float *)c->bias[0].p : nullptr,
                                        (float *)c->bias1.p, s));
            HIP_TRY(c, launch_fold_w0(m, b, c->mfma, s));
        }
    }
    HIP_TRY(c, mark(2));
    if (c->mfma.attn)
        HIP_TRY(c, launch_attn_mfma(m, b, c->X.p, c->mfma, fused || staged_proj, s, attn_indexes ? c->table : nullptr,
                                    attn_indexes ? (int32_t *)c->bad.p : nullptr));
    else
        HIP_TRY(c, launch_attn_generic(m, b, c->X.p, c->has_wq ? (const float *)c->wq.p : nullptr, c->max_seq_len, s));
    HIP_TRY(c, mark(3));
    if (c->mfma.mlp) {
        const float *bf[MAX_LAYERS];
        for (int l = 0; l < m.n_layers; ++l) bf[l] = c->has_bias[l] ? (const float *)c->bias[l].p : nullptr;
        HIP_TRY(c, launch_mlp_mfma(m, b, c->X.p, c->mfma, bf, (const float *)c->wt[m.n_layers - 1].p,
                                   (const float *)c->bias1.p, s));
    } else {
        MlpGenericWeights gw{};
        for (int l = 0; l < m.n_layers; ++l) {
            gw.wt[l] = (const float *)c->wt[l].p;
            gw.bias[l] = c->has_bias[l] ? (const float *)c->bias[l].p : nullptr;
        }
        HIP_TRY(c, launch_mlp_generic(m, b, c->X.p, gw, (const float *)c->bias1.p, s));
    }
    HIP_TRY(c, mark(4));
    if (k > 0) {
        hipEvent_t *pt = nullptr;
        if (c->prof_on && (c->prof_mask & (1u << AIF_STAGE_TOPK)) && c->prof_topk_calls < c->prof_max &&
            c->prof_seen_topk++ % c->prof_every == 0)
            pt = &c->prof_topk[(size_t)2 * c->prof_topk_calls++];
        if (pt) HIP_TRY(c, hipEventRecord(pt[0], s));
        if (n_req <= TOPK_FEW)                   // the lists' descriptors in the kernel's arguments: a round trip less in its chain
            HIP_TRY(c, launch_topk_few((const TopkDesc *)(h + toff), n_req, k, idx_out, val_out, s));
        else {
            int n_max = 0;
            for (int r = 0; r < n_req; ++r) n_max = std::max(n_max, (int)((const TopkDesc *)(h + toff))[r].n);
            HIP_TRY(c, launch_topk((const TopkDesc *)(d + toff), n_req, n_max, k, idx_out, val_out, s));
        }
        if (pt) HIP_TRY(c, hipEventRecord(pt[1], s));
    }
    // The event guards the slot's pinned host memory against the next call that takes the slot.  When the descriptors
    // travelled in the launch arguments the device never reads that memory: no event, and the stream ends on the last
    // kernel (an event after it is one more thing the device completes before the caller's wait returns).
    c->ev_live[slot] = !stage_fills;
    if (!stage_fills) HIP_TRY(c, hipEventRecord(c->ev[slot], s));
    return AIF_OK;
}

aif_status aif_score_batch(aif_ctx *c, const aif_request *reqs, int32_t n_req, void *hip_stream)
{
    return score_impl(c, reqs, n_req, 0, nullptr, nullptr, hip_stream);
}

aif_status aif_score_topk(aif_ctx *c, const aif_request *reqs, int32_t n_req, int32_t k, int32_t *idx_out,
                          float *val_out, void *hip_stream)
{
    if (!c) return AIF_EINVAL;
    if (k <= 0) return fail(c, AIF_EINVAL, "k must be positive");
    return score_impl(c, reqs, n_req, k, idx_out, val_out, hip_stream);
}

// One request scored (and its k best selected) with every per-call buffer inside the file-scope scratch array: the
// same kernels as score_impl on a one-request batch, with the descriptor tables written by k_static_fill from kernel
// arguments.  No allocation, no pinned staging, no event, no copy or memset command.
aif_status aif_score_topk_static(aif_ctx *c, const aif_request *req, int32_t k, int32_t *idx_out, float *val_out,
                                 void *hip_stream)
{
    if (!c) return AIF_EINVAL;
    if (!req) return fail(c, AIF_EINVAL, "NULL request");
    if (k < 0) return fail(c, AIF_EINVAL, "k must not be negative");
    if (k > 0 && (!idx_out || !val_out)) return fail(c, AIF_EINVAL, "NULL idx_out or val_out");
    if (k > TOPK_MAX) return fail(c, AIF_ERANGE, "k %d exceeds %d", k, TOPK_MAX);
    const Model &m = c->m;
    const aif_request &q = *req;
    if (q.n_cand < 0 || q.seq_len < 0) return fail(c, AIF_EINVAL, "negative n_cand or seq_len");
    if (q.seq_len > c->max_seq_len) return fail(c, AIF_ERANGE, "seq_len %d exceeds max_seq_len %d", q.seq_len, c->max_seq_len);
    if ((m.d_user > 0 && !q.user_vec) || (q.seq_len > 0 && (!q.seq_keys || !q.seq_vals)) || (q.n_cand > 0 && (!q.cand_ids || !q.logits_out)))
        return fail(c, AIF_EINVAL, "NULL tensor pointer");
    if (((uintptr_t)q.user_vec | (uintptr_t)q.cross_vecs | (uintptr_t)q.seq_keys | (uintptr_t)q.seq_vals) % 16)
        return fail(c, AIF_EINVAL, "user tensors must be 16-byte aligned");
    if ((m.cross_mode == AIF_CROSS_SEGDOT || m.cross_mode == AIF_CROSS_BEA) && !q.cross_vecs)
        return fail(c, AIF_EINVAL, "SEGDOT and BEA need cross_vecs");
    if (m.cross_mode == AIF_CROSS_HADAMARD && !q.cross_vecs && m.d_user != m.d_item)
        return fail(c, AIF_ESHAPE, "HADAMARD without cross_vecs needs d_user == d_item");
    aif_status st = check_device(c);
    if (st != AIF_OK) return st;

    // ---- the call's buffers, laid out in the scratch array ------------------------------------------------------
    const int esz = m.dtype == 0 ? 4 : 2, H1 = m.dims[1];
    const int rows = round_up(q.n_cand, ROW_BLOCK), n_blk = rows / ROW_BLOCK;
    ReqDesc rd{};
    rd.user_vec = q.user_vec;
    rd.cross_vecs = q.cross_vecs ? q.cross_vecs : q.user_vec;
    rd.seq_keys = q.seq_keys;
    rd.seq_vals = q.seq_vals;
    rd.cand_ids = q.cand_ids;
    rd.logits_out = q.logits_out;
    rd.scores_out = q.scores_out;
    rd.seq_len = q.seq_len;
    rd.n_cand = q.n_cand;
    AttnGroup tmp[STATIC_MAX_GROUPS];
    if (c->mfma.attn && attn_max_groups((size_t)rows, 1) > (size_t)STATIC_MAX_GROUPS)
        return fail(c, AIF_ERANGE, "n_cand %d: more attention groups than the static call holds (%d)", q.n_cand, STATIC_MAX_GROUPS);
    int n_streamed = 0;
    AttnPlanInfo plan_info{};
    const int n_groups = c->mfma.attn ? attn_plan_groups(m, &rd, 1, c->n_cu, tmp, &n_streamed, &plan_info) : 0;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off = align_up(off + bytes, 256);
        return at;
    };
    const size_t o_req = take(sizeof(ReqDesc)), o_blk = take((size_t)(n_blk + 1) * 4), o_bsl = take((size_t)(n_blk + 1) * 4),
                 o_srq = take(4), o_grp = take((size_t)(n_groups + 1) * sizeof(AttnGroup)), o_tk = take(sizeof(TopkDesc)),
                 o_b1 = take((size_t)H1 * 4);
    size_t o_kmax = 0, o_kv = 0, o_h0 = 0, o_h1 = 0;
    if (c->mfma.attn) {
        o_kmax = take((size_t)m.n_heads * (c->mfma.nktp / 2 + 1) * 4);
        o_kv = take(c->mfma.pack_stride + 16);
    }
    const bool layered = c->mfma.mlp && c->mfma.mlp_variant == MLP_VARIANT_LAYERS;
    if (layered) {
        o_h0 = take(mlp_layers_buf_bytes(m, (size_t)rows, 0));
        o_h1 = take(mlp_layers_buf_bytes(m, (size_t)rows, 1));
    }
    const size_t o_w0 = m.cross_in_mlp == 2 ? take(c->mfma.w0_stride) : 0;
    const size_t o_x = take((size_t)rows * m.ldx * esz);
    if (off > (size_t)AIF_STATIC_SCRATCH_BYTES)
        return fail(c, AIF_ERANGE, "request of %d candidates (sequence of up to %d) needs %zu bytes of workspace, the static call holds %zu",
                    q.n_cand, c->max_seq_len, off, (size_t)AIF_STATIC_SCRATCH_BYTES);
    if (q.n_cand == 0) return AIF_OK;
    hipStream_t s = (hipStream_t)hip_stream;
    unsigned char *base = c->scratch_dev;        // the device address, never the array's name

    FewFill f{};
    f.rd[0] = rd;
    f.td[0] = TopkDesc{q.logits_out, q.n_cand};
    f.reqs = (ReqDesc *)(base + o_req);
    f.blk_req = (int32_t *)(base + o_blk);
    f.blk_slot = (int32_t *)(base + o_bsl);
    f.slot_req_dev = (int32_t *)(base + o_srq);
    f.groups = (AttnGroup *)(base + o_grp);
    f.topk = k > 0 ? (TopkDesc *)(base + o_tk) : nullptr;
    f.n_req = 1;
    f.n_slots = 1;
    f.n_blk = n_blk;
    f.n_groups = n_groups;
    f.per = plan_info.per;
    f.resident = plan_info.resident;
    const bool fused = stage_fusable(m, c->mfma);
    if (!fused) {                                // else the staging launch writes the tables
        hipLaunchKernelGGL(k_static_fill, dim3((few_fill_items(f) + 255) / 256), dim3(256), 0, s, f);
        HIP_TRY(c, hipGetLastError());
    }

    Batch b{};
    b.reqs = f.reqs;
    b.blk_req = f.blk_req;
    b.blk_slot = f.blk_slot;
    b.slot_req = f.slot_req_dev;
    b.groups = f.groups;
    b.n_req = 1;
    b.n_blk = n_blk;
    b.n_groups = n_groups;
    b.n_streamed = n_streamed;
    b.n_slots = 1;
    MfmaPlan plan = c->mfma;                     // the context's packed weights, this call's buffers
    plan.kmax = (float *)(base + o_kmax);
    plan.kvpack = (char *)(base + o_kv);
    plan.hbuf[0] = layered ? (char *)(base + o_h0) : nullptr;
    plan.hbuf[1] = layered ? (char *)(base + o_h1) : nullptr;
    plan.w0_user = m.cross_in_mlp == 2 ? (char *)(base + o_w0) : nullptr;
    void *X = base + o_x;
    float *bias1 = (float *)(base + o_b1);
    int32_t *bad = (int32_t *)c->bad.p;
    const float *b1 = c->has_bias[0] ? (const float *)c->bias[0].p : nullptr;

    c->row_base.clear();                         // aif_peek_features has nothing to show for this call
    c->last_slots = 1;
    const bool attn_indexes = plan.attn && !c->separate_gather && attn_gathers(m, b, plan);
    const bool staged_proj = !fused && stage_proj_fusable(m, plan);
    c->attn_indexed = attn_indexes;
    if (fused) {
        HIP_TRY(c, launch_stage(m, b, c->table, X, bad, (const float *)c->w1u.p, b1, bias1, plan, !attn_indexes, s, nullptr, &f));
    } else {
        if (!attn_indexes) HIP_TRY(c, launch_gather(m, b, c->table, X, bad, s));
        if (staged_proj) {
            HIP_TRY(c, launch_stage_proj(m, b, (const float *)c->w1u.p, b1, bias1, plan, s));
        } else {
            HIP_TRY(c, launch_user_fold(m, b, (const float *)c->w1u.p, b1, bias1, s));
            HIP_TRY(c, launch_fold_w0(m, b, plan, s));
        }
    }
    if (plan.attn)
        HIP_TRY(c, launch_attn_mfma(m, b, X, plan, fused || staged_proj, s, attn_indexes ? c->table : nullptr, attn_indexes ? bad : nullptr));
    else
        HIP_TRY(c, launch_attn_generic(m, b, X, c->has_wq ? (const float *)c->wq.p : nullptr, c->max_seq_len, s));
    if (plan.mlp) {
        const float *bf[MAX_LAYERS];
        for (int l = 0; l < m.n_layers; ++l) bf[l] = c->has_bias[l] ? (const float *)c->bias[l].p : nullptr;
        HIP_TRY(c, launch_mlp_mfma(m, b, X, plan, bf, (const float *)c->wt[m.n_layers - 1].p, bias1, s));
    } else {
        MlpGenericWeights gw{};
        for (int l = 0; l < m.n_layers; ++l) {
            gw.wt[l] = (const float *)c->wt[l].p;
            gw.bias[l] = c->has_bias[l] ? (const float *)c->bias[l].p : nullptr;
        }
        HIP_TRY(c, launch_mlp_generic(m, b, X, gw, bias1, s));
    }
    if (k > 0) HIP_TRY(c, launch_topk_few(&f.td[0], 1, k, idx_out, val_out, s));
    return AIF_OK;
}

aif_status aif_score_request(aif_ctx *ctx, const aif_request *req, void *hip_stream)
{
    if (!ctx) return AIF_EINVAL;
    if (!req) return fail(ctx, AIF_EINVAL, "NULL request");
    return aif_score_batch(ctx, req, 1, hip_stream);
}

aif_status aif_topk(aif_ctx *c, const float *const *logits, const int32_t *n_cand, int32_t n_req, int32_t k,
                    int32_t *idx_out, float *val_out, void *hip_stream)
{
    if (!c) return AIF_EINVAL;
    if (n_req < 0 || (n_req > 0 && (!logits || !n_cand || !idx_out || !val_out)))
        return fail(c, AIF_EINVAL, "NULL argument or negative n_req");
    if (k <= 0) return fail(c, AIF_EINVAL, "k must be positive");
    if (k > TOPK_MAX) return fail(c, AIF_ERANGE, "k %d exceeds %d", k, TOPK_MAX);
    if (n_req > c->max_users) return fail(c, AIF_ERANGE, "n_req %d exceeds max_users %d", n_req, c->max_users);
    for (int r = 0; r < n_req; ++r) {
        if (n_cand[r] < 0) return fail(c, AIF_EINVAL, "request %d: negative n_cand", r);
        if (n_cand[r] > 0 && !logits[r]) return fail(c, AIF_EINVAL, "request %d: NULL logits", r);
    }
    aif_status st = check_device(c);
    if (st != AIF_OK) return st;
    if (n_req == 0) return AIF_OK;
    hipStream_t s = (hipStream_t)hip_stream;
    if (n_req <= TOPK_FEW) {                     // the descriptors in the kernel's arguments: no staging slot, no upload
        TopkDesc few[TOPK_FEW];
        for (int r = 0; r < n_req; ++r) few[r] = TopkDesc{logits[r], n_cand[r]};
        hipEvent_t *pe = nullptr;
        if (c->prof_on && (c->prof_mask & (1u << AIF_STAGE_TOPK)) && c->prof_topk_calls < c->prof_max &&
            c->prof_seen_topk++ % c->prof_every == 0)
            pe = &c->prof_topk[(size_t)2 * c->prof_topk_calls++];
        if (pe) HIP_TRY(c, hipEventRecord(pe[0], s));
        HIP_TRY(c, launch_topk_few(few, n_req, k, idx_out, val_out, s));
        if (pe) HIP_TRY(c, hipEventRecord(pe[1], s));
        return AIF_OK;
    }
    int slot;
    st = take_slot(c, &slot);
    if (st != AIF_OK) return st;
    TopkDesc *h = (TopkDesc *)(c->h_stage + (size_t)slot * c->slot_bytes);
    TopkDesc *d = (TopkDesc *)((char *)c->d_stage.p + (size_t)slot * c->slot_bytes);
    for (int r = 0; r < n_req; ++r) {
        h[r].logits = logits[r];
        h[r].n = n_cand[r];
    }
    HIP_TRY(c, upload(c, slot, (size_t)n_req * sizeof(TopkDesc), s));
    hipEvent_t *pe = nullptr;
    if (c->prof_on && (c->prof_mask & (1u << AIF_STAGE_TOPK)) && c->prof_topk_calls < c->prof_max &&
        c->prof_seen_topk++ % c->prof_every == 0)
        pe = &c->prof_topk[(size_t)2 * c->prof_topk_calls++];
    if (pe) HIP_TRY(c, hipEventRecord(pe[0], s));
    HIP_TRY(c, launch_topk(d, n_req, *std::max_element(n_cand, n_cand + n_req), k, idx_out, val_out, s));
    if (pe) HIP_TRY(c, hipEventRecord(pe[1], s));
    HIP_TRY(c, hipEventRecord(c->ev[slot], s));
    c->ev_live[slot] = true;
    return AIF_OK;
}

aif_status aif_update_rows(aif_ctx *c, const int32_t *ids, const void *rows, int32_t n, void *hip_stream)
{
    if (!c) return AIF_EINVAL;
    if (n < 0 || (n > 0 && (!ids || !rows))) return fail(c, AIF_EINVAL, "NULL ids or rows, or negative n");
    if ((uintptr_t)rows % 16 || (uintptr_t)ids % 4) return fail(c, AIF_EINVAL, "rows must be 16-byte aligned, ids 4-byte aligned");
    aif_status st = check_device(c);
    if (st != AIF_OK) return st;
    HIP_TRY(c, launch_update_rows(c->m, const_cast<void *>(c->table), ids, rows, n, (int32_t *)c->bad.p, (hipStream_t)hip_stream));
    return AIF_OK;
}

aif_status aif_swap_table(aif_ctx *c, const void *new_table, int64_t n_items)
{
    if (!c) return AIF_EINVAL;
    if (!new_table || n_items <= 0) return fail(c, AIF_EINVAL, "NULL table or non-positive n_items");
    if ((uintptr_t)new_table % 16) return fail(c, AIF_EINVAL, "item_table must be 16-byte aligned");
    c->table = new_table;
    c->m.n_items = n_items;
    return AIF_OK;
}

aif_status aif_poll_device_errors(aif_ctx *c, int32_t *n_bad_ids)
{
    if (!c) return AIF_EINVAL;
    if (!n_bad_ids) return fail(c, AIF_EINVAL, "NULL n_bad_ids");
    aif_status st = check_device(c);
    if (st != AIF_OK) return st;
    HIP_TRY(c, hipMemcpy(n_bad_ids, c->bad.p, 4, hipMemcpyDeviceToHost));
    HIP_TRY(c, hipMemset(c->bad.p, 0, 4));
    return AIF_OK;
}

aif_status aif_peek_features(aif_ctx *c, int32_t request, int32_t first_row, int32_t n_rows, void *out)
{
    if (!c) return AIF_EINVAL;
    if (request < 0 || (size_t)request >= c->row_base.size()) return fail(c, AIF_EINVAL, "request %d is not in the last batch", request);
    if (first_row < 0 || n_rows < 0 || !out) return fail(c, AIF_EINVAL, "bad row range or NULL out");
    const Model &m = c->m;
    const size_t row0 = (size_t)c->row_base[request] + first_row;
    if (row0 + n_rows > c->x_rows) return fail(c, AIF_EINVAL, "rows beyond the workspace");
    aif_status st = check_device(c);
    if (st != AIF_OK) return st;
    if (n_rows == 0) return AIF_OK;
    // whole tiles to the host, then piece by piece into row-major order
    const XLayout xl = x_layout(m);
    const size_t t0 = row0 / X_TILE, t1 = (row0 + n_rows - 1) / X_TILE + 1;
    std::vector<char> tiles((t1 - t0) * xl.tile_bytes);
    HIP_TRY(c, hipMemcpy(tiles.data(), (const char *)c->X.p + t0 * xl.tile_bytes, tiles.size(), hipMemcpyDeviceToHost));
    const uint32_t row_bytes = xl.tile_bytes / X_TILE, pieces = row_bytes / 16;
    for (int32_t i = 0; i < n_rows; ++i)
        for (uint32_t p = 0; p < pieces; ++p)
            memcpy((char *)out + (size_t)i * row_bytes + 16 * p,
                   tiles.data() + x_offset(xl, (uint32_t)(row0 + i - t0 * X_TILE), p), 16);
    if (m.cross_in_mlp) {
        // The workspace's cross block is not written on this route (the MLP chain forms c = u (.) e in registers, or the
        // block is folded into the user's layer-1 weights): show the block as the kernels that write it would form it
        // -- fp32 arithmetic on the bf16 values, rounded to nearest even -- from the item block and the request's operand.
        const size_t n_op = m.cross_mode == 1 ? (size_t)m.d_item : (size_t)m.n_cross * m.d_cv;
        std::vector<uint16_t> u(n_op);
        HIP_TRY(c, hipMemcpy(u.data(), c->peek_cross[request], n_op * 2, hipMemcpyDeviceToHost));
        auto widen = [](uint16_t b) { uint32_t w = (uint32_t)b << 16; float f; memcpy(&f, &w, 4); return f; };
        auto narrow = [](float f) {
            uint32_t w;
            memcpy(&w, &f, 4);
            if ((w & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((w >> 16) | 0x40u);
            w += 0x7FFFu + ((w >> 16) & 1u);
            return (uint16_t)(w >> 16);
        };
        for (int32_t i = 0; i < n_rows; ++i) {
            uint16_t *row = (uint16_t *)((char *)out + (size_t)i * row_bytes);
            if (m.cross_mode == 3) {            // Algorithm 1 step 4: the row's last n_cross entries weigh the user-side vectors
                for (int f = 0; f < m.d_cv; ++f) {
                    float acc = 0.f;
                    for (int j = 0; j < m.n_cross; ++j) acc = fmaf(widen(row[m.d_item - m.n_cross + j]), widen(u[(size_t)j * m.d_cv + f]), acc);
                    row[m.d_item + m.d_attn + f] = narrow(acc);
                }
            } else if (m.cross_mode == 2) {     // segment dots: c[j S + s] = <Vc_j, e_s>
                const int S = m.d_item / m.d_cv;
                for (int j = 0; j < m.n_cross; ++j)
                    for (int sg = 0; sg < S; ++sg) {
                        float acc = 0.f;
                        for (int k = 0; k < m.d_cv; ++k) acc = fmaf(widen(u[(size_t)j * m.d_cv + k]), widen(row[sg * m.d_cv + k]), acc);
                        row[m.d_item + m.d_attn + j * S + sg] = narrow(acc);
                    }
            } else
                for (int k = 0; k < m.d_item; ++k) row[m.d_item + m.d_attn + k] = narrow(widen(row[k]) * widen(u[k]));
        }
    }
    return AIF_OK;
}

aif_status aif_profile_begin(aif_ctx *c, int32_t max_calls)
{
    return aif_profile_begin_stages(c, max_calls, (1u << AIF_STAGE_COUNT) - 1);
}

aif_status aif_profile_begin_stages(aif_ctx *c, int32_t max_calls, uint32_t stage_mask)
{
    return aif_profile_begin_sampled(c, max_calls, stage_mask, 1);
}

aif_status aif_profile_begin_sampled(aif_ctx *c, int32_t max_calls, uint32_t stage_mask, int32_t every)
{
    if (!c) return AIF_EINVAL;
    if (every < 1) return fail(c, AIF_EINVAL, "every must be at least 1");
    if (max_calls <= 0 || max_calls > 100000) return fail(c, AIF_EINVAL, "max_calls out of range");
    if (stage_mask == 0 || stage_mask >= (1u << AIF_STAGE_COUNT)) return fail(c, AIF_EINVAL, "stage_mask names no stage");
    aif_status st = check_device(c);
    if (st != AIF_OK) return st;
    while ((int)c->prof_batch.size() < 5 * max_calls) {
        hipEvent_t e;
        HIP_TRY(c, hipEventCreateWithFlags(&e, hipEventDisableSystemFence));
        c->prof_batch.push_back(e);
    }
    while ((int)c->prof_topk.size() < 2 * max_calls) {
        hipEvent_t e;
        HIP_TRY(c, hipEventCreateWithFlags(&e, hipEventDisableSystemFence));
        c->prof_topk.push_back(e);
    }
    c->prof_max = max_calls;
    c->prof_mask = stage_mask;
    c->prof_every = every;
    c->prof_seen_batch = c->prof_seen_topk = 0;
    c->prof_batch_calls = c->prof_topk_calls = 0;
    c->prof_on = true;
    return AIF_OK;
}

aif_status aif_profile_end(aif_ctx *c, double *ms_sum, int32_t *n_calls)
{
    if (!c) return AIF_EINVAL;
    if (!ms_sum || !n_calls) return fail(c, AIF_EINVAL, "NULL output");
    c->prof_on = false;
    for (int i = 0; i < AIF_STAGE_COUNT; ++i) {
        ms_sum[i] = 0.0;
        n_calls[i] = 0;
    }
    for (int j = 0; j < c->prof_batch_calls; ++j) {
        hipEvent_t *pe = &c->prof_batch[(size_t)5 * j];
        for (int st = 0; st < 4; ++st) {
            if (!(c->prof_mask & (1u << st))) continue;
            HIP_TRY(c, hipEventSynchronize(pe[st + 1]));
            float ms = 0.f;
            HIP_TRY(c, hipEventElapsedTime(&ms, pe[st], pe[st + 1]));
            ms_sum[st] += ms;
            n_calls[st] += 1;
        }
    }
    for (int j = 0; j < c->prof_topk_calls; ++j) {
        hipEvent_t *pe = &c->prof_topk[(size_t)2 * j];
        HIP_TRY(c, hipEventSynchronize(pe[1]));
        float ms = 0.f;
        HIP_TRY(c, hipEventElapsedTime(&ms, pe[0], pe[1]));
        ms_sum[AIF_STAGE_TOPK] += ms;
        n_calls[AIF_STAGE_TOPK] += 1;
    }
    c->prof_batch_calls = c->prof_topk_calls = 0;
    return AIF_OK;
}

int32_t aif_last_user_slots(const aif_ctx *c) { return c ? c->last_slots : -1; }
int32_t aif_mlp_layer1_width(const aif_ctx *c) { return !c ? -1 : (c->m.cross_in_mlp == 2 ? c->m.d_item + c->m.d_attn : c->m.k1); }

int32_t aif_stage_kind(const aif_ctx *c, int32_t stage)
{
    if (!c) return -1;
    if (stage == AIF_STAGE_GATHER) return c->attn_indexed ? 2 : 0;
    if (stage == AIF_STAGE_ATTENTION) return c->mfma.attn ? 1 : 0;
    if (stage == AIF_STAGE_MLP) return c->mfma.mlp ? 1 : 0;
    return 0;
}

}  // extern "C"
