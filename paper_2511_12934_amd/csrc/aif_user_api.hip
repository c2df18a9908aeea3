// C ABI of the user-side network (include/aif_user.h): context, validation, per-call staging of the
// descriptors and the launch sequence
//   projections (Eq. 1) -> K/V packing + attention of every position and of the profile (Eq. 2, Eq. 3)
//   -> FFN + partial pooling -> pooling + combined vector.
// The attention stage is the library's target-attention kernels run on a workspace whose "candidates" are the
// user's sequence positions plus one row for the profile.
#include "../../include/aif_user.h"
#include "aif_user_dev.h"
#include "k_mfma.h"

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

using namespace aif;

namespace {
constexpr int USER_NSLOT = 8;
constexpr int USER_EV_PER_CALL = 4;
thread_local std::string g_user_init_error = "";
}  // namespace

struct aif_user_ctx {
    Model m{};                      // the attention kernels' view: d_item = d_attn = d, one head, no cross, no MLP
    UserWeights w{};
    int device = 0, n_cu = 256;
    int max_seq_len = 0, max_users = 0;
    size_t x_rows = 0;
    void *wseq_t = nullptr, *wprof = nullptr, *wffn_t = nullptr, *b_ffn = nullptr;   // fp32 copies (owned)
    void *wseq_frag = nullptr, *wffn_frag = nullptr;                                  // bf16 MFMA fragments (owned)
    void *X = nullptr, *part = nullptr;                                               // workspace (owned)
    MfmaPlan mfma{};
    char *h_stage = nullptr, *h_stage_dev = nullptr;   // pinned ring of descriptor tables, its device mapping (or null)
    void *d_stage = nullptr;
    size_t slot_bytes = 0;
    hipEvent_t ev[USER_NSLOT] = {};
    bool ev_live[USER_NSLOT] = {};
    int next_slot = 0;
    bool prof_on = false;
    int prof_max = 0, prof_calls = 0;
    std::vector<hipEvent_t> prof;
    std::string err;
};

namespace {

aif_status ufail(aif_user_ctx *c, aif_status st, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (c)
        c->err = buf;
    else
        g_user_init_error = buf;
    return st;
}

#define USER_TRY(ctxp, expr)                                                                          \
    do {                                                                                              \
        hipError_t e_ = (expr);                                                                       \
        if (e_ != hipSuccess)                                                                         \
            return ufail(ctxp, e_ == hipErrorOutOfMemory ? AIF_ENOMEM : AIF_EDEVICE, "%s: %s", #expr, \
                         hipGetErrorString(e_));                                                      \
    } while (0)

int round_up(int v, int a) { return (v + a - 1) / a * a; }

void udestroy(aif_user_ctx *c)
{
    if (!c) return;
    for (void *p : {c->wseq_t, c->wprof, c->wffn_t, c->b_ffn, c->wseq_frag, c->wffn_frag, c->X, c->part, c->d_stage})
        if (p) (void)hipFree(p);
    mfma_release(c->mfma);
    if (c->h_stage) (void)hipHostFree(c->h_stage);
    for (int i = 0; i < USER_NSLOT; ++i)
        if (c->ev[i]) (void)hipEventDestroy(c->ev[i]);
    for (auto e : c->prof) (void)hipEventDestroy(e);
    delete c;
}

aif_status ucheck_device(aif_user_ctx *c)
{
    int cur = -1;
    USER_TRY(c, hipGetDevice(&cur));
    if (cur != c->device) return ufail(c, AIF_EDEVICE, "context belongs to device %d, current device is %d", c->device, cur);
    return AIF_OK;
}

aif_status uinit(const aif_user_config *cfg, const aif_user_weights *wts, aif_user_ctx *c)
{
    if (cfg->dtype != AIF_F32 && cfg->dtype != AIF_BF16) return ufail(nullptr, AIF_EINVAL, "unknown dtype %d", (int)cfg->dtype);
    if (cfg->d_raw <= 0 || cfg->d <= 0 || cfg->max_seq_len < 0 || cfg->max_users <= 0)
        return ufail(nullptr, AIF_EINVAL, "non-positive size in aif_user_config");
    if (!wts->w_profile || !wts->w_seq || !wts->w_ffn) return ufail(nullptr, AIF_EINVAL, "NULL weight");
    const int esz = cfg->dtype == AIF_F32 ? 4 : 2, vec = 16 / esz;
    if (cfg->d_raw % vec || cfg->d % vec) return ufail(nullptr, AIF_ESHAPE, "d_raw and d must be multiples of %d elements", vec);
    if (user_project_lds_bytes(cfg->d_raw) > 160 * 1024 || user_ffn_lds_bytes(cfg->d) > 160 * 1024)
        return ufail(nullptr, AIF_ESHAPE, "d_raw %d or d %d beyond the LDS budget of the projection / FFN kernels", cfg->d_raw, cfg->d);

    Model &m = c->m;
    m.dtype = cfg->dtype == AIF_F32 ? 0 : 1;
    m.n_items = 1;
    m.d_item = m.d_attn = m.d_head = cfg->d;
    m.d_user = 0;
    m.n_heads = 1;
    m.cross_mode = 0;
    m.n_cross = m.d_cv = m.d_cross = 0;
    m.ldx = 2 * cfg->d;
    m.x_tiled = 0;
    m.n_layers = 0;
    m.k1 = 0;
    c->max_seq_len = cfg->max_seq_len;
    c->max_users = cfg->max_users;
    USER_TRY(nullptr, hipGetDevice(&c->device));
    {
        hipDeviceProp_t prop;
        USER_TRY(nullptr, hipGetDeviceProperties(&prop, c->device));
        c->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    }

    hipStream_t s = nullptr;
    const size_t pw = (size_t)cfg->d_raw * cfg->d * 4, fw = (size_t)cfg->d * cfg->d * 4;
    USER_TRY(nullptr, hipMalloc(&c->wseq_t, pw));
    USER_TRY(nullptr, hipMalloc(&c->wprof, pw));
    USER_TRY(nullptr, hipMalloc(&c->wffn_t, fw));
    USER_TRY(nullptr, launch_pack_transposed(m.dtype, wts->w_seq, cfg->d, cfg->d_raw, 0, cfg->d_raw, (float *)c->wseq_t, s));
    USER_TRY(nullptr, launch_to_f32(m.dtype, wts->w_profile, cfg->d, cfg->d_raw, cfg->d_raw, 0, (float *)c->wprof, s));
    USER_TRY(nullptr, launch_pack_transposed(m.dtype, wts->w_ffn, cfg->d, cfg->d, 0, cfg->d, (float *)c->wffn_t, s));
    if (wts->b_ffn) {
        USER_TRY(nullptr, hipMalloc(&c->b_ffn, (size_t)cfg->d * 4));
        USER_TRY(nullptr, launch_to_f32(m.dtype, wts->b_ffn, 1, cfg->d, cfg->d, 0, (float *)c->b_ffn, s));
    }
    c->w = UserWeights{(const float *)c->wseq_t, (const float *)c->wprof, (const float *)c->wffn_t,
                       (const float *)c->b_ffn, cfg->d_raw, cfg->d, m.dtype, nullptr, nullptr, USER_FFN_ROWS};
    {
        const char *force = getenv("AIF_FORCE_GENERIC");
        const bool generic = force && force[0] == '1';
        if (!generic && m.dtype == 1 && (cfg->d == 32 || cfg->d == 64 || cfg->d == 128) && cfg->d_raw % 16 == 0) {
            USER_TRY(nullptr, hipMalloc(&c->wseq_frag, (size_t)cfg->d * cfg->d_raw * 2));
            USER_TRY(nullptr, hipMalloc(&c->wffn_frag, (size_t)cfg->d * cfg->d * 2));
            USER_TRY(nullptr, pack_frag(wts->w_seq, cfg->d_raw, 0, cfg->d, cfg->d_raw, false, c->wseq_frag, s));
            USER_TRY(nullptr, pack_frag(wts->w_ffn, cfg->d, 0, cfg->d, cfg->d, false, c->wffn_frag, s));
            c->w.wseq_frag = c->wseq_frag;
            c->w.wffn_frag = c->wffn_frag;
            c->w.part_rows = 32;
        }
    }

    // the attention kernels: MFMA when the shape is one they serve, else the shape-agnostic one
    const void *no_w[1] = {nullptr};
    USER_TRY(nullptr, mfma_plan(m, c->max_seq_len, c->max_users, 0, nullptr, no_w, c->mfma, s));
    if (!c->mfma.attn && attn_generic_lds_bytes(m, c->max_seq_len) > 160 * 1024)
        return ufail(nullptr, AIF_ESHAPE, "max_seq_len %d needs more LDS than a compute unit has", c->max_seq_len);

    c->x_rows = (size_t)c->max_users * round_up(c->max_seq_len + 1, ROW_BLOCK);
    USER_TRY(nullptr, hipMalloc(&c->X, c->x_rows * m.ldx * esz));
    USER_TRY(nullptr, hipMalloc(&c->part, c->x_rows / 32 * cfg->d * 4));
    const size_t n_blk_max = c->x_rows / ROW_BLOCK;
    const size_t sb = (size_t)c->max_users * (sizeof(ReqDesc) + sizeof(UserDesc)) + (n_blk_max + 4) * sizeof(int32_t) + 16 +
                      attn_max_groups(c->x_rows, c->max_users) * sizeof(AttnGroup);
    c->slot_bytes = (sb + 255) / 256 * 256;
    USER_TRY(nullptr, staging_alloc(c->slot_bytes * USER_NSLOT, &c->h_stage, &c->h_stage_dev));
    USER_TRY(nullptr, hipMalloc(&c->d_stage, c->slot_bytes * USER_NSLOT));
    for (int i = 0; i < USER_NSLOT; ++i)
        USER_TRY(nullptr, hipEventCreateWithFlags(&c->ev[i], hipEventDisableTiming | hipEventDisableSystemFence));
    USER_TRY(nullptr, hipStreamSynchronize(s));
    return AIF_OK;
}

}  // namespace

extern "C" {

aif_status aif_user_init(const aif_user_config *cfg, const aif_user_weights *weights, aif_user_ctx **out)
{
    if (!cfg || !weights || !out) return ufail(nullptr, AIF_EINVAL, "NULL argument");
    aif_user_ctx *c = new (std::nothrow) aif_user_ctx();
    if (!c) return ufail(nullptr, AIF_ENOMEM, "out of host memory");
    const aif_status st = uinit(cfg, weights, c);
    if (st != AIF_OK) {
        udestroy(c);
        return st;
    }
    *out = c;
    return AIF_OK;
}

void aif_user_destroy(aif_user_ctx *ctx) { udestroy(ctx); }

const char *aif_user_last_error(const aif_user_ctx *ctx) { return ctx ? ctx->err.c_str() : g_user_init_error.c_str(); }

int32_t aif_user_attention_kind(const aif_user_ctx *ctx) { return !ctx ? -1 : (ctx->mfma.attn ? 1 : 0); }

aif_status aif_user_precompute(aif_user_ctx *c, const aif_user_request *users, int32_t n_users, void *hip_stream)
{
    if (!c) return AIF_EINVAL;
    if (n_users < 0 || (n_users > 0 && !users)) return ufail(c, AIF_EINVAL, "NULL user array or negative n_users");
    if (n_users > c->max_users) return ufail(c, AIF_ERANGE, "n_users %d exceeds max_users %d", n_users, c->max_users);
    for (int r = 0; r < n_users; ++r) {
        const aif_user_request &q = users[r];
        if (q.seq_len < 0) return ufail(c, AIF_EINVAL, "user %d: negative seq_len", r);
        if (q.seq_len > c->max_seq_len) return ufail(c, AIF_ERANGE, "user %d: seq_len %d exceeds max_seq_len %d", r, q.seq_len, c->max_seq_len);
        if (!q.profile || !q.user_vec_out || (q.seq_len > 0 && (!q.seq || !q.seq_out)))
            return ufail(c, AIF_EINVAL, "user %d: NULL tensor pointer", r);
        if (((uintptr_t)q.profile | (uintptr_t)q.seq | (uintptr_t)q.user_vec_out | (uintptr_t)q.seq_out) % 16)
            return ufail(c, AIF_EINVAL, "user %d: tensors must be 16-byte aligned", r);
    }
    aif_status st = ucheck_device(c);
    if (st != AIF_OK) return st;
    if (n_users == 0) return AIF_OK;
    hipStream_t s = (hipStream_t)hip_stream;
    const Model &m = c->m;

    const int slot = c->next_slot;
    c->next_slot = (slot + 1) % USER_NSLOT;
    if (c->ev_live[slot]) USER_TRY(c, hipEventSynchronize(c->ev[slot]));
    char *h = c->h_stage + (size_t)slot * c->slot_bytes;
    char *d = (char *)c->d_stage + (size_t)slot * c->slot_bytes;
    ReqDesc *hr = (ReqDesc *)h;
    UserDesc *hu = (UserDesc *)(h + (size_t)n_users * sizeof(ReqDesc));
    int32_t *hb = (int32_t *)(h + (size_t)n_users * (sizeof(ReqDesc) + sizeof(UserDesc)));
    int rows = 0;
    for (int r = 0; r < n_users; ++r) {
        const aif_user_request &q = users[r];
        ReqDesc &e = hr[r];
        memset(&e, 0, sizeof e);
        e.seq_keys = q.seq_out;             // keys and values: the projected sequence
        e.seq_vals = q.seq_out;
        e.seq_len = q.seq_len;
        e.n_cand = q.seq_len + 1;           // every position, and the profile, is a query
        e.row_base = rows;
        e.index = r;
        e.slot = r;                         // every user of the call is a user slot of its own
        hu[r] = UserDesc{q.profile, q.seq, q.user_vec_out, q.seq_out, q.seq_len, rows};
        const int nb = round_up(e.n_cand, ROW_BLOCK) / ROW_BLOCK;
        for (int j = 0; j < nb; ++j) hb[rows / ROW_BLOCK + j] = r;
        rows += nb * ROW_BLOCK;
    }
    Batch b;
    b.reqs = (const ReqDesc *)d;
    const UserDesc *du = (const UserDesc *)(d + (size_t)n_users * sizeof(ReqDesc));
    b.blk_req = (const int32_t *)(d + (size_t)n_users * (sizeof(ReqDesc) + sizeof(UserDesc)));
    b.n_req = n_users;
    b.n_slots = n_users;
    b.blk_slot = nullptr;                   // read by the MLP kernels only
    b.slot_req = nullptr;                   // slot s = request s
    b.n_blk = rows / ROW_BLOCK;
    const size_t goff = ((size_t)n_users * (sizeof(ReqDesc) + sizeof(UserDesc)) + (size_t)b.n_blk * sizeof(int32_t) + 15) / 16 * 16;
    b.n_streamed = 0;
    b.n_groups = c->mfma.attn ? attn_plan_groups(m, hr, n_users, c->n_cu, (AttnGroup *)(h + goff), &b.n_streamed) : 0;
    b.groups = (const AttnGroup *)(d + goff);
    USER_TRY(c, staging_upload(c->h_stage, c->h_stage_dev, (size_t)slot * c->slot_bytes, d,
                               goff + (size_t)b.n_groups * sizeof(AttnGroup), s));

    hipEvent_t *pe = nullptr;
    if (c->prof_on && c->prof_calls < c->prof_max) pe = &c->prof[(size_t)USER_EV_PER_CALL * c->prof_calls++];
    if (pe) USER_TRY(c, hipEventRecord(pe[0], s));
    USER_TRY(c, launch_user_project(c->w, du, b.blk_req, b.n_blk, c->X, s));
    if (pe) USER_TRY(c, hipEventRecord(pe[1], s));
    if (c->mfma.attn)
        USER_TRY(c, launch_attn_mfma(m, b, c->X, c->mfma, false, s));
    else
        USER_TRY(c, launch_attn_generic(m, b, c->X, nullptr, c->max_seq_len, s));
    if (pe) USER_TRY(c, hipEventRecord(pe[2], s));
    USER_TRY(c, launch_user_ffn_partial(c->w, du, b.blk_req, b.n_blk, c->X, (float *)c->part, s));
    USER_TRY(c, launch_user_combine(c->w, du, n_users, c->X, (const float *)c->part, s));
    if (pe) USER_TRY(c, hipEventRecord(pe[3], s));
    USER_TRY(c, hipEventRecord(c->ev[slot], s));
    c->ev_live[slot] = true;
    return AIF_OK;
}

aif_status aif_user_profile_begin(aif_user_ctx *c, int32_t max_calls)
{
    if (!c) return AIF_EINVAL;
    if (max_calls <= 0 || max_calls > 100000) return ufail(c, AIF_EINVAL, "max_calls out of range");
    aif_status st = ucheck_device(c);
    if (st != AIF_OK) return st;
    while ((int)c->prof.size() < USER_EV_PER_CALL * max_calls) {
        hipEvent_t e;
        USER_TRY(c, hipEventCreateWithFlags(&e, hipEventDisableSystemFence));
        c->prof.push_back(e);
    }
    c->prof_max = max_calls;
    c->prof_calls = 0;
    c->prof_on = true;
    return AIF_OK;
}

aif_status aif_user_profile_end(aif_user_ctx *c, double *ms, int32_t *calls)
{
    if (!c) return AIF_EINVAL;
    if (!ms || !calls) return ufail(c, AIF_EINVAL, "NULL output");
    c->prof_on = false;
    for (int i = 0; i < AIF_USER_N_STAGES; ++i) {
        ms[i] = 0.0;
        calls[i] = 0;
    }
    for (int j = 0; j < c->prof_calls; ++j) {
        hipEvent_t *pe = &c->prof[(size_t)USER_EV_PER_CALL * j];
        USER_TRY(c, hipEventSynchronize(pe[USER_EV_PER_CALL - 1]));
        for (int i = 0; i < AIF_USER_N_STAGES; ++i) {
            float t = 0.f;
            USER_TRY(c, hipEventElapsedTime(&t, pe[i], pe[i + 1]));
            ms[i] += t;
            ++calls[i];
        }
    }
    c->prof_calls = 0;
    return AIF_OK;
}

}  // extern "C"
