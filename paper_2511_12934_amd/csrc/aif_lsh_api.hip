// C ABI of the LSH behaviour-modelling path (include/aif_lsh.h): context, validation, per-call
// staging of the request descriptors and the launch sequence
//   user-side partial sums -> their reduction -> LSH-DIN -> SimTier.
#include "../../include/aif_lsh.h"
#include "aif_lsh_dev.h"
#include "aif_dev.h"

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

using namespace aif;

namespace {
constexpr int LSH_NSLOT = 8;
constexpr int LSH_EV_PER_CALL = 4;
thread_local std::string g_lsh_init_error = "";
}  // namespace

struct aif_lsh_ctx {
    LshModel m{};
    int device = 0;
    int max_seq_len = 0, max_candidates = 0, max_users = 0, max_chunks = 0;
    const uint8_t *table = nullptr;
    void *part = nullptr, *A = nullptr, *bad = nullptr;     // device workspace (owned)
    void *hist = nullptr;                                   // the requests' history signatures as matrix operands (or null: SimTier on the vector ALU)
    void *parts = nullptr;                                  // partial tier counts of a batch whose histories are cut into parts
    void *din_pieces = nullptr;                             // the requests' LSH-DIN tables as bf16 matrix operands (or null: LSH-DIN on the vector ALU)
    size_t hist_stride = 0;
    char *h_stage = nullptr, *h_stage_dev = nullptr;        // pinned ring of descriptor tables, its device mapping (or null)
    void *d_stage = nullptr;
    size_t slot_bytes = 0;
    hipEvent_t ev[LSH_NSLOT] = {};
    bool ev_live[LSH_NSLOT] = {};
    int next_slot = 0;
    bool prof_on = false;
    int prof_max = 0, prof_calls = 0;
    std::vector<hipEvent_t> prof;
    std::string err;
};

namespace {

aif_status lfail(aif_lsh_ctx *c, aif_status st, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (c)
        c->err = buf;
    else
        g_lsh_init_error = buf;
    return st;
}

#define LSH_TRY(ctxp, expr)                                                                           \
    do {                                                                                              \
        hipError_t e_ = (expr);                                                                       \
        if (e_ != hipSuccess)                                                                         \
            return lfail(ctxp, e_ == hipErrorOutOfMemory ? AIF_ENOMEM : AIF_EDEVICE, "%s: %s", #expr, \
                         hipGetErrorString(e_));                                                      \
    } while (0)

void ldestroy(aif_lsh_ctx *c)
{
    if (!c) return;
    if (c->part) (void)hipFree(c->part);
    if (c->A) (void)hipFree(c->A);
    if (c->bad) (void)hipFree(c->bad);
    if (c->hist) (void)hipFree(c->hist);
    if (c->parts) (void)hipFree(c->parts);
    if (c->din_pieces) (void)hipFree(c->din_pieces);
    if (c->d_stage) (void)hipFree(c->d_stage);
    if (c->h_stage) (void)hipHostFree(c->h_stage);
    for (int i = 0; i < LSH_NSLOT; ++i)
        if (c->ev[i]) (void)hipEventDestroy(c->ev[i]);
    for (auto e : c->prof) (void)hipEventDestroy(e);
    delete c;
}

aif_status lcheck_device(aif_lsh_ctx *c)
{
    int cur = -1;
    LSH_TRY(c, hipGetDevice(&cur));
    if (cur != c->device) return lfail(c, AIF_EDEVICE, "context belongs to device %d, current device is %d", c->device, cur);
    return AIF_OK;
}

aif_status linit(const aif_lsh_config *cfg, const uint8_t *table, aif_lsh_ctx *c)
{
    if (cfg->dtype != AIF_F32 && cfg->dtype != AIF_BF16) return lfail(nullptr, AIF_EINVAL, "unknown dtype %d", (int)cfg->dtype);
    if (cfg->n_items <= 0 || cfg->max_seq_len < 0 || cfg->max_candidates <= 0 || cfg->max_users <= 0)
        return lfail(nullptr, AIF_EINVAL, "non-positive size in aif_lsh_config");
    if (cfg->d_bits < 32 || cfg->d_bits > 256 || cfg->d_bits % 32)
        return lfail(nullptr, AIF_ESHAPE, "d_bits = %d: a multiple of 32 in 32..256 is required", cfg->d_bits);
    if (cfg->d_out < 16 || cfg->d_out > 256 || cfg->d_out % 16)
        return lfail(nullptr, AIF_ESHAPE, "d_out = %d: a multiple of 16 in 16..256 is required", cfg->d_out);
    if (cfg->n_tiers < 1 || cfg->n_tiers > LSH_MAX_TIERS) return lfail(nullptr, AIF_ESHAPE, "n_tiers = %d: 1..%d", cfg->n_tiers, LSH_MAX_TIERS);
    if ((uintptr_t)table % 4) return lfail(nullptr, AIF_EINVAL, "sig_table must be 4-byte aligned");
    LshModel &m = c->m;
    m.n_items = cfg->n_items;
    m.d_bits = cfg->d_bits;
    m.d_out = cfg->d_out;
    m.n_tiers = cfg->n_tiers;
    m.dtype = cfg->dtype == AIF_F32 ? 0 : 1;
    m.tier_mul = ((1 << 20) + cfg->d_bits - 1) / cfg->d_bits;
    c->table = table;
    c->max_seq_len = cfg->max_seq_len;
    c->max_candidates = cfg->max_candidates;
    c->max_users = cfg->max_users;
    c->max_chunks = std::min(LSH_MAX_CHUNKS, (cfg->max_seq_len + LSH_TCHUNK - 1) / LSH_TCHUNK);   // a shorter history never has more chunks than a longer one's cap
    LSH_TRY(nullptr, hipGetDevice(&c->device));
    const size_t tab = (size_t)2 * m.d_bits * m.d_out * 4;
    LSH_TRY(nullptr, hipMalloc(&c->part, tab * (size_t)c->max_users * (c->max_chunks > 0 ? c->max_chunks : 1)));
    LSH_TRY(nullptr, hipMalloc(&c->A, tab * (size_t)c->max_users));
    {
        const char *valu = getenv("AIF_LSH_SIMTIER_VALU");      // testing and measurement: SimTier on the vector ALU whatever the shape
        if (lsh_simtier_on_mfma(m) && c->max_seq_len > 0 && !(valu && valu[0] == '1')) {
            c->hist_stride = lsh_hist_stride(m, c->max_seq_len);
            LSH_TRY(nullptr, hipMalloc(&c->hist, c->hist_stride * 16 * (size_t)c->max_users));
            LSH_TRY(nullptr, hipMalloc(&c->parts, lsh_simtier_parts_bytes()));
        }
    }
    {
        const char *valu = getenv("AIF_LSH_DIN_VALU");          // testing and measurement: LSH-DIN on the vector ALU whatever the shape
        if (lsh_din_on_mfma(m) && !(valu && valu[0] == '1'))
            LSH_TRY(nullptr, hipMalloc(&c->din_pieces, lsh_din_pieces_stride(m) * 16 * (size_t)c->max_users));
    }
    LSH_TRY(nullptr, hipMalloc(&c->bad, 16));
    LSH_TRY(nullptr, hipMemset(c->bad, 0, 16));
    const size_t n_blk_max = (size_t)c->max_users * ((c->max_candidates + LSH_BLOCK - 1) / LSH_BLOCK);
    c->slot_bytes = ((size_t)c->max_users * sizeof(LshReqDesc) + n_blk_max * sizeof(int32_t) + 255) / 256 * 256;
    LSH_TRY(nullptr, staging_alloc(c->slot_bytes * LSH_NSLOT, &c->h_stage, &c->h_stage_dev));
    LSH_TRY(nullptr, hipMalloc(&c->d_stage, c->slot_bytes * LSH_NSLOT));
    for (int i = 0; i < LSH_NSLOT; ++i)
        LSH_TRY(nullptr, hipEventCreateWithFlags(&c->ev[i], hipEventDisableTiming | hipEventDisableSystemFence));
    LSH_TRY(nullptr, hipDeviceSynchronize());
    return AIF_OK;
}

}  // namespace

extern "C" {

aif_status aif_lsh_init(const aif_lsh_config *cfg, const uint8_t *sig_table, aif_lsh_ctx **out)
{
    if (!cfg || !sig_table || !out) return lfail(nullptr, AIF_EINVAL, "NULL argument");
    aif_lsh_ctx *c = new (std::nothrow) aif_lsh_ctx();
    if (!c) return lfail(nullptr, AIF_ENOMEM, "out of host memory");
    const aif_status st = linit(cfg, sig_table, c);
    if (st != AIF_OK) {
        ldestroy(c);
        return st;
    }
    *out = c;
    return AIF_OK;
}

void aif_lsh_destroy(aif_lsh_ctx *ctx) { ldestroy(ctx); }

const char *aif_lsh_last_error(const aif_lsh_ctx *ctx) { return ctx ? ctx->err.c_str() : g_lsh_init_error.c_str(); }

aif_status aif_lsh_batch(aif_lsh_ctx *c, const aif_lsh_request *reqs, int32_t n_req, void *hip_stream)
{
    if (!c) return AIF_EINVAL;
    if (n_req < 0 || (n_req > 0 && !reqs)) return lfail(c, AIF_EINVAL, "NULL request array or negative n_req");
    if (n_req > c->max_users) return lfail(c, AIF_ERANGE, "n_req %d exceeds max_users %d", n_req, c->max_users);
    const LshModel &m = c->m;
    for (int r = 0; r < n_req; ++r) {
        const aif_lsh_request &q = reqs[r];
        if (q.n_cand < 0 || q.seq_len < 0) return lfail(c, AIF_EINVAL, "request %d: negative n_cand or seq_len", r);
        if (q.n_cand > c->max_candidates) return lfail(c, AIF_ERANGE, "request %d: n_cand %d exceeds max_candidates %d", r, q.n_cand, c->max_candidates);
        if (q.seq_len > c->max_seq_len) return lfail(c, AIF_ERANGE, "request %d: seq_len %d exceeds max_seq_len %d", r, q.seq_len, c->max_seq_len);
        if ((q.seq_len > 0 && (!q.seq_sigs || !q.seq_emb)) || (q.n_cand > 0 && (!q.cand_ids || !q.din_out || !q.tier_out)))
            return lfail(c, AIF_EINVAL, "request %d: NULL tensor pointer", r);
        if ((uintptr_t)q.seq_sigs % 4 || (uintptr_t)q.seq_emb % 16 || (uintptr_t)q.din_out % 16 || (uintptr_t)q.tier_out % 4)
            return lfail(c, AIF_EINVAL, "request %d: misaligned tensor", r);
    }
    aif_status st = lcheck_device(c);
    if (st != AIF_OK) return st;
    if (n_req == 0) return AIF_OK;
    hipStream_t s = (hipStream_t)hip_stream;

    const int slot = c->next_slot;
    c->next_slot = (slot + 1) % LSH_NSLOT;
    if (c->ev_live[slot]) LSH_TRY(c, hipEventSynchronize(c->ev[slot]));
    char *h = c->h_stage + (size_t)slot * c->slot_bytes;
    char *d = (char *)c->d_stage + (size_t)slot * c->slot_bytes;
    LshReqDesc *hd = (LshReqDesc *)h;
    int32_t *hb = (int32_t *)(h + (size_t)n_req * sizeof(LshReqDesc));
    int slots = 0, max_chunks = 0, longest = 0;
    for (int r = 0; r < n_req; ++r) {
        const aif_lsh_request &q = reqs[r];
        LshReqDesc &e = hd[r];
        e.seq_sigs = q.seq_sigs;
        e.seq_emb = q.seq_emb;
        e.cand_ids = q.cand_ids;
        e.din_out = q.din_out;
        e.tier_out = q.tier_out;
        e.seq_len = q.seq_len;
        e.n_cand = q.n_cand;
        e.cand_base = slots;
        e.index = r;
        const int nb = (q.n_cand + LSH_BLOCK - 1) / LSH_BLOCK;
        for (int j = 0; j < nb; ++j) hb[slots / LSH_BLOCK + j] = r;
        slots += nb * LSH_BLOCK;
        const int ch = lsh_chunks(q.seq_len);
        if (ch > max_chunks) max_chunks = ch;
        if (q.seq_len > longest) longest = q.seq_len;
    }
    LshBatch b;
    b.reqs = (const LshReqDesc *)d;
    b.blk_req = (const int32_t *)(d + (size_t)n_req * sizeof(LshReqDesc));
    b.n_req = n_req;
    b.n_blk = slots / LSH_BLOCK;
    const size_t bytes = (size_t)n_req * sizeof(LshReqDesc) + (size_t)b.n_blk * sizeof(int32_t);
    LSH_TRY(c, staging_upload(c->h_stage, c->h_stage_dev, (size_t)slot * c->slot_bytes, d, bytes, s));

    hipEvent_t *pe = nullptr;
    if (c->prof_on && c->prof_calls < c->prof_max) pe = &c->prof[(size_t)LSH_EV_PER_CALL * c->prof_calls++];
    if (pe) LSH_TRY(c, hipEventRecord(pe[0], s));
    LSH_TRY(c, launch_lsh_user_partial(m, b, max_chunks, c->max_chunks, (float *)c->part, s));
    LSH_TRY(c, launch_lsh_user_reduce(m, b, c->max_chunks, (const float *)c->part, (float *)c->A, s));
    if (pe) LSH_TRY(c, hipEventRecord(pe[1], s));
    if (c->din_pieces)
        LSH_TRY(c, launch_lsh_din_mfma(m, b, c->table, (const float *)c->A, c->din_pieces, (int32_t *)c->bad, s));
    else
        LSH_TRY(c, launch_lsh_din(m, b, c->table, (const float *)c->A, (int32_t *)c->bad, s));
    if (pe) LSH_TRY(c, hipEventRecord(pe[2], s));
    if (c->hist)
        LSH_TRY(c, launch_lsh_simtier_mfma(m, b, c->table, c->hist, c->hist_stride, longest, c->parts, s));
    else
        LSH_TRY(c, launch_lsh_simtier(m, b, c->table, s));
    if (pe) LSH_TRY(c, hipEventRecord(pe[3], s));
    LSH_TRY(c, hipEventRecord(c->ev[slot], s));
    c->ev_live[slot] = true;
    return AIF_OK;
}

int32_t aif_lsh_simtier_kind(const aif_lsh_ctx *ctx) { return !ctx ? -1 : (ctx->hist ? 1 : 0); }

int32_t aif_lsh_din_kind(const aif_lsh_ctx *ctx) { return !ctx ? -1 : (ctx->din_pieces ? 1 : 0); }

aif_status aif_lsh_poll_device_errors(aif_lsh_ctx *c, int32_t *n_bad_ids)
{
    if (!c) return AIF_EINVAL;
    if (!n_bad_ids) return lfail(c, AIF_EINVAL, "NULL n_bad_ids");
    aif_status st = lcheck_device(c);
    if (st != AIF_OK) return st;
    LSH_TRY(c, hipMemcpy(n_bad_ids, c->bad, 4, hipMemcpyDeviceToHost));
    LSH_TRY(c, hipMemset(c->bad, 0, 4));
    return AIF_OK;
}

aif_status aif_lsh_profile_begin(aif_lsh_ctx *c, int32_t max_calls)
{
    if (!c) return AIF_EINVAL;
    if (max_calls <= 0 || max_calls > 100000) return lfail(c, AIF_EINVAL, "max_calls out of range");
    aif_status st = lcheck_device(c);
    if (st != AIF_OK) return st;
    while ((int)c->prof.size() < LSH_EV_PER_CALL * max_calls) {
        hipEvent_t e;
        LSH_TRY(c, hipEventCreateWithFlags(&e, hipEventDisableSystemFence));
        c->prof.push_back(e);
    }
    c->prof_max = max_calls;
    c->prof_calls = 0;
    c->prof_on = true;
    return AIF_OK;
}

aif_status aif_lsh_profile_end(aif_lsh_ctx *c, double *ms, int32_t *calls)
{
    if (!c) return AIF_EINVAL;
    if (!ms || !calls) return lfail(c, AIF_EINVAL, "NULL output");
    c->prof_on = false;
    for (int i = 0; i < AIF_LSH_N_STAGES; ++i) {
        ms[i] = 0.0;
        calls[i] = 0;
    }
    for (int j = 0; j < c->prof_calls; ++j) {
        hipEvent_t *pe = &c->prof[(size_t)LSH_EV_PER_CALL * j];
        LSH_TRY(c, hipEventSynchronize(pe[LSH_EV_PER_CALL - 1]));
        for (int i = 0; i < AIF_LSH_N_STAGES; ++i) {
            float t = 0.f;
            LSH_TRY(c, hipEventElapsedTime(&t, pe[i], pe[i + 1]));
            ms[i] += t;
            ++calls[i];
        }
    }
    c->prof_calls = 0;
    return AIF_OK;
}

}  // extern "C"
