"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the
same seeded inputs, element by element."""
import os

import numpy as np
import pytest

import oracle
from paper_2511_12934_amd import workloads as wl

from helpers import (assert_features_close, assert_logits_close, check_topk_against_oracle_logits, key_rounding_term,
                     oracle_scores, oracle_scores_rows)

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[case] {msg}", flush=True)


@pytest.fixture(scope="module")
def R():
    from paper_2511_12934_amd import runner
    return runner


@pytest.fixture(scope="module")
def torch():
    import torch
    return torch


def run_batch(R, torch, cfg, model, table_dev, users_ids, *, ctx=None, k=None, max_seq_len=None):
    """Score a list of (user, ids) requests in one aif_score_batch; returns per-request logits,
    scores, the device requests and the context."""
    dm = R.DeviceModel(cfg, model)
    own = ctx is None
    if own:
        ctx = R.make_context(cfg, dm, table_dev, max_users=max(len(users_ids), 1),
                             max_candidates=max([len(i) for _, i in users_ids] + [1]),
                             max_seq_len=max([u.seq_keys.shape[0] for u, _ in users_ids] + [1])
                             if max_seq_len is None else max_seq_len)
    drs = [R.upload_request(cfg, u, ids) for u, ids in users_ids]
    ctx.aif_score_batch([d.req for d in drs])
    torch.cuda.synchronize()
    return [d.logits.cpu().numpy() for d in drs], [d.scores.cpu().numpy() for d in drs], drs, ctx


def small_cfg(dtype="f32", **kw):
    base = dict(name="S", index=8, dtype=dtype, n_users=1, n_cand=40, n_items=300, d_item=16,
                id_dist="uniform", seq_len=9, d_attn=8, n_heads=1, use_wq=False,
                cross_mode=wl.CROSS_HADAMARD, n_cross=0, d_cross_vec=0, d_user=16,
                mlp_dims=(56, 24, 12, 1), top_k=5)
    base.update(kw)
    c = wl.Config(**base)
    assert c.d_in == c.mlp_dims[0], c.d_in
    return c


# ---------------------------------------------------------------------------
# configuration 1, full size, fp32: every output element by element
# ---------------------------------------------------------------------------
def test_c1_fp32_whole_request(R, torch):
    cfg = wl.CONFIGS["C1"]
    _say("C1 fp32 1x1000 whole request")
    rng = np.random.default_rng(cfg.seed)
    model = wl.make_model(cfg)
    table = wl.make_table_host(cfg, rng)
    req = wl.make_requests(cfg)[0]
    table_dev = R.to_device(table, cfg.dtype)
    (z,), (y,), drs, ctx = run_batch(R, torch, cfg, model, table_dev, [(req.user, req.ids)])
    ref = oracle_scores(cfg, model, table, req.user, req.ids)

    X = R.peek_features(ctx, cfg, 0, cfg.n_cand)
    assert np.array_equal(X[:, :cfg.d_item], table[req.ids]), "gather is not an exact row copy"
    assert_features_close("f32", X[:, cfg.d_item:cfg.d_item + cfg.d_attn], ref.attn, "attention")
    assert_features_close("f32", X[:, cfg.d_item + cfg.d_attn:], ref.cross, "cross")
    assert_logits_close("f32", z, ref.logits, "C1")
    assert np.allclose(y, ref.scores, rtol=1e-5, atol=1e-7)

    idx = torch.empty(cfg.top_k, dtype=torch.int32, device="cuda")
    val = torch.empty(cfg.top_k, dtype=torch.float32, device="cuda")
    ctx.aif_topk([drs[0].logits], cfg.top_k, idx, val)
    torch.cuda.synchronize()
    oi, ov = oracle.topk(z.astype(np.float64), cfg.top_k)        # K4 alone, on the GPU's own logits
    assert np.array_equal(idx.cpu().numpy(), oi)
    assert np.array_equal(val.cpu().numpy().astype(np.float64), ov)
    check_topk_against_oracle_logits("f32", idx.cpu().numpy(), ref.logits, cfg.top_k)
    assert ctx.aif_poll_device_errors() == 0


def test_c1_minibatch_split_is_bitwise_on_gpu(R, torch):
    cfg = wl.CONFIGS["C1"]
    _say("C1 mini-batch invariance 1x1000 vs 10x100 vs ragged")
    rng = np.random.default_rng(cfg.seed)
    model = wl.make_model(cfg)
    table_dev = R.to_device(wl.make_table_host(cfg, rng), cfg.dtype)
    req = wl.make_requests(cfg)[0]
    dm = R.DeviceModel(cfg, model)
    ctx = R.make_context(cfg, dm, table_dev, max_users=16, max_candidates=1000)
    whole = R.upload_request(cfg, req.user, req.ids)
    ctx.aif_score_request(whole.req)
    torch.cuda.synchronize()
    z0 = whole.logits.cpu().numpy().copy()
    for cuts in ([0, 100, 200, 300, 400, 500, 600, 700, 800, 900, 1000], [0, 1, 17, 256, 257, 777, 1000]):
        whole.logits.fill_(float("nan"))
        parts = [R.slice_request(cfg, whole, lo, hi) for lo, hi in zip(cuts[:-1], cuts[1:])]
        ctx.aif_score_batch([p.req for p in parts])
        torch.cuda.synchronize()
        assert np.array_equal(whole.logits.cpu().numpy(), z0), cuts
    # determinism: the same call twice
    ctx.aif_score_request(whole.req)
    torch.cuda.synchronize()
    assert np.array_equal(whole.logits.cpu().numpy(), z0)


# ---------------------------------------------------------------------------
# configuration 2, full size, bf16: whole and as ten 1,000-item mini-batches
# ---------------------------------------------------------------------------
def test_c2_bf16_whole_and_minibatched(R, torch):
    cfg = wl.CONFIGS["C2"]
    _say("C2 bf16 1x10000, whole and 10x1000")
    rng = np.random.default_rng(cfg.seed)
    model = wl.make_model(cfg)
    table = wl.make_table_host(cfg, rng)
    req = wl.make_requests(cfg)[0]
    table_dev = R.to_device(table, cfg.dtype)
    dm = R.DeviceModel(cfg, model)
    ctx = R.make_context(cfg, dm, table_dev, max_users=10, max_candidates=cfg.n_cand)
    whole = R.upload_request(cfg, req.user, req.ids)
    ctx.aif_score_request(whole.req)
    torch.cuda.synchronize()
    z = whole.logits.cpu().numpy().copy()
    ref = oracle_scores(cfg, model, table, req.user, req.ids)
    X = R.peek_features(ctx, cfg, 0, cfg.n_cand)
    assert np.array_equal(X[:, :cfg.d_item], table[req.ids])
    assert_features_close("bf16", X[:, cfg.d_item:cfg.d_item + cfg.d_attn], ref.attn, "attention",
                          key_rounding_term(cfg, model, table[req.ids], req.user))
    assert_features_close("bf16", X[:, cfg.d_item + cfg.d_attn:], ref.cross, "cross")
    assert_logits_close("bf16", z, ref.logits, "C2 whole")
    # the error actually seen is far inside the 2e-2 bar; keep an eye on it
    assert np.abs(z - ref.logits).max() < 5e-3

    whole.logits.fill_(float("nan"))
    parts = [R.slice_request(cfg, whole, lo, lo + 1000) for lo in range(0, cfg.n_cand, 1000)]
    ctx.aif_score_batch([p.req for p in parts])
    torch.cuda.synchronize()
    assert np.array_equal(whole.logits.cpu().numpy(), z), "mini-batched scores differ from whole-request scores"
    assert ctx.aif_last_user_slots() == 1, "ten slices of one user: the user side is staged once"

    idx = torch.empty(cfg.top_k, dtype=torch.int32, device="cuda")
    val = torch.empty(cfg.top_k, dtype=torch.float32, device="cuda")
    ctx.aif_topk([whole.logits], cfg.top_k, idx, val)
    torch.cuda.synchronize()
    oi, ov = oracle.topk(z.astype(np.float64), cfg.top_k)
    assert np.array_equal(idx.cpu().numpy(), oi)
    assert np.array_equal(val.cpu().numpy().astype(np.float64), ov)
    check_topk_against_oracle_logits("bf16", idx.cpu().numpy(), ref.logits, cfg.top_k)


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_user_side_is_staged_once_per_user_across_slices(R, torch, name):
    """Sec. 3.1: user-level work is not repeated per mini-batch.  A call that mixes the slices of three users'
    candidate lists (interleaved) stages three users -- one folded bias, one packed K/V each, shared by the slices --
    and every candidate gets the bits it gets when its user is scored alone and whole.  The same tensors with another
    sequence length are another user."""
    cfg = wl.CONFIGS[name].scaled(n_items=4000, seq_len=min(wl.CONFIGS[name].seq_len, 300))
    _say(f"{name} shape: slices of three users in one call")
    rng = np.random.default_rng(1234)
    model = wl.make_model(cfg, bias_scale=0.05)
    table = wl.make_table_host(cfg, rng, n_items=4000)
    table_dev = R.to_device(table, cfg.dtype)
    dm = R.DeviceModel(cfg, model)
    sampler = wl.IdSampler(cfg, 4000)
    users = [wl.make_user(cfg, rng) for _ in range(3)]
    ids = [sampler.sample(rng, n) for n in (900, 300, 517)]
    ctx = R.make_context(cfg, dm, table_dev, max_users=8, max_candidates=1000)
    wholes = [R.upload_request(cfg, u, i) for u, i in zip(users, ids)]
    alone = []
    for w in wholes:
        ctx.aif_score_batch([w.req])
        torch.cuda.synchronize()
        assert ctx.aif_last_user_slots() == 1
        alone.append(w.logits.cpu().numpy().copy())
        w.logits.fill_(float("nan"))
    a, b, c = wholes
    parts = [R.slice_request(cfg, a, 0, 256), b, R.slice_request(cfg, c, 0, 100), R.slice_request(cfg, a, 256, 700),
             R.slice_request(cfg, c, 100, 517), R.slice_request(cfg, a, 700, 900)]
    ctx.aif_score_batch([p.req for p in parts])
    torch.cuda.synchronize()
    assert ctx.aif_last_user_slots() == 3
    for w, z in zip(wholes, alone):
        assert np.array_equal(w.logits.cpu().numpy(), z)
    assert_logits_close(cfg.dtype, alone[0], oracle_scores(cfg, model, table, users[0], ids[0]).logits, "user 0")
    # a shorter view of the same sequence is a different user-side input: a slot of its own, and its own scores
    if cfg.seq_len > 40:
        import copy
        short = R.slice_request(cfg, a, 0, 300)
        short.req = copy.copy(short.req)
        short.req.seq_len = 40
        z_short = torch.full((300,), float("nan"), device="cuda")
        short.req.logits_out = z_short
        ctx.aif_score_batch([R.slice_request(cfg, a, 300, 900).req, short.req])
        torch.cuda.synchronize()
        assert ctx.aif_last_user_slots() == 2
        assert np.array_equal(a.logits.cpu().numpy()[300:], alone[0][300:])
        u40 = wl.User(users[0].user_vec, users[0].seq_keys[:40], users[0].seq_vals[:40], users[0].cross_vecs)
        assert_logits_close(cfg.dtype, z_short.cpu().numpy(), oracle_scores(cfg, model, table, u40, ids[0][:300]).logits, "40 keys")


# ---------------------------------------------------------------------------
# small shapes: ragged tails, several users, heads, W_q, both cross modes
# ---------------------------------------------------------------------------
SHAPES = {
    "hadamard": dict(),
    "heads_wq": dict(d_item=24, d_user=24, d_attn=16, n_heads=4, use_wq=True, seq_len=13, mlp_dims=(88, 40, 1)),
    "segdot": dict(d_item=32, d_user=12, d_attn=16, n_heads=2, use_wq=True, seq_len=7, cross_mode=wl.CROSS_SEGDOT,
                   n_cross=4, d_cross_vec=8, mlp_dims=(76, 32, 16, 8, 1)),
    "nocross_1layer": dict(cross_mode=wl.CROSS_NONE, mlp_dims=(40, 1)),
}


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", list(SHAPES))
@pytest.mark.parametrize("sigma", [0.1, 1.0])
def test_small_shapes_ragged_batches(R, torch, dtype, shape, sigma):
    cfg = small_cfg(dtype, **SHAPES[shape])
    _say(f"small {shape} {dtype} sigma={sigma}")
    rng = np.random.default_rng(1234)
    model = wl.make_model(cfg, seed=77, bias_scale=0.3)
    table = wl.make_table_host(cfg, rng, sigma=sigma)
    table_dev = R.to_device(table, cfg.dtype)
    sampler = wl.IdSampler(cfg)
    users_ids = []
    for n, L in [(1, 9), (15, 1), (16, 0), (17, 5), (255, 9), (256, 3), (257, 9), (0, 4), (300, 8)]:
        u = wl.make_user(cfg, rng, sigma=sigma, seq_len=L)
        ids = sampler.sample(rng, n) if n <= cfg.n_items else rng.integers(0, cfg.n_items, n).astype(np.int32)
        users_ids.append((u, ids))
    zs, ys, drs, ctx = run_batch(R, torch, cfg, model, table_dev, users_ids, max_seq_len=9)
    for r, ((u, ids), z, y) in enumerate(zip(users_ids, zs, ys)):
        if ids.size == 0:
            continue
        ref = oracle_scores(cfg, model, table, u, ids, n_threads=1)
        X = R.peek_features(ctx, cfg, r, ids.size)
        assert np.array_equal(X[:, :cfg.d_item], table[ids])
        a = X[:, cfg.d_item:cfg.d_item + cfg.d_attn]
        c = X[:, cfg.d_item + cfg.d_attn:]
        assert_features_close(dtype, a, ref.attn, f"req {r} attention", key_rounding_term(cfg, model, table[ids], u))
        if cfg.d_cross:
            assert_features_close(dtype, c, ref.cross, f"req {r} cross")
        if dtype == "f32":
            assert_logits_close("f32", z, ref.logits, f"req {r}")
        else:
            # inputs far above the configurations' scale: judge bf16 logits
            # relative to the request's scale (2e-2 absolute is for N(0,0.1))
            scale = max(1.0, float(np.abs(ref.logits).max()))
            assert np.abs(z - ref.logits).max() <= 2e-2 * scale, f"req {r}"
        assert np.allclose(y, ref.scores, atol=1e-2 if dtype == "bf16" else 1e-6)


# shapes the bf16 MFMA kernels serve (attention d_head 64 / 32, the MLP chains of C2-C4), with
# ragged sequence lengths and candidate counts, at the configurations' scale and far above it
MFMA_SHAPES = {
    "c3_like": dict(d_item=64, d_user=64, d_attn=64, n_heads=1, mlp_dims=(256, 512, 256, 1)),
    "c2_like": dict(d_item=64, d_user=64, d_attn=64, n_heads=1, mlp_dims=(256, 256, 128, 1)),
    "c4_like": dict(d_item=128, d_user=128, d_attn=128, n_heads=4, mlp_dims=(512, 256, 1)),
}


@pytest.mark.parametrize("shape", list(MFMA_SHAPES))
@pytest.mark.parametrize("sigma", [0.1, 1.0, 4.0])
def test_mfma_kernels_ragged_and_large_inputs(R, torch, shape, sigma):
    cfg = small_cfg("bf16", n_items=5000, seq_len=200, **MFMA_SHAPES[shape])
    _say(f"mfma {shape} sigma={sigma}")
    rng = np.random.default_rng(4321)
    model = wl.make_model(cfg, seed=11, bias_scale=0.2)
    table = wl.make_table_host(cfg, rng, sigma=sigma)
    table_dev = R.to_device(table, cfg.dtype)
    sampler = wl.IdSampler(cfg)
    users_ids = []
    for n, L in [(1, 200), (31, 1), (32, 0), (33, 31), (255, 32), (256, 33), (257, 63), (700, 64), (64, 65), (300, 199)]:
        users_ids.append((wl.make_user(cfg, rng, sigma=sigma, seq_len=L), sampler.sample(rng, n)))
    zs, ys, drs, ctx = run_batch(R, torch, cfg, model, table_dev, users_ids, max_seq_len=200)
    assert ctx.aif_stage_kind("attention") == 1 and ctx.aif_stage_kind("mlp") == 1, "MFMA kernels not selected"
    for r, ((u, ids), z) in enumerate(zip(users_ids, zs)):
        ref = oracle_scores(cfg, model, table, u, ids, n_threads=4)
        X = R.peek_features(ctx, cfg, r, ids.size)
        assert np.array_equal(X[:, :cfg.d_item], table[ids])
        assert_features_close("bf16", X[:, cfg.d_item:cfg.d_item + cfg.d_attn], ref.attn, f"req {r} attention",
                              key_rounding_term(cfg, model, table[ids], u))
        assert_features_close("bf16", X[:, cfg.d_item + cfg.d_attn:], ref.cross, f"req {r} cross")
        if sigma == 0.1:
            assert_logits_close("bf16", z, ref.logits, f"req {r}")
        else:
            scale = max(1.0, float(np.abs(ref.logits).max()))
            assert np.abs(z - ref.logits).max() <= 2e-2 * scale, f"req {r}"


@pytest.mark.parametrize("shape", list(MFMA_SHAPES))
def test_mlp_chain_blocks_that_take_two_tiles(R, torch, shape):
    """A batch with more 256-candidate tiles than twice the compute units: the MLP chain's blocks then take two
    tiles each, here mostly of two different requests (different layer-1 biases, outputs, ragged ends).
    Sampled requests against the oracle; every request bit for bit against the same request scored alone
    (few tiles: one per block)."""
    cfg = small_cfg("bf16", n_items=5000, seq_len=12, **MFMA_SHAPES[shape])
    _say(f"two-tile blocks {shape}")
    rng = np.random.default_rng(977)
    model = wl.make_model(cfg, seed=12, bias_scale=0.2)
    table = wl.make_table_host(cfg, rng, sigma=1.0)
    table_dev = R.to_device(table, cfg.dtype)
    sampler = wl.IdSampler(cfg)
    sizes = [200, 300, 257, 256, 31, 513, 1]
    users_ids = []
    for r in range(640):
        users_ids.append((wl.make_user(cfg, rng, sigma=1.0, seq_len=int(rng.integers(0, 13))),
                          sampler.sample(rng, sizes[r % len(sizes)])))
    n_tiles = sum((ids.size + 255) // 256 for _, ids in users_ids)
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    assert n_tiles > 2 * n_cu + 64, "the batch is too small for two-tile blocks on this device"
    zs, ys, drs, ctx = run_batch(R, torch, cfg, model, table_dev, users_ids, max_seq_len=12)
    assert ctx.aif_stage_kind("mlp") == 1, "MFMA chain not selected"
    assert ctx.aif_poll_device_errors() == 0
    for r in list(range(24)) + list(range(len(users_ids) - 8, len(users_ids))):
        u, ids = users_ids[r]
        ref = oracle_scores(cfg, model, table, u, ids, n_threads=8)
        scale = max(1.0, float(np.abs(ref.logits).max()))
        assert np.all(np.isfinite(zs[r])) and np.abs(zs[r] - ref.logits).max() <= 2e-2 * scale, f"req {r}"
    for r, (u, ids) in enumerate(users_ids):
        alone = R.upload_request(cfg, u, ids)
        ctx.aif_score_request(alone.req)
        torch.cuda.synchronize()
        assert np.array_equal(alone.logits.cpu().numpy(), zs[r]), f"req {r}: batch and single call differ"


def test_resident_and_streaming_attention_give_the_same_bits(R, torch):
    """A request whose K/V fit in LDS is served by the resident attention kernel; in a batch with a
    request whose K/V do not fit, by the streaming one.  Its results must not depend on the company."""
    cfg = small_cfg("bf16", n_items=5000, seq_len=1100, **MFMA_SHAPES["c3_like"])
    _say("resident vs streaming attention, same request")
    rng = np.random.default_rng(99)
    model = wl.make_model(cfg, seed=5, bias_scale=0.2)
    table = wl.make_table_host(cfg, rng)
    table_dev = R.to_device(table, cfg.dtype)
    sampler = wl.IdSampler(cfg)
    ua, ia = wl.make_user(cfg, rng, seq_len=333), sampler.sample(rng, 777)
    ub, ib = wl.make_user(cfg, rng, seq_len=1100), sampler.sample(rng, 300)     # 35 key tiles x 8 KB > LDS
    dm = R.DeviceModel(cfg, model)
    ctx = R.make_context(cfg, dm, table_dev, max_users=2, max_candidates=1024, max_seq_len=1100)
    da, db = R.upload_request(cfg, ua, ia), R.upload_request(cfg, ub, ib)
    ctx.aif_score_batch([da.req])
    torch.cuda.synchronize()
    z_alone = da.logits.cpu().numpy().copy()
    x_alone = R.peek_features(ctx, cfg, 0, ia.size)
    assert ctx.aif_stage_kind("gather") == 2, "the resident attention kernel indexes the item table itself"
    da.logits.fill_(float("nan"))
    ctx.aif_score_batch([da.req, db.req])
    torch.cuda.synchronize()
    assert ctx.aif_stage_kind("gather") == 0, "with the streaming kernel the gather is a launch of its own"
    assert np.array_equal(R.peek_features(ctx, cfg, 0, ia.size), x_alone)
    assert np.array_equal(da.logits.cpu().numpy(), z_alone)
    assert_logits_close("bf16", z_alone, oracle_scores(cfg, model, table, ua, ia, n_threads=4).logits, "resident")
    assert_logits_close("bf16", db.logits.cpu().numpy(), oracle_scores(cfg, model, table, ub, ib, n_threads=4).logits, "streaming")


@pytest.mark.parametrize("shape", ["c2_like", "c4_like"])
def test_streamed_requests_give_the_same_bits_alone_and_in_any_company(R, torch, shape):
    """Requests whose K/V exceed LDS go to the streaming kernels: one workgroup per 32-candidate tile with the keys
    split over its waves when the batch is small, one wave per tile otherwise (two- or eight-wave workgroups).  All
    sum a candidate's keys in the same runs and add the runs in the same order, so a request has the same bits
    alone, in a medium batch and in a large one.  Sequence lengths cover runs of one stage, empty runs (fewer
    stages than waves), an odd number of key tiles and a ragged last tile; every request against the oracle."""
    heads = MFMA_SHAPES[shape]["n_heads"]
    long_l = 1100 if heads == 1 else 700            # > 152 KB of packed K/V either way
    cfg = small_cfg("bf16", n_items=5000, seq_len=2100, **MFMA_SHAPES[shape])
    _say(f"streamed requests alone / medium / large batch, {shape}")
    rng = np.random.default_rng(2024)
    model = wl.make_model(cfg, seed=9, bias_scale=0.2)
    table = wl.make_table_host(cfg, rng)
    table_dev = R.to_device(table, cfg.dtype)
    sampler = wl.IdSampler(cfg)
    dm = R.DeviceModel(cfg, model)
    ctx = R.make_context(cfg, dm, table_dev, max_users=40, max_candidates=2048, max_seq_len=2100)
    probes = [(long_l, 300), (long_l + 37, 33), (2100, 64), (long_l + 64 * 3 + 1, 257)]
    probes = [(wl.make_user(cfg, rng, seq_len=L), sampler.sample(rng, n)) for L, n in probes]
    alone = []
    for u, ids in probes:
        d = R.upload_request(cfg, u, ids)
        ctx.aif_score_batch([d.req])
        torch.cuda.synchronize()
        z = d.logits.cpu().numpy().copy()
        assert_logits_close("bf16", z, oracle_scores(cfg, model, table, u, ids, n_threads=4).logits, "alone")
        alone.append(z)
    filler_user = wl.make_user(cfg, rng, seq_len=long_l)
    for n_fill, what in [(10, "medium batch: a wave per tile, two-wave workgroups"),
                         (36, "large batch: eight-wave workgroups")]:
        fill = [R.upload_request(cfg, filler_user, sampler.sample(rng, 2000)) for _ in range(n_fill)]
        ds = [R.upload_request(cfg, u, ids) for u, ids in probes]
        ctx.aif_score_batch([f.req for f in fill[: n_fill // 2]] + [d.req for d in ds] + [f.req for f in fill[n_fill // 2:]])
        torch.cuda.synchronize()
        for i, d in enumerate(ds):
            assert np.array_equal(d.logits.cpu().numpy(), alone[i]), f"probe {i}: {what}"


def test_mfma_attention_with_item_vector_wider_than_attention(R, torch):
    """d_item > d_attn without W_q: the query is the leading slice, the Hadamard cross still spans the whole
    item vector; the MLP of this shape has no MFMA variant, so the workspace stays row-major."""
    cfg = small_cfg("bf16", n_items=4000, seq_len=150, d_item=128, d_user=128, d_attn=64, n_heads=1,
                    mlp_dims=(448, 64, 1))
    _say("MFMA attention, d_item 128 > d_attn 64, generic MLP")
    rng = np.random.default_rng(123)
    model = wl.make_model(cfg, seed=2, bias_scale=0.2)
    table = wl.make_table_host(cfg, rng)
    sampler = wl.IdSampler(cfg)
    users_ids = [(wl.make_user(cfg, rng, seq_len=L), sampler.sample(rng, n)) for n, L in [(600, 150), (45, 77)]]
    zs, _, _, ctx = run_batch(R, torch, cfg, model, R.to_device(table, "bf16"), users_ids, max_seq_len=150)
    assert ctx.aif_stage_kind("attention") == 1 and ctx.aif_stage_kind("mlp") == 0
    for r, ((u, ids), z) in enumerate(zip(users_ids, zs)):
        ref = oracle_scores(cfg, model, table, u, ids, n_threads=4)
        X = R.peek_features(ctx, cfg, r, ids.size)
        assert np.array_equal(X[:, :cfg.d_item], table[ids])
        assert_features_close("bf16", X[:, cfg.d_item:cfg.d_item + cfg.d_attn], ref.attn, f"req {r} attention",
                              key_rounding_term(cfg, model, table[ids], u))
        assert_features_close("bf16", X[:, cfg.d_item + cfg.d_attn:], ref.cross, f"req {r} cross")
        assert_logits_close("bf16", z, ref.logits, f"req {r}")


def test_forced_generic_kernels_on_bf16_config(R, torch, monkeypatch):
    """The shape-agnostic kernels must also serve a bf16 model the MFMA kernels cover."""
    monkeypatch.setenv("AIF_FORCE_GENERIC", "1")
    cfg = wl.CONFIGS["C3"].scaled(n_items=3000)
    _say("C3 shape on the generic kernels")
    rng = np.random.default_rng(7)
    model = wl.make_model(cfg)
    table = wl.make_table_host(cfg, rng, n_items=3000)
    u = wl.make_user(cfg, rng)
    ids = wl.IdSampler(cfg, 3000).sample(rng, 300)
    (z,), _, drs, ctx = run_batch(R, torch, cfg, model, R.to_device(table, "bf16"), [(u, ids)])
    assert ctx.aif_stage_kind("attention") == 0 and ctx.aif_stage_kind("mlp") == 0
    assert_logits_close("bf16", z, oracle_scores(cfg, model, table, u, ids).logits)
    # the fall-back is not silent: the context says which stages left the matrix cores
    dm = R.DeviceModel(cfg, model)
    ctx2 = R.make_context(cfg, dm, R.to_device(table, "bf16"), max_candidates=300, max_users=1)
    note = ctx2.aif_last_error()
    assert "shape-agnostic" in note and "attention" in note and "MLP" in note, note
    monkeypatch.delenv("AIF_FORCE_GENERIC")
    ctx3 = R.make_context(cfg, dm, R.to_device(table, "bf16"), max_candidates=300, max_users=1)
    assert ctx3.aif_last_error() == ""


def test_mfma_kernels_on_row_major_workspace(R, torch, monkeypatch):
    """The MFMA kernels take the workspace in either layout (fragment order when both of them consume it,
    row-major when one consumer is a shape-agnostic kernel): same results, bit for bit."""
    cfg = wl.CONFIGS["C3"].scaled(n_items=3000)
    _say("C3 shape, MFMA kernels, row-major workspace vs fragment order")
    rng = np.random.default_rng(11)
    model = wl.make_model(cfg)
    table = wl.make_table_host(cfg, rng, n_items=3000)
    u = wl.make_user(cfg, rng)
    ids = wl.IdSampler(cfg, 3000).sample(rng, 333)
    (z0,), _, _, ctx0 = run_batch(R, torch, cfg, model, R.to_device(table, "bf16"), [(u, ids)])
    X0 = R.peek_features(ctx0, cfg, 0, ids.size)
    monkeypatch.setenv("AIF_X_ROW_MAJOR", "1")
    (z1,), _, _, ctx1 = run_batch(R, torch, cfg, model, R.to_device(table, "bf16"), [(u, ids)])
    assert ctx1.aif_stage_kind("attention") == 1 and ctx1.aif_stage_kind("mlp") == 1
    X1 = R.peek_features(ctx1, cfg, 0, ids.size)
    assert np.array_equal(X0, X1)
    assert np.array_equal(z0, z1)
    assert_logits_close("bf16", z1, oracle_scores(cfg, model, table, u, ids).logits)


def test_descriptor_tables_uploaded_by_kernel_or_by_copy_give_the_same_bits(R, torch, monkeypatch):
    """The call's descriptor tables reach the device by a kernel that reads the mapped pinned slot (inside the staging
    launch when the attention kernel indexes the table) or, where the mapping is refused, by a copy command."""
    cfg = wl.CONFIGS["C3"].scaled(n_items=3000)
    _say("C3 shape, descriptor upload by kernel vs by copy command")
    rng = np.random.default_rng(13)
    model = wl.make_model(cfg)
    table = wl.make_table_host(cfg, rng, n_items=3000)
    reqs = [(wl.make_user(cfg, rng), wl.IdSampler(cfg, 3000).sample(rng, n)) for n in (333, 1, 64, 700)]
    z0, _, _, ctx0 = run_batch(R, torch, cfg, model, R.to_device(table, "bf16"), reqs)
    assert ctx0.aif_stage_kind("gather") == 2
    monkeypatch.setenv("AIF_STAGING_COPY", "1")
    z1, _, _, ctx1 = run_batch(R, torch, cfg, model, R.to_device(table, "bf16"), reqs)
    assert ctx1.aif_stage_kind("gather") == 2
    for r, (u, ids) in enumerate(reqs):
        assert np.array_equal(z0[r], z1[r]), f"request {r}"
    assert_logits_close("bf16", z1[0], oracle_scores(cfg, model, table, reqs[0][0], reqs[0][1]).logits)


def test_stale_workspace_rows_do_not_change_a_candidates_bits(R, torch):
    """Rows of the workspace past the end of a request keep what an earlier call left there.  A call with
    huge-valued rows (their softmax takes the true maximum instead of the norm bound) is followed, on the same
    context, by a shorter request at the configurations' scale whose last tile ends among those rows: its
    candidates must come out bit for bit as on a fresh context."""
    cfg = wl.CONFIGS["C3"].scaled(n_items=3000)
    _say("C3 shape, stale huge rows in the padded tail of the last tile")
    rng = np.random.default_rng(23)
    model = wl.make_model(cfg)
    table = wl.make_table_host(cfg, rng, n_items=3000)
    table[:1500] = wl.round_storage(table[:1500] * 300.0, "bf16")
    u_big = wl.make_user(cfg, rng, sigma=30.0)
    u = wl.make_user(cfg, rng)
    ids_big = rng.permutation(1500)[:64].astype(np.int32)
    ids = (1500 + rng.permutation(1500)[:40]).astype(np.int32)
    table_dev = R.to_device(table, "bf16")
    (zb,), _, _, ctx = run_batch(R, torch, cfg, model, table_dev, [(u_big, ids_big)], max_seq_len=cfg.seq_len)
    assert np.all(np.isfinite(zb))
    (z1,), _, _, _ = run_batch(R, torch, cfg, model, table_dev, [(u, ids)], ctx=ctx)
    X1 = R.peek_features(ctx, cfg, 0, ids.size)
    (z0,), _, _, ctx0 = run_batch(R, torch, cfg, model, table_dev, [(u, ids)], max_seq_len=cfg.seq_len)
    X0 = R.peek_features(ctx0, cfg, 0, ids.size)
    assert np.array_equal(X0, X1)
    assert np.array_equal(z0, z1)
    assert_logits_close("bf16", z1, oracle_scores(cfg, model, table, u, ids).logits)


# ---------------------------------------------------------------------------
# Bridge Embedding Approximation as the cross block (Sec. 4.1, Algorithm 1 step 4)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,n_bridges,d_out", [("f32", 5, 12), ("f32", 16, 4), ("bf16", 10, 40), ("bf16", 3, 8)])
def test_bea_cross_on_the_shape_agnostic_kernels(R, torch, dtype, n_bridges, d_out):
    d_item = 24
    cfg = small_cfg(dtype, d_item=d_item, d_user=8, d_attn=8, seq_len=7, cross_mode=wl.CROSS_BEA, n_cross=n_bridges,
                    d_cross_vec=d_out, mlp_dims=(8 + d_item + 8 + d_out, 16, 1), n_cand=75)
    _say(f"BEA generic {dtype} n={n_bridges} d'={d_out}")
    rng = np.random.default_rng(31)
    model = wl.make_model(cfg, seed=4, bias_scale=0.3)
    table = wl.make_table_host(cfg, rng)
    u = wl.make_user(cfg, rng, sigma=1.0)
    ids = wl.IdSampler(cfg).sample(rng, cfg.n_cand)
    (z,), _, _, ctx = run_batch(R, torch, cfg, model, R.to_device(table, dtype), [(u, ids)])
    assert ctx.aif_stage_kind("attention") == 0
    ref = oracle_scores(cfg, model, table, u, ids)
    X = R.peek_features(ctx, cfg, 0, ids.size)
    assert np.array_equal(X[:, :d_item], table[ids])
    assert_features_close(dtype, X[:, d_item + cfg.d_attn:], ref.cross, "BEA cross")
    assert_logits_close(dtype, z, ref.logits, "BEA generic")


@pytest.mark.parametrize("shape", ["resident_16", "resident_pad_10", "resident_two_ksteps_20", "streaming_16",
                                   "heads32_wide_item"])
@pytest.mark.parametrize("fold", [False, True])
def test_bea_cross_on_the_mfma_kernels(R, torch, monkeypatch, shape, fold):
    """The weighted sum as an MFMA inside both attention kernels: 16 bridges (one k-step), 10 (window entries in
    front of the weights meet zero rows), 20 (two k-steps), the streaming kernel (L = 1000), and 4 heads of 32 with
    a 128-wide row and a 32-wide output.  fold: the default route where the head is a fused chain -- the block's share
    of layer 1, sum_j w^_j (W1c V^T)[n, j], is folded into each user's layer-1 weights at the bridge weights' columns
    and no kernel forms the block (the library then shows it as computed from the row and the user's vectors);
    without (AIF_CROSS_FOLD=0) the attention kernels write it."""
    if not fold:
        monkeypatch.setenv("AIF_CROSS_FOLD", "0")
    base = wl.CONFIGS["B3"]
    if shape == "resident_16":
        cfg = base.scaled(n_items=3000)
    elif shape == "resident_pad_10":
        cfg = base.scaled(n_items=3000, n_cross=10)
    elif shape == "resident_two_ksteps_20":
        cfg = base.scaled(n_items=3000, n_cross=20)
    elif shape == "streaming_16":
        cfg = base.scaled(n_items=3000, seq_len=1000, mlp_dims=(256, 256, 128, 1))
    else:
        cfg = wl.CONFIGS["C4"].scaled(n_items=3000, cross_mode=wl.CROSS_BEA, n_cross=16, d_cross_vec=32, d_user=96,
                                      mlp_dims=(384, 64, 1))
    assert cfg.d_in == cfg.mlp_dims[0]
    _say(f"BEA MFMA {shape}")
    rng = np.random.default_rng(37)
    model = wl.make_model(cfg, bias_scale=0.05)
    table = wl.make_table_host(cfg, rng, n_items=3000)
    users = [wl.make_user(cfg, rng, sigma=s) for s in (0.1, 1.0)]
    sampler = wl.IdSampler(cfg, 3000)
    reqs = [(users[0], sampler.sample(rng, 333)), (users[1], sampler.sample(rng, 600))]
    zs, _, _, ctx = run_batch(R, torch, cfg, model, R.to_device(table, "bf16"), reqs)
    assert ctx.aif_stage_kind("attention") == 1
    folded = fold and shape != "heads32_wide_item"          # that head is no fused chain: nothing to fold into
    assert ctx.aif_mlp_layer1_width() == (cfg.d_item + cfg.d_attn if folded else cfg.d_in - cfg.d_user)
    # the resident kernel indexes the table itself and takes the bridge weights from the table row
    assert ctx.aif_stage_kind("gather") == (0 if shape == "streaming_16" else 2)
    for i, (u, ids) in enumerate(reqs):
        ref = oracle_scores(cfg, model, table, u, ids)
        X = R.peek_features(ctx, cfg, i, ids.size)
        assert np.array_equal(X[:, :cfg.d_item], table[ids])
        assert_features_close("bf16", X[:, cfg.d_item:cfg.d_item + cfg.d_attn], ref.attn, "attention",
                              key_rounding_term(cfg, model, table[ids], u))
        # fp32 accumulation of at most 32 products of bf16 values, one rounding to bf16 on the way out
        c = X[:, cfg.d_item + cfg.d_attn:]
        tol = 2.0 ** -8 * np.abs(ref.cross) + 2.0 ** -16 * np.abs(ref.cross).max() + 1e-30
        assert np.all(np.abs(c - ref.cross) <= tol), f"BEA cross, request {i}"
        if i == 0:
            assert_logits_close("bf16", zs[i], ref.logits, f"BEA {shape}")
        else:                                               # inputs of unit scale: relative to the request's logits
            from helpers import assert_bf16_logits_tight
            assert_bf16_logits_tight(zs[i], ref.logits, f"BEA {shape}, request {i}")


# ---------------------------------------------------------------------------
# wide heads: the MLP one launch per layer
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("shape", ["two_hidden_tiled", "three_hidden_tiled", "row_major_after_generic_attention"])
def test_layered_mlp_for_wide_heads(R, torch, shape):
    """Hidden widths that are multiples of 256 and not one of the fused chains: layer by layer through HBM in
    fragment order.  Ragged requests, non-zero biases, both workspace layouts."""
    base = wl.CONFIGS["C3"].scaled(n_items=3000)
    if shape == "two_hidden_tiled":
        cfg = base.scaled(mlp_dims=(256, 256, 256, 1))
    elif shape == "three_hidden_tiled":
        cfg = base.scaled(mlp_dims=(256, 512, 256, 256, 1))
    else:
        cfg = base.scaled(mlp_dims=(256, 768, 256, 1), use_wq=True)
    _say(f"layered MLP {shape} {cfg.mlp_dims}")
    rng = np.random.default_rng(53)
    model = wl.make_model(cfg, bias_scale=0.05)
    table = wl.make_table_host(cfg, rng, n_items=3000)
    sampler = wl.IdSampler(cfg, 3000)
    reqs = [(wl.make_user(cfg, rng), sampler.sample(rng, n)) for n in (300, 1, 257, 600)]
    zs, _, _, ctx = run_batch(R, torch, cfg, model, R.to_device(table, "bf16"), reqs)
    assert ctx.aif_stage_kind("mlp") == 1
    assert ctx.aif_stage_kind("attention") == (0 if cfg.use_wq else 1)
    for i, (u, ids) in enumerate(reqs):
        assert_logits_close("bf16", zs[i], oracle_scores(cfg, model, table, u, ids).logits, f"layered {shape} request {i}")
    # slices of a request give the same bits as the whole
    u, ids = reqs[3]
    parts, _, _, _ = run_batch(R, torch, cfg, model, R.to_device(table, "bf16"), [(u, ids[:256]), (u, ids[256:])])
    assert np.array_equal(np.concatenate(parts), zs[3])


# ---------------------------------------------------------------------------
# query projection + 16-wide heads on the matrix cores (the shape of configuration 5)
# ---------------------------------------------------------------------------
PROJ_SHAPES = {
    # C5's model: 8 heads of 16 over a 256-wide item vector, 16 cross vectors x 4 segments, layered MLP
    "c5_like": dict(d_item=256, d_user=576, d_attn=128, n_heads=8, use_wq=True, cross_mode=wl.CROSS_SEGDOT,
                    n_cross=16, d_cross_vec=64, mlp_dims=(1024, 1024, 512, 256, 1)),
    # Hadamard cross, fused MLP chain (workspace in fragment order)
    "hadamard_4_heads": dict(d_item=64, d_user=64, d_attn=64, n_heads=4, use_wq=True, mlp_dims=(256, 256, 128, 1)),
    # fewer cross vectors than MFMA rows, narrow segments, shape-agnostic MLP (row-major workspace)
    "segdot_6_vectors_2_heads": dict(d_item=128, d_user=16, d_attn=32, n_heads=2, use_wq=True,
                                     cross_mode=wl.CROSS_SEGDOT, n_cross=6, d_cross_vec=32, mlp_dims=(200, 64, 1)),
    "no_cross_8_heads": dict(d_item=64, d_user=8, d_attn=128, n_heads=8, use_wq=True, cross_mode=wl.CROSS_NONE,
                             mlp_dims=(200, 32, 1)),
}


def _projected_attention_tolerance(cfg, model, rows, user, ref_attn):
    """The kernel rounds the projected, scaled query to bf16 (unit roundoff 2^-8) before the score product; the
    oracle never rounds.  A score moves by at most ds = 2^-8 sum_k |q_k K_tk| / sqrt(d_h), the softmax weights by
    at most 2 max_t ds in total, the output by that times max |V|.  Added to the bf16 tolerance of the block."""
    from helpers import feature_tolerance
    dh = cfg.d_attn // cfg.n_heads
    q = np.abs(rows.astype(np.float64) @ model.w_q.astype(np.float64).T)               # [n, d_attn]
    K = np.abs(user.seq_keys.astype(np.float64))
    tol = feature_tolerance("bf16", ref_attn)
    if K.shape[0] == 0:
        return tol
    vmax = np.abs(user.seq_vals.astype(np.float64)).max(axis=0)                        # [d_attn]
    extra = np.zeros_like(tol)
    for h in range(cfg.n_heads):
        sl = slice(h * dh, (h + 1) * dh)
        ds = 2.0 ** -8 * (q[:, sl] @ K[:, sl].T).max(axis=1) / np.sqrt(dh)             # [n]
        extra[:, sl] = 2.0 * ds[:, None] * vmax[None, sl]
    return tol + extra


@pytest.mark.parametrize("shape", list(PROJ_SHAPES))
@pytest.mark.parametrize("sigma", [0.1, 1.0, 4.0])
def test_projection_attention_with_16_wide_heads(R, torch, shape, sigma):
    """W_q, heads of 16, Hadamard / segment-dot / no cross: ragged candidate counts and sequence lengths (none, one
    key, around the 32-key tile and the 256-key stage), at the configurations' scale and far above it (the
    softmax then needs the true maximum instead of the norm bound)."""
    cfg = small_cfg("bf16", n_items=5000, seq_len=530, **PROJ_SHAPES[shape])
    _say(f"projection attention {shape} sigma={sigma}")
    rng = np.random.default_rng(777)
    model = wl.make_model(cfg, seed=13, bias_scale=0.2)
    table = wl.make_table_host(cfg, rng, sigma=sigma)
    table_dev = R.to_device(table, cfg.dtype)
    sampler = wl.IdSampler(cfg)
    users_ids = []
    for n, L in [(1, 530), (31, 1), (32, 0), (33, 31), (255, 32), (256, 33), (257, 255), (700, 256), (64, 257),
                 (300, 513)]:
        users_ids.append((wl.make_user(cfg, rng, sigma=sigma, seq_len=L), sampler.sample(rng, n)))
    zs, ys, drs, ctx = run_batch(R, torch, cfg, model, table_dev, users_ids, max_seq_len=530)
    assert ctx.aif_stage_kind("attention") == 1, "MFMA attention not selected"
    assert ctx.aif_stage_kind("gather") == 2, "the projection kernel indexes the item table itself"
    for r, ((u, ids), z) in enumerate(zip(users_ids, zs)):
        ref = oracle_scores(cfg, model, table, u, ids, n_threads=4)
        X = R.peek_features(ctx, cfg, r, ids.size)
        assert np.array_equal(X[:, :cfg.d_item], table[ids])
        a = X[:, cfg.d_item:cfg.d_item + cfg.d_attn]
        assert np.all(np.isfinite(a)), f"req {r}: non-finite attention"
        tol = _projected_attention_tolerance(cfg, model, table[ids], u, ref.attn)
        err = np.abs(a.astype(np.float64) - ref.attn)
        w = np.unravel_index(int(np.argmax(err - tol)), err.shape)
        assert np.all(err <= tol), f"req {r} attention: worst at {w}: got {a[w]!r} ref {ref.attn[w]!r} tol {tol[w]:.3e}"
        if cfg.d_cross:
            assert_features_close("bf16", X[:, cfg.d_item + cfg.d_attn:], ref.cross, f"req {r} cross")
        if sigma == 0.1:
            assert_logits_close("bf16", z, ref.logits, f"req {r}")
        else:
            # far above the configurations' scale the logit is a small difference of large terms: the MLP input is
            # stored in bf16, and a segment-dot entry of magnitude c (here up to ~200) carries up to 2^-9 c of
            # rounding into layer 1.  Judge relative to the larger of the logits and 5 % of the largest input.
            x_max = float(np.abs(ref.cross).max()) if cfg.d_cross else 0.0
            scale = max(1.0, float(np.abs(ref.logits).max()), 0.05 * x_max)
            assert np.abs(z - ref.logits).max() <= 2e-2 * scale, f"req {r}"
    # slices of a request give the same bits as the whole, whatever shares their waves
    u, ids = users_ids[7]
    parts, _, _, _ = run_batch(R, torch, cfg, model, table_dev, [(u, ids[:256]), (u, ids[256:300]), (u, ids[300:])],
                               max_seq_len=530)
    assert np.array_equal(np.concatenate(parts), zs[7])


@pytest.mark.parametrize("name", ["C2", "C3", "C4"])
def test_hadamard_cross_formed_in_the_mlp_chain_gives_the_same_bits(R, torch, monkeypatch, name):
    """Where the MLP is a fused chain and the cross block is u (.) e, the chain can form the products itself from the
    item block it reads anyway (AIF_CROSS_FOLD=0), the attention kernel leaving the workspace's cross block unwritten.
    Same products, same rounding: logits and scores are those of the route that writes the block
    (AIF_CROSS_MATERIALIZED=1, whose cross block is compared with the oracle's element by element), bit for bit, and
    the feature matrix the library shows is the same."""
    base = wl.CONFIGS[name]
    cfg = base.scaled(n_items=6000, seq_len=min(base.seq_len, 700))
    _say(f"{name} shape: Hadamard cross in the MLP chain vs written to the workspace")
    rng = np.random.default_rng(4242)
    model = wl.make_model(cfg, bias_scale=0.05)
    table = wl.make_table_host(cfg, rng, n_items=6000, sigma=1.0)
    sampler = wl.IdSampler(cfg, 6000)
    reqs = [(wl.make_user(cfg, rng, sigma=1.0), sampler.sample(rng, n)) for n in (1500, 1, 257, 700)]
    table_dev = R.to_device(table, "bf16")
    monkeypatch.setenv("AIF_CROSS_FOLD", "0")
    z0, y0, _, ctx0 = run_batch(R, torch, cfg, model, table_dev, reqs)
    assert ctx0.aif_mlp_layer1_width() == cfg.d_in - cfg.d_user
    X0 = [R.peek_features(ctx0, cfg, r, ids.size) for r, (_, ids) in enumerate(reqs)]
    monkeypatch.setenv("AIF_CROSS_MATERIALIZED", "1")
    z1, y1, _, ctx1 = run_batch(R, torch, cfg, model, table_dev, reqs)
    X1 = [R.peek_features(ctx1, cfg, r, ids.size) for r, (_, ids) in enumerate(reqs)]
    for r, (u, ids) in enumerate(reqs):
        assert np.array_equal(z0[r], z1[r]) and np.array_equal(y0[r], y1[r]), f"request {r}"
        assert np.array_equal(X0[r], X1[r]), f"request {r}: feature matrix"
        ref = oracle_scores(cfg, model, table, u, ids, n_threads=8)
        assert_features_close("bf16", X1[r][:, cfg.d_item + cfg.d_attn:], ref.cross, f"request {r} cross")


@pytest.mark.parametrize("name", ["C2", "C3", "C4"])
@pytest.mark.parametrize("sigma", [0.1, 1.0])
def test_hadamard_cross_folded_into_the_users_layer1_weights(R, torch, monkeypatch, name, sigma):
    """The default route where the MLP is a fused chain and the cross block is u (.) e: the block's share of layer 1,
    sum_k W1c[n, k] u_k e_k, is linear in the item vector, so the staging launch folds it into each user's layer-1
    weights, W' = W1e + u W1c, and the chain contracts over [item | attention] only.  Not the same roundings as the
    route that forms the block (W' is rounded to bf16 instead of the products): both against the oracle to the
    scale-aware bound, whole requests; users in one call get their own weights (four users, one of them as two slices
    that share a slot); the feature matrix the library shows is the same."""
    from helpers import assert_bf16_logits_tight
    base = wl.CONFIGS[name]
    cfg = base.scaled(n_items=6000, seq_len=min(base.seq_len, 700))
    _say(f"{name} shape, sigma {sigma}: Hadamard cross folded into the users' layer-1 weights")
    rng = np.random.default_rng(777)
    model = wl.make_model(cfg, bias_scale=0.05)
    table = wl.make_table_host(cfg, rng, n_items=6000, sigma=sigma)
    sampler = wl.IdSampler(cfg, 6000)
    reqs = [(wl.make_user(cfg, rng, sigma=sigma), sampler.sample(rng, n)) for n in (1500, 1, 257, 700)]
    table_dev = R.to_device(table, "bf16")
    z0, y0, _, ctx0 = run_batch(R, torch, cfg, model, table_dev, reqs)
    assert ctx0.aif_mlp_layer1_width() == cfg.d_item + cfg.d_attn, "the fold is the default on these shapes"
    X0 = [R.peek_features(ctx0, cfg, r, ids.size) for r, (_, ids) in enumerate(reqs)]
    monkeypatch.setenv("AIF_CROSS_MATERIALIZED", "1")
    z1, y1, _, ctx1 = run_batch(R, torch, cfg, model, table_dev, reqs)
    X1 = [R.peek_features(ctx1, cfg, r, ids.size) for r, (_, ids) in enumerate(reqs)]
    monkeypatch.delenv("AIF_CROSS_MATERIALIZED")
    for r, (u, ids) in enumerate(reqs):
        ref = oracle_scores(cfg, model, table, u, ids, n_threads=8)
        assert np.array_equal(X0[r], X1[r]), f"request {r}: feature matrix"
        if ids.size > 1:
            e0 = assert_bf16_logits_tight(z0[r], ref.logits, f"folded, request {r}")
            e1 = assert_bf16_logits_tight(z1[r], ref.logits, f"materialized, request {r}")
            print(f"    request {r}: rms error folded {e0[1]:.3e}, materialized {e1[1]:.3e}, rms z {e0[2]:.3e}", flush=True)
        else:
            assert_logits_close("bf16", z0[r], ref.logits, f"folded, request {r}")
    # slices of one request share its user's weights and give the whole request's bits
    u, ids = reqs[0]
    whole = R.upload_request(cfg, u, ids)
    parts = [R.slice_request(cfg, whole, lo, min(lo + 600, ids.size)) for lo in range(0, ids.size, 600)]
    other = R.upload_request(cfg, reqs[3][0], reqs[3][1])
    ctx0.aif_score_batch([p.req for p in parts[:1]] + [other.req] + [p.req for p in parts[1:]])
    torch.cuda.synchronize()
    assert ctx0.aif_last_user_slots() == 2
    assert np.array_equal(whole.logits.cpu().numpy(), z0[0]) and np.array_equal(other.logits.cpu().numpy(), z0[3])


def test_descriptors_in_the_launch_arguments_and_uploaded_give_the_same_results(R, torch):
    """Up to 16 requests travel in the staging launch's arguments and the device tables (block -> request, slot ->
    request, attention groups, top-k lists) are written by that launch; more are uploaded from the pinned slot.
    The same 16 requests -- users that repeat (shared slots), an empty request, one whose K/V exceed LDS beside
    resident ones -- scored as a batch of 16 and inside a batch of 17: same logits, same selection; each request
    against the oracle."""
    cfg = small_cfg("bf16", n_items=5000, seq_len=1100, **MFMA_SHAPES["c3_like"])
    _say("16 requests in the arguments vs 17 uploaded")
    rng = np.random.default_rng(1617)
    model = wl.make_model(cfg, seed=21, bias_scale=0.1)
    table = wl.make_table_host(cfg, rng)
    table_dev = R.to_device(table, cfg.dtype)
    sampler = wl.IdSampler(cfg)
    users = [wl.make_user(cfg, rng, seq_len=L) for L in (200, 64, 1100, 333, 1)]
    sizes = [300, 1, 257, 0, 700, 33, 256, 100, 512, 31, 32, 1000, 7, 64, 129, 400]
    dm = R.DeviceModel(cfg, model)
    ctx = R.make_context(cfg, dm, table_dev, max_users=17, max_candidates=1024, max_seq_len=1100)
    du = [R.upload_request(cfg, u, sampler.sample(rng, 1)) for u in users]           # the users' tensors on the device, once
    def request(u, ids):                                    # a request that brings user u's tensors (same pointers: same slot)
        d = R.upload_request(cfg, users[u], ids)
        q, b = d.req, du[u].req
        d.req = type(q)(b.user_vec, b.seq_keys, b.seq_vals, q.cand_ids, q.logits_out, q.scores_out, b.cross_vecs, b.seq_len)
        return d
    ids = [sampler.sample(rng, n) for n in sizes]
    who = [i % len(users) for i in range(16)]
    k = 20
    out = {}
    for n_req in (16, 17):
        ds = [request(who[i], ids[i]) for i in range(16)]
        extra = [request(2, sampler.sample(rng, 50))] if n_req == 17 else []
        idx = torch.full((n_req, k), -7, dtype=torch.int32, device="cuda")
        val = torch.zeros((n_req, k), dtype=torch.float32, device="cuda")
        ctx.aif_score_topk([d.req for d in ds + extra], k, idx, val)
        torch.cuda.synchronize()
        assert ctx.aif_last_user_slots() == len(users)
        out[n_req] = ([d.logits.cpu().numpy().copy() for d in ds], idx.cpu().numpy()[:16].copy(), val.cpu().numpy()[:16].copy())
    for i in range(16):
        assert np.array_equal(out[16][0][i], out[17][0][i]), f"request {i}: logits"
        assert np.array_equal(out[16][1][i], out[17][1][i]) and np.array_equal(out[16][2][i], out[17][2][i]), f"request {i}: top-k"
        if sizes[i]:
            ref = oracle_scores(cfg, model, table, users[who[i]], ids[i], n_threads=4)
            assert_logits_close("bf16", out[16][0][i], ref.logits, f"request {i}")
            oi, ov = oracle.topk(out[16][0][i].astype(np.float64), k)           # the selection alone, on the GPU's own logits
            assert np.array_equal(out[16][1][i], oi), f"request {i}: selection"
        else:
            assert np.all(out[16][1][i] == -1) and np.all(np.isneginf(out[16][2][i]))


def test_cross_fold_with_the_shape_agnostic_attention_kernel(R, torch):
    """A bf16 model whose attention has no matrix-core kernel (four heads of 16 without W_q) but whose head is a
    fused chain: the cross block is still folded into the users' layer-1 weights -- by a launch of its own, the
    staging not being the fused one -- and the shape-agnostic attention kernel leaves the block unwritten."""
    from helpers import assert_bf16_logits_tight
    cfg = small_cfg("bf16", n_items=4000, seq_len=150, d_item=64, d_user=64, d_attn=64, n_heads=4, mlp_dims=(256, 512, 256, 1))
    _say("cross fold beside the generic attention kernel")
    rng = np.random.default_rng(515)
    model = wl.make_model(cfg, seed=3, bias_scale=0.1)
    table = wl.make_table_host(cfg, rng)
    sampler = wl.IdSampler(cfg)
    reqs = [(wl.make_user(cfg, rng, seq_len=L), sampler.sample(rng, n)) for n, L in ((700, 150), (33, 7), (256, 64))]
    zs, _, _, ctx = run_batch(R, torch, cfg, model, R.to_device(table, cfg.dtype), reqs, max_seq_len=150)
    assert ctx.aif_stage_kind("attention") == 0 and ctx.aif_stage_kind("mlp") == 1
    assert ctx.aif_mlp_layer1_width() == cfg.d_item + cfg.d_attn
    for i, (u, ids) in enumerate(reqs):
        ref = oracle_scores(cfg, model, table, u, ids, n_threads=4)
        assert_logits_close("bf16", zs[i], ref.logits, f"request {i}")
        assert_bf16_logits_tight(zs[i], ref.logits, f"request {i}")
        X = R.peek_features(ctx, cfg, i, ids.size)
        assert_features_close("bf16", X[:, cfg.d_item + cfg.d_attn:], ref.cross, f"request {i}: the cross block the library shows")


def test_widest_head_as_one_fused_chain(R, torch, monkeypatch):
    """C5's head (448 -> 1024 -> 512 -> 256 -> 1 after the user fold) runs as ONE launch with a candidate's activations
    in registers.  Enough candidates (more 128-candidate tiles than compute units) that blocks take two tiles each as
    well as one; non-zero biases; against the oracle to the scale-aware bound -- with the segment-dot cross block
    folded into the users' layer-1 weights (the default: layer 1 over 384 columns) and with the block written by the
    attention kernel (AIF_CROSS_FOLD=0) --, the latter against the one-launch-per-layer route (AIF_MLP_LAYERED=1: same
    products, hidden activations through HBM) within two roundings, and sliced vs whole bit for bit."""
    from helpers import assert_bf16_logits_tight
    cfg = wl.CONFIGS["C5"].scaled(n_items=20000, seq_len=64)
    _say("C5 head, fused chain: 3 requests x 12000 candidates")
    rng = np.random.default_rng(97)
    model = wl.make_model(cfg, seed=5, bias_scale=0.02)
    table = wl.make_table_host(cfg, rng, n_items=20000)
    table_dev = R.to_device(table, "bf16")
    sampler = wl.IdSampler(cfg, 20000)
    reqs = [(wl.make_user(cfg, rng), sampler.sample(rng, n)) for n in (12000, 11999, 12001)]
    zs, _, _, ctx = run_batch(R, torch, cfg, model, table_dev, reqs)
    assert ctx.aif_stage_kind("mlp") == 1 and ctx.aif_last_error() == ""
    assert ctx.aif_mlp_layer1_width() == cfg.d_item + cfg.d_attn
    X_fold = R.peek_features(ctx, cfg, 1, 500)
    refs = [oracle_scores(cfg, model, table, u, ids, n_threads=16) for u, ids in reqs]
    for i, (u, ids) in enumerate(reqs):
        assert_logits_close("bf16", zs[i], refs[i].logits, f"request {i}")
        e_max, e_rms, z_rms = assert_bf16_logits_tight(zs[i], refs[i].logits, f"request {i}")
        print(f"[case] folded, request {i}: max |dz| {e_max:.3e}, rms dz {e_rms:.3e}, rms z {z_rms:.3e}", flush=True)
    u, ids = reqs[2]
    parts, _, _, _ = run_batch(R, torch, cfg, model, table_dev, [(u, ids[:1000]), (u, ids[1000:1300]), (u, ids[1300:])])
    assert np.array_equal(np.concatenate(parts), zs[2])
    monkeypatch.setenv("AIF_CROSS_FOLD", "0")
    zs, _, _, ctx = run_batch(R, torch, cfg, model, table_dev, reqs)
    assert ctx.aif_stage_kind("mlp") == 1 and ctx.aif_mlp_layer1_width() == cfg.d_in - cfg.d_user
    assert_features_close("bf16", X_fold[:, cfg.d_item + cfg.d_attn:], R.peek_features(ctx, cfg, 1, 500)[:, cfg.d_item + cfg.d_attn:],
                          "the cross block the library shows on the two routes")
    for i in range(3):
        e_max, e_rms, z_rms = assert_bf16_logits_tight(zs[i], refs[i].logits, f"request {i}, cross block written")
        print(f"[case] written, request {i}: max |dz| {e_max:.3e}, rms dz {e_rms:.3e}, rms z {z_rms:.3e}", flush=True)
    monkeypatch.setenv("AIF_MLP_LAYERED", "1")
    zl, _, _, ctx_l = run_batch(R, torch, cfg, model, table_dev, reqs)
    assert ctx_l.aif_stage_kind("mlp") == 1
    for i in range(3):
        d = np.abs(zl[i] - zs[i]).max()
        assert d <= 2.0 ** -6 * np.sqrt(np.mean(np.square(zs[i]))) + 1e-6, (i, d)


# ---------------------------------------------------------------------------
# nearline maintenance of the item table (Sec. 3.4): incremental and full updates
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["C1", "C2"])
def test_incremental_table_update_is_exact_and_ordered_with_the_stream(R, torch, name):
    """aif_update_rows against the oracle's update, bit for bit on the whole table; a scoring call enqueued before
    the update reads the old rows and one enqueued after it the new ones, with no host synchronisation between."""
    cfg = wl.CONFIGS[name].scaled(n_items=5000)
    _say(f"{name} incremental update of 700 (+3 bad) of 5000 rows")
    rng = np.random.default_rng(41)
    model = wl.make_model(cfg)
    table = wl.make_table_host(cfg, rng, n_items=5000)
    u = wl.make_user(cfg, rng)
    ids = wl.IdSampler(cfg, 5000).sample(rng, 600)
    others = rng.permutation(np.setdiff1d(np.arange(5000, dtype=np.int32), ids))[:400]
    upd_ids = np.concatenate([ids[:300], others]).astype(np.int32)      # distinct; half of the scored candidates change
    upd_ids = np.concatenate([upd_ids, np.array([-1, 5000, 2 ** 30], np.int32)])
    upd_rows = wl.round_storage(rng.standard_normal((703, cfg.d_item)).astype(np.float32) * 0.1, cfg.dtype)
    new_table, skipped = oracle.update_rows(table, upd_ids, upd_rows)
    assert skipped == 3

    table_dev = R.to_device(table, cfg.dtype)
    dm = R.DeviceModel(cfg, model)
    ctx = R.make_context(cfg, dm, table_dev, max_users=1, max_candidates=600, max_seq_len=cfg.seq_len)
    before, after = R.upload_request(cfg, u, ids), R.upload_request(cfg, u, ids)
    di = torch.from_numpy(upd_ids).to("cuda:0")
    dr = R.to_device(upd_rows, cfg.dtype)
    ctx.aif_score_batch([before.req])
    ctx.aif_update_rows(di, dr)
    ctx.aif_score_batch([after.req])
    torch.cuda.synchronize()
    assert ctx.aif_poll_device_errors() == 3
    assert np.array_equal(R.from_device_f32(table_dev), new_table), "table after the update"
    z0, z1 = before.logits.cpu().numpy(), after.logits.cpu().numpy()
    assert_logits_close(cfg.dtype, z0, oracle_scores(cfg, model, table, u, ids).logits, "before the update")
    assert_logits_close(cfg.dtype, z1, oracle_scores(cfg, model, new_table, u, ids).logits, "after the update")
    assert np.array_equal(z0[300:], z1[300:]) and not np.array_equal(z0[:300], z1[:300])
    # empty update and host-side errors
    ctx.aif_update_rows(di[:0], dr[:0])
    from paper_2511_12934_amd import binding as B
    with pytest.raises(B.AifError):
        ctx.aif_update_rows(di, None)


def test_full_table_update_swaps_the_table_for_later_calls(R, torch):
    cfg = wl.CONFIGS["C2"].scaled(n_items=3000)
    _say("C2 full update: swap to a table of another size")
    rng = np.random.default_rng(43)
    model = wl.make_model(cfg)
    t0 = wl.make_table_host(cfg, rng, n_items=3000)
    t1 = wl.make_table_host(cfg, rng, n_items=4000)
    u = wl.make_user(cfg, rng)
    ids = np.concatenate([wl.IdSampler(cfg, 3000).sample(rng, 400), np.array([3500], np.int32)])
    d0, d1 = R.to_device(t0, "bf16"), R.to_device(t1, "bf16")
    ctx = R.make_context(cfg, R.DeviceModel(cfg, model), d0, max_users=1, max_candidates=401, max_seq_len=cfg.seq_len)
    a, b = R.upload_request(cfg, u, ids), R.upload_request(cfg, u, ids)
    ctx.aif_score_batch([a.req])
    ctx.aif_swap_table(d1)
    ctx.aif_score_batch([b.req])
    torch.cuda.synchronize()
    za, zb = a.logits.cpu().numpy(), b.logits.cpu().numpy()
    assert np.isnan(za[400]) and ctx.aif_poll_device_errors() == 1      # row 3500 exists in the new table only
    assert_logits_close("bf16", za[:400], oracle_scores(cfg, model, t0, u, ids[:400]).logits, "old table")
    assert_logits_close("bf16", zb, oracle_scores(cfg, model, t1, u, ids).logits, "new table")


def test_large_scores_do_not_overflow(R, torch):
    """|score| far beyond the fp32 exp range: softmax must subtract its maximum."""
    cfg = small_cfg("f32", d_item=32, d_user=32, d_attn=32, seq_len=33, mlp_dims=(128, 16, 1))
    _say("large scores fp32")
    rng = np.random.default_rng(5)
    model = wl.make_model(cfg, seed=3)
    table = wl.make_table_host(cfg, rng, sigma=30.0)
    u = wl.make_user(cfg, rng, sigma=30.0)
    ids = wl.IdSampler(cfg).sample(rng, 64)
    (z,), _, drs, ctx = run_batch(R, torch, cfg, model, R.to_device(table, "f32"), [(u, ids)])
    ref = oracle_scores(cfg, model, table, u, ids)
    X = R.peek_features(ctx, cfg, 0, ids.size)
    a = X[:, cfg.d_item:cfg.d_item + cfg.d_attn]
    assert np.all(np.isfinite(a))
    # scores are ~ +-5000: fp32 rounding of the score itself (ulp ~ 5e-4) moves
    # the weights, so compare with a tolerance on the dominant-key structure
    assert np.abs(a - ref.attn).max() <= 2e-2 * np.abs(ref.attn).max()


# ---------------------------------------------------------------------------
# top-k alone: bit-exact against the oracle's full stable sort
# ---------------------------------------------------------------------------
def _topk_cases(rng):
    n = 10_000
    z = rng.standard_normal(n).astype(np.float32) * 0.05
    cases = {"random": z.copy(), "equal": np.full(n, 0.25, np.float32),
             "sorted": np.sort(z)[::-1].copy(), "reversed": np.sort(z),
             "dups": rng.integers(0, 7, n).astype(np.float32),
             "narrow": (0.0123 + rng.integers(0, 50, n) * 1e-9).astype(np.float32)}
    s = z.copy()
    s[[3, 77, 9000]] = np.inf
    s[[5, 100, 200]] = -np.inf
    s[[0, 9, 128, 9999]] = np.nan
    s[[11, 12]] = [0.0, -0.0]
    cases["special"] = s
    cases["all_nan"] = np.full(300, np.nan, np.float32)
    cases["tiny"] = np.array([1.0, 2.0, 2.0], np.float32)
    cases["big"] = rng.standard_normal(20_000).astype(np.float32)
    # more candidates than the kernel keeps in registers (the tail is re-read from memory in every pass), with ties
    cases["bigger"] = np.round(rng.standard_normal(23_456).astype(np.float32), 2)
    cases["bigger_dups"] = rng.integers(0, 3, 30_000).astype(np.float32)
    # aimed at the value-bin shortcut: ties straddling the cut inside one bin, an outlier that squeezes every other
    # logit into one bin, fewer candidates than k, only two distinct values, huge range
    cases["coarse"] = np.round(z, 3)
    o = z.copy()
    o[4321] = 1e6
    cases["outlier"] = o
    cases["few"] = rng.standard_normal(700).astype(np.float32)
    cases["two_values"] = np.where(rng.random(n) < 0.01, 1.0, -1.0).astype(np.float32)
    h = z.copy()
    h[[1, 2]] = [3e38, -3e38]
    cases["huge_range"] = h
    # lengths between the register sizes the kernel is built for, with the special values among them
    t = rng.standard_normal(2_000).astype(np.float32)
    t[[0, 1999]] = np.inf
    t[[7, 1024]] = -np.inf
    t[[3, 1023, 1025]] = np.nan
    cases["two_thousand"] = t
    cases["five_thousand"] = np.round(rng.standard_normal(5_000).astype(np.float32), 1)
    cases["one_past"] = rng.standard_normal(10_241).astype(np.float32)
    return cases


@pytest.mark.parametrize("k", [1, 100, 200, 1024, 4096])
def test_topk_equals_full_stable_sort(R, torch, k):
    from paper_2511_12934_amd import binding as B
    _say(f"topk k={k}")
    rng = np.random.default_rng(99)
    cases = _topk_cases(rng)
    cfg = small_cfg("f32")
    model = wl.make_model(cfg)
    table_dev = R.to_device(wl.make_table_host(cfg, rng), "f32")
    ctx = R.make_context(cfg, R.DeviceModel(cfg, model), table_dev, max_users=len(cases) + 1, max_candidates=64)
    names = list(cases)
    dev = [torch.from_numpy(cases[nm]).cuda() for nm in names]
    dev.append(torch.empty(0, dtype=torch.float32, device="cuda"))        # an empty request
    idx = torch.full((len(dev), k), -7, dtype=torch.int32, device="cuda")
    val = torch.full((len(dev), k), -7.0, dtype=torch.float32, device="cuda")
    ctx.aif_topk(dev, k, idx, val)
    torch.cuda.synchronize()
    idx, val = idx.cpu().numpy(), val.cpu().numpy()
    for r, nm in enumerate(names):
        oi, ov = oracle.topk(cases[nm].astype(np.float64), k)
        assert np.array_equal(idx[r], oi), (nm, k)
        assert np.array_equal(val[r].astype(np.float64), ov, equal_nan=True), (nm, k)
    assert np.all(idx[-1] == -1) and np.all(np.isneginf(val[-1]))
    # every list alone: the kernel is then the one built for that list's length (together, the longest decides)
    i1 = torch.empty((1, k), dtype=torch.int32, device="cuda")
    v1 = torch.empty((1, k), dtype=torch.float32, device="cuda")
    for r, nm in enumerate(names):
        i1.fill_(-7)
        v1.fill_(-7.0)
        ctx.aif_topk([dev[r]], k, i1, v1)
        torch.cuda.synchronize()
        assert np.array_equal(i1.cpu().numpy()[0], idx[r]), (nm, k)
        assert np.array_equal(v1.cpu().numpy()[0], val[r], equal_nan=True), (nm, k)
    for kk in (2, 3, 4):                                                   # k around n for the 3-element case
        i2 = torch.empty((1, kk), dtype=torch.int32, device="cuda")
        v2 = torch.empty((1, kk), dtype=torch.float32, device="cuda")
        ctx.aif_topk([dev[names.index("tiny")]], kk, i2, v2)
        torch.cuda.synchronize()
        oi, ov = oracle.topk(cases["tiny"].astype(np.float64), kk)
        assert np.array_equal(i2.cpu().numpy()[0], oi)
        assert np.array_equal(v2.cpu().numpy()[0].astype(np.float64), ov)


def test_score_topk_is_score_batch_followed_by_topk(R, torch):
    """The one-call form leaves exactly what the two calls leave: logits and selections, bit for bit, for ragged
    requests including one shorter than k and an empty one."""
    cfg = wl.CONFIGS["C2"].scaled(n_items=4000)
    _say("aif_score_topk vs aif_score_batch + aif_topk")
    rng = np.random.default_rng(47)
    model = wl.make_model(cfg)
    table_dev = R.to_device(wl.make_table_host(cfg, rng, n_items=4000), "bf16")
    sampler = wl.IdSampler(cfg, 4000)
    sizes = (1500, 37, 0, 700)
    users = [wl.make_user(cfg, rng) for _ in sizes]
    k = 200
    dm = R.DeviceModel(cfg, model)
    outs = []
    for fused in (False, True):
        ctx = R.make_context(cfg, dm, table_dev, max_users=len(sizes), max_candidates=max(sizes), max_seq_len=cfg.seq_len)
        drs = [R.upload_request(cfg, u, sampler.sample(np.random.default_rng(100 + i), n)) for i, (u, n) in enumerate(zip(users, sizes))]
        idx = torch.full((len(sizes), k), -7, dtype=torch.int32, device="cuda")
        val = torch.full((len(sizes), k), -7.0, dtype=torch.float32, device="cuda")
        if fused:
            ctx.aif_score_topk([d.req for d in drs], k, idx, val)
        else:
            ctx.aif_score_batch([d.req for d in drs])
            ctx.aif_topk([d.logits for d in drs], k, idx, val)
        torch.cuda.synchronize()
        outs.append(([d.logits.cpu().numpy() for d in drs], idx.cpu().numpy(), val.cpu().numpy()))
    for a, b in zip(outs[0][0], outs[1][0]):
        assert np.array_equal(a, b)
    assert np.array_equal(outs[0][1], outs[1][1]) and np.array_equal(outs[0][2], outs[1][2])
    for r, n in enumerate(sizes):
        oi, _ = oracle.topk(outs[1][0][r].astype(np.float64), k)
        assert np.array_equal(outs[1][1][r], oi)


# ---------------------------------------------------------------------------
# duplicates, bad ids, host-side errors
# ---------------------------------------------------------------------------
def test_duplicate_candidates_and_bad_ids(R, torch):
    cfg = small_cfg("f32")
    _say("duplicates and out-of-range ids")
    rng = np.random.default_rng(8)
    model = wl.make_model(cfg, seed=5, bias_scale=0.2)
    table = wl.make_table_host(cfg, rng, sigma=1.0)
    u = wl.make_user(cfg, rng, sigma=1.0)
    ids = np.array([7, 3, 7, 299, 3, 7, 0], np.int32)
    (z,), _, drs, ctx = run_batch(R, torch, cfg, model, R.to_device(table, "f32"), [(u, ids)])
    assert z[0] == z[2] == z[5] and z[1] == z[4]
    ref = oracle_scores(cfg, model, table, u, ids)
    assert_logits_close("f32", z, ref.logits)
    idx = torch.empty(7, dtype=torch.int32, device="cuda")
    val = torch.empty(7, dtype=torch.float32, device="cuda")
    ctx.aif_topk([drs[0].logits], 7, idx, val)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), oracle.topk(z.astype(np.float64), 7)[0])
    assert ctx.aif_poll_device_errors() == 0

    bad = np.array([5, -1, 300, 2, 2_000_000_000], np.int32)
    d = R.upload_request(cfg, u, bad)
    ctx.aif_score_request(d.req)
    torch.cuda.synchronize()
    zb = d.logits.cpu().numpy()
    yb = d.scores.cpu().numpy()
    assert np.isnan(zb[[1, 2, 4]]).all() and np.isnan(yb[[1, 2, 4]]).all()
    good = oracle_scores(cfg, model, table, u, bad[[0, 3]])
    assert_logits_close("f32", zb[[0, 3]], good.logits)
    assert ctx.aif_poll_device_errors() == 3
    assert ctx.aif_poll_device_errors() == 0


@pytest.mark.parametrize("shape", ["c3_like", "c4_like"])
def test_bad_ids_on_the_fragment_order_workspace(R, torch, shape):
    """The MFMA path (gather through LDS into the fragment-order workspace): out-of-range ids give NaN logits and
    are counted once each, their neighbours are untouched; ragged request sizes around the 32-row tile."""
    cfg = small_cfg("bf16", n_items=3000, seq_len=40, **MFMA_SHAPES[shape])
    _say(f"bad ids, fragment-order workspace, {shape}")
    rng = np.random.default_rng(31)
    model = wl.make_model(cfg, seed=3, bias_scale=0.1)
    table = wl.make_table_host(cfg, rng)
    u = wl.make_user(cfg, rng)
    ids = rng.integers(0, 3000, 300).astype(np.int32)
    bad_pos = np.array([0, 31, 32, 255, 256, 299])
    ids_bad = ids.copy()
    ids_bad[bad_pos] = [-1, 3000, 2_000_000_000, -5, 3001, -2_000_000_000]
    (z_bad,), _, _, ctx = run_batch(R, torch, cfg, model, R.to_device(table, "bf16"), [(u, ids_bad)])
    assert ctx.aif_stage_kind("attention") == 1 and ctx.aif_stage_kind("mlp") == 1
    assert ctx.aif_poll_device_errors() == bad_pos.size
    assert np.isnan(z_bad[bad_pos]).all()
    good = np.setdiff1d(np.arange(ids.size), bad_pos)
    ref = oracle_scores(cfg, model, table, u, ids[good], n_threads=4)
    assert_logits_close("bf16", z_bad[good], ref.logits, "neighbours of bad ids")
    (z_ok,), _, _, ctx2 = run_batch(R, torch, cfg, model, R.to_device(table, "bf16"), [(u, ids)])
    assert np.array_equal(z_ok[good], z_bad[good])
    assert ctx2.aif_poll_device_errors() == 0


@pytest.mark.parametrize("shape", ["c5_like", "hadamard_4_heads", "segdot_6_vectors_2_heads"])
def test_bad_ids_when_the_projection_kernel_indexes_the_table(R, torch, shape):
    """W_q models: the attention kernel reads the table rows itself.  Out-of-range ids give NaN logits and are
    counted once each, their neighbours keep their bits; with the layered MLP, the MLP chain and the
    shape-agnostic MLP behind it."""
    cfg = small_cfg("bf16", n_items=3000, seq_len=40, **PROJ_SHAPES[shape])
    _say(f"bad ids, projection attention, {shape}")
    rng = np.random.default_rng(33)
    model = wl.make_model(cfg, seed=5, bias_scale=0.1)
    table = wl.make_table_host(cfg, rng)
    u = wl.make_user(cfg, rng)
    ids = rng.integers(0, 3000, 300).astype(np.int32)
    bad_pos = np.array([0, 31, 32, 255, 256, 299])
    ids_bad = ids.copy()
    ids_bad[bad_pos] = [-1, 3000, 2_000_000_000, -5, 3001, -2_000_000_000]
    (z_bad,), _, _, ctx = run_batch(R, torch, cfg, model, R.to_device(table, "bf16"), [(u, ids_bad)])
    assert ctx.aif_stage_kind("attention") == 1 and ctx.aif_stage_kind("gather") == 2
    assert ctx.aif_poll_device_errors() == bad_pos.size
    assert np.isnan(z_bad[bad_pos]).all()
    good = np.setdiff1d(np.arange(ids.size), bad_pos)
    ref = oracle_scores(cfg, model, table, u, ids[good], n_threads=4)
    assert_logits_close("bf16", z_bad[good], ref.logits, "neighbours of bad ids")
    (z_ok,), _, _, ctx2 = run_batch(R, torch, cfg, model, R.to_device(table, "bf16"), [(u, ids)])
    assert np.array_equal(z_ok[good], z_bad[good])
    assert ctx2.aif_poll_device_errors() == 0


@pytest.mark.parametrize("shape", ["c3", "b3", "c5_like"])
def test_gather_inside_the_attention_kernel_or_on_its_own_gives_the_same_bits(R, torch, monkeypatch, shape):
    """The attention kernels that index the item table themselves against the same kernels behind a separate gather
    (AIF_SEPARATE_GATHER=1): workspace and logits bit for bit, ragged requests."""
    if shape == "c3":
        cfg = wl.CONFIGS["C3"].scaled(n_items=3000)
    elif shape == "b3":
        cfg = wl.CONFIGS["B3"].scaled(n_items=3000)
    else:
        cfg = small_cfg("bf16", n_items=3000, seq_len=300, **PROJ_SHAPES["c5_like"])
    _say(f"gather routes, {shape}")
    rng = np.random.default_rng(41)
    model = wl.make_model(cfg, bias_scale=0.05)
    table = wl.make_table_host(cfg, rng, n_items=3000)
    sampler = wl.IdSampler(cfg, 3000)
    reqs = [(wl.make_user(cfg, rng), sampler.sample(rng, n)) for n in (333, 1, 600, 32)]
    z0, _, _, ctx0 = run_batch(R, torch, cfg, model, R.to_device(table, "bf16"), reqs)
    assert ctx0.aif_stage_kind("gather") == 2
    X0 = [R.peek_features(ctx0, cfg, i, ids.size) for i, (_, ids) in enumerate(reqs)]
    monkeypatch.setenv("AIF_SEPARATE_GATHER", "1")
    z1, _, _, ctx1 = run_batch(R, torch, cfg, model, R.to_device(table, "bf16"), reqs)
    assert ctx1.aif_stage_kind("gather") != 2 and ctx1.aif_stage_kind("attention") == 1
    for i, (_, ids) in enumerate(reqs):
        assert np.array_equal(X0[i], R.peek_features(ctx1, cfg, i, ids.size)), f"workspace, request {i}"
        assert np.array_equal(z0[i], z1[i]), f"logits, request {i}"


def test_profiling_times_the_selected_stages_only(R, torch):
    """aif_profile_begin brackets every stage of a scoring call with events, aif_profile_begin_stages only the
    stages named; the results are the same either way.  The batch's K/V fit one compute unit's LDS and there is
    no W_q, so the attention kernel indexes the item table itself and the library says so."""
    cfg = small_cfg("bf16", n_items=5000, seq_len=40, **MFMA_SHAPES["c3_like"])
    _say("profiling")
    rng = np.random.default_rng(5)
    model = wl.make_model(cfg, seed=3)
    table = wl.make_table_host(cfg, rng)
    table_dev = R.to_device(table, cfg.dtype)
    sampler = wl.IdSampler(cfg)
    users_ids = [(wl.make_user(cfg, rng, seq_len=40), sampler.sample(rng, 300)) for _ in range(3)]
    zs, _, drs, ctx = run_batch(R, torch, cfg, model, table_dev, users_ids, max_seq_len=40)
    assert ctx.aif_stage_kind("gather") == 2 and ctx.aif_stage_kind("attention") == 1
    ctx.aif_profile_begin(4)
    for _ in range(2):
        ctx.aif_score_batch([d.req for d in drs])
    torch.cuda.synchronize()
    prof = ctx.aif_profile_end()
    for st in ("gather", "user_fold", "attention", "mlp"):
        assert prof[st][1] == 2 and prof[st][0] >= 0.0, (st, prof[st])
    assert prof["topk"][1] == 0
    ctx.aif_profile_begin_stages(4, ["mlp"])
    ctx.aif_score_batch([d.req for d in drs])
    torch.cuda.synchronize()
    prof = ctx.aif_profile_end()
    assert prof["mlp"][1] == 1 and prof["mlp"][0] > 0.0
    assert all(prof[st] == (0.0, 0) for st in ("gather", "user_fold", "attention", "topk")), prof
    for d, z in zip(drs, zs):
        assert np.array_equal(d.logits.cpu().numpy(), z)
    ctx.aif_profile_begin_sampled(4, ["mlp"], 2)                 # every second call: calls 0 and 2 of 3
    for _ in range(3):
        ctx.aif_score_batch([d.req for d in drs])
    torch.cuda.synchronize()
    prof = ctx.aif_profile_end()
    assert prof["mlp"][1] == 2 and prof["mlp"][0] > 0.0, prof
    with pytest.raises(Exception):
        ctx.aif_profile_begin_stages(4, [])
    with pytest.raises(Exception):
        ctx.aif_profile_begin_sampled(4, ["mlp"], 0)


def test_host_side_errors_enqueue_nothing(R, torch):
    from paper_2511_12934_amd import binding as B
    cfg = small_cfg("f32")
    _say("host-side validation")
    rng = np.random.default_rng(8)
    model = wl.make_model(cfg)
    table = wl.make_table_host(cfg, rng)
    table_dev = R.to_device(table, "f32")
    dm = R.DeviceModel(cfg, model)
    ctx = R.make_context(cfg, dm, table_dev, max_users=2, max_candidates=50, max_seq_len=9)
    u = wl.make_user(cfg, rng)
    ok = R.upload_request(cfg, u, np.arange(10, dtype=np.int32))
    too_many = R.upload_request(cfg, u, np.arange(51, dtype=np.int32) % 300)
    long_seq = R.upload_request(cfg, wl.make_user(cfg, rng, seq_len=10), np.arange(4, dtype=np.int32))
    for reqs, status in (([too_many.req], B.AIF_ERANGE), ([long_seq.req], B.AIF_ERANGE),
                         ([ok.req, ok.req, ok.req], B.AIF_ERANGE)):
        with pytest.raises(B.AifError) as ei:
            ctx.aif_score_batch(reqs)
        assert ei.value.status == status
    torch.cuda.synchronize()
    assert np.isnan(too_many.logits.cpu().numpy()).all()           # nothing was written
    idx = torch.empty(4, dtype=torch.int32, device="cuda")
    val = torch.empty(4, dtype=torch.float32, device="cuda")
    for k, status in ((0, B.AIF_EINVAL), (4097, B.AIF_ERANGE)):
        with pytest.raises(B.AifError) as ei:
            ctx.aif_topk([ok.logits], k, idx, val)
        assert ei.value.status == status
    # bad configurations are refused by aif_score_init
    with pytest.raises(B.AifError) as ei:
        R.make_context(cfg.scaled(mlp_dims=(57, 24, 12, 1)), dm, table_dev)
    assert ei.value.status == B.AIF_ESHAPE
    with pytest.raises(B.AifError) as ei:
        R.make_context(cfg.scaled(n_heads=3), dm, table_dev)
    assert ei.value.status == B.AIF_ESHAPE
    ctx.aif_score_batch([])                                           # empty batch is a no-op
    ctx.aif_score_request(ok.req)
    torch.cuda.synchronize()
    assert np.isfinite(ok.logits.cpu().numpy()).all()
