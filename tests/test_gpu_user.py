"""GPU parity of the user-side asynchronous network (Sec. 3.1, Eq. 1-3; include/aif_user.h) against the CPU
oracle on the same seeded inputs, element by element, and of the chain user network -> real-time scoring."""
import numpy as np
import pytest

import oracle
from paper_2511_12934_amd import workloads as wl

from helpers import assert_features_close, assert_logits_close

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


def oracle_user(model, user):
    return oracle.user_network(profile=user.profile, seq=user.seq, w_profile=model.w_profile, w_seq=model.w_seq,
                               w_ffn=model.w_ffn, b_ffn=model.b_ffn)


def run_users(R, torch, cfg, model, users, ctx=None):
    if ctx is None:
        ctx = R.make_user_context(cfg, model, max_users=max(len(users), 1),
                                  max_seq_len=max([u.seq.shape[0] for u in users] + [1]))
    dev = [R.upload_raw_user(cfg, u) for u in users]
    ctx.aif_user_precompute([d.req for d in dev])
    torch.cuda.synchronize()
    return [(R.from_device_f32(d.user_vec), R.from_device_f32(d.seq_out)[:u.seq.shape[0]]) for d, u in zip(dev, users)], dev, ctx


def check_user(dtype, got, ref, d, what):
    (uv, sh), (ruv, rsh) = got, ref
    assert np.all(np.isfinite(uv)) and np.all(np.isfinite(sh)), what
    if rsh.size:
        # Eq. 1: fp32 accumulation, one rounding to the storage type
        tol = (2.0 ** -8 if dtype == "bf16" else 2e-6) * np.abs(rsh) + 2e-6 * np.abs(rsh).max() + 1e-30
        assert np.all(np.abs(sh - rsh) <= tol), f"{what}: projected sequence"
    assert_features_close(dtype, uv[d:], ruv[d:], f"{what}: profile attention (Eq. 3)")
    assert_features_close(dtype, uv[:d], ruv[:d], f"{what}: pooled self-attention (Eq. 2)")


def test_u1_fp32_whole_configuration(R, torch):
    cfg = wl.USER_CONFIGS["U1"]
    _say("U1 fp32")
    model = wl.make_user_net_model(cfg, bias_scale=0.2)
    users = wl.make_raw_users(cfg, 3, sigma=1.0)
    got, _, ctx = run_users(R, torch, cfg, model, users)
    assert ctx.aif_user_attention_kind() == 0
    for i, u in enumerate(users):
        check_user("f32", got[i], oracle_user(model, u), cfg.d, f"U1 user {i}")


@pytest.mark.parametrize("dtype,d_raw,d,lens", [("f32", 12, 8, (0, 1, 7, 65)), ("bf16", 24, 16, (3, 33, 130)),
                                                ("bf16", 40, 72, (50,)), ("f32", 256, 128, (40,)),
                                                ("bf16", 64, 128, (70, 33, 128))])
def test_shape_agnostic_kernels_on_odd_shapes(R, torch, dtype, d_raw, d, lens):
    cfg = wl.UserNetConfig("T", 9, dtype, len(lens), max(lens), d_raw, d)
    _say(f"user net generic {dtype} d_raw={d_raw} d={d} lens={lens}")
    model = wl.make_user_net_model(cfg, bias_scale=0.3)
    rng = np.random.default_rng(5)
    users = [wl.make_raw_user(cfg, rng, sigma=1.0, seq_len=L) for L in lens]
    got, _, ctx = run_users(R, torch, cfg, model, users)
    assert ctx.aif_user_attention_kind() == 0
    for i, u in enumerate(users):
        check_user(dtype, got[i], oracle_user(model, u), d, f"generic user {i} (L={lens[i]})")


@pytest.mark.parametrize("d,lens,sigma", [(64, (500, 333, 31, 1, 0, 256, 255), 0.1), (64, (500, 97), 1.0),
                                          (32, (200, 64, 5), 0.5), (64, (1000, 700), 0.1)])
def test_mfma_attention_path(R, torch, d, lens, sigma):
    """bf16, d = 64 or 32: both attentions run on the MFMA target-attention kernels (resident K/V for short
    sequences, the streaming kernel for L = 1000), ragged lengths in one call."""
    cfg = wl.UserNetConfig("T", 10, "bf16", len(lens), max(lens), 128, d)
    _say(f"user net MFMA d={d} lens={lens} sigma={sigma}")
    model = wl.make_user_net_model(cfg, bias_scale=0.05)
    rng = np.random.default_rng(6)
    users = [wl.make_raw_user(cfg, rng, sigma=sigma, seq_len=L) for L in lens]
    got, _, ctx = run_users(R, torch, cfg, model, users)
    assert ctx.aif_user_attention_kind() == 1
    for i, u in enumerate(users):
        check_user("bf16", got[i], oracle_user(model, u), d, f"MFMA user {i} (L={lens[i]})")


def test_forced_generic_kernels_agree_with_the_oracle_on_the_mfma_shape(R, torch, monkeypatch):
    monkeypatch.setenv("AIF_FORCE_GENERIC", "1")
    cfg = wl.UserNetConfig("T", 12, "bf16", 2, 140, 128, 64)
    _say("user net, bf16 d=64 on the shape-agnostic kernels")
    model = wl.make_user_net_model(cfg, bias_scale=0.05)
    rng = np.random.default_rng(8)
    users = [wl.make_raw_user(cfg, rng, seq_len=L) for L in (140, 65)]
    got, _, ctx = run_users(R, torch, cfg, model, users)
    assert ctx.aif_user_attention_kind() == 0
    for i, u in enumerate(users):
        check_user("bf16", got[i], oracle_user(model, u), cfg.d, f"forced generic user {i}")


def test_a_users_result_does_not_depend_on_its_batch(R, torch):
    cfg = wl.USER_CONFIGS["U3"].scaled(n_users=5)
    _say("user net: alone vs in a batch, twice")
    model = wl.make_user_net_model(cfg)
    users = wl.make_raw_users(cfg, 5)
    got, _, ctx = run_users(R, torch, cfg, model, users)
    again, _, _ = run_users(R, torch, cfg, model, users, ctx=ctx)
    alone, _, _ = run_users(R, torch, cfg, model, users[3:4])
    for a, b in zip(got, again):
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert np.array_equal(got[3][0], alone[0][0]) and np.array_equal(got[3][1], alone[0][1])


def test_u3_full_size_sampled_users(R, torch):
    cfg = wl.USER_CONFIGS["U3"]
    _say("U3 full size: 64 users x 500 positions")
    w = R.UserNetWorkload(cfg)
    w.step()
    torch.cuda.synchronize()
    assert w.ctx.aif_user_attention_kind() == 1
    for i in (0, 17, 63):
        d = w.dev[i]
        got = (R.from_device_f32(d.user_vec), R.from_device_f32(d.seq_out))
        check_user("bf16", got, oracle_user(w.model, w.users[i]), cfg.d, f"U3 user {i}")


def test_chain_user_network_into_real_time_scoring(R, torch):
    """The cached tensors the asynchronous phase leaves are what the real-time phase reads (Sec. 3.1): user
    network on the GPU -> aif_score_batch on its outputs, against the oracle's own chain."""
    from paper_2511_12934_amd import binding as B
    ucfg = wl.USER_CONFIGS["U3"].scaled(n_users=2)
    cfg = wl.CONFIGS["A3"].scaled(n_items=4000, n_users=2, n_cand=700)
    _say("chain U3 -> A3")
    umodel = wl.make_user_net_model(ucfg)
    users = wl.make_raw_users(ucfg, 2)
    got, udev, _ = run_users(R, torch, ucfg, umodel, users)
    model = wl.make_model(cfg)
    rng = np.random.default_rng(9)
    table = wl.make_table_host(cfg, rng, n_items=4000)
    table_dev = R.to_device(table, "bf16")
    dm = R.DeviceModel(cfg, model)
    ctx = R.make_context(cfg, dm, table_dev, max_users=2, max_candidates=700, max_seq_len=ucfg.seq_len)
    sampler = wl.IdSampler(cfg, 4000)
    reqs, outs, ids_all = [], [], []
    for d in udev:
        ids = sampler.sample(rng, 700)
        idt = torch.from_numpy(ids).to("cuda:0")
        z = torch.full((700,), float("nan"), dtype=torch.float32, device="cuda:0")
        reqs.append(B.Request(d.user_vec, d.seq_out, d.seq_out, idt, z, None, d.user_vec[ucfg.d:], d.seq_out.shape[0]))
        outs.append(z)
        ids_all.append(ids)
    ctx.aif_score_batch(reqs)
    torch.cuda.synchronize()
    assert ctx.aif_stage_kind("attention") == 1 and ctx.aif_stage_kind("mlp") == 1
    for i, u in enumerate(users):
        uv, sh = oracle_user(umodel, u)
        ref = oracle.score(table=table, ids=ids_all[i], user_vec=uv, seq_keys=sh, seq_vals=sh, dims=model.dims,
                           weights=model.weights, biases=model.biases, cross_mode=oracle.CROSS_HADAMARD,
                           cross_vecs=uv[ucfg.d:], n_threads=8)
        assert_logits_close("bf16", outs[i].cpu().numpy(), ref.logits, f"chain user {i}")


def test_host_side_errors_enqueue_nothing(R, torch):
    from paper_2511_12934_amd import binding as B
    cfg = wl.UserNetConfig("T", 11, "bf16", 1, 20, 16, 16)
    model = wl.make_user_net_model(cfg)
    ctx = R.make_user_context(cfg, model, max_users=1, max_seq_len=20)
    rng = np.random.default_rng(1)
    d = R.upload_raw_user(cfg, wl.make_raw_user(cfg, rng, seq_len=21))
    with pytest.raises(B.AifError) as ei:
        ctx.aif_user_precompute([d.req])
    assert ei.value.status == B.AIF_ERANGE
    ok = R.upload_raw_user(cfg, wl.make_raw_user(cfg, rng))
    with pytest.raises(B.AifError) as ei:
        ctx.aif_user_precompute([ok.req, ok.req])
    assert ei.value.status == B.AIF_ERANGE
    bad = B.UserRequest(ok.req.profile, ok.req.seq, None, ok.req.seq_out)
    with pytest.raises(B.AifError) as ei:
        ctx.aif_user_precompute([bad])
    assert ei.value.status == B.AIF_EINVAL
    with pytest.raises(B.AifError):
        R.make_user_context(wl.UserNetConfig("T", 11, "bf16", 1, 20, 12, 16), model)      # d_raw not a multiple of 8
    ctx.aif_user_precompute([ok.req])
    torch.cuda.synchronize()
    assert torch.all(torch.isfinite(ok.user_vec.float()))
