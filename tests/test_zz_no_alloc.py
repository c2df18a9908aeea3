"""aif_score_topk_static -- the entry point that allocates nothing (its per-call workspace is a fixed array the
library holds on the GPU) -- against aif_score_topk, through the C ABI: identical logits, scores and top-k, on
two calls in a row, the second with a smaller input (the array keeps the first call's contents); the size limit;
and, since the call is meant for code under HIP graph capture, a captured call replayed several times with eager
work in between."""
import numpy as np
import pytest

from paper_2511_12934_amd import binding as B
from paper_2511_12934_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch as t
    if not t.cuda.is_available():
        pytest.skip("no GPU")
    return t


@pytest.fixture(scope="module")
def R():
    from paper_2511_12934_amd import runner
    return runner


def _setup(R, cfg, seed, n_items):
    rng = np.random.default_rng(seed)
    model = wl.make_model(cfg, bias_scale=0.05)
    table = wl.make_table_host(cfg, rng, n_items=n_items)
    dm = R.DeviceModel(cfg, model)
    table_dev = R.to_device(table, cfg.dtype)
    sampler = wl.IdSampler(cfg, n_items)
    return rng, dm, table_dev, sampler


def _both(R, torch, ctx, cfg, user, ids, k):
    """(logits, scores, idx, val) of the allocating call and of the static one, on separate output buffers."""
    out = []
    for static in (False, True):
        dr = R.upload_request(cfg, user, ids)
        idx = torch.full((k,), -7, dtype=torch.int32, device="cuda")
        val = torch.full((k,), float("nan"), dtype=torch.float32, device="cuda")
        if static:
            ctx.aif_score_topk_static(dr.req, k, idx, val)
        else:
            ctx.aif_score_topk([dr.req], k, idx, val)
        torch.cuda.synchronize()
        out.append((dr.logits.cpu().numpy(), dr.scores.cpu().numpy(), idx.cpu().numpy(), val.cpu().numpy()))
    return out


@pytest.mark.parametrize("name,n_first,n_second", [("C2", 10000, 777), ("C3", 5000, 1), ("C4", 3000, 2999),
                                                    ("C1", 1000, 300), ("C5", 4000, 513)])
def test_static_call_gives_the_bits_of_the_allocating_call(R, torch, name, n_first, n_second):
    base = wl.CONFIGS[name]
    cfg = base.scaled(n_items=20000, seq_len=min(base.seq_len, 1000))
    print(f"[case] {name} shape: static vs allocating call, {n_first} then {n_second} candidates", flush=True)
    rng, dm, table_dev, sampler = _setup(R, cfg, 2025, 20000)
    ctx = R.make_context(cfg, dm, table_dev, max_users=1, max_candidates=max(n_first, n_second))
    for n, L in ((n_first, cfg.seq_len), (n_second, max(1, cfg.seq_len // 3))):
        user = wl.make_user(cfg, rng, seq_len=L)
        ids = sampler.sample(rng, n)
        k = min(cfg.top_k, 4096)
        (z0, y0, i0, v0), (z1, y1, i1, v1) = _both(R, torch, ctx, cfg, user, ids, k)
        assert np.all(np.isfinite(z0))
        assert np.array_equal(z0, z1), f"{name} n={n}: logits differ"
        assert np.array_equal(y0, y1), f"{name} n={n}: scores differ"
        assert np.array_equal(i0, i1) and np.array_equal(v0, v1), f"{name} n={n}: top-k differs"
    assert ctx.aif_poll_device_errors() == 0
    # k = 0: scores only
    dr = R.upload_request(cfg, user, ids)
    ctx.aif_score_topk_static(dr.req, 0)
    torch.cuda.synchronize()
    assert np.array_equal(dr.logits.cpu().numpy(), z0)
    # a bad id is counted and answered with NaN, as in the allocating call
    bad_ids = ids.copy()
    bad_ids[0] = -5
    dr = R.upload_request(cfg, user, bad_ids)
    ctx.aif_score_topk_static(dr.req, 0)
    torch.cuda.synchronize()
    z = dr.logits.cpu().numpy()
    assert np.isnan(z[0]) and np.array_equal(z[1:], z0[1:])
    assert ctx.aif_poll_device_errors() == 1


def test_static_call_rejects_what_does_not_fit(R, torch):
    cfg = wl.CONFIGS["C5"].scaled(n_items=30000, seq_len=64)
    rng, dm, table_dev, sampler = _setup(R, cfg, 7, 30000)
    ctx = R.make_context(cfg, dm, table_dev, max_users=1, max_candidates=30000)
    user = wl.make_user(cfg, rng)
    dr = R.upload_request(cfg, user, sampler.sample(rng, 30000))      # 30000 rows x 448 x 2 bytes > 16 MiB
    with pytest.raises(B.AifError) as e:
        ctx.aif_score_topk_static(dr.req, 10, torch.empty(10, dtype=torch.int32, device="cuda"),
                                  torch.empty(10, dtype=torch.float32, device="cuda"))
    assert e.value.status == B.AIF_ERANGE and "static call holds" in str(e.value)
    torch.cuda.synchronize()
    assert torch.isnan(dr.logits).all(), "a rejected call enqueues nothing"


def test_static_call_replayed_from_a_graph(R, torch):
    """Captured once, replayed four times with the program's own eager work and synchronisations between the
    replays (another request through the same array, which a replay must overwrite completely); every replay
    is checked against the eager result."""
    cfg = wl.CONFIGS["C2"].scaled(n_items=20000)
    print("[case] C2 shape: static call under graph capture", flush=True)
    rng, dm, table_dev, sampler = _setup(R, cfg, 99, 20000)
    ctx = R.make_context(cfg, dm, table_dev, max_users=1, max_candidates=10000)
    user, ids = wl.make_user(cfg, rng), sampler.sample(rng, 10000)
    other_user, other_ids = wl.make_user(cfg, rng, seq_len=333), sampler.sample(rng, 4321)
    k = cfg.top_k
    (z_ref, y_ref, i_ref, v_ref), _ = _both(R, torch, ctx, cfg, user, ids, k)
    dr = R.upload_request(cfg, user, ids)
    other = R.upload_request(cfg, other_user, other_ids)
    idx = torch.empty(k, dtype=torch.int32, device="cuda")
    val = torch.empty(k, dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ctx.aif_score_topk_static(dr.req, k, idx, val)          # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        ctx.aif_score_topk_static(dr.req, k, idx, val)
    for rep in range(4):
        dr.logits.fill_(float("nan"))
        idx.fill_(-3)
        ctx.aif_score_topk_static(other.req, 0)                 # eager work through the same array
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(dr.logits.cpu().numpy(), z_ref), f"replay {rep}: logits"
        assert np.array_equal(idx.cpu().numpy(), i_ref) and np.array_equal(val.cpu().numpy(), v_ref), f"replay {rep}: top-k"
