"""Configurations 3-5 (and C3 with the BEA cross block) at full size, in the launch configuration the benchmark
times (one aif_score_batch over all users + one aif_topk): sampled candidates
against the oracle one by one, top-k of every user against the oracle's full
stable sort of the GPU's logits, and the properties that hold at any size."""
import numpy as np
import pytest

import oracle
from paper_2511_12934_amd import workloads as wl

from helpers import assert_features_close, assert_logits_close, oracle_scores_rows

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["C3", "C4", "C5", "B3"])
def test_full_size_batched_config(name):
    import torch
    from paper_2511_12934_amd import runner as R
    cfg = wl.CONFIGS[name]
    print(f"[case] {name} full size {cfg.n_users}x{cfg.n_cand}, table {cfg.n_items}x{cfg.d_item}", flush=True)
    w = R.Workload(cfg)
    w.step()
    torch.cuda.synchronize()
    print("[case] step done", flush=True)
    assert w.ctx.aif_poll_device_errors() == 0
    rng = np.random.default_rng(2024)
    idx = w.idx.cpu().numpy()
    val = w.val.cpu().numpy()
    # top-k of every user, bit-exact on the GPU's own logits
    for u in range(cfg.n_users):
        z = w.dev[u].logits.cpu().numpy()
        assert np.all(np.isfinite(z)), f"user {u}: non-finite logits"
        oi, ov = oracle.topk(z.astype(np.float64), cfg.top_k)
        assert np.array_equal(idx[u], oi), f"user {u}"
        assert np.array_equal(val[u].astype(np.float64), ov), f"user {u}"
    # sampled candidates of sampled users against the oracle
    users = sorted({0, 1, cfg.n_users - 1, int(rng.integers(0, cfg.n_users))})
    for u in users:
        pos = np.unique(np.concatenate([[0, 255, 256, cfg.n_cand - 1], rng.integers(0, cfg.n_cand, 124)]))
        rows = w.rows_of(u, pos)
        ref = oracle_scores_rows(cfg, w.model, rows, w.requests[u].user)
        z = w.dev[u].logits.cpu().numpy()[pos]
        assert_logits_close(cfg.dtype, z, ref.logits, f"{name} user {u}")
        X = R.peek_features(w.ctx, cfg, u, cfg.n_cand)[pos]
        assert np.array_equal(X[:, :cfg.d_item], rows), "gather is not an exact row copy"
        assert_features_close(cfg.dtype, X[:, cfg.d_item:cfg.d_item + cfg.d_attn], ref.attn, "attention")
        assert_features_close(cfg.dtype, X[:, cfg.d_item + cfg.d_attn:], ref.cross, "cross")
        print(f"[case] user {u}: max |dz| = {np.abs(z - ref.logits).max():.3e}", flush=True)
    # determinism of the whole step
    z0 = [d.logits.clone() for d in w.dev[:2]]
    w.step()
    torch.cuda.synchronize()
    for a, d in zip(z0, w.dev[:2]):
        assert torch.equal(a, d.logits)
    assert np.array_equal(w.idx.cpu().numpy(), idx)
