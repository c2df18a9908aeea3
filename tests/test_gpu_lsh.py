"""GPU parity of the LSH path (include/aif_lsh.h) against its CPU oracle: SimTier counts bit-exact,
LSH-DIN within a tolerance derived from the fp32 summation."""
import numpy as np
import pytest

import oracle
from paper_2511_12934_amd import workloads as wl

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


def din_tolerance(u_seq, L, d_bits):
    """Per output feature j.  Every U~[t, j] enters the GPU's sum exactly d' times (once per bit, in the table
    of the value the candidate's bit takes) through chains of at most 128 (staged items) + 4 (stagings per
    chunk of 512) + chunks + d' (bits) fp32 additions, then one division by d'.  The standard bound for a sum,
    n u sum|x| with u = 2^-24, over the d' copies and divided by d' gives  n 2^-24 sum_t |U~[t, j]|.
    (A history of more than 64 chunks is cut into 64 longer ones: 4 m stagings and about chunks / m partial sums with
    m = ceil(chunks / 64), fewer additions in a row than the 4 + chunks counted here.)"""
    n = 128 + 4 + (L + 511) // 512 + d_bits + 2
    return n * 2.0 ** -24 * np.abs(u_seq.astype(np.float64)).sum(0) + 1e-30


def check(R, torch, cfg, table, users_ids, ctx=None):
    if ctx is None:
        tdev = torch.from_numpy(table).cuda()
        ctx = R.make_lsh_context(cfg, tdev, max_users=len(users_ids), max_candidates=max([i.size for _, i in users_ids] + [1]),
                                 max_seq_len=max([u.seq_sigs.shape[0] for u, _ in users_ids] + [1]))
    drs = [R.upload_lsh_request(cfg, u, ids) for u, ids in users_ids]
    ctx.aif_lsh_batch([d.req for d in drs])
    torch.cuda.synchronize()
    for r, ((u, ids), d) in enumerate(zip(users_ids, drs)):
        ref = oracle.lsh_request(sig_table=table, ids=ids, seq_sig=u.seq_sigs, u_seq=u.seq_emb, n_tiers=cfg.n_tiers, n_threads=8)
        tiers = d.tiers.cpu().numpy()
        assert np.array_equal(tiers, ref.tiers), f"req {r}: SimTier counts differ"
        din = d.din.cpu().numpy().astype(np.float64)
        tol = din_tolerance(u.seq_emb, u.seq_sigs.shape[0], cfg.d_bits)
        assert np.all(np.abs(din - ref.din) <= tol[None, :]), (r, np.abs(din - ref.din).max(), tol.max())
    assert ctx.aif_lsh_poll_device_errors() == 0
    return ctx, drs


def test_l1_full_size(R, torch):
    cfg = wl.LSH_CONFIGS["L1"]
    _say("L1 fp32 1 x 1000 candidates, 2000 history items")
    table = wl.make_sig_table_host(cfg)
    rq = wl.make_lsh_requests(cfg)[0]
    ctx = R.make_lsh_context(cfg, torch.from_numpy(table).cuda(), max_users=8)
    ctx, drs = check(R, torch, cfg, table, [(rq.user, rq.ids)], ctx=ctx)
    # mini-batch invariance: ten slices give the same bits
    whole = drs[0]
    d0, t0 = whole.din.cpu().numpy().copy(), whole.tiers.cpu().numpy().copy()
    whole.din.fill_(float("nan"))
    whole.tiers.fill_(-9)
    parts = [R.slice_lsh_request(whole, lo, hi) for lo, hi in zip([0, 1, 100, 257, 512, 999], [1, 100, 257, 512, 999, 1000])]
    ctx.aif_lsh_batch([p.req for p in parts])
    torch.cuda.synchronize()
    assert np.array_equal(whole.din.cpu().numpy(), d0) and np.array_equal(whole.tiers.cpu().numpy(), t0)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d_bits,d_out,n_tiers", [(64, 64, 8), (32, 16, 1), (96, 48, 5), (128, 128, 8), (256, 256, 7), (160, 32, 3),
                                                   (128, 64, 4), (64, 128, 2), (32, 16, 8), (64, 32, 4), (32, 32, 2), (128, 16, 1),
                                                   (128, 32, 2), (64, 16, 1), (256, 64, 8), (64, 64, 7)])
def test_shapes_ragged(R, torch, dtype, d_bits, d_out, n_tiers):
    cfg = wl.LshConfig("S", 9, dtype, 1, 10, 3000, d_bits, d_out, n_tiers, 50, n_clusters=16, flip=0.2)
    _say(f"lsh {dtype} d'={d_bits} d={d_out} N={n_tiers}")
    table = wl.make_sig_table_host(cfg)
    rng = np.random.default_rng(d_bits + d_out)
    users_ids = []
    for n, L in [(1, 1), (5, 0), (255, 15), (256, 16), (257, 17), (700, 255), (33, 256), (64, 513), (300, 1100)]:
        users_ids.append((wl.make_lsh_user(cfg, rng, seq_len=L, sigma=1.0), rng.integers(0, cfg.n_items, n).astype(np.int32)))
    ctx, _ = check(R, torch, cfg, table, users_ids)
    # the matrix-core SimTier serves exactly the shapes whose tiers are a power of two of equal-bit counts wide
    width = 2 * d_bits / n_tiers
    assert ctx.aif_lsh_simtier_kind() == int(d_bits in (32, 64, 128) and width == int(width) and int(width) & (int(width) - 1) == 0)
    assert ctx.aif_lsh_din_kind() == int(d_out % 32 == 0 and d_out <= 128)


@pytest.mark.parametrize("d_bits,d_out,n_tiers", [(64, 64, 8), (128, 128, 8), (32, 32, 4), (256, 96, 8)])
def test_vector_alu_kernels_give_the_same_results(R, torch, monkeypatch, d_bits, d_out, n_tiers):
    """SimTier and LSH-DIN on the matrix cores and on the vector ALU, both against the oracle on the same requests (a
    context reads the switches when it is made): the same counts, the same DIN within the fp32 bound."""
    cfg = wl.LshConfig("S", 12, "bf16", 1, 10, 3000, d_bits, d_out, n_tiers, 50, n_clusters=16, flip=0.2)
    _say(f"lsh both kernel families, d'={d_bits} d={d_out} N={n_tiers}")
    table = wl.make_sig_table_host(cfg)
    rng = np.random.default_rng(5)
    users_ids = [(wl.make_lsh_user(cfg, rng, seq_len=L, sigma=1.0), rng.integers(0, cfg.n_items, n).astype(np.int32))
                 for n, L in [(300, 777), (17, 31), (256, 128)]]
    ctx, drs = check(R, torch, cfg, table, users_ids)
    assert ctx.aif_lsh_simtier_kind() == int(d_bits <= 128) and ctx.aif_lsh_din_kind() == 1
    on_mfma = [d.tiers.cpu().numpy().copy() for d in drs]
    monkeypatch.setenv("AIF_LSH_SIMTIER_VALU", "1")
    monkeypatch.setenv("AIF_LSH_DIN_VALU", "1")
    ctx2, drs2 = check(R, torch, cfg, table, users_ids)
    assert ctx2.aif_lsh_simtier_kind() == 0 and ctx2.aif_lsh_din_kind() == 0
    for a, d in zip(on_mfma, drs2):
        assert np.array_equal(a, d.tiers.cpu().numpy())


@pytest.mark.parametrize("d_bits,seq_len", [(64, 250_123), (128, 130_001), (32, 40_000)])
def test_simtier_long_history_few_candidates(R, torch, d_bits, seq_len):
    """A batch too small to fill the chip: the histories are cut into parts, a block each, and a second kernel adds the
    parts' counts up; a history this long also makes every wave read its counting planes out more than once."""
    cfg = wl.LshConfig("S", 13, "bf16", 1, 10, 5000, d_bits, 64 if d_bits == 128 else 16, 8, 50, n_clusters=16, flip=0.2)
    _say(f"lsh long history d'={d_bits} L={seq_len}")
    table = wl.make_sig_table_host(cfg)
    rng = np.random.default_rng(6)
    users_ids = [(wl.make_lsh_user(cfg, rng, seq_len=seq_len, sigma=1.0), rng.integers(0, cfg.n_items, 300).astype(np.int32)),
                 (wl.make_lsh_user(cfg, rng, seq_len=999, sigma=1.0), rng.integers(0, cfg.n_items, 70).astype(np.int32))]
    users_ids[0][0].seq_sigs[seq_len // 2] = table[users_ids[0][1][5]]         # one history item equal to a candidate
    ctx, _ = check(R, torch, cfg, table, users_ids)
    assert ctx.aif_lsh_simtier_kind() == 1


def test_extreme_similarities_and_tier_edges(R, torch):
    """History items equal to, and complementary to, candidates: similarities 1 and 0 land in the outer tiers."""
    cfg = wl.LshConfig("S", 10, "f32", 1, 10, 500, 64, 32, 8, 50, n_clusters=4, flip=0.3)
    _say("lsh extreme similarities")
    table = wl.make_sig_table_host(cfg)
    rng = np.random.default_rng(3)
    ids = np.arange(100, dtype=np.int32)
    u = wl.make_lsh_user(cfg, rng, seq_len=300, sigma=1.0)
    u.seq_sigs[:100] = table[:100]
    u.seq_sigs[100:200] = np.bitwise_not(table[:100])
    for e in range(65):                                   # every possible number of equal bits with candidate 0
        bits = np.unpackbits(table[0])
        bits[:64 - e] ^= 1
        u.seq_sigs[200 + e] = np.packbits(bits)
    check(R, torch, cfg, table, [(u, ids)])


def test_bad_ids_and_host_errors(R, torch):
    cfg = wl.LshConfig("S", 11, "f32", 1, 10, 100, 64, 16, 4, 20, n_clusters=4)
    _say("lsh bad ids / host errors")
    table = wl.make_sig_table_host(cfg)
    rng = np.random.default_rng(4)
    u = wl.make_lsh_user(cfg, rng, seq_len=20)
    ids = np.array([0, 5, 100, -1, 7], dtype=np.int32)
    ctx = R.make_lsh_context(cfg, torch.from_numpy(table).cuda(), max_users=2, max_candidates=16, max_seq_len=20)
    d = R.upload_lsh_request(cfg, u, ids)
    ctx.aif_lsh_batch([d.req])
    torch.cuda.synchronize()
    din, tiers = d.din.cpu().numpy(), d.tiers.cpu().numpy()
    assert np.isnan(din[2]).all() and np.isnan(din[3]).all() and (tiers[2] == -1).all() and (tiers[3] == -1).all()
    good = [0, 1, 4]
    ref = oracle.lsh_request(sig_table=table, ids=ids[good], seq_sig=u.seq_sigs, u_seq=u.seq_emb, n_tiers=cfg.n_tiers)
    assert np.array_equal(tiers[good], ref.tiers)
    assert ctx.aif_lsh_poll_device_errors() == 2
    from paper_2511_12934_amd.binding import AifError
    big = R.upload_lsh_request(cfg, u, np.zeros(17, np.int32))
    with pytest.raises(AifError):
        ctx.aif_lsh_batch([big.req])                      # n_cand beyond max_candidates
    with pytest.raises(AifError):
        ctx.aif_lsh_batch([d.req, d.req, d.req])          # more requests than max_users


@pytest.mark.parametrize("name", ["L2", "L3"])
def test_full_size_config_sampled(R, torch, name):
    """The configurations bench.py can time, at full size and in its launch configuration (one aif_lsh_batch over
    all users): sampled candidates against the oracle one by one, and properties that hold at any size."""
    cfg = wl.LSH_CONFIGS[name]
    _say(f"{name} full size {cfg.n_users} x {cfg.n_cand} x {cfg.seq_len}")
    w = R.LshWorkload(cfg)
    w.step()
    torch.cuda.synchronize()
    _say("step done")
    assert w.ctx.aif_lsh_poll_device_errors() == 0
    rng = np.random.default_rng(77)
    for u in sorted({0, cfg.n_users - 1, int(rng.integers(0, cfg.n_users))}):
        rq = w.requests[u]
        tiers = w.dev[u].tiers.cpu().numpy()
        assert np.all(tiers.sum(1) == cfg.seq_len), "a candidate's tier counts must add up to the history length"
        pos = np.unique(np.concatenate([[0, 255, 256, cfg.n_cand - 1], rng.integers(0, cfg.n_cand, 60)]))
        ref = oracle.lsh_request(sig_table=w.table_host, ids=rq.ids[pos], seq_sig=rq.user.seq_sigs, u_seq=rq.user.seq_emb,
                                 n_tiers=cfg.n_tiers, n_threads=8)
        assert np.array_equal(tiers[pos], ref.tiers), f"user {u}"
        din = w.dev[u].din.cpu().numpy()[pos].astype(np.float64)
        tol = din_tolerance(rq.user.seq_emb, cfg.seq_len, cfg.d_bits)
        assert np.all(np.abs(din - ref.din) <= tol[None, :]), (u, np.abs(din - ref.din).max(), tol.max())
        _say(f"user {u}: max |d DIN| = {np.abs(din - ref.din).max():.3e} (bar {tol.min():.3e})")
    d0, t0 = w.dev[0].din.clone(), w.dev[0].tiers.clone()
    w.step()
    torch.cuda.synchronize()
    assert torch.equal(d0, w.dev[0].din) and torch.equal(t0, w.dev[0].tiers)
