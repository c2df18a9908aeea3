"""Pins of the CPU oracle against things other than itself.

The paper prints no number for the online scoring path, so every step is
pinned by what the mathematics fixes: closed forms, invariants, special cases
that reduce to a textbook routine (NumPy float64 / torch SDPA float64), and
brute force against an independently written vectorised NumPy reference.
"""
import numpy as np
import pytest

import oracle
from paper_2511_12934_amd import workloads as wl

RNG = lambda s: np.random.default_rng(s)


# --------------------------------------------------------------------------
# an independently written reference (vectorised NumPy float64) of the whole
# path; used for brute force on tiny inputs.  Shares nothing with the C code.
# --------------------------------------------------------------------------
def numpy_path(table, ids, u, K, V, dims, Ws, bs, w_q=None, H=1, cross_mode=1, cv=None):
    T = np.asarray(table, np.float64)
    E = T[np.asarray(ids)]                                          # [n, d_item]
    d_attn = K.shape[1]
    Q = E @ np.asarray(w_q, np.float64).T if w_q is not None else E[:, :d_attn]
    K64, V64 = np.asarray(K, np.float64), np.asarray(V, np.float64)
    n, L = E.shape[0], K64.shape[0]
    dh = d_attn // H
    A = np.zeros((n, d_attn))
    if L:
        Qh = Q.reshape(n, H, dh)
        Kh = K64.reshape(L, H, dh)
        Vh = V64.reshape(L, H, dh)
        S = np.einsum("nhd,lhd->nhl", Qh, Kh) / np.sqrt(dh)
        S = S - S.max(axis=2, keepdims=True)
        P = np.exp(S)
        P /= P.sum(axis=2, keepdims=True)
        A = np.einsum("nhl,lhd->nhd", P, Vh).reshape(n, d_attn)
    u64 = np.asarray(u, np.float64)
    if cross_mode == wl.CROSS_HADAMARD:
        Cx = E * (u64 if cv is None else np.asarray(cv, np.float64))[None, :]
    elif cross_mode == wl.CROSS_SEGDOT:
        cv64 = np.asarray(cv, np.float64)                             # [n_cross, d_c]
        S_ = E.shape[1] // cv64.shape[1]
        Eseg = E.reshape(n, S_, cv64.shape[1])
        Cx = np.einsum("jm,nsm->njs", cv64, Eseg).reshape(n, -1)
    elif cross_mode == wl.CROSS_BEA:
        cv64 = np.asarray(cv, np.float64)                             # V [n_bridges, d']
        Cx = E[:, E.shape[1] - cv64.shape[0]:] @ cv64
    else:
        Cx = np.zeros((n, 0))
    X = np.concatenate([np.broadcast_to(u64, (n, u64.size)), E, A, Cx], axis=1)
    Hh = X
    for l, (W, b) in enumerate(zip(Ws, bs)):
        Hh = Hh @ np.asarray(W, np.float64).T + (0 if b is None else np.asarray(b, np.float64))
        if l + 1 < len(Ws):
            Hh = np.maximum(Hh, 0)
    return Hh[:, 0], A, Cx


def tiny_cfg(**kw):
    base = dict(name="T", index=9, dtype="f32", n_users=1, n_cand=8, n_items=20, d_item=4,
                id_dist="uniform", seq_len=3, d_attn=4, n_heads=1, use_wq=False,
                cross_mode=wl.CROSS_HADAMARD, n_cross=0, d_cross_vec=0, d_user=4,
                mlp_dims=(16, 5, 1), top_k=3)
    base.update(kw)
    c = wl.Config(**base)
    assert c.d_in == c.mlp_dims[0]
    return c


# ------------------------------------------------- nearline table update
def test_update_rows_is_an_indexed_assignment_that_skips_bad_ids():
    rng = RNG(12)
    t = rng.standard_normal((50, 6)).astype(np.float32)
    ids = rng.permutation(50)[:20].astype(np.int32)
    rows = rng.standard_normal((20, 6)).astype(np.float32)
    got, skipped = oracle.update_rows(t, ids, rows)
    ref = t.copy()
    ref[ids] = rows                                      # NumPy's own indexed assignment (distinct ids)
    assert skipped == 0 and np.array_equal(got, ref)
    untouched = np.setdiff1d(np.arange(50), ids)
    assert np.array_equal(got[untouched], t[untouched]) and not np.array_equal(got[ids], t[ids])
    # ids outside the table are skipped and counted; a later entry for an id replaces an earlier one
    ids2 = np.array([3, -1, 50, 3, 7], np.int32)
    rows2 = np.arange(30, dtype=np.float32).reshape(5, 6)
    got2, skipped2 = oracle.update_rows(t, ids2, rows2)
    assert skipped2 == 2
    assert np.array_equal(got2[3], rows2[3]) and np.array_equal(got2[7], rows2[4])
    rest = np.setdiff1d(np.arange(50), [3, 7])
    assert np.array_equal(got2[rest], t[rest])
    # scoring reads the updated row
    assert np.array_equal(oracle.gather(got2, np.array([7], np.int32))[0], rows2[4].astype(np.float64))


# ------------------------------------------------------------------ gather
def test_gather_is_row_copy_and_rejects_bad_ids():
    rng = RNG(1)
    T = rng.standard_normal((50, 6)).astype(np.float32)
    ids = np.array([0, 49, 7, 7, 13], np.int32)
    E = oracle.gather(T, ids)
    assert E.dtype == np.float64
    assert np.array_equal(E, T[ids].astype(np.float64))
    for bad in (-1, 50):
        with pytest.raises(oracle.OracleError) as ei:
            oracle.gather(T, np.array([1, bad], np.int32))
        assert ei.value.code == oracle.ERANGE


# ------------------------------------------------------------------- query
def test_query_slice_and_projection():
    e = np.arange(1.0, 7.0)
    assert np.array_equal(oracle.query(e, None, 4), e[:4])
    Wq = np.array([[1, 0, 0, 0, 0, 2], [0, -1, 0.5, 0, 0, 0]], np.float32)
    # by hand: row0 = 1*1 + 2*6 = 13 ; row1 = -2 + 1.5 = -0.5
    assert np.array_equal(oracle.query(e, Wq, 2), np.array([13.0, -0.5]))


# --------------------------------------------------------------- attention
@pytest.mark.parametrize("scale", [0.1, 1.0, 8.0, 30.0])
@pytest.mark.parametrize("H", [1, 2, 4])
def test_attention_weights_are_a_distribution(scale, H):
    rng = RNG(2)
    L, d = 37, 8
    q = rng.standard_normal(d) * scale
    K = (rng.standard_normal((L, d)) * scale).astype(np.float32)
    V = rng.standard_normal((L, d)).astype(np.float32)
    a, p = oracle.attention(q, K, V, H, return_weights=True)
    assert p.shape == (H, L)
    assert np.all(p >= 0) and np.all(np.isfinite(p))
    assert np.allclose(p.sum(axis=1), 1.0, atol=1e-12, rtol=0)
    assert np.all(np.isfinite(a))


def test_attention_single_key_returns_its_value():
    rng = RNG(3)
    q = rng.standard_normal(6) * 5
    K = rng.standard_normal((1, 6)).astype(np.float32)
    V = rng.standard_normal((1, 6)).astype(np.float32)
    assert np.array_equal(oracle.attention(q, K, V, 1), V[0].astype(np.float64))
    assert np.array_equal(oracle.attention(q, K, V, 3), V[0].astype(np.float64))


def test_attention_equal_keys_or_zero_query_gives_mean_value():
    rng = RNG(4)
    L, d = 11, 4
    V = rng.standard_normal((L, d)).astype(np.float32)
    K = np.tile(rng.standard_normal((1, d)).astype(np.float32), (L, 1))
    q = rng.standard_normal(d) * 3
    assert np.allclose(oracle.attention(q, K, V), V.astype(np.float64).mean(0), atol=1e-14)
    K2 = rng.standard_normal((L, d)).astype(np.float32)
    assert np.allclose(oracle.attention(np.zeros(d), K2, V), V.astype(np.float64).mean(0), atol=1e-14)


def test_attention_empty_sequence_is_zero():
    a = oracle.attention(np.ones(4), np.zeros((0, 4), np.float32), np.zeros((0, 4), np.float32))
    assert np.array_equal(a, np.zeros(4))


def test_attention_shift_invariance_in_keys():
    # K_t + kappa for every t adds q.kappa to every score: softmax unchanged.
    rng = RNG(5)
    L, d = 23, 8
    q = rng.standard_normal(d)
    # values on a coarse binary grid so K + kappa is exact in float32
    K = (rng.integers(-64, 64, (L, d)) / 16.0).astype(np.float32)
    kappa = (rng.integers(-64, 64, d) / 16.0).astype(np.float32)
    V = rng.standard_normal((L, d)).astype(np.float32)
    a0 = oracle.attention(q, K, V, 2)
    a1 = oracle.attention(q, K + kappa[None, :], V, 2)
    assert np.allclose(a0, a1, atol=1e-12)


def test_attention_dominant_key_and_large_scores_do_not_overflow():
    rng = RNG(6)
    L, d = 9, 4
    K = rng.standard_normal((L, d)).astype(np.float32)
    V = rng.standard_normal((L, d)).astype(np.float32)
    q = K[5].astype(np.float64) * 400.0      # |s| far above 88 (float exp range) and 709
    a, p = oracle.attention(q, K, V, 1, return_weights=True)
    assert np.all(np.isfinite(a))
    s = K.astype(np.float64) @ q / 2.0
    top = int(s.argmax())
    assert np.sort(s)[-1] - np.sort(s)[-2] > 50          # one key dominates
    assert p[0].argmax() == top and p[0, top] > 1 - 1e-12
    assert np.allclose(a, V[top], atol=1e-9)


def test_attention_heads_equal_independent_single_head_calls():
    rng = RNG(7)
    L, d, H = 13, 12, 3
    dh = d // H
    q = rng.standard_normal(d) * 2
    K = rng.standard_normal((L, d)).astype(np.float32)
    V = rng.standard_normal((L, d)).astype(np.float32)
    a = oracle.attention(q, K, V, H)
    for h in range(H):
        sl = slice(h * dh, (h + 1) * dh)
        ah = oracle.attention(q[sl], np.ascontiguousarray(K[:, sl]), np.ascontiguousarray(V[:, sl]), 1)
        assert np.array_equal(a[sl], ah)


def test_attention_scale_is_inverse_sqrt_of_head_width():
    # two keys, d_h = 4: p_0 = sigmoid((s0 - s1)) with s = q.k / 2
    q = np.array([1.0, 2.0, 0.0, -1.0])
    K = np.array([[1, 0, 0, 0], [0, 1, 0, 0]], np.float32)
    V = np.array([[1, 0, 0, 0], [0, 1, 0, 0]], np.float32)
    a = oracle.attention(q, K, V, 1)
    s0, s1 = 1.0 / 2.0, 2.0 / 2.0
    p0 = 1.0 / (1.0 + np.exp(s1 - s0))
    assert np.allclose(a, [p0, 1 - p0, 0, 0], atol=1e-15)
    # with H = 2 (d_h = 2) the scale becomes 1/sqrt(2) and heads are separate
    a2 = oracle.attention(q, K, V, 2)
    t0, t1 = 1.0 / np.sqrt(2), 2.0 / np.sqrt(2)
    p0 = 1.0 / (1.0 + np.exp(t1 - t0))
    assert np.allclose(a2[:2], [p0, 1 - p0], atol=1e-15)
    assert np.allclose(a2[2:], [0, 0], atol=1e-15)      # head 2: V slice is zero


@pytest.mark.parametrize("scale", [0.1, 1.0, 8.0])
def test_attention_matches_torch_sdpa_float64(scale):
    torch = pytest.importorskip("torch")
    rng = RNG(8)
    n, L, d, H = 5, 29, 16, 4
    Q = rng.standard_normal((n, d)) * scale
    K = (rng.standard_normal((L, d)) * scale).astype(np.float32)
    V = rng.standard_normal((L, d)).astype(np.float32)
    dh = d // H
    tq = torch.tensor(Q).reshape(n, H, dh).permute(1, 0, 2)[None]          # [1,H,n,dh]
    tk = torch.tensor(K, dtype=torch.float64).reshape(L, H, dh).permute(1, 0, 2)[None]
    tv = torch.tensor(V, dtype=torch.float64).reshape(L, H, dh).permute(1, 0, 2)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0].permute(1, 0, 2).reshape(n, d)
    got = np.stack([oracle.attention(Q[i], K, V, H) for i in range(n)])
    assert np.allclose(got, ref.numpy(), atol=1e-12, rtol=1e-12)


# ------------------------------------------------------------------- cross
def test_cross_hadamard_by_hand_and_identity():
    e = np.array([2.0, -3.0, 0.5])
    assert np.array_equal(oracle.cross(oracle.CROSS_HADAMARD, [4, 0.5, -2], e), [8.0, -1.5, -1.0])
    assert np.array_equal(oracle.cross(oracle.CROSS_HADAMARD, np.ones(3), e), e)


def test_cross_segdot_by_hand_one_hot_and_layout():
    e = np.array([1.0, 2.0, 3.0, 4.0, 5.0, 6.0])          # S = 3 segments of d_c = 2
    Vc = np.array([[1, 0], [0, 1], [1, 1], [2, -1]], np.float32)
    c = oracle.cross(oracle.CROSS_SEGDOT, Vc, e, n_cross=4, d_c=2)
    # c[j*S + s] = <Vc_j, e[2s:2s+2]>
    want = [1, 3, 5,  2, 4, 6,  3, 7, 11,  0, 2, 4]
    assert np.array_equal(c, np.array(want, np.float64))
    with pytest.raises(oracle.OracleError):
        oracle.cross(oracle.CROSS_SEGDOT, Vc, np.ones(5), n_cross=4, d_c=2)


# --------------------------------------------------------------------- MLP
def test_mlp_zero_weights_give_last_bias():
    dims = (6, 4, 3, 1)
    Ws = [np.zeros((dims[i + 1], dims[i]), np.float32) for i in range(3)]
    bs = [np.full(4, 2.0, np.float32), np.full(3, -1.0, np.float32), np.array([0.75], np.float32)]
    assert oracle.mlp(np.arange(6.0), dims, Ws, bs)[0] == 0.75


def test_mlp_single_layer_is_a_dot_product():
    x = np.array([1.0, -2.0, 0.5])
    z = oracle.mlp(x, (3, 1), [np.array([[2, 1, 4]], np.float32)], [np.array([0.25], np.float32)])
    assert z[0] == 2 - 2 + 2 + 0.25


def test_mlp_relu_kills_negated_copy_and_last_layer_is_linear():
    # hidden = [w.x, -w.x]; relu keeps one of them; output = h0 - h1 = |w.x| sign-restored
    w = np.array([[1.0, 2.0], [-1.0, -2.0]], np.float32)
    out = np.array([[1.0, -1.0]], np.float32)
    for x in ([3.0, 1.0], [-3.0, -1.0]):
        z = oracle.mlp(np.array(x), (2, 2, 1), [w, out], None)[0]
        assert z == x[0] + 2 * x[1]            # relu(a) - relu(-a) = a
    # a negative final pre-activation must survive (no ReLU on the last layer)
    z = oracle.mlp(np.array([1.0]), (1, 1, 1), [np.array([[1.0]], np.float32), np.array([[-3.0]], np.float32)], None)
    assert z[0] == -3.0


def test_mlp_matches_numpy_float64_chain():
    rng = RNG(9)
    dims = (24, 16, 8, 1)
    Ws = [rng.standard_normal((dims[i + 1], dims[i])).astype(np.float32) for i in range(3)]
    bs = [rng.standard_normal(dims[i + 1]).astype(np.float32) for i in range(3)]
    x = rng.standard_normal(24)
    h = x
    for l in range(3):
        h = Ws[l].astype(np.float64) @ h + bs[l].astype(np.float64)
        if l < 2:
            h = np.maximum(h, 0)
    assert np.allclose(oracle.mlp(x, dims, Ws, bs), h, rtol=1e-13, atol=1e-13)


def test_sigmoid_values():
    assert oracle.sigmoid(0.0) == 0.5
    assert abs(oracle.sigmoid(np.log(3.0)) - 0.75) < 1e-15
    assert abs(oracle.sigmoid(2.0) + oracle.sigmoid(-2.0) - 1.0) < 1e-15


# ------------------------------------------------------------------- top-k
def _full_sort_topk(z, k):
    z = np.asarray(z, np.float64)
    key = np.where(np.isnan(z), -np.inf, z)
    # NaN below every number including -inf: sort by (is_nan, -value) stably
    order = np.lexsort((np.arange(z.size), -key, np.isnan(z)))
    idx = np.full(k, -1, np.int32)
    val = np.full(k, -np.inf)
    m = min(k, z.size)
    idx[:m] = order[:m]
    val[:m] = z[order[:m]]
    return idx, val


@pytest.mark.parametrize("kind", ["random", "equal", "sorted", "reversed", "inf", "nan", "dups", "zeros"])
def test_topk_equals_full_stable_sort(kind):
    rng = RNG(10)
    n = 257
    z = rng.standard_normal(n)
    if kind == "equal":
        z[:] = 1.5
    elif kind == "sorted":
        z = np.sort(z)[::-1].copy()
    elif kind == "reversed":
        z = np.sort(z)
    elif kind == "inf":
        z[[3, 77]] = np.inf
        z[[5, 100, 200]] = -np.inf
    elif kind == "nan":
        z[[0, 9, 128]] = np.nan
        z[[4]] = -np.inf
    elif kind == "dups":
        z = rng.integers(0, 5, n).astype(np.float64)
    elif kind == "zeros":
        z = rng.integers(-1, 2, n).astype(np.float64)
        z[z == 0] = np.where(rng.random((z == 0).sum()) < 0.5, 0.0, -0.0)
    for k in (1, 7, n - 1, n, n + 1, n + 10):
        idx, val = oracle.topk(z, k)
        ridx, rval = _full_sort_topk(z, k)
        assert np.array_equal(idx, ridx), (kind, k)
        assert np.array_equal(val, rval, equal_nan=True), (kind, k)


def test_topk_numpy_argsort_agreement_without_special_values():
    rng = RNG(11)
    z = rng.integers(0, 40, 1000).astype(np.float64)
    idx, _ = oracle.topk(z, 100)
    assert np.array_equal(idx, np.argsort(-z, kind="stable")[:100])


def test_topk_rejects_bad_k():
    with pytest.raises(oracle.OracleError):
        oracle.topk(np.zeros(4), 0)


# -------------------------------------------------------------- whole path
def _tiny_inputs(cfg, seed, sigma=1.0, bias_scale=0.5):
    rng = RNG(seed)
    model = wl.make_model(cfg, seed=seed, bias_scale=bias_scale)
    table = wl.make_table_host(cfg, rng, sigma=sigma)
    user = wl.make_user(cfg, rng, sigma=sigma)
    ids = wl.IdSampler(cfg).sample(rng, cfg.n_cand)
    return model, table, user, ids


def _score(cfg, model, table, user, ids, **kw):
    return oracle.score(table=table, ids=ids, user_vec=user.user_vec, seq_keys=user.seq_keys,
                        seq_vals=user.seq_vals, dims=model.dims, weights=model.weights,
                        biases=model.biases, w_q=model.w_q, n_heads=cfg.n_heads,
                        cross_mode=cfg.cross_mode, cross_vecs=user.cross_vecs, **kw)


@pytest.mark.parametrize("variant", ["hadamard", "wq_heads", "segdot", "bea"])
def test_whole_path_brute_force_against_numpy_reference(variant):
    if variant == "hadamard":
        cfg = tiny_cfg()
    elif variant == "wq_heads":
        cfg = tiny_cfg(d_item=6, d_user=6, d_attn=4, n_heads=2, use_wq=True, seq_len=4,
                       mlp_dims=(22, 7, 3, 1))
    elif variant == "bea":
        cfg = tiny_cfg(d_item=8, d_user=5, d_attn=4, n_heads=2, seq_len=4,
                       cross_mode=wl.CROSS_BEA, n_cross=3, d_cross_vec=5, mlp_dims=(22, 6, 1))
    else:
        cfg = tiny_cfg(d_item=8, d_user=5, d_attn=4, n_heads=2, use_wq=True, seq_len=4,
                       cross_mode=wl.CROSS_SEGDOT, n_cross=3, d_cross_vec=4, mlp_dims=(23, 6, 1))
    for seed in range(3):
        model, table, user, ids = _tiny_inputs(cfg, 100 + seed)
        got = _score(cfg, model, table, user, ids)
        z, A, Cx = numpy_path(table, ids, user.user_vec, user.seq_keys, user.seq_vals, model.dims,
                              model.weights, model.biases, model.w_q, cfg.n_heads, cfg.cross_mode,
                              user.cross_vecs)
        assert np.allclose(got.attn, A, rtol=1e-12, atol=1e-13)
        assert np.allclose(got.cross, Cx, rtol=1e-12, atol=1e-13)
        assert np.allclose(got.logits, z, rtol=1e-11, atol=1e-12)
        assert np.allclose(got.scores, 1 / (1 + np.exp(-z)), rtol=1e-12)


def test_whole_path_config1_shape_against_numpy_reference():
    cfg = wl.CONFIGS["C1"].scaled(n_items=500, n_cand=40)
    model, table, user, ids = _tiny_inputs(cfg, 7, sigma=0.1, bias_scale=0.0)
    got = _score(cfg, model, table, user, ids)
    z, A, Cx = numpy_path(table, ids, user.user_vec, user.seq_keys, user.seq_vals, model.dims,
                          model.weights, model.biases, model.w_q, cfg.n_heads, cfg.cross_mode, None)
    assert np.allclose(got.logits, z, rtol=1e-11, atol=1e-13)
    assert np.allclose(got.attn, A, rtol=1e-11, atol=1e-13)


def test_user_fold_identity():
    # [u|e|a|c] W1^T = u W1u^T (once per request) + [e|a|c] W1rest^T
    cfg = tiny_cfg()
    model, table, user, ids = _tiny_inputs(cfg, 21)
    got = _score(cfg, model, table, user, ids)
    W1 = model.weights[0].astype(np.float64)
    du = cfg.d_user
    fold_bias = W1[:, :du] @ user.user_vec.astype(np.float64) + model.biases[0]
    E = oracle.gather(table, ids)
    rest = np.concatenate([E, got.attn, got.cross], axis=1)
    h1 = np.maximum(rest @ W1[:, du:].T + fold_bias, 0)
    z = h1 @ model.weights[1].astype(np.float64).T + model.biases[1]
    assert np.allclose(got.logits, z[:, 0], rtol=1e-12, atol=1e-13)


def test_permutation_equivariance_is_bitwise():
    cfg = tiny_cfg(n_cand=16, n_items=64)
    model, table, user, ids = _tiny_inputs(cfg, 33)
    perm = RNG(0).permutation(ids.size)
    z0 = _score(cfg, model, table, user, ids).logits
    z1 = _score(cfg, model, table, user, ids[perm]).logits
    assert np.array_equal(z1, z0[perm])
    k = 5
    i0, _ = oracle.topk(z0, k)
    i1, _ = oracle.topk(z1, k)
    if len(set(z0.tolist())) == z0.size:                     # no ties
        assert np.array_equal(perm[i1], i0)


def test_minibatch_split_is_bitwise_and_thread_count_does_not_matter():
    cfg = wl.CONFIGS["C1"].scaled(n_items=2000, n_cand=300)
    model, table, user, ids = _tiny_inputs(cfg, 44, sigma=0.1, bias_scale=0.0)
    whole = _score(cfg, model, table, user, ids).logits
    parts = np.concatenate([_score(cfg, model, table, user, ids[i:i + 100]).logits
                            for i in range(0, 300, 100)])
    assert np.array_equal(whole, parts)
    threaded = _score(cfg, model, table, user, ids, n_threads=4).logits
    assert np.array_equal(whole, threaded)


def test_duplicate_candidates_score_identically_and_tie_break_by_position():
    cfg = tiny_cfg(n_cand=6, n_items=30)
    model, table, user, ids = _tiny_inputs(cfg, 55)
    ids = np.array([ids[0], ids[1], ids[0], ids[2], ids[1], ids[0]], np.int32)
    z = _score(cfg, model, table, user, ids).logits
    assert z[0] == z[2] == z[5] and z[1] == z[4]
    idx, _ = oracle.topk(z, 6)
    pos = {int(p): r for r, p in enumerate(idx)}
    assert pos[0] < pos[2] < pos[5] and pos[1] < pos[4]


def test_whole_path_shape_errors():
    cfg = tiny_cfg()
    model, table, user, ids = _tiny_inputs(cfg, 66)
    with pytest.raises(oracle.OracleError):
        oracle.score(table=table, ids=ids, user_vec=user.user_vec, seq_keys=user.seq_keys,
                     seq_vals=user.seq_vals, dims=(15, 5, 1), weights=[np.zeros((5, 15)), np.zeros((1, 5))])
    with pytest.raises(oracle.OracleError) as ei:
        _score(cfg, model, table, user, np.array([0, cfg.n_items], np.int32))
    assert ei.value.code == oracle.ERANGE
