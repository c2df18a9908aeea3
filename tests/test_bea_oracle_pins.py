"""Pins of the oracle's Bridge Embedding Approximation (Sec. 4.1, Algorithm 1) against things other
than itself: closed forms, special cases, library routines (scipy softmax, NumPy float64 matmul).
The paper prints no number for Algorithm 1."""
import numpy as np
import pytest
from scipy.special import softmax

import oracle
from paper_2511_12934_amd import workloads as wl

RNG = lambda s: np.random.default_rng(s)


# ---- steps 1 and 3: softmax cross-attention between bridges and embeddings ----
def test_attention_weight_rows_are_distributions():
    rng = RNG(1)
    for scale in (0.1, 1.0, 30.0):
        I = (rng.standard_normal((7, 6)) * scale).astype(np.float32)
        B = (rng.standard_normal((5, 6)) * scale).astype(np.float32)
        w = oracle.bea_attention_weights(I, B)
        assert w.shape == (7, 5)
        assert np.all(w >= 0) and np.all(np.isfinite(w))
        assert np.allclose(w.sum(axis=1), 1.0, rtol=0, atol=1e-12)


def test_attention_weights_hand_worked_two_bridges():
    # d = 4, item (2,0,0,0), bridges (1,0,0,0) and 0: logits 2/sqrt(4) = 1 and 0 -> e/(1+e), 1/(1+e)
    I = np.array([[2, 0, 0, 0]], np.float32)
    B = np.array([[1, 0, 0, 0], [0, 0, 0, 0]], np.float32)
    w = oracle.bea_attention_weights(I, B)
    e = np.e
    assert np.allclose(w, [[e / (1 + e), 1 / (1 + e)]], rtol=1e-15)
    # the scale is 1/sqrt(d) of the embedding width, not of the number of bridges: d = 1 gives e^2
    w1 = oracle.bea_attention_weights(np.array([[2]], np.float32), np.array([[1], [0]], np.float32))
    assert np.allclose(w1, [[e * e / (1 + e * e), 1 / (1 + e * e)]], rtol=1e-15)


def test_zero_item_gives_uniform_weights_and_dominant_bridge_gives_one_hot():
    rng = RNG(2)
    B = rng.standard_normal((6, 8)).astype(np.float32)
    w = oracle.bea_attention_weights(np.zeros((3, 8), np.float32), B)
    assert np.allclose(w, 1.0 / 6, rtol=0, atol=1e-15)
    I = (B[4:5] * 500).astype(np.float32)                 # far along bridge 4: logits differ by hundreds
    w = oracle.bea_attention_weights(I, B)
    assert np.argmax(w[0]) == 4 and w[0, 4] > 1 - 1e-12 and np.all(np.isfinite(w))


def test_attention_weights_match_scipy_softmax_and_step1_is_the_same_operator():
    rng = RNG(3)
    U = rng.standard_normal((9, 5)).astype(np.float32)    # m user-side embeddings
    I = rng.standard_normal((4, 5)).astype(np.float32)    # b item-side embeddings
    B = rng.standard_normal((3, 5)).astype(np.float32)    # n bridges
    ref3 = softmax(I.astype(np.float64) @ B.astype(np.float64).T / np.sqrt(5), axis=1)      # [b, n]
    ref1 = softmax(B.astype(np.float64) @ U.astype(np.float64).T / np.sqrt(5), axis=1)      # [n, m]
    assert np.allclose(oracle.bea_attention_weights(I, B), ref3, rtol=1e-13, atol=1e-15)
    assert np.allclose(oracle.bea_attention_weights(B, U), ref1, rtol=1e-13, atol=1e-15)
    # a transposed operand or a softmax over the wrong axis would not give rows summing to one here
    assert not np.allclose(ref3.sum(axis=0), 1.0)


# ---- step 4: the online weighted sum -------------------------------------------
def test_weighted_sum_matches_numpy_matmul_and_is_not_its_transpose():
    rng = RNG(4)
    w = rng.random((6, 4))
    V = rng.standard_normal((4, 4)).astype(np.float32)    # square on purpose: a transposed V still has a valid shape
    got = oracle.bea_weighted_sum(w, V)
    assert np.allclose(got, w @ V.astype(np.float64), rtol=1e-14, atol=1e-15)
    assert not np.allclose(got, w @ V.astype(np.float64).T)


def test_one_hot_weights_select_a_row_and_a_single_bridge_returns_it():
    rng = RNG(5)
    V = rng.standard_normal((5, 7)).astype(np.float32)
    for j in range(5):
        w = np.zeros((1, 5))
        w[0, j] = 1.0
        assert np.array_equal(oracle.bea_weighted_sum(w, V)[0], V[j].astype(np.float64))
    assert np.array_equal(oracle.bea_weighted_sum(np.ones((3, 1)), V[:1]), np.repeat(V[:1].astype(np.float64), 3, 0))


def test_convex_weights_stay_inside_the_hull_of_the_user_vectors():
    rng = RNG(6)
    V = rng.standard_normal((10, 16)).astype(np.float32)
    w = rng.exponential(size=(200, 10))
    w /= w.sum(axis=1, keepdims=True)
    v = oracle.bea_weighted_sum(w, V)
    assert np.all(v <= V.max(axis=0) + 1e-12) and np.all(v >= V.min(axis=0) - 1e-12)
    # uniform weights = mean of the user-side vectors
    assert np.allclose(oracle.bea_weighted_sum(np.full((1, 10), 0.1), V)[0], V.astype(np.float64).mean(axis=0), atol=1e-15)


def test_steps_3_and_4_compose_like_numpy():
    rng = RNG(7)
    I = rng.standard_normal((12, 8)).astype(np.float32)
    B = rng.standard_normal((10, 8)).astype(np.float32)
    V = rng.standard_normal((10, 6)).astype(np.float32)
    v = oracle.bea_weighted_sum(oracle.bea_attention_weights(I, B), V)
    ref = softmax(I.astype(np.float64) @ B.astype(np.float64).T / np.sqrt(8), axis=1) @ V.astype(np.float64)
    assert np.allclose(v, ref, rtol=1e-12, atol=1e-14)


# ---- the cross block of the scoring path -----------------------------------------
def test_cross_block_is_step_4_on_the_rows_trailing_weights():
    rng = RNG(8)
    n, d_out, d_item = 4, 6, 12
    e = rng.standard_normal(d_item)
    V = rng.standard_normal((n, d_out)).astype(np.float32)
    c = oracle.cross(oracle.CROSS_BEA, V, e, n_cross=n, d_c=d_out)
    assert c.shape == (d_out,)
    assert np.allclose(c, e[d_item - n:] @ V.astype(np.float64), rtol=1e-14, atol=1e-15)
    # leading entries of the row (the item vector proper) do not enter
    e2 = e.copy()
    e2[:d_item - n] += 5.0
    assert np.array_equal(oracle.cross(oracle.CROSS_BEA, V, e2, n_cross=n, d_c=d_out), c)
    with pytest.raises(oracle.OracleError):
        oracle.cross(oracle.CROSS_BEA, V, e, n_cross=d_item + 1, d_c=d_out)


def test_workload_tables_carry_simplex_weights_in_the_row_tail():
    cfg = wl.Config(name="B", index=11, dtype="bf16", n_users=1, n_cand=8, n_items=50, d_item=24, id_dist="uniform",
                    seq_len=3, d_attn=8, n_heads=1, use_wq=False, cross_mode=wl.CROSS_BEA, n_cross=10,
                    d_cross_vec=16, d_user=8, mlp_dims=(56, 8, 1), top_k=3)
    assert cfg.d_cross == 16 and cfg.d_in == 56
    t = wl.make_table_host(cfg, RNG(9))
    w = t[:, 14:]
    assert np.all(w >= 0) and np.allclose(w.sum(axis=1), 1.0, atol=2e-2)       # bf16-rounded weights
    u = wl.make_user(cfg, RNG(10))
    assert u.cross_vecs.shape == (10, 16)
