"""Pins of the oracle's user-side network (Sec. 3.1, Eq. 1-3) against things other than itself: NumPy float64
matmul, torch scaled-dot-product attention in float64, closed forms and special cases.  The paper prints no
number for these equations."""
import numpy as np
import pytest

import oracle

RNG = lambda s: np.random.default_rng(s)
f32 = lambda a: np.asarray(a, np.float32)


def _weights(rng, d, d_raw, bias=0.3):
    return (f32(rng.standard_normal((d, d_raw)) / np.sqrt(d_raw)), f32(rng.standard_normal((d, d_raw)) / np.sqrt(d_raw)),
            f32(rng.standard_normal((d, d)) / np.sqrt(d)), f32(rng.standard_normal(d) * bias))


def numpy_user_network(profile, seq, wp, ws, wf, bf):
    """Independently written vectorised float64 reference of Eq. 1-3 with the same readings."""
    P = np.asarray(profile, np.float64)[None, :] @ np.asarray(wp, np.float64).T
    S = np.asarray(seq, np.float64) @ np.asarray(ws, np.float64).T
    d = S.shape[1]

    def attend(Q):
        z = Q @ S.T / np.sqrt(d)
        z = np.exp(z - z.max(axis=1, keepdims=True))
        return (z / z.sum(axis=1, keepdims=True)) @ S

    ffn = np.maximum(attend(S) @ np.asarray(wf, np.float64).T + (0 if bf is None else np.asarray(bf, np.float64)), 0)
    return np.concatenate([ffn.mean(axis=0), attend(P)[0]]), S


def test_projection_is_a_matmul_with_the_transposed_weight():
    rng = RNG(1)
    x, W = f32(rng.standard_normal((7, 5))), f32(rng.standard_normal((5, 5)))     # square: a missing transpose keeps the shape
    got = oracle.user_project(x, W)
    assert np.allclose(got, x.astype(np.float64) @ W.astype(np.float64).T, rtol=1e-14, atol=1e-15)
    assert not np.allclose(got, x.astype(np.float64) @ W.astype(np.float64))


@pytest.mark.parametrize("scale", [0.1, 1.0, 8.0, 40.0])
def test_attention_core_matches_torch_sdpa_float64(scale):
    torch = pytest.importorskip("torch")
    rng = RNG(2)
    S = rng.standard_normal((23, 8)) * scale
    Q = rng.standard_normal((5, 8)) * scale
    ref = torch.nn.functional.scaled_dot_product_attention(torch.tensor(Q)[None], torch.tensor(S)[None], torch.tensor(S)[None])[0].numpy()
    got = oracle.user_attend(Q, S)
    assert np.all(np.isfinite(got))
    assert np.allclose(got, ref, rtol=1e-11, atol=1e-13)


def test_attention_core_special_cases_and_scale():
    rng = RNG(3)
    S = rng.standard_normal((6, 4))
    Q = rng.standard_normal((3, 4))
    assert np.allclose(oracle.user_attend(Q, S[:1]), np.repeat(S[:1], 3, 0), atol=1e-15)          # l = 1
    same = np.repeat(S[2:3], 6, 0)
    assert np.allclose(oracle.user_attend(Q, same), np.repeat(S[2:3], 3, 0), atol=1e-15)           # equal rows
    assert np.allclose(oracle.user_attend(np.zeros((1, 4)), S)[0], S.mean(axis=0), atol=1e-15)    # q = 0: uniform
    assert np.array_equal(oracle.user_attend(Q, np.zeros((0, 4))), np.zeros((3, 4)))              # l = 0
    # hand case, d = 4: q = (2,0,0,0), rows (1,0,0,0) and 0 -> logits 1 and 0 -> weight e/(1+e) on the first row
    out = oracle.user_attend(np.array([[2.0, 0, 0, 0]]), np.array([[1.0, 0, 0, 0], [0, 0, 0, 0]]))
    assert np.allclose(out[0], [np.e / (1 + np.e), 0, 0, 0], rtol=1e-15)


def test_ffn_and_pooling_special_cases():
    rng = RNG(4)
    x = rng.standard_normal((9, 6))
    eye = np.eye(6, dtype=np.float32)
    assert np.array_equal(oracle.user_ffn(np.abs(x), eye), np.abs(x))                  # identity weight, non-negative input
    assert np.array_equal(oracle.user_ffn(x, eye), np.maximum(x, 0))                   # ReLU
    b = f32([0.5, -0.5, 0, 1, -1, 2])
    assert np.array_equal(oracle.user_ffn(x, np.zeros((6, 6), np.float32), b), np.repeat(np.maximum(b, 0)[None].astype(np.float64), 9, 0))
    W = f32(rng.standard_normal((6, 6)))
    assert np.allclose(oracle.user_ffn(x, W, b), np.maximum(x @ W.astype(np.float64).T + b, 0), rtol=1e-13, atol=1e-14)
    assert not np.allclose(oracle.user_ffn(x, W, b), np.maximum(x @ W.astype(np.float64) + b, 0))
    assert np.allclose(oracle.user_pool(x), x.mean(axis=0), rtol=1e-14, atol=1e-16)
    assert np.array_equal(oracle.user_pool(np.zeros((0, 6))), np.zeros(6))


def test_network_identity_ffn_reduces_to_pooled_sdpa():
    """W_seq = identity on non-negative embeddings and W_ffn = identity: Eq. 2 is the mean over positions of
    plain self-attention, Eq. 3 plain attention of the projected profile -- both available from torch."""
    torch = pytest.importorskip("torch")
    rng = RNG(5)
    d = 8
    seq = f32(np.abs(rng.standard_normal((17, d))))
    profile = f32(rng.standard_normal(d))
    eye = np.eye(d, dtype=np.float32)
    wp = f32(rng.standard_normal((d, d)))
    uv, sh = oracle.user_network(profile=profile, seq=seq, w_profile=wp, w_seq=eye, w_ffn=eye)
    assert np.array_equal(sh, seq.astype(np.float64))
    S = torch.tensor(seq.astype(np.float64))[None]
    sa = torch.nn.functional.scaled_dot_product_attention(S, S, S)[0].numpy()
    assert np.allclose(uv[:d], sa.mean(axis=0), rtol=1e-12, atol=1e-14)
    P = torch.tensor(profile.astype(np.float64) @ wp.astype(np.float64).T)[None, None]
    pa = torch.nn.functional.scaled_dot_product_attention(P, S, S)[0, 0].numpy()
    assert np.allclose(uv[d:], pa, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("l,d_raw,d", [(1, 3, 2), (5, 6, 4), (33, 12, 8)])
def test_network_brute_force_against_numpy_reference(l, d_raw, d):
    for seed in range(3):
        rng = RNG(100 + seed)
        wp, ws, wf, bf = _weights(rng, d, d_raw)
        profile, seq = f32(rng.standard_normal(d_raw)), f32(rng.standard_normal((l, d_raw)))
        uv, sh = oracle.user_network(profile=profile, seq=seq, w_profile=wp, w_seq=ws, w_ffn=wf, b_ffn=bf)
        ruv, rsh = numpy_user_network(profile, seq, wp, ws, wf, bf)
        assert np.allclose(sh, rsh, rtol=1e-13, atol=1e-14)
        assert np.allclose(uv, ruv, rtol=1e-11, atol=1e-13)


def test_network_empty_sequence_and_order_of_the_combined_vector():
    rng = RNG(7)
    d, d_raw = 4, 5
    wp, ws, wf, bf = _weights(rng, d, d_raw)
    uv, sh = oracle.user_network(profile=f32(rng.standard_normal(d_raw)), seq=np.zeros((0, d_raw), np.float32),
                                 w_profile=wp, w_seq=ws, w_ffn=wf, b_ffn=bf)
    assert sh.shape == (0, d) and np.array_equal(uv, np.zeros(2 * d))
    # permuting the sequence permutes U^_seq and leaves both halves of the combined vector unchanged
    profile, seq = f32(rng.standard_normal(d_raw)), f32(rng.standard_normal((9, d_raw)))
    uv0, sh0 = oracle.user_network(profile=profile, seq=seq, w_profile=wp, w_seq=ws, w_ffn=wf, b_ffn=bf)
    perm = rng.permutation(9)
    uv1, sh1 = oracle.user_network(profile=profile, seq=seq[perm], w_profile=wp, w_seq=ws, w_ffn=wf, b_ffn=bf)
    assert np.array_equal(sh1, sh0[perm]) and np.allclose(uv1, uv0, rtol=1e-13, atol=1e-15)
    # the profile enters the second half only
    uv2, _ = oracle.user_network(profile=profile + 1, seq=seq, w_profile=wp, w_seq=ws, w_ffn=wf, b_ffn=bf)
    assert np.array_equal(uv2[:d], uv0[:d]) and not np.allclose(uv2[d:], uv0[d:])
