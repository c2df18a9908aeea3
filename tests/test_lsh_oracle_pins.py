"""Pins of the LSH oracle (Sec. 4.3, Eq. 5-9, Table 3) against what the paper
prints and what the mathematics fixes; none of them re-types the oracle."""
import math
import os

import numpy as np
import pytest

import oracle

GOLD = {}
with open(os.path.join(os.path.dirname(__file__), "golden", "lsh_paper_values.txt")) as f:
    for ln in f:
        if ln.strip() and not ln.startswith("#"):
            k, v = ln.split()[:2]
            GOLD[k] = v


def unpack(sig):
    """bits of signatures by NumPy's own routine (most significant bit first)."""
    return np.unpackbits(np.asarray(sig, dtype=np.uint8), axis=-1, bitorder="big")


def test_paper_byte_example():
    bits = [int(c) for c in GOLD["byte_example_bits"]]
    assert oracle.lsh_pack_bits(bits).tolist() == [int(GOLD["byte_example_value"])]


def test_signature_bits_are_signs_of_projections():
    rng = np.random.default_rng(0)
    M = rng.standard_normal((40, 24)).astype(np.float32)
    W = rng.standard_normal((64, 24)).astype(np.float32)
    sig = oracle.lsh_sign(M, W)
    assert sig.shape == (40, 8)
    proj = M.astype(np.float64) @ W.astype(np.float64).T
    assert np.array_equal(unpack(sig), (proj > 0).astype(np.uint8))
    # the signature of a negated embedding is the complement
    assert np.array_equal(oracle.lsh_sign(-M, W), np.bitwise_not(sig))
    # scaling an embedding by a positive number does not change it (hyperplanes through the origin)
    assert np.array_equal(oracle.lsh_sign(3.5 * M, W), sig)


def test_self_and_complement_similarity():
    rng = np.random.default_rng(1)
    for nb in (1, 8, 16, 32):
        h = rng.integers(0, 256, nb, dtype=np.uint8)
        assert oracle.lsh_equal_bits(h, h) == 8 * nb                 # M_sim(h, h) = 1
        assert oracle.lsh_equal_bits(h, np.bitwise_not(h)) == 0      # M_sim(h, ~h) = 0
        g = rng.integers(0, 256, nb, dtype=np.uint8)
        eq = oracle.lsh_equal_bits(h, g)
        assert eq == oracle.lsh_equal_bits(g, h)
        hamming = int((unpack(h) != unpack(g)).sum())
        assert eq + hamming == 8 * nb


@pytest.mark.parametrize("theta", [0.2, math.pi / 3, math.pi / 2, 2.5])
def test_simhash_collision_law(theta):
    """Two vectors at angle theta agree on a random-hyperplane bit with probability 1 - theta / pi."""
    rng = np.random.default_rng(int(theta * 1000))
    d, d_bits = 32, 8192
    a = rng.standard_normal(d)
    b = rng.standard_normal(d)
    b -= a * (a @ b) / (a @ a)
    a /= np.linalg.norm(a)
    b /= np.linalg.norm(b)
    x, y = a, math.cos(theta) * a + math.sin(theta) * b
    W = rng.standard_normal((d_bits, d)).astype(np.float32)
    sig = oracle.lsh_sign(np.stack([x, y]).astype(np.float32), W)
    m = oracle.lsh_equal_bits(sig[0], sig[1]) / d_bits
    p = 1 - theta / math.pi
    assert abs(m - p) < 3 * math.sqrt(p * (1 - p) / d_bits) + 1e-3


def test_din_and_simtier_against_numpy_on_unpacked_bits():
    rng = np.random.default_rng(5)
    n_items, L, d, nb, n_tiers = 200, 77, 12, 8, 8
    table = rng.integers(0, 256, (n_items, nb), dtype=np.uint8)
    seq = rng.integers(0, 256, (L, nb), dtype=np.uint8)
    seq[:10] = table[:10]                                        # some exact matches
    seq[10:20] = np.bitwise_not(table[:10])                      # and exact opposites
    U = rng.standard_normal((L, d)).astype(np.float32)
    ids = rng.permutation(n_items)[:50].astype(np.int32)
    res = oracle.lsh_request(sig_table=table, ids=ids, seq_sig=seq, u_seq=U, n_tiers=n_tiers, want_equal=True)
    bi, bs = unpack(table[ids]).astype(np.int64), unpack(seq).astype(np.int64)
    equal = (bi[:, None, :] == bs[None, :, :]).sum(-1)           # [n, L]
    assert np.array_equal(res.equal, equal)
    msim = equal / (8 * nb)
    assert np.allclose(res.din, msim @ U.astype(np.float64), rtol=1e-13, atol=1e-13)
    tier = np.minimum(n_tiers - 1, np.floor(msim * n_tiers).astype(np.int64))
    hist = np.stack([(tier == j).sum(1) for j in range(n_tiers)], axis=1)
    assert np.array_equal(res.tiers, hist)
    assert np.all(res.tiers.sum(1) == L)


def test_din_special_cases():
    rng = np.random.default_rng(6)
    L, d, nb = 9, 5, 4
    U = rng.standard_normal((L, d)).astype(np.float32)
    h = rng.integers(0, 256, (1, nb), dtype=np.uint8)
    same = np.repeat(h, L, axis=0)
    r = oracle.lsh_request(sig_table=h, ids=[0], seq_sig=same, u_seq=U, n_tiers=4)
    assert np.allclose(r.din[0], U.astype(np.float64).sum(0), rtol=1e-14)         # all weights 1
    assert r.tiers[0].tolist() == [0, 0, 0, L]                                   # m = 1 falls in the last tier
    r = oracle.lsh_request(sig_table=h, ids=[0], seq_sig=np.bitwise_not(same), u_seq=U, n_tiers=4)
    assert np.all(r.din[0] == 0.0) and r.tiers[0].tolist() == [L, 0, 0, 0]       # all weights 0
    # one history item: a = m * U~_0
    g = h.copy()
    g[0, 0] ^= 0b00000111                                                        # three bits differ
    r = oracle.lsh_request(sig_table=h, ids=[0], seq_sig=g, u_seq=U[:1], n_tiers=4)
    assert np.allclose(r.din[0], (8 * nb - 3) / (8 * nb) * U[0].astype(np.float64), rtol=1e-14)
    # empty history
    r = oracle.lsh_request(sig_table=h, ids=[0], seq_sig=np.zeros((0, nb), np.uint8), u_seq=np.zeros((0, d), np.float32),
                           n_tiers=4)
    assert np.all(r.din == 0) and np.all(r.tiers == 0)


def test_tier_edges():
    # d' = 64, N = 8: tier j holds 8 j <= equal < 8 j + 8, the last one also equal = 64
    eq = np.arange(65, dtype=np.int32)
    t = oracle.simtier(eq, 64, 8)
    assert t.tolist() == [8, 8, 8, 8, 8, 8, 8, 9]
    # N that does not divide d': tier(m) = floor(m N) still
    t = oracle.simtier(eq, 64, 5)
    ref = np.bincount(np.minimum(4, (eq * 5) // 64), minlength=5)
    assert t.tolist() == ref.tolist()


def test_out_of_range_id_is_an_error():
    h = np.zeros((3, 8), np.uint8)
    with pytest.raises(oracle.OracleError):
        oracle.lsh_request(sig_table=h, ids=[3], seq_sig=h, u_seq=np.zeros((3, 2), np.float32), n_tiers=2)


def test_linear_form_of_lsh_din():
    """M_sim is affine in the candidate's sign vector, so Eq. 8 equals 1/2 sum_t U~_t + S_i G / (2 d') with
    G = sum_t S_t^T U~_t (S = +-1 signs): the form the GPU path uses.  Checked here against the definition."""
    rng = np.random.default_rng(8)
    n_items, L, d, nb = 50, 300, 16, 8
    table = rng.integers(0, 256, (n_items, nb), dtype=np.uint8)
    seq = rng.integers(0, 256, (L, nb), dtype=np.uint8)
    U = rng.standard_normal((L, d)).astype(np.float32)
    ids = np.arange(n_items, dtype=np.int32)
    res = oracle.lsh_request(sig_table=table, ids=ids, seq_sig=seq, u_seq=U, n_tiers=8)
    Si = 2.0 * unpack(table) - 1.0
    St = 2.0 * unpack(seq) - 1.0
    G = St.T @ U.astype(np.float64)
    lin = 0.5 * U.astype(np.float64).sum(0) + Si @ G / (2 * 8 * nb)
    assert np.allclose(res.din, lin, rtol=1e-12, atol=1e-12)


def test_table3_reductions():
    b, l, d_lsh = 1e4, 1e5, 8.0
    d_id = d_mm = 8 * d_lsh
    base = oracle.lsh_similarity_cost(b, l, [d_id, d_mm])                        # DIN + SimTier
    red = lambda widths: 1 - oracle.lsh_similarity_cost(b, l, widths) / base
    assert red([d_lsh, d_mm]) == pytest.approx(float(GOLD["reduction_lsh_din_simtier"]))
    assert red([d_id, d_lsh]) == pytest.approx(float(GOLD["reduction_din_lsh_simtier"]))
    assert red([d_mm]) == pytest.approx(float(GOLD["reduction_mm_din_simtier"]))
    assert red([d_lsh]) == pytest.approx(float(GOLD["reduction_lsh_both"]))
