"""Pins for the PQ / ADC oracle (CPU only).

The paper cites product quantisation and gives only its size (Sec. 3
"Storage composition"); the oracle is the textbook definition, pinned by brute
force over decoded vectors, k-means invariants, closed-form degenerate cases and
scipy's Lloyd iteration for the one-subspace case.
"""
import numpy as np
import pytest
from scipy.cluster.vq import kmeans2

import leann_inputs as li


def data(n, d, seed, clusters=0):
    rng = np.random.default_rng(seed)
    if clusters:
        cent = rng.standard_normal((clusters, d)) * 4
        return (cent[rng.integers(0, clusters, n)] + 0.3 * rng.standard_normal((n, d))).astype(np.float32)
    return rng.standard_normal((n, d)).astype(np.float32)


def test_adc_equals_negated_squared_distance_to_decoded_vector(orc):
    x = data(600, 32, 0)
    cb, _ = orc.pq_train(x, 4, 5, 7)
    codes = orc.pq_encode(x, cb)
    dec = orc.pq_decode(codes, cb)
    q = data(3, 32, 1)
    ids = np.random.default_rng(2).integers(0, 600, 100).astype(np.uint32)
    for qi in q:
        lut = orc.lut(qi, cb)
        s, l1 = orc.adc(lut, codes, ids)
        want = -((dec[ids].astype(np.float64) - qi.astype(np.float64)) ** 2).sum(1)
        assert np.abs(s - want).max() <= 1e-6 * np.abs(want).max()
        np.testing.assert_allclose(l1, -s, rtol=1e-6)  # every term has the same sign
    # lut entries themselves: -|q_m - centroid|^2
    diff = q[0].reshape(4, 1, 8).astype(np.float64) - cb.astype(np.float64)
    np.testing.assert_allclose(orc.lut(q[0], cb), -(diff ** 2).sum(-1), rtol=1e-5, atol=1e-6)
    # sign and transposition check on a hand case: q = (1,2 | 0,0), centroid 0 of both subspaces at the origin,
    # centroid 1 of subspace 0 at (1,2)
    cb2 = np.zeros((2, 256, 2), np.float32)
    cb2[0, 1] = [1.0, 2.0]
    lut2 = orc.lut(np.array([1.0, 2.0, 0.0, 0.0], np.float32), cb2)
    assert lut2[0, 0] == -5.0 and lut2[0, 1] == 0.0 and lut2[1, 0] == 0.0
    s2, _ = orc.adc(lut2, np.array([[0, 0], [1, 0]], np.uint8), np.array([0, 1], np.uint32))
    assert list(s2) == [-5.0, 0.0]


def test_decode_layout_and_code_is_true_argmin(orc):
    x = data(500, 24, 3)
    cb, _ = orc.pq_train(x, 3, 4, 11)
    codes = orc.pq_encode(x, cb)
    dec = orc.pq_decode(codes, cb)
    for m in range(3):
        sub = x[:, m * 8:(m + 1) * 8].astype(np.float64)
        dist = ((sub[:, None, :] - cb[m][None].astype(np.float64)) ** 2).sum(-1)
        best = dist.min(1)
        chosen = dist[np.arange(500), codes[:, m]]
        assert np.all(chosen <= best + 1e-5)
        np.testing.assert_array_equal(dec[:, m * 8:(m + 1) * 8], cb[m][codes[:, m]])
    assert codes.dtype == np.uint8 and codes.shape == (500, 3)  # bytes per vector = number of subspaces


def test_objective_non_increasing(orc):
    x = data(3000, 16, 4, clusters=40)
    _, obj = orc.pq_train(x, 2, 12, 5, ksub=32)
    assert np.all(np.diff(obj) <= 1e-6 * obj[0])
    assert obj[-1] < obj[0]


def test_enough_centroids_means_zero_error(orc):
    rng = np.random.default_rng(6)
    base = rng.standard_normal((40, 16)).astype(np.float32)
    x = base[rng.integers(0, 40, 300)]
    x[:40] = base
    cb, obj = orc.pq_train(x, 2, 6, 9)  # 256 centroids >= 40 distinct points per subspace
    codes = orc.pq_encode(x, cb)
    np.testing.assert_array_equal(orc.pq_decode(codes, cb), x)
    q = rng.standard_normal(16).astype(np.float32)
    s, _ = orc.adc(orc.lut(q, cb), codes, np.arange(300, dtype=np.uint32))
    np.testing.assert_allclose(s, -((x.astype(np.float64) - q.astype(np.float64)) ** 2).sum(1), rtol=1e-5)
    # for unit vectors the ADC score is then 2<q,x> - 2: the same ranking as the inner product
    xu = x / np.linalg.norm(x, axis=1, keepdims=True)
    qu = q / np.linalg.norm(q)
    cbu, _ = orc.pq_train(xu, 2, 6, 9)
    su, _ = orc.adc(orc.lut(qu, cbu), orc.pq_encode(xu, cbu), np.arange(300, dtype=np.uint32))
    np.testing.assert_allclose(su, 2 * (xu.astype(np.float64) @ qu.astype(np.float64)) - 2, atol=1e-5)


def test_single_centroid_is_the_mean(orc):
    x = data(1000, 12, 7)
    cb, _ = orc.pq_train(x, 3, 3, 1, ksub=1)
    np.testing.assert_allclose(cb.reshape(-1), x.astype(np.float64).mean(0), atol=1e-6)


def test_one_subspace_matches_scipy_lloyd(orc):
    x = data(2000, 8, 8, clusters=16)
    iters, k = 6, 16
    perm = orc.permutation(2000, 123)
    init = x[perm[:k]].astype(np.float64)
    cb, _ = orc.pq_train(x, 1, iters, 123, ksub=k)
    want, _ = kmeans2(x.astype(np.float64), init, iter=iters, minit="matrix", missing="raise")
    np.testing.assert_allclose(cb[0], want, atol=1e-4)


def test_permutation_is_a_seeded_permutation(orc):
    p = orc.permutation(1000, 42)
    assert np.array_equal(np.sort(p), np.arange(1000))
    assert np.array_equal(p, orc.permutation(1000, 42))
    assert not np.array_equal(p, orc.permutation(1000, 43))
    # splitmix64 reference output for state 0 (published test vector): first draw 0xE220A8397B1DCDAF
    # i = 1 of a 2-element shuffle uses that draw: j = draw mod 2 = 1 -> identity
    assert np.array_equal(orc.permutation(2, 0), np.array([0, 1]))


def test_permutation_sequence_against_the_published_generator_outputs(orc):
    """The whole sequence, not only its first draw: the generator's published outputs for state 1234567 (the test
    vector that accompanies the public-domain splitmix64 reference code) drive a textbook Fisher-Yates shuffle of six
    elements written out here (i from n-1 down to 1, j = draw mod (i+1), the draws in the order the generator yields
    them); the oracle must return that permutation.  A different draw order, modulus or loop direction fails."""
    draws = [6457827717110365317, 3203168211198807973, 9817491932198370423, 4593380528125082431, 16408922859458223821]
    want = list(range(6))
    for i, dr in zip(range(5, 0, -1), draws):
        j = dr % (i + 1)
        want[i], want[j] = want[j], want[i]
    assert list(orc.permutation(6, 1234567)) == want
    assert want != list(range(6))  # the case is not the identity


def test_training_sample_is_capped(orc):
    """More rows than the training cap: still a valid codebook, built from the permutation's prefix only."""
    x = data(70000, 4, 10)
    cb, _ = orc.pq_train(x, 1, 1, 3, ksub=4)
    perm = orc.permutation(70000, 3)
    tr = x[perm[:65536]].astype(np.float64)
    init = tr[:4]
    a = ((tr[:, None] - init[None]) ** 2).sum(-1).argmin(1)
    want = np.stack([tr[a == c].mean(0) for c in range(4)])
    np.testing.assert_allclose(cb[0], want, atol=1e-5)


def test_size_accounting_matches_paper():
    """Sec. 3: PQ table ~ 4*N*dim/100 bytes; dim 768 -> ~31 B, the configurations use 32 B per vector."""
    assert abs(4 * 768 / 100 - 32) <= 2
    # Table 1: 60 M vectors -> about 2 GB of PQ codes; fp32 embeddings -> 173 GB
    assert round(60e6 * 32 / 2 ** 30, 1) == 1.8
    assert round(60e6 * 768 * 4 / 2 ** 30) in (171, 172, 173)


def test_bad_arguments(orc):
    x = data(10, 6, 0)
    with pytest.raises(RuntimeError):
        orc.pq_train(x, 4, 1, 0)  # 6 not divisible by 4
