"""GPU parity: leann_adc / leann_build_pq / PQ import-export against the PQ oracle.

ADC bound (spec: 1e-4 relative): |gpu - oracle| <= 1e-4 * |oracle| (every term of the sum has the same
sign, so the sum's own magnitude is its forward-error scale).  k-means itself is not compared bit for bit (Lloyd iterations amplify rounding); the built table
is judged by its invariants and by its quantisation error against the oracle's.
"""
import numpy as np
import pytest

import leann_inputs as li
from gpu_util import say, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def L():
    import paper_2506_08276_amd as L
    L.load_library()
    return L


@pytest.fixture(scope="module")
def ctx(L):
    c = L.leann_create(li.TINY, to_dev(li.encoder_weights(li.TINY, 1)))
    yield c
    L.leann_destroy(c)


def unit_rows(n, d, seed, clusters=20):
    rng = np.random.default_rng(seed)
    cent = rng.standard_normal((clusters, d))
    x = cent[rng.integers(0, clusters, n)] + 0.4 * rng.standard_normal((n, d))
    return (x / np.linalg.norm(x, axis=1, keepdims=True)).astype(np.float32)


@pytest.mark.parametrize("d,m_sub,n,nc", [(128, 16, 3000, 77), (768, 32, 5000, 1500), (64, 4, 300, 1)])
def test_adc_matches_oracle(L, orc, ctx, d, m_sub, n, nc):
    say(f"adc d={d} m_sub={m_sub} n={n} nc={nc}")
    x = unit_rows(n, d, 3)
    cb, _ = orc.pq_train(x, m_sub, 3, 5)
    codes = orc.pq_encode(x, cb)
    pq = L.leann_pq_import(ctx, cb, codes)
    rng = np.random.default_rng(4)
    nq = 9
    queries = unit_rows(nq, d, 6)
    cand = rng.integers(0, n, size=(nq, nc)).astype(np.uint32)
    cand[0, 0], cand[-1, -1] = 0, n - 1
    got = L.leann_adc(ctx, to_dev(queries), pq, to_dev(cand)).cpu().numpy()
    for qi in range(nq):
        want, l1 = orc.adc(orc.lut(queries[qi], cb), codes, cand[qi])
        assert np.all(np.abs(got[qi] - want) <= 1e-4 * np.maximum(np.abs(want), l1))
    cb2, codes2 = L.leann_pq_export(ctx, pq)
    assert np.array_equal(cb2, cb) and np.array_equal(codes2, codes)
    assert L.leann_pq_info(pq) == (n, d, m_sub)
    # wrapped device-resident codes give the same scores
    import torch
    codes_dev = to_dev(codes)
    pq_w = L.leann_pq_wrap(ctx, cb, codes_dev)
    got_w = L.leann_adc(ctx, to_dev(queries), pq_w, to_dev(cand))
    assert torch.equal(got_w.cpu(), torch.from_numpy(got))
    L.leann_pq_free(pq_w)
    # an id outside the table is reported
    cand[2, 0] = n
    with pytest.raises(L.LeannError):
        L.leann_adc(ctx, to_dev(queries), pq, to_dev(cand))
    L.leann_pq_free(pq)


@pytest.mark.parametrize("m_sub,d", [(32, 768), (16, 128)])
def test_adc_many_queries_several_rounds_per_block(L, orc, ctx, m_sub, d):
    """Launch shapes in which a block of the scorer goes through several rounds of 2048 candidates with its lookup
    table kept in LDS, and a query's candidates are split over several blocks (9000 queries x 4100 candidates: two
    blocks per query, two rounds in the first, a ragged one in the second): sampled queries against the oracle, and
    the whole result against the same candidates scored 1500 at a time (one round per block)."""
    import torch
    n, nq, nc = 5000, 9000, 4100
    say(f"adc multi-round d={d} m_sub={m_sub} nq={nq} nc={nc}")
    x = unit_rows(n, d, 3)
    cb, _ = orc.pq_train(x, m_sub, 2, 5)
    codes = orc.pq_encode(x, cb)
    pq = L.leann_pq_import(ctx, cb, codes)
    queries = unit_rows(nq, d, 8)
    g = torch.Generator(device="cpu").manual_seed(5)
    cand = torch.randint(0, n, (nq, nc), dtype=torch.int32, generator=g)
    qd, cd = to_dev(queries), cand.to("cuda:0")
    got = L.leann_adc(ctx, qd, pq, cd)
    for s0 in range(0, nc, 1500):
        part = L.leann_adc(ctx, qd, pq, cd[:, s0:s0 + 1500].contiguous())
        assert torch.equal(got[:, s0:s0 + 1500], part), s0
    got = got.cpu().numpy()
    cand = cand.numpy().view(np.uint32)
    for qi in (0, 4499, 8999):
        want, l1 = orc.adc(orc.lut(queries[qi], cb), codes, cand[qi])
        assert np.all(np.abs(got[qi] - want) <= 1e-4 * np.maximum(np.abs(want), l1))
    L.leann_pq_free(pq)


@pytest.mark.parametrize("n,d,m_sub,iters", [(2000, 128, 16, 10), (70000, 48, 2, 3)])
def test_build_pq_invariants_and_error(L, orc, ctx, n, d, m_sub, iters):
    say(f"build_pq n={n} d={d} m_sub={m_sub} iters={iters}")
    x = unit_rows(n, d, 11, clusters=300)
    pq = L.leann_build_pq(ctx, to_dev(x), m_sub, iters, 99)
    cb, codes = L.leann_pq_export(ctx, pq)
    L.leann_pq_free(pq)
    assert cb.shape == (m_sub, 256, d // m_sub) and codes.shape == (n, m_sub) and np.isfinite(cb).all()
    dsub = d // m_sub
    sample = np.random.default_rng(0).choice(n, 500, replace=False)
    err_gpu = 0.0
    for m in range(m_sub):
        sub = x[sample, m * dsub:(m + 1) * dsub].astype(np.float64)
        dist = ((sub[:, None, :] - cb[m][None].astype(np.float64)) ** 2).sum(-1)
        chosen = dist[np.arange(len(sample)), codes[sample, m]]
        assert np.all(chosen <= dist.min(1) + 1e-5)  # every code is a true arg-min of its own codebook
        err_gpu += chosen.sum()
    cb_o, _ = orc.pq_train(x, m_sub, iters, 99)
    dec_o = orc.pq_decode(orc.pq_encode(x[sample], cb_o), cb_o)
    err_orc = ((dec_o.astype(np.float64) - x[sample]) ** 2).sum()
    assert abs(err_gpu - err_orc) <= 0.01 * err_orc  # quantisation error within 1 % of the oracle's
    # same seed, same permutation: the first Lloyd step starts from the same rows, so with iters small and
    # well separated data most centroids agree closely
    close = np.isclose(cb, cb_o, atol=1e-3).all(-1).mean()
    print(f"centroids agreeing with the oracle's to 1e-3: {close:.3f}")
    assert close > 0.5


def test_build_pq_rejects_bad_shapes(L, ctx):
    say("build_pq bad shapes")
    x = to_dev(np.zeros((10, 130), np.float32))
    with pytest.raises(L.LeannError):
        L.leann_build_pq(ctx, x, 4, 1, 0)      # 130 % 4 != 0
    with pytest.raises(L.LeannError):
        L.leann_build_pq(ctx, x, 2, 1, 0)      # sub-vector longer than 32
