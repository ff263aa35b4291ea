"""GPU graph construction (Algorithm 3) against the construction oracle, through the C ABI.

Integer-valued embeddings make every inner product exact in fp32 whatever the order of summation, so the device and
the oracle must agree edge for edge (and there are many equal similarities, which exercises the tie rules).  On
real-valued embeddings the two may part at a rounding-level tie (the construction is a heuristic whose later steps
depend on earlier ones); there the graph's promises and its quality are compared.
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
    cfg = li.TINY
    c = L.leann_create(cfg, to_dev(li.encoder_weights(cfg, 1)))
    yield c
    L.leann_destroy(c)


def gpu_csr(rp, ci):
    return rp.cpu().numpy().view(np.uint64), ci.cpu().numpy().view(np.uint32)


@pytest.mark.parametrize("n,batch,ramp,hubs", [(300, 1, 1, False), (300, 1, 1, True), (301, 8, 2, True),
                                                (700, 256, 8, False), (3000, 1024, 2, True), (257, 32, 1, True)])
def test_construction_identical_on_exact_arithmetic(L, orc, ctx, n, batch, ramp, hubs):
    rng = np.random.default_rng(n + batch)
    d, efC, M, m = 8, 24, 8, 3
    emb = rng.integers(-5, 6, size=(n, d)).astype(np.float32)
    is_hub = (rng.random(n) < 0.1).astype(np.uint8) if hubs else None
    say(f"build n={n} batch={batch} ramp={ramp} hubs={hubs}")
    rp, ci = L.leann_build_graph(ctx, to_dev(emb), efC, M, m if hubs else M, to_dev(is_hub) if hubs else None, batch, ramp)
    rp, ci = gpu_csr(rp, ci)
    want_rp, want_ci, st = orc.build_graph(emb, efC, M, m if hubs else M, is_hub, batch, ramp)
    np.testing.assert_array_equal(rp, want_rp)
    np.testing.assert_array_equal(ci, want_ci)
    assert len(ci) == st["edges"]


def test_top_degree_matches_oracle(L, orc, ctx):
    rng = np.random.default_rng(0)
    emb = rng.integers(-5, 6, size=(500, 8)).astype(np.float32)
    rp, ci = L.leann_build_graph(ctx, to_dev(emb), 24, 8, batch=16, ramp=2)
    for beta in (0.0, 0.02, 0.1, 0.5, 1.0):
        got = L.leann_top_degree(ctx, rp, beta).cpu().numpy()
        np.testing.assert_array_equal(got, orc.top_degree(rp.cpu().numpy().view(np.uint64), beta))


def test_real_valued_corpus_promises_and_quality(L, orc, ctx):
    """Clustered unit vectors: degree caps, forward-edge caps, edge count close to the oracle's, and Algorithm 1 on
    the device-built graph finds the exact neighbours as well as on the oracle-built one."""
    rng = np.random.default_rng(5)
    n, d, efC, M, m = 2500, 128, 48, 16, 4  # d = the context's hidden size (the search checks it)
    cent = rng.standard_normal((40, d))
    emb = cent[rng.integers(0, 40, n)] + 0.7 * rng.standard_normal((n, d))
    emb = (emb / np.linalg.norm(emb, axis=1, keepdims=True)).astype(np.float32)
    say("real-valued build, sequential and batched, with hubs")
    rp0, _ = L.leann_build_graph(ctx, to_dev(emb), efC, M, batch=64, ramp=8)
    is_hub = L.leann_top_degree(ctx, rp0, 0.02)
    want0 = orc.build_graph(emb, efC, M, batch=64, ramp=8)
    hub_o = orc.top_degree(want0[0], 0.02)
    graphs = {}
    for name, batch in (("sequential", 1), ("batched", 64)):
        rp, ci = gpu_csr(*L.leann_build_graph(ctx, to_dev(emb), efC, M, m, is_hub, batch, 8))
        flags = is_hub.cpu().numpy()
        deg = np.diff(rp.astype(np.int64))
        assert deg.max() <= M
        for v in range(n):
            nb = ci[int(rp[v]):int(rp[v + 1])]
            assert len(set(nb.tolist())) == len(nb) and v not in nb and (nb < n).all()
            assert (nb < v).sum() <= (M if flags[v] else m)
        o_rp, o_ci, o_st = orc.build_graph(emb, efC, M, m, hub_o, batch, 8)
        assert abs(len(ci) - o_st["edges"]) <= 0.02 * o_st["edges"]
        graphs[name] = ((rp, ci), (o_rp, o_ci))
    # quality: exact-distance search (alpha = 1, stored embeddings for every node) on both graphs
    cb, _ = orc.pq_train(emb, 8, 4, 1)
    codes = orc.pq_encode(emb, cb)
    pq = L.leann_pq_import(ctx, cb, codes)
    try:
        import torch
        q = emb[rng.integers(0, n, 64)] + 0.1 * rng.standard_normal((64, d)).astype(np.float32)
        q = (q / np.linalg.norm(q, axis=1, keepdims=True)).astype(np.float32)
        truth = np.argsort(-(q @ emb.T), axis=1)[:, :3]
        cache = (to_dev(np.arange(n, dtype=np.int32)), to_dev(emb))
        tokens = to_dev(np.ones((n, 4), np.int32))
        lengths = to_dev(np.full(n, 4, np.int32))
        for name, (dev_g, orc_g) in graphs.items():
            rec = []
            for rp, ci in (dev_g, orc_g):
                ids, _, _ = L.leann_search(ctx, to_dev(q), (to_dev(rp), to_dev(ci), 0), pq, tokens, lengths, 32, 3, 1.0, 1,
                                           cache=cache)
                ids = ids.cpu().numpy()
                rec.append(np.mean([len(set(ids[i]) & set(truth[i])) / 3 for i in range(len(q))]))
            print(f"{name}: recall@3 at ef=32 device-built {rec[0]:.3f}, oracle-built {rec[1]:.3f}")
            assert rec[0] >= 0.9 and rec[0] >= rec[1] - 0.03
    finally:
        L.leann_pq_free(pq)


def test_argument_checks(L, ctx):
    emb = to_dev(np.ones((10, 4), np.float32))
    for kw in (dict(efC=0, M=4), dict(efC=300, M=4), dict(efC=8, M=65), dict(efC=8, M=4, m=5),
               dict(efC=8, M=4, batch=1025), dict(efC=8, M=4, ramp=0)):
        with pytest.raises(L.LeannError) as ei:
            L.leann_build_graph(ctx, emb, **kw)
        assert ei.value.status == -1
