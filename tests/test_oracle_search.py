"""Pins for the search oracle (CPU only).

Algorithm 2 + dynamic batching is an order-dependent heuristic; the paper prints
no worked example, so the oracle is pinned by a hand trace
(tests/golden/search_trace.txt), by its reduction to an independently written
Algorithm 1 at alpha = 1 / batch = 1, by brute-force exact top-k (Eq. 1) when
ef >= N on a strongly connected graph, and by invariants of the queues.
"""
import math
import os

import numpy as np
import pytest

import leann_inputs as li

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- fixtures
def unit(x):
    return (x / np.linalg.norm(x, axis=1, keepdims=True)).astype(np.float32)


def clustered(n, d, seed, clusters=12):
    rng = np.random.default_rng(seed)
    cent = rng.standard_normal((clusters, d))
    return unit(cent[rng.integers(0, clusters, n)] + 0.5 * rng.standard_normal((n, d)))


@pytest.fixture(scope="module")
def world(orc):
    n, d, deg = 400, 16, 8
    table = clustered(n, d, 1)
    nbr, _ = li.knn_graph(table, deg)
    entry, _ = li.max_in_degree_node(nbr)
    row_ptr, col_idx = li.to_csr(li.add_ring(list(nbr)))
    cb, _ = orc.pq_train(table, 4, 6, 5)
    codes = orc.pq_encode(table, cb)
    rng = np.random.default_rng(2)
    queries = unit(table[rng.integers(0, n, 12)] + 0.2 * rng.standard_normal((12, d)))
    return dict(n=n, d=d, table=table, row_ptr=row_ptr, col_idx=col_idx, entry=entry, cb=cb, codes=codes,
                queries=queries)


def brute_topk(q, table, k):
    s = table.astype(np.float32) @ q.astype(np.float32)
    order = np.lexsort((np.arange(len(s)), -s))[:k]
    return order, s[order]


def best_first_alg1(q, table, row_ptr, col_idx, entry, ef, k):
    """Algorithm 1 written independently of the oracle: sorted Python list, exact distance for every neighbour."""
    score = lambda v: float(np.float32(np.dot(table[v].astype(np.float32), q.astype(np.float32))))
    key = lambda t: (-t[0], t[1])
    cand = [(score(entry), entry)]          # the bounded queue C
    visited, computed, order = set(), {entry}, []
    while True:
        todo = [t for t in sorted(cand, key=key) if t[1] not in visited]
        if not todo:
            break
        u = todo[0][1]
        visited.add(u)
        order.append(u)
        for v in col_idx[int(row_ptr[u]):int(row_ptr[u + 1])]:
            v = int(v)
            if v in computed:
                continue
            computed.add(v)
            cand.append((score(v), v))
            cand.sort(key=key)
            del cand[ef:]
    return [t[1] for t in sorted(cand, key=key)[:k]], order, computed


# ---------------------------------------------------------------- golden trace
def load_trace():
    cases = []
    for line in open(os.path.join(GOLD, "search_trace.txt")):
        if line.startswith("#") or not line.strip():
            continue
        f = dict(t.split("=") for t in line.split())
        cases.append(f)
    return cases


@pytest.mark.parametrize("case", load_trace(), ids=lambda c: c["case"])
def test_hand_traced_example(orc, case):
    exact = [0.10, 0.50, 0.30, 0.70, 0.90, 0.40, 0.20]
    approx = [0.0, 0.45, 0.60, 0.20, 0.80, 0.40, 0.10]
    table = np.array([[x, 0.5] for x in exact], np.float32)
    cb = np.zeros((1, 256, 2), np.float32)
    cb[0, :7, 0] = approx
    cb[0, :7, 1] = 3.0                     # same offset for every node: ADC order = order of the first coordinate
    codes = np.arange(7, dtype=np.uint8).reshape(7, 1)
    adj = [[1, 2, 3], [4, 0], [5, 6], [4], [3], [], []]
    row_ptr, col_idx = li.to_csr([np.array(a, np.int64) for a in adj])
    r = orc.search_table(np.array([1.0, 0.0], np.float32), row_ptr, col_idx, 0, cb, codes, table, ef=3, k=2,
                         alpha=0.5, batch=int(case["batch"]), alpha_mode=int(case["alpha_mode"]))
    ints = lambda s: [int(t) for t in s.split(",")]
    assert list(r["ids"]) == ints(case["ids"])
    st = r["stats"]
    assert [st["hops"], st["adc_candidates"], st["recomputed"], st["flushes"]] == ints(case["stats"])
    assert list(r["visit_order"]) == ints(case["visit"])
    assert list(r["log_ids"]) == ints(case["log"])
    np.testing.assert_allclose(r["scores"], [exact[i] for i in ints(case["ids"])], atol=1e-7)


# ---------------------------------------------------------------- reductions
def test_alpha_one_batch_one_is_algorithm_1(orc, world):
    w = world
    for q in w["queries"]:
        for ef in (4, 16):
            r = orc.search_table(q, w["row_ptr"], w["col_idx"], w["entry"], w["cb"], w["codes"], w["table"],
                                 ef=ef, k=3, alpha=1.0, batch=1)
            ids, order, computed = best_first_alg1(q, w["table"], w["row_ptr"], w["col_idx"], w["entry"], ef, 3)
            assert list(r["ids"]) == ids
            assert list(r["visit_order"]) == order
            assert set(r["log_ids"]) == computed
            assert r["stats"]["recomputed"] == len(computed) == r["stats"]["adc_candidates"] + 1


def test_ef_at_least_n_gives_exact_topk(orc, world):
    w = world
    for q in w["queries"][:6]:
        for alpha_mode in (0, 1):
            r = orc.search_table(q, w["row_ptr"], w["col_idx"], w["entry"], w["cb"], w["codes"], w["table"],
                                 ef=w["n"], k=5, alpha=1.0, batch=7, alpha_mode=alpha_mode)
            ids, sc = brute_topk(q, w["table"], 5)
            assert list(r["ids"]) == list(ids)
            np.testing.assert_allclose(r["scores"], sc, atol=1e-6)
            assert r["stats"]["recomputed"] == w["n"]  # every node scored exactly once


def test_equal_scores_are_ordered_by_id(orc):
    """The total order is (score descending, id ascending): with duplicated vectors (integer coordinates, so equal
    vectors give bit-equal scores) every tie has to come out lower id first, in the result and in the queue rule."""
    rng = np.random.default_rng(4)
    base = rng.integers(-3, 4, size=(40, 8)).astype(np.float32)
    table = base[rng.integers(0, 40, 160)]                      # every vector about four times
    n, d = table.shape
    nbr, _ = li.knn_graph(table, 6)
    row_ptr, col_idx = li.to_csr(li.add_ring(list(nbr)))
    cb, _ = orc.pq_train(table, 2, 3, 1, ksub=16)
    codes = orc.pq_encode(table, cb)
    for qi in range(5):
        q = base[qi] + 0.0
        r = orc.search_table(q, row_ptr, col_idx, 0, cb, codes, table, ef=n, k=12, alpha=1.0, batch=5)
        s = table @ q
        want = np.lexsort((np.arange(n), -s))[:12]              # written out: score descending, then id ascending
        assert list(r["ids"]) == list(want)
        assert len(set(s[want].tolist())) < 12                  # the case does contain ties
        # a short queue: the tail of EQ is decided by the same rule
        r2 = orc.search_table(q, row_ptr, col_idx, 0, cb, codes, table, ef=6, k=6, alpha=1.0, batch=1)
        order = np.lexsort((r2["log_ids"], -r2["log_scores"].astype(np.float64)))[:6]
        assert list(r2["ids"]) == list(r2["log_ids"][order])


def test_exact_topk_is_brute_force(orc, world):
    w = world
    for q in w["queries"][:4]:
        ids, sc = orc.exact_topk(q, w["table"], 7)
        want, wsc = brute_topk(q, w["table"], 7)
        assert list(ids) == list(want)
        np.testing.assert_allclose(sc, wsc, atol=1e-6)
    ids, sc = orc.exact_topk(w["queries"][0], w["table"][:2], 4)
    assert list(ids[2:]) == [-1, -1] and np.all(np.isinf(sc[2:]))


# ---------------------------------------------------------------- invariants
@pytest.mark.parametrize("alpha,batch", [(0.2, 1), (0.2, 8), (0.5, 32), (0.1, 1000), (1.0, 16)])
def test_queue_invariants(orc, world, alpha, batch):
    w = world
    for q in w["queries"]:
        r = orc.search_table(q, w["row_ptr"], w["col_idx"], w["entry"], w["cb"], w["codes"], w["table"],
                             ef=12, k=3, alpha=alpha, batch=batch)
        log_ids, log_sc = r["log_ids"], r["log_scores"]
        # no chunk is recomputed twice; the entry point is the first
        assert len(set(log_ids)) == len(log_ids) and log_ids[0] == w["entry"]
        assert r["stats"]["recomputed"] == len(log_ids)
        # logged scores are the true inner products
        np.testing.assert_allclose(log_sc, w["table"][log_ids] @ q, atol=1e-6)
        # result = top-k of everything scored exactly (ef >= k)
        order = np.lexsort((log_ids, -log_sc))[:3]
        assert list(r["ids"]) == list(log_ids[order])
        # every recomputed node other than the entry point was ADC-scored, i.e. is a neighbour of a visited node
        reach = set()
        for u in r["visit_order"]:
            reach.update(int(v) for v in w["col_idx"][int(w["row_ptr"][u]):int(w["row_ptr"][u + 1])])
        assert set(log_ids[1:]) <= reach
        # visited nodes were in the exact queue, hence scored exactly
        assert set(r["visit_order"]) <= set(log_ids)
        assert r["stats"]["hops"] == len(r["visit_order"]) == len(set(r["visit_order"]))
        assert r["stats"]["adc_candidates"] == len(reach - {w["entry"]})
        # a flush holds fewer than batch + max-degree chunks
        assert r["stats"]["flushes"] >= math.ceil(len(log_ids) / (batch + 9))


def test_selection_count_per_hop(orc, world):
    """batch = 1: each flush after the first holds exactly ceil(alpha * new) chunks, best ADC first."""
    w = world
    q = w["queries"][3]
    alpha = 0.3
    r = orc.search_table(q, w["row_ptr"], w["col_idx"], w["entry"], w["cb"], w["codes"], w["table"],
                         ef=10, k=3, alpha=alpha, batch=1)
    seen, aq, pos = {w["entry"]}, {}, 1
    lut = orc.lut(q, w["cb"])
    for u in r["visit_order"]:
        new = []
        for v in w["col_idx"][int(w["row_ptr"][u]):int(w["row_ptr"][u + 1])]:
            if int(v) not in seen:
                seen.add(int(v))
                new.append(int(v))
        if new:
            s, _ = orc.adc(lut, w["codes"], np.array(new, np.uint32))
            aq.update(dict(zip(new, s)))
        take = min(int(np.ceil(np.float32(alpha) * np.float32(len(new)))), len(aq))
        best = sorted(aq, key=lambda v: (-aq[v], v))[:take]
        assert list(r["log_ids"][pos:pos + take]) == best
        for v in best:
            del aq[v]
        pos += take
    assert pos == len(r["log_ids"])


def test_trends_recompute_and_recall(orc, world):
    """Fewer recomputations at smaller alpha; recall does not drop as ef grows (averages, Sec. 2 / Sec. 7)."""
    w = world

    def run(alpha, ef):
        rec, hit = 0, 0
        for q in w["queries"]:
            r = orc.search_table(q, w["row_ptr"], w["col_idx"], w["entry"], w["cb"], w["codes"], w["table"],
                                 ef=ef, k=3, alpha=alpha, batch=8)
            rec += r["stats"]["recomputed"]
            hit += len(set(r["ids"]) & set(brute_topk(q, w["table"], 3)[0]))
        return rec / len(w["queries"]), hit / (3 * len(w["queries"]))

    r_small, _ = run(0.2, 16)
    r_full, _ = run(1.0, 16)
    assert r_small < r_full
    recalls = [run(0.5, ef)[1] for ef in (3, 8, 32, 128)]
    assert recalls[-1] >= recalls[0] and recalls[-1] >= 0.9


def test_huge_batch_terminates_and_duplicates_tolerated(orc, world):
    w = world
    col = w["col_idx"].copy()
    col[1] = col[0]  # duplicate neighbour id in node 0's list
    r = orc.search_table(w["queries"][0], w["row_ptr"], col, w["entry"], w["cb"], w["codes"], w["table"],
                         ef=8, k=3, alpha=0.5, batch=10 ** 6)
    assert len(set(r["log_ids"])) == len(r["log_ids"])
    assert r["stats"]["flushes"] >= 2


def test_fewer_than_k_reachable_pads(orc):
    table = unit(np.random.default_rng(0).standard_normal((5, 4)))
    row_ptr, col_idx = li.to_csr([np.array([1]), np.array([0]), np.array([]), np.array([]), np.array([])])
    cb = np.zeros((1, 256, 4), np.float32)
    codes = np.zeros((5, 1), np.uint8)
    r = orc.search_table(table[0], row_ptr, col_idx, 0, cb, codes, table, ef=4, k=3, alpha=1.0, batch=2)
    assert list(r["ids"][:2]) == [0, 1] and r["ids"][2] == -1 and np.isinf(r["scores"][2])


def test_argument_checks(orc, world):
    w = world
    args = (w["queries"][0], w["row_ptr"], w["col_idx"], w["entry"], w["cb"], w["codes"], w["table"])
    for kw in (dict(ef=2, k=3, alpha=0.5, batch=1), dict(ef=4, k=3, alpha=0.0, batch=1),
               dict(ef=4, k=3, alpha=1.5, batch=1), dict(ef=4, k=3, alpha=0.5, batch=0)):
        with pytest.raises(RuntimeError):
            orc.search_table(*args, **kw)


def test_search_with_true_recomputation_equals_table_lookup(orc):
    """The encoder-backed search and the table-backed search agree (batch-composition invariance)."""
    cfg = dict(layers=1, hidden=16, heads=2, ffn=32, vocab=60, max_pos=8, ln_eps=1e-12)
    e = orc.desc(**cfg)
    w = li.encoder_weights(cfg, 3, std=0.4)
    tokens, lengths = li.uniform_chunks(80, 8, 1, 60, 2, 8, 4)
    table = orc.embed(e, w, tokens, lengths)
    nbr, _ = li.knn_graph(table, 6)
    entry, _ = li.max_in_degree_node(nbr)
    row_ptr, col_idx = li.to_csr(nbr)
    cb, _ = orc.pq_train(table, 4, 4, 1)
    codes = orc.pq_encode(table, cb)
    for qi in (5, 17):
        a = orc.search_table(table[qi], row_ptr, col_idx, entry, cb, codes, table, ef=8, k=3, alpha=0.3, batch=4)
        b = orc.search_encoder(table[qi], row_ptr, col_idx, entry, cb, codes, e, w, tokens, lengths, ef=8, k=3,
                               alpha=0.3, batch=4)
        assert list(a["ids"]) == list(b["ids"]) and a["stats"] == b["stats"]
        assert np.array_equal(a["scores"], b["scores"])


# ---------------------------------------------------------------- pending updates (App. B)
def top_ef_of_log(r, ef):
    """The exact queue at the end of a search = the best ef of everything exactly scored (score desc, id asc)."""
    order = np.lexsort((r["log_ids"], -r["log_scores"].astype(np.float64)))[:ef]
    return r["log_ids"][order], r["log_scores"][order]


def test_soft_delete_filters_the_exact_queue_not_the_traversal(orc, world):
    w, ef, k = world, 24, 5
    rng = np.random.default_rng(11)
    for qi, q in enumerate(w["queries"][:6]):
        plain = orc.search_table(q, w["row_ptr"], w["col_idx"], w["entry"], w["cb"], w["codes"], w["table"], ef, k, 0.3, 4)
        deleted = np.zeros(w["n"], np.uint8)
        deleted[plain["ids"][[0, 2]]] = 1                       # two of the answers ...
        deleted[rng.integers(0, w["n"], 40)] = 1                # ... and a random 10 %
        r = orc.search_table(q, w["row_ptr"], w["col_idx"], w["entry"], w["cb"], w["codes"], w["table"], ef, k, 0.3, 4,
                             deleted=deleted)
        # deleted nodes are still traversed: the trajectory and every count are those of the plain search
        assert list(r["visit_order"]) == list(plain["visit_order"]) and list(r["log_ids"]) == list(plain["log_ids"])
        assert r["stats"] == plain["stats"]
        # the answer is the exact queue without the flagged nodes, first k (written out independently)
        eq_ids, eq_sc = top_ef_of_log(plain, ef)
        keep = [i for i in range(len(eq_ids)) if not deleted[eq_ids[i]]][:k]
        want = list(eq_ids[keep]) + [-1] * (k - len(keep))
        assert list(r["ids"]) == want and not any(deleted[i] for i in r["ids"] if i >= 0)
        np.testing.assert_array_equal(r["scores"][:len(keep)], eq_sc[keep])
    # everything deleted: nothing to return
    r = orc.search_table(w["queries"][0], w["row_ptr"], w["col_idx"], w["entry"], w["cb"], w["codes"], w["table"], ef, k,
                         0.3, 4, deleted=np.ones(w["n"], np.uint8))
    assert list(r["ids"]) == [-1] * k and np.all(np.isneginf(r["scores"]))


def test_add_buffer_is_scanned_and_merged(orc, world):
    w, ef, k = world, 24, 5
    rng = np.random.default_rng(12)
    nb = 30
    buf_ids = np.arange(w["n"], w["n"] + nb, dtype=np.int64)
    for qi, q in enumerate(w["queries"][:6]):
        # buffered chunks: a few near the query (they must surface), the rest random
        near = unit(q[None, :] + 0.15 * rng.standard_normal((4, w["d"])))
        buf = np.concatenate([near, unit(rng.standard_normal((nb - 4, w["d"])))]).astype(np.float32)
        plain = orc.search_table(q, w["row_ptr"], w["col_idx"], w["entry"], w["cb"], w["codes"], w["table"], ef, k, 0.3, 4)
        r = orc.search_table(q, w["row_ptr"], w["col_idx"], w["entry"], w["cb"], w["codes"], w["table"], ef, k, 0.3, 4,
                             buffer=(buf_ids, buf))
        assert list(r["visit_order"]) == list(plain["visit_order"]) and r["stats"] == plain["stats"]
        # brute force over (exact queue) U (buffer), written out independently
        eq_ids, eq_sc = top_ef_of_log(plain, ef)
        bs = np.array([np.float32(sum(np.float32(a) * np.float32(b) for a, b in zip(q, e))) for e in buf], np.float32)
        ids = np.concatenate([eq_ids, buf_ids])
        sc = np.concatenate([eq_sc, bs])
        order = np.lexsort((ids, -sc.astype(np.float64)))[:k]
        assert list(r["ids"]) == list(ids[order])
        np.testing.assert_allclose(r["scores"], sc[order], rtol=0, atol=1e-6)
        assert any(i >= w["n"] for i in r["ids"])           # the near-duplicates of the query do surface
    # both kinds of update together, and k larger than what is left
    deleted = np.ones(w["n"], np.uint8)
    r = orc.search_table(w["queries"][0], w["row_ptr"], w["col_idx"], w["entry"], w["cb"], w["codes"], w["table"], ef, k,
                         0.3, 4, deleted=deleted, buffer=(buf_ids[:3], buf[:3]))
    assert sorted(r["ids"][:3]) == list(buf_ids[:3]) and list(r["ids"][3:]) == [-1, -1]
