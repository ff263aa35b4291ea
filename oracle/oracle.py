"""ctypes binding of oracle/leann_oracle.c (test infrastructure only).

Every function here is a thin marshalling layer over the C oracle; the
arithmetic lives in the C file, which cites the passages it follows.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# LEANN_ORACLE_SRC points the binding at another copy of the source (the test that plants mistakes in the oracle and
# checks that the pins notice uses it); the library is then built next to that copy
_SRC = os.environ.get("LEANN_ORACLE_SRC") or os.path.join(_HERE, "leann_oracle.c")
_LIB = os.path.join(os.path.dirname(_SRC), "libleann_oracle.so")
_lib = None

__all__ = [
    "build", "EncoderDesc", "desc", "weight_count", "embed", "permutation", "pq_train", "pq_encode", "pq_decode",
    "lut", "adc", "exact_topk", "search_table", "search_encoder", "search_callback", "build_graph", "top_degree", "shrink",
]


def build(force=False):
    """Compile the C oracle with gcc (-O2, no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                               "-Wall", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class EncoderDesc(C.Structure):
    _fields_ = [("layers", C.c_int32), ("hidden", C.c_int32), ("heads", C.c_int32), ("ffn", C.c_int32),
                ("vocab", C.c_int32), ("max_pos", C.c_int32), ("ln_eps", C.c_float)]


class _Stats(C.Structure):
    _fields_ = [("hops", C.c_int64), ("adc_candidates", C.c_int64), ("recomputed", C.c_int64),
                ("flushes", C.c_int64)]


_EMBED_FN = C.CFUNCTYPE(C.c_int, C.c_void_p, C.POINTER(C.c_int64), C.c_int64, C.POINTER(C.c_float))


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.orc_weight_count.restype = C.c_int64
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t)) if a is not None else None


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with status {rc}")


def desc(layers, hidden, heads, ffn, vocab, max_pos, ln_eps=1e-12):
    return EncoderDesc(layers, hidden, heads, ffn, vocab, max_pos, ln_eps)


def weight_count(e):
    return int(_load().orc_weight_count(C.byref(e)))


def embed(e, weights, tokens, lengths, ids=None, precision=0):
    """Embeddings [n_ids][d] of the chunks `ids` (all chunks when None)."""
    lib = _load()
    weights = _f32(weights)
    assert weights.size == weight_count(e), (weights.size, weight_count(e))
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    lengths = np.ascontiguousarray(lengths, dtype=np.int32)
    n, seq = tokens.shape
    if ids is not None:
        ids = np.ascontiguousarray(ids, dtype=np.int64)
    n_ids = n if ids is None else ids.size
    out = np.empty((n_ids, e.hidden), dtype=np.float32)
    rc = lib.orc_embed(C.byref(e), _p(weights, C.c_float), _p(tokens, C.c_int32), _p(lengths, C.c_int32),
                       C.c_int64(n), C.c_int32(seq), _p(ids, C.c_int64), C.c_int64(n_ids), C.c_int32(precision),
                       _p(out, C.c_float))
    _check(rc, "embed")
    return out


def permutation(n, seed):
    perm = np.empty(n, dtype=np.int64)
    _check(_load().orc_permutation(C.c_int64(n), C.c_uint64(seed), _p(perm, C.c_int64)), "permutation")
    return perm


def pq_train(x, m_sub, iters, seed, ksub=256):
    """Returns (codebook [m_sub][ksub][dsub], objective per iteration)."""
    x = _f32(x)
    n, d = x.shape
    cb = np.empty((m_sub, ksub, d // m_sub), dtype=np.float32)
    obj = np.zeros(max(iters, 1), dtype=np.float64)
    rc = _load().orc_pq_train(_p(x, C.c_float), C.c_int64(n), C.c_int32(d), C.c_int32(m_sub), C.c_int32(ksub),
                              C.c_int32(iters), C.c_uint64(seed), _p(cb, C.c_float), _p(obj, C.c_double))
    _check(rc, "pq_train")
    return cb, obj[:iters]


def pq_encode(x, codebook):
    x = _f32(x)
    codebook = _f32(codebook)
    n, d = x.shape
    m_sub, ksub, _ = codebook.shape
    codes = np.empty((n, m_sub), dtype=np.uint8)
    rc = _load().orc_pq_encode(_p(x, C.c_float), C.c_int64(n), C.c_int32(d), C.c_int32(m_sub), C.c_int32(ksub),
                               _p(codebook, C.c_float), _p(codes, C.c_uint8))
    _check(rc, "pq_encode")
    return codes


def pq_decode(codes, codebook):
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    codebook = _f32(codebook)
    m_sub, ksub, dsub = codebook.shape
    n = codes.shape[0]
    out = np.empty((n, m_sub * dsub), dtype=np.float32)
    rc = _load().orc_pq_decode(_p(codes, C.c_uint8), C.c_int64(n), C.c_int32(m_sub * dsub), C.c_int32(m_sub),
                               C.c_int32(ksub), _p(codebook, C.c_float), _p(out, C.c_float))
    _check(rc, "pq_decode")
    return out


def lut(q, codebook):
    q = _f32(q)
    codebook = _f32(codebook)
    m_sub, ksub, dsub = codebook.shape
    out = np.empty((m_sub, ksub), dtype=np.float32)
    rc = _load().orc_lut(_p(q, C.c_float), C.c_int32(q.size), C.c_int32(m_sub), C.c_int32(ksub),
                         _p(codebook, C.c_float), _p(out, C.c_float))
    _check(rc, "lut")
    return out


def adc(lut_, codes, ids):
    """Returns (similarities, l1 mass of the summed terms) for node ids."""
    lut_ = _f32(lut_)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    ids = np.ascontiguousarray(ids, dtype=np.uint32)
    m_sub, ksub = lut_.shape
    out = np.empty(ids.size, dtype=np.float32)
    l1 = np.empty(ids.size, dtype=np.float32)
    rc = _load().orc_adc(_p(lut_, C.c_float), C.c_int32(m_sub), C.c_int32(ksub), _p(codes, C.c_uint8),
                         _p(ids, C.c_uint32), C.c_int64(ids.size), _p(out, C.c_float), _p(l1, C.c_float))
    _check(rc, "adc")
    return out, l1


def exact_topk(q, table, k):
    q = _f32(q)
    table = _f32(table)
    n, d = table.shape
    ids = np.empty(k, dtype=np.int64)
    sc = np.empty(k, dtype=np.float32)
    rc = _load().orc_exact_topk(_p(q, C.c_float), _p(table, C.c_float), C.c_int64(n), C.c_int32(d), C.c_int32(k),
                                _p(ids, C.c_int64), _p(sc, C.c_float))
    _check(rc, "exact_topk")
    return ids, sc


def _graph_args(row_ptr, col_idx):
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.uint64)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.uint32)
    return row_ptr, col_idx


def _search_common(call, n, ef, k):
    out_ids = np.empty(k, dtype=np.int64)
    out_sc = np.empty(k, dtype=np.float32)
    st = _Stats()
    cap = int(n) + 1
    log_ids = np.empty(cap, dtype=np.int64)
    log_sc = np.empty(cap, dtype=np.float32)
    visit = np.empty(cap, dtype=np.int64)
    log_n = C.c_int64(0)
    visit_n = C.c_int64(0)
    rc = call(out_ids, out_sc, st, log_ids, log_sc, cap, log_n, visit, visit_n)
    _check(rc, "search")
    ln, vn = min(log_n.value, cap), min(visit_n.value, cap)
    return {
        "ids": out_ids, "scores": out_sc,
        "stats": {"hops": st.hops, "adc_candidates": st.adc_candidates, "recomputed": st.recomputed,
                  "flushes": st.flushes},
        "log_ids": log_ids[:ln].copy(), "log_scores": log_sc[:ln].copy(), "visit_order": visit[:vn].copy(),
    }


def search_table(q, row_ptr, col_idx, entry, codebook, codes, table, ef, k, alpha, batch, alpha_mode=0,
                 deleted=None, buffer=None):
    """Algorithm 2 + dynamic batching with exact embeddings looked up in `table`.
    deleted: optional uint8 flags [n] (soft-deleted nodes, filtered at the output stage);
    buffer: optional (ids int64 [nb], emb float32 [nb][d]) of added chunks that are scanned exhaustively."""
    lib = _load()
    q = _f32(q)
    table = _f32(table)
    codebook = _f32(codebook)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    row_ptr, col_idx = _graph_args(row_ptr, col_idx)
    n, d = table.shape
    m_sub = codebook.shape[0]

    if deleted is not None:
        deleted = np.ascontiguousarray(deleted, dtype=np.uint8)
        assert deleted.shape == (n,)
    buf_ids = buf_emb = None
    if buffer is not None:
        buf_ids = np.ascontiguousarray(buffer[0], dtype=np.int64)
        buf_emb = _f32(buffer[1])
        assert buf_emb.shape == (len(buf_ids), d)

    def call(out_ids, out_sc, st, log_ids, log_sc, cap, log_n, visit, visit_n):
        if deleted is not None or buffer is not None:
            return lib.orc_search_table_updates(
                _p(q, C.c_float), C.c_int32(d), _p(row_ptr, C.c_uint64), _p(col_idx, C.c_uint32), C.c_int64(n),
                C.c_uint32(entry), _p(codebook, C.c_float), _p(codes, C.c_uint8), C.c_int32(m_sub),
                _p(table, C.c_float), C.c_int32(ef), C.c_int32(k), C.c_float(alpha), C.c_int32(batch),
                C.c_int32(alpha_mode), _p(deleted, C.c_uint8) if deleted is not None else None,
                _p(buf_emb, C.c_float) if buffer is not None else None,
                _p(buf_ids, C.c_int64) if buffer is not None else None,
                C.c_int64(len(buf_ids) if buffer is not None else 0),
                _p(out_ids, C.c_int64), _p(out_sc, C.c_float), C.byref(st),
                _p(log_ids, C.c_int64), _p(log_sc, C.c_float), C.c_int64(cap), C.byref(log_n),
                _p(visit, C.c_int64), C.c_int64(cap), C.byref(visit_n))
        return lib.orc_search_table(
            _p(q, C.c_float), C.c_int32(d), _p(row_ptr, C.c_uint64), _p(col_idx, C.c_uint32), C.c_int64(n),
            C.c_uint32(entry), _p(codebook, C.c_float), _p(codes, C.c_uint8), C.c_int32(m_sub),
            _p(table, C.c_float), C.c_int32(ef), C.c_int32(k), C.c_float(alpha), C.c_int32(batch),
            C.c_int32(alpha_mode), _p(out_ids, C.c_int64), _p(out_sc, C.c_float), C.byref(st),
            _p(log_ids, C.c_int64), _p(log_sc, C.c_float), C.c_int64(cap), C.byref(log_n),
            _p(visit, C.c_int64), C.c_int64(cap), C.byref(visit_n))

    return _search_common(call, n, ef, k)


def search_callback(q, row_ptr, col_idx, n, entry, codebook, codes, embed_fn, ef, k, alpha, batch, alpha_mode=0):
    """Algorithm 2 with a Python embedder: embed_fn(ids ndarray) -> [len(ids)][d] float32."""
    lib = _load()
    q = _f32(q)
    d = q.size
    codebook = _f32(codebook)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    row_ptr, col_idx = _graph_args(row_ptr, col_idx)
    m_sub = codebook.shape[0]

    def _cb(_user, ids_p, cnt, out_p):
        ids = np.ctypeslib.as_array(ids_p, shape=(cnt,)).copy()
        res = _f32(embed_fn(ids))
        np.ctypeslib.as_array(out_p, shape=(cnt, d))[:] = res
        return 0

    cb = _EMBED_FN(_cb)

    def call(out_ids, out_sc, st, log_ids, log_sc, cap, log_n, visit, visit_n):
        return lib.orc_search(
            _p(q, C.c_float), C.c_int32(d), _p(row_ptr, C.c_uint64), _p(col_idx, C.c_uint32), C.c_int64(n),
            C.c_uint32(entry), _p(codebook, C.c_float), _p(codes, C.c_uint8), C.c_int32(m_sub), cb, None,
            C.c_int32(ef), C.c_int32(k), C.c_float(alpha), C.c_int32(batch), C.c_int32(alpha_mode),
            _p(out_ids, C.c_int64), _p(out_sc, C.c_float), C.byref(st), _p(log_ids, C.c_int64),
            _p(log_sc, C.c_float), C.c_int64(cap), C.byref(log_n), _p(visit, C.c_int64), C.c_int64(cap),
            C.byref(visit_n))

    return _search_common(call, n, ef, k)


def search_encoder(q, row_ptr, col_idx, entry, codebook, codes, e, weights, tokens, lengths, ef, k, alpha, batch,
                   precision=0, alpha_mode=0):
    """Algorithm 2 with true recomputation: each flush runs the encoder oracle."""
    lib = _load()
    q = _f32(q)
    weights = _f32(weights)
    codebook = _f32(codebook)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    lengths = np.ascontiguousarray(lengths, dtype=np.int32)
    row_ptr, col_idx = _graph_args(row_ptr, col_idx)
    n, seq = tokens.shape
    m_sub = codebook.shape[0]
    out_ids = np.empty(k, dtype=np.int64)
    out_sc = np.empty(k, dtype=np.float32)
    st = _Stats()
    rc = lib.orc_search_encoder(
        _p(q, C.c_float), _p(row_ptr, C.c_uint64), _p(col_idx, C.c_uint32), C.c_int64(n), C.c_uint32(entry),
        _p(codebook, C.c_float), _p(codes, C.c_uint8), C.c_int32(m_sub), C.byref(e), _p(weights, C.c_float),
        _p(tokens, C.c_int32), _p(lengths, C.c_int32), C.c_int32(seq), C.c_int32(precision), C.c_int32(ef),
        C.c_int32(k), C.c_float(alpha), C.c_int32(batch), C.c_int32(alpha_mode), _p(out_ids, C.c_int64),
        _p(out_sc, C.c_float), C.byref(st))
    _check(rc, "search_encoder")
    return {"ids": out_ids, "scores": out_sc,
            "stats": {"hops": st.hops, "adc_candidates": st.adc_candidates, "recomputed": st.recomputed,
                      "flushes": st.flushes}}


def build_graph(emb, efC, M, m=None, is_hub=None, batch=1, ramp=1):
    """Algorithm 3: graph construction by insertion with RNG neighbour selection; nodes flagged in is_hub (uint8 [n],
    None = all) may keep M forward edges, the others m.  Returns (row_ptr uint64 [n+1], col_idx uint32 [E], stats)."""
    emb = _f32(emb)
    n, d = emb.shape
    m = M if m is None else m
    if is_hub is not None:
        is_hub = np.ascontiguousarray(is_hub, dtype=np.uint8)
        assert is_hub.shape == (n,)
    row_ptr = np.empty(n + 1, dtype=np.uint64)
    col_idx = np.empty(n * M, dtype=np.uint32)
    n_edges, searched = C.c_int64(0), C.c_int64(0)
    rc = _load().orc_build_graph(_p(emb, C.c_float), C.c_int64(n), C.c_int32(d), _p(is_hub, C.c_uint8), C.c_int32(efC),
                                 C.c_int32(M), C.c_int32(m), C.c_int32(batch), C.c_int32(ramp), _p(row_ptr, C.c_uint64),
                                 _p(col_idx, C.c_uint32), C.byref(n_edges), C.byref(searched))
    _check(rc, "build_graph")
    return row_ptr, col_idx[:n_edges.value].copy(), {"edges": n_edges.value, "searched": searched.value}


def top_degree(row_ptr, beta):
    """uint8 flags [n] of the ceil(beta * n) nodes of largest out-degree (ties: lower id)."""
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.uint64)
    n = len(row_ptr) - 1
    out = np.empty(n, dtype=np.uint8)
    _check(_load().orc_top_degree(_p(row_ptr, C.c_uint64), C.c_int64(n), C.c_double(beta), _p(out, C.c_uint8)), "top_degree")
    return out


def shrink(emb, anchor, ids, cap):
    """RNG neighbour selection around node `anchor` among candidate node ids; returns the kept ids, best first."""
    emb = _f32(emb)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    out = np.empty(max(cap, 1), dtype=np.int32)
    n_out = C.c_int32(0)
    _check(_load().orc_shrink(_p(emb, C.c_float), C.c_int64(emb.shape[0]), C.c_int32(emb.shape[1]), C.c_int64(anchor),
                              _p(ids, C.c_int32), C.c_int32(len(ids)), C.c_int32(cap), _p(out, C.c_int32),
                              C.byref(n_out)), "shrink")
    return out[:n_out.value].copy()
