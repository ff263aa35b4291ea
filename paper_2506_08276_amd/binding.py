"""Thin ctypes binding of libleann.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/leann.h).
Device buffers are torch CUDA tensors (PyTorch is used for device memory and
the stream, nothing else); the raw data_ptr() values are handed to the library.
There is no fallback: if the shared library is missing, loading raises.
"""
import ctypes as C
import os

import numpy as np
import torch  # imported before libleann.so so that both share the HIP runtime torch ships (same soname)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libleann.so")
_lib = None

LEANN_F32, LEANN_BF16 = 0, 1
STATUS = {0: "LEANN_OK", -1: "LEANN_EINVAL", -2: "LEANN_ENOMEM", -3: "LEANN_EDEVICE", -4: "LEANN_ESHAPE",
          -5: "LEANN_ECAPACITY"}
EXPORTS = ["leann_last_error", "leann_create", "leann_destroy", "leann_embed", "leann_build_pq", "leann_pq_export",
           "leann_pq_import", "leann_pq_wrap", "leann_pq_info", "leann_pq_free", "leann_adc", "leann_adc_noalloc", "leann_search",
           "leann_search_updates", "leann_build_graph", "leann_top_degree",
           "leann_set_limits", "leann_set_call_memo", "leann_set_gemm_tiles", "leann_profile_begin", "leann_profile_end", "leann_bench_mfma", "leann_bench_gather", "leann_bench_l1pull"]
PROF_KINDS = ["gemm_qkv", "gemm_o", "gemm_ffn1", "gemm_ffn2", "attention", "layernorm", "enc_other", "traverse",
              "collect", "score_insert", "lut", "adc"]


class LeannError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{STATUS.get(status, status)}: {message}")
        self.status = status


class EncoderDesc(C.Structure):
    _fields_ = [("layers", C.c_int32), ("hidden", C.c_int32), ("heads", C.c_int32), ("ffn", C.c_int32),
                ("vocab", C.c_int32), ("max_pos", C.c_int32), ("ln_eps", C.c_float)]


class Graph(C.Structure):
    _fields_ = [("row_ptr", C.c_void_p), ("col_idx", C.c_void_p), ("n", C.c_int64), ("entry", C.c_uint32)]


class Chunks(C.Structure):
    _fields_ = [("tokens", C.c_void_p), ("lengths", C.c_void_p), ("n", C.c_int64), ("seq", C.c_int32)]


class EmbCache(C.Structure):
    _fields_ = [("slot_of", C.c_void_p), ("emb", C.c_void_p), ("rows", C.c_int64)]


class SearchStats(C.Structure):
    _fields_ = [("hops", C.c_int64), ("adc_candidates", C.c_int64), ("recomputed_chunks", C.c_int64),
                ("encoded_chunks", C.c_int64), ("encoded_tokens", C.c_int64), ("flushes", C.c_int64),
                ("rounds", C.c_int64), ("cache_hits", C.c_int64), ("memo_hits", C.c_int64), ("encoder_ms", C.c_float),
                ("traverse_ms", C.c_float),
                ("total_ms", C.c_float)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class Profile(C.Structure):
    _fields_ = [("ms", C.c_double * len(PROF_KINDS)), ("launches", C.c_int64 * len(PROF_KINDS)),
                ("tokens", C.c_int64)]


def load_library(path=LIB_PATH):
    """Load libleann.so; raises when it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(path):
            raise FileNotFoundError(f"{path} not found: build it with `python -m paper_2506_08276_amd.build` "
                                    "(or __graft_entry__.build())")
        lib = C.CDLL(path)
        lib.leann_last_error.restype = C.c_char_p
        for name in EXPORTS:
            getattr(lib, name)
        lib.leann_destroy.restype = None
        lib.leann_pq_free.restype = None
        _lib = lib
    return _lib


def _check(rc):
    if rc != 0:
        raise LeannError(rc, load_library().leann_last_error(None).decode())


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else None


def _dev(t, dtype, what):
    assert isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == dtype, \
        f"{what}: need a contiguous CUDA tensor of {dtype}"
    return t


def leann_create(desc, weights, device=0, stream=None):
    """desc: dict of encoder dimensions; weights: packed CUDA tensor (float32 or bfloat16).  Returns a ctx handle."""
    lib = load_library()
    assert weights.is_cuda and weights.is_contiguous() and weights.dtype in (torch.float32, torch.bfloat16)
    d = EncoderDesc(desc["layers"], desc["hidden"], desc["heads"], desc["ffn"], desc["vocab"], desc["max_pos"],
                    desc.get("ln_eps", 1e-12))
    ctx = C.c_void_p()
    if stream is None:
        stream = torch.cuda.current_stream(device).cuda_stream
    _check(lib.leann_create(C.byref(ctx), C.byref(d), _ptr(weights),
                            LEANN_F32 if weights.dtype == torch.float32 else LEANN_BF16, C.c_int(device),
                            C.c_void_p(stream)))
    return ctx


def leann_destroy(ctx):
    load_library().leann_destroy(ctx)


def leann_set_limits(ctx, max_tokens_per_pass=0, aq_capacity=0):
    _check(load_library().leann_set_limits(ctx, C.c_int64(max_tokens_per_pass), C.c_int32(aq_capacity)))


def leann_set_call_memo(ctx, max_rows):
    """Per-call embedding memo of leann_search: up to max_rows embeddings kept within a call (0 = off)."""
    _check(load_library().leann_set_call_memo(ctx, C.c_int64(max_rows)))


def leann_set_gemm_tiles(ctx, large_tile=0, small_rows=2048):
    _check(load_library().leann_set_gemm_tiles(ctx, C.c_int32(large_tile), C.c_int32(small_rows)))


def _chunks(tokens, lengths):
    _dev(tokens, torch.int32, "tokens")
    _dev(lengths, torch.int32, "lengths")
    assert tokens.dim() == 2 and lengths.numel() == tokens.shape[0]
    return Chunks(tokens.data_ptr(), lengths.data_ptr(), tokens.shape[0], tokens.shape[1])


def leann_embed(ctx, tokens, lengths, ids=None, n_ids=None, hidden=None, out=None):
    """Embeddings fp32 [n_ids][hidden] of chunks `ids` (int64 CUDA tensor) or of the first n_ids chunks."""
    lib = load_library()
    ch = _chunks(tokens, lengths)
    if ids is not None:
        _dev(ids, torch.int64, "ids")
        n_ids = ids.numel()
    elif n_ids is None:
        n_ids = tokens.shape[0]
    if out is None:
        out = torch.empty((n_ids, hidden), dtype=torch.float32, device=tokens.device)
    _dev(out, torch.float32, "out")
    _check(lib.leann_embed(ctx, C.byref(ch), _ptr(ids), C.c_int64(n_ids), _ptr(out)))
    return out


def leann_build_pq(ctx, emb, m_sub, iters, seed):
    _dev(emb, torch.float32, "emb")
    pq = C.c_void_p()
    _check(load_library().leann_build_pq(ctx, _ptr(emb), C.c_int64(emb.shape[0]), C.c_int32(emb.shape[1]),
                                         C.c_int32(m_sub), C.c_int32(iters), C.c_uint64(seed), C.byref(pq)))
    return pq


def leann_pq_info(pq):
    n, d, m = C.c_int64(), C.c_int32(), C.c_int32()
    _check(load_library().leann_pq_info(pq, C.byref(n), C.byref(d), C.byref(m)))
    return n.value, d.value, m.value


def leann_pq_export(ctx, pq):
    """Returns (codebook float32 [m_sub][256][dsub], codes uint8 [n][m_sub]) as numpy arrays."""
    n, d, m = leann_pq_info(pq)
    cb = np.empty((m, 256, d // m), dtype=np.float32)
    codes = np.empty((n, m), dtype=np.uint8)
    _check(load_library().leann_pq_export(ctx, pq, cb.ctypes.data_as(C.c_void_p), codes.ctypes.data_as(C.c_void_p)))
    return cb, codes


def leann_pq_import(ctx, codebook, codes):
    codebook = np.ascontiguousarray(codebook, dtype=np.float32)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    m, ksub, dsub = codebook.shape
    assert ksub == 256 and codes.shape[1] == m
    pq = C.c_void_p()
    _check(load_library().leann_pq_import(ctx, codebook.ctypes.data_as(C.c_void_p), codes.ctypes.data_as(C.c_void_p),
                                          C.c_int64(codes.shape[0]), C.c_int32(m * dsub), C.c_int32(m), C.byref(pq)))
    return pq


def leann_pq_wrap(ctx, codebook, codes_dev):
    codebook = np.ascontiguousarray(codebook, dtype=np.float32)
    _dev(codes_dev, torch.uint8, "codes")
    m, ksub, dsub = codebook.shape
    assert ksub == 256 and codes_dev.shape[1] == m
    pq = C.c_void_p()
    _check(load_library().leann_pq_wrap(ctx, codebook.ctypes.data_as(C.c_void_p), _ptr(codes_dev),
                                        C.c_int64(codes_dev.shape[0]), C.c_int32(m * dsub), C.c_int32(m),
                                        C.byref(pq)))
    return pq


def leann_pq_free(pq):
    load_library().leann_pq_free(pq)


def leann_adc(ctx, queries, pq, cand_ids, out=None):
    """ADC similarities fp32 [nq][nc] of candidate node ids (uint32 stored in an int32 CUDA tensor)."""
    _dev(queries, torch.float32, "queries")
    _dev(cand_ids, torch.int32, "cand_ids")
    nq, nc = cand_ids.shape
    if out is None:
        out = torch.empty((nq, nc), dtype=torch.float32, device=queries.device)
    _check(load_library().leann_adc(ctx, _ptr(queries), C.c_int64(nq), pq, _ptr(cand_ids), C.c_int32(nc), _ptr(out)))
    return out


def leann_adc_noalloc(ctx, queries, pq, cand_ids, out):
    """leann_adc through the library's fixed workspace (no allocation, no synchronisation); `out` is required."""
    _dev(queries, torch.float32, "queries")
    _dev(cand_ids, torch.int32, "cand_ids")
    _dev(out, torch.float32, "out")
    nq, nc = cand_ids.shape
    assert out.shape == (nq, nc)
    _check(load_library().leann_adc_noalloc(ctx, _ptr(queries), C.c_int64(nq), pq, _ptr(cand_ids), C.c_int32(nc),
                                            _ptr(out)))
    return out


class Updates(C.Structure):
    _fields_ = [("deleted_bits", C.c_void_p), ("buffer_emb", C.c_void_p), ("buffer_ids", C.c_void_p),
                ("buffer_n", C.c_int64)]


def _search(entry_point, ctx, queries, graph, pq, tokens, lengths, ef, k, rerank_ratio, batch, cache, updates):
    _dev(queries, torch.float32, "queries")
    row_ptr, col_idx, entry = graph
    _dev(row_ptr, torch.int64, "row_ptr")
    _dev(col_idx, torch.int32, "col_idx")
    g = Graph(row_ptr.data_ptr(), col_idx.data_ptr(), row_ptr.numel() - 1, int(entry))
    ch = _chunks(tokens, lengths)
    nq = queries.shape[0]
    ids = torch.empty((nq, k), dtype=torch.int64, device=queries.device)
    scores = torch.empty((nq, k), dtype=torch.float32, device=queries.device)
    st = SearchStats()
    cref = None
    if cache is not None:
        slot_of, emb = cache
        _dev(slot_of, torch.int32, "slot_of")
        _dev(emb, torch.float32, "cache emb")
        cstruct = EmbCache(slot_of.data_ptr(), emb.data_ptr(), emb.shape[0])
        cref = C.byref(cstruct)
    head = (ctx, _ptr(queries), C.c_int64(nq), C.byref(g), pq, C.byref(ch), cref)
    tail = (C.c_int32(ef), C.c_int32(k), C.c_float(rerank_ratio), C.c_int32(batch), _ptr(ids), _ptr(scores), C.byref(st))
    if entry_point == "leann_search":
        _check(load_library().leann_search(*head, *tail))
    else:
        deleted_bits, buffer = updates
        u = Updates(None, None, None, 0)
        if deleted_bits is not None:
            _dev(deleted_bits, torch.int32, "deleted_bits")
            assert deleted_bits.numel() >= (g.n + 31) // 32
            u.deleted_bits = deleted_bits.data_ptr()
        if buffer is not None:
            buf_ids, buf_emb = buffer
            _dev(buf_ids, torch.int32, "buffer ids")
            _dev(buf_emb, torch.float32, "buffer emb")
            assert buf_emb.shape == (buf_ids.numel(), queries.shape[1])
            u.buffer_emb, u.buffer_ids, u.buffer_n = buf_emb.data_ptr(), buf_ids.data_ptr(), buf_ids.numel()
        _check(load_library().leann_search_updates(*head, C.byref(u), *tail))
    return ids, scores, st.as_dict()


def leann_search(ctx, queries, graph, pq, tokens, lengths, ef, k, rerank_ratio, batch, cache=None):
    """graph = (row_ptr int64 CUDA tensor holding uint64 values, col_idx int32 CUDA tensor holding uint32, entry).
    cache = (slot_of int32 [n], emb float32 [rows][d]) or None.
    Returns (ids int64 [nq][k], scores float32 [nq][k], stats dict)."""
    return _search("leann_search", ctx, queries, graph, pq, tokens, lengths, ef, k, rerank_ratio, batch, cache, None)


def leann_search_updates(ctx, queries, graph, pq, tokens, lengths, ef, k, rerank_ratio, batch, cache=None,
                         deleted_bits=None, buffer=None):
    """leann_search with pending updates: deleted_bits = int32 CUDA tensor of (n + 31) // 32 words (bit v set: node v
    is soft-deleted) or None; buffer = (ids int32 CUDA tensor holding uint32 [nb], emb float32 [nb][d]) or None."""
    return _search("leann_search_updates", ctx, queries, graph, pq, tokens, lengths, ef, k, rerank_ratio, batch, cache,
                   (deleted_bits, buffer))


def leann_build_graph(ctx, emb, efC, M, m=None, is_hub=None, batch=256, ramp=8):
    """Algorithm 3 on the device.  emb float32 CUDA [n][d]; is_hub uint8 CUDA [n] or None.
    Returns (row_ptr int64 CUDA tensor holding uint64 [n+1], col_idx int32 CUDA tensor holding uint32 [E])."""
    _dev(emb, torch.float32, "emb")
    n, d = emb.shape
    m = M if m is None else m
    if is_hub is not None:
        _dev(is_hub, torch.uint8, "is_hub")
        assert is_hub.numel() == n
    row_ptr = torch.empty(n + 1, dtype=torch.int64, device=emb.device)
    col_idx = torch.empty(n * M, dtype=torch.int32, device=emb.device)
    edges = C.c_int64(0)
    _check(load_library().leann_build_graph(ctx, _ptr(emb), C.c_int64(n), C.c_int32(d), _ptr(is_hub), C.c_int32(efC),
                                            C.c_int32(M), C.c_int32(m), C.c_int32(batch), C.c_int32(ramp),
                                            _ptr(row_ptr), _ptr(col_idx), C.byref(edges)))
    return row_ptr, col_idx[:edges.value].clone()


def leann_top_degree(ctx, row_ptr, beta):
    """uint8 CUDA flags [n] of the ceil(beta * n) nodes of largest out-degree (ties: lower id)."""
    _dev(row_ptr, torch.int64, "row_ptr")
    n = row_ptr.numel() - 1
    out = torch.empty(n, dtype=torch.uint8, device=row_ptr.device)
    _check(load_library().leann_top_degree(ctx, _ptr(row_ptr), C.c_int64(n), C.c_double(beta), _ptr(out)))
    return out


def leann_profile_begin(ctx):
    _check(load_library().leann_profile_begin(ctx))


def leann_profile_end(ctx):
    """Returns {"ms": {kind: summed ms}, "launches": {kind: count}, "tokens": valid tokens encoded}."""
    p = Profile()
    _check(load_library().leann_profile_end(ctx, C.byref(p)))
    return {"ms": {k: p.ms[i] for i, k in enumerate(PROF_KINDS)},
            "launches": {k: p.launches[i] for i, k in enumerate(PROF_KINDS)}, "tokens": p.tokens}


def leann_bench_mfma(ctx, operand_kind, blocks_per_cu=2, iters=4000, launches=40):
    """(TFLOP/s, ms per launch) of a loop of independent bf16 MFMAs; operand_kind 0 zeros, 1 near one, 2 random bits."""
    tf, ms = C.c_double(), C.c_double()
    _check(load_library().leann_bench_mfma(ctx, C.c_int32(operand_kind), C.c_int32(blocks_per_cu), C.c_int32(iters),
                                           C.c_int32(launches), C.byref(tf), C.byref(ms)))
    return tf.value, ms.value


def leann_bench_gather(ctx, table, launches=5):
    """(rows/s, ms per launch) of uniformly random 32-byte row gathers from `table` (uint8 CUDA tensor [rows][32])."""
    _dev(table, torch.uint8, "table")
    assert table.dim() == 2 and table.shape[1] == 32
    rps, ms = C.c_double(), C.c_double()
    _check(load_library().leann_bench_gather(ctx, _ptr(table), C.c_int64(table.shape[0]), C.c_int32(launches),
                                             C.byref(rps), C.byref(ms)))
    return rps.value, ms.value


def leann_bench_l1pull(ctx, panel_rows, launches=5):
    """(bytes/s, ms per launch) of eight waves per CU doing only the GEMM's operand loads over a panel of 1536-byte rows."""
    bps, ms = C.c_double(), C.c_double()
    _check(load_library().leann_bench_l1pull(ctx, C.c_int64(panel_rows), C.c_int32(launches), C.byref(bps), C.byref(ms)))
    return bps.value, ms.value
