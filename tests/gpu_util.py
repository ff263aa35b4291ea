"""Helpers shared by the GPU parity tests: device upload and the config-1 ("Tiny") world built by the oracle."""
import numpy as np

import leann_inputs as li


def say(*a):
    """Name the case before each GPU step (flushed, so a fault leaves a trace)."""
    print("[gpu-case]", *a, flush=True)


def to_dev(a):
    import torch
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint64:
        a = a.view(np.int64)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).to("cuda:0")


def tiny_world(orc, n=2000, n_queries=16, seed=li.config_seed(1), ragged=False):
    """Config 1: N chunks of 32 token ids in [1,1000), 2-layer encoder, kNN-16 graph over the oracle's fp32
    embeddings, PQ 16 x 256 trained for 10 iterations, queries = embeddings of random chunks."""
    cfg = li.TINY
    w = li.encoder_weights(cfg, seed)
    tokens, lengths = li.uniform_chunks(n, 32, 1, 1000, 4 if ragged else 32, 32, seed + 1)
    e = orc.desc(**cfg)
    emb = orc.embed(e, w, tokens, lengths)
    nbr, _ = li.knn_graph(emb, 16)
    entry, _ = li.max_in_degree_node(nbr)
    row_ptr, col_idx = li.to_csr(nbr)
    cb, _ = orc.pq_train(emb, 16, 10, seed + 2)
    codes = orc.pq_encode(emb, cb)
    qids = np.random.Generator(np.random.Philox(seed + 3)).choice(n, n_queries, replace=False)
    return dict(cfg=cfg, w=w, tokens=tokens, lengths=lengths, desc=e, emb=emb, row_ptr=row_ptr, col_idx=col_idx,
                entry=entry, cb=cb, codes=codes, qids=qids, queries=emb[qids].copy(), n=n)
