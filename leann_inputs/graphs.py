"""Graph fixtures: brute-force kNN graphs over a given embedding matrix, CSR packing.

These build *inputs* for the search (the paper takes its graph from an HNSW
build followed by its pruning algorithm; here a kNN graph stands in).  The
functions accept numpy arrays, or torch tensors (any device) for large N.
"""
import numpy as np


def knn_graph(emb, deg, block=4096):
    """neighbours [n][deg] (int64) by inner product, self excluded, best first, plus their similarities."""
    try:
        import torch
    except ImportError:  # pragma: no cover
        torch = None
    if torch is not None and isinstance(emb, torch.Tensor):
        n = emb.shape[0]
        nbr = torch.empty((n, deg), dtype=torch.int64, device=emb.device)
        sim = torch.empty((n, deg), dtype=torch.float32, device=emb.device)
        for s in range(0, n, block):
            e = min(n, s + block)
            sc = emb[s:e].float() @ emb.float().T
            sc[torch.arange(e - s, device=emb.device), torch.arange(s, e, device=emb.device)] = -float("inf")
            v, i = torch.topk(sc, deg, dim=1)
            nbr[s:e], sim[s:e] = i, v
        return nbr.cpu().numpy(), sim.cpu().numpy()
    emb = np.asarray(emb, dtype=np.float32)
    n = emb.shape[0]
    nbr = np.empty((n, deg), dtype=np.int64)
    sim = np.empty((n, deg), dtype=np.float32)
    for s in range(0, n, block):
        e = min(n, s + block)
        sc = emb[s:e] @ emb.T
        sc[np.arange(e - s), np.arange(s, e)] = -np.inf
        order = np.argsort(-sc, axis=1, kind="stable")[:, :deg]
        nbr[s:e] = order
        sim[s:e] = np.take_along_axis(sc, order, axis=1)
    return nbr, sim


def max_in_degree_node(nbr, n=None):
    """Node with the highest in-degree in the un-pruned graph (ties: lowest id)."""
    n = nbr.shape[0] if n is None else n
    indeg = np.bincount(np.asarray(nbr).reshape(-1), minlength=n)
    return int(np.argmax(indeg)), indeg


def to_csr(lists):
    """Adjacency (2-D array or list of 1-D arrays) -> (row_ptr uint64 [n+1], col_idx uint32 [E])."""
    lens = np.array([len(r) for r in lists], dtype=np.uint64)
    row_ptr = np.zeros(len(lists) + 1, dtype=np.uint64)
    np.cumsum(lens, out=row_ptr[1:])
    if isinstance(lists, np.ndarray) and lists.ndim == 2:
        col_idx = lists.reshape(-1).astype(np.uint32)
    else:
        col_idx = np.concatenate([np.asarray(r, dtype=np.uint32) for r in lists]) if len(lists) else \
            np.zeros(0, np.uint32)
    return row_ptr, col_idx


def add_ring(nbr_lists):
    """Append the edge i -> (i+1) mod n to every node so the graph is strongly connected."""
    n = len(nbr_lists)
    return [np.concatenate([np.asarray(r, dtype=np.int64), np.array([(i + 1) % n], dtype=np.int64)])
            for i, r in enumerate(nbr_lists)]


def hub_prune_fixture(nbr, sim, hub_frac=0.02, hub_deg=64, low_deg=16):
    """Degree-skewed fixture in the spirit of the paper's high-degree-preserving pruning (Alg. 3).

    Hubs = top ceil(hub_frac * n) nodes by in-degree of the kNN graph (ties: lower id).
    A hub keeps the hub_deg most similar of (its own kNN list + its reverse edges);
    every other node keeps the first low_deg entries of its own list.
    Returns (list of neighbour arrays, hub ids, in-degree array).
    """
    nbr = np.asarray(nbr)
    sim = np.asarray(sim)
    n, deg = nbr.shape
    indeg = np.bincount(nbr.reshape(-1), minlength=n)
    n_hub = int(np.ceil(hub_frac * n))
    hubs = np.lexsort((np.arange(n), -indeg))[:n_hub]
    is_hub = np.zeros(n, dtype=bool)
    is_hub[hubs] = True
    src = np.repeat(np.arange(n, dtype=np.int64), deg)
    dst = nbr.reshape(-1)
    s = sim.reshape(-1)
    sel = is_hub[dst]
    r_dst, r_src, r_sim = dst[sel], src[sel], s[sel]
    order = np.argsort(r_dst, kind="stable")
    r_dst, r_src, r_sim = r_dst[order], r_src[order], r_sim[order]
    starts = np.searchsorted(r_dst, hubs, side="left")
    ends = np.searchsorted(r_dst, hubs, side="right")
    out = [nbr[i, :low_deg].astype(np.int64) for i in range(n)]
    for h, a, b in zip(hubs, starts, ends):
        ids = np.concatenate([nbr[h], r_src[a:b]])
        sc = np.concatenate([sim[h], r_sim[a:b]])
        ids, first = np.unique(ids, return_index=True)
        sc = sc[first]
        keep = np.lexsort((ids, -sc))[:hub_deg]
        out[h] = ids[keep].astype(np.int64)
    return out, hubs, indeg
