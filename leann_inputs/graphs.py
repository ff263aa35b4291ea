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


def hub_slots(row_ptr, col_idx, frac):
    """Stored-embedding table layout for the nodes of highest degree in a CSR graph: the ceil(frac * n) nodes with the
    largest in-degree + out-degree (ties: lower id), in id order.  Returns (ids int64 [rows], slot_of int32 [n])
    with slot_of[v] = row of v in the table, -1 for the others."""
    n = len(row_ptr) - 1
    deg = np.diff(np.asarray(row_ptr).astype(np.int64)) + np.bincount(np.asarray(col_idx).astype(np.int64), minlength=n)
    rows = int(np.ceil(frac * n))
    order = np.lexsort((np.arange(n), -deg))
    ids = np.sort(order[:rows]).astype(np.int64)
    slot_of = np.full(n, -1, dtype=np.int32)
    slot_of[ids] = np.arange(rows, dtype=np.int32)
    return ids, slot_of


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


def _diversify(emb, nbr, sim, block=8192):
    """Relative-neighbourhood selection over each node's candidate list (best first): candidate c is kept when it
    is more similar to the node than to every candidate kept before it.  Returns a bool mask [n][k]."""
    try:
        import torch
    except ImportError:  # pragma: no cover
        torch = None
    n, k = nbr.shape
    keep = np.zeros((n, k), dtype=bool)
    if torch is not None and isinstance(emb, torch.Tensor):
        nb = torch.from_numpy(np.ascontiguousarray(nbr)).to(emb.device)
        sm = torch.from_numpy(np.ascontiguousarray(sim)).to(emb.device)
        for s in range(0, n, block):
            e = min(n, s + block)
            c = emb[nb[s:e]].float()
            pair = torch.bmm(c, c.transpose(1, 2))
            kp = torch.zeros((e - s, k), dtype=torch.bool, device=emb.device)
            for i in range(k):
                kp[:, i] = ~((pair[:, i, :] >= sm[s:e, i:i + 1]) & kp).any(1)
            keep[s:e] = kp.cpu().numpy()
        return keep
    emb = np.asarray(emb, dtype=np.float32)
    for s in range(0, n, block):
        e = min(n, s + block)
        c = emb[nbr[s:e]]
        pair = np.einsum("bid,bjd->bij", c, c)
        kp = np.zeros((e - s, k), dtype=bool)
        for i in range(k):
            kp[:, i] = ~((pair[:, i, :] >= sim[s:e, i:i + 1]) & kp).any(1)
        keep[s:e] = kp
    return keep


def navigable_fixture(emb, nbr, sim, hub_frac=0.02, hub_deg=64, low_deg=16):
    """Degree-skewed, navigable graph fixture in the spirit of the paper's high-degree-preserving pruning
    (Alg. 3: hubs keep up to M edges, other nodes m, edges are added in both directions).

    Hubs = top ceil(hub_frac * n) nodes by in-degree of the kNN graph (ties: lower id).  Every node first takes
    the relative-neighbourhood-diversified subset of its kNN list (at most its cap), then reverse edges of other
    nodes' selections, most similar first, while it has room (cap hub_deg for hubs, low_deg otherwise); a node
    still below low_deg is filled with its nearest unselected kNN entries.
    Returns (list of neighbour arrays, hub ids, in-degree array).
    """
    nbr = np.asarray(nbr)
    sim = np.asarray(sim)
    n, k = nbr.shape
    indeg = np.bincount(nbr.reshape(-1), minlength=n)
    n_hub = int(np.ceil(hub_frac * n))
    hubs = np.lexsort((np.arange(n), -indeg))[:n_hub]
    cap = np.full(n, low_deg, dtype=np.int64)
    cap[hubs] = hub_deg
    keep = _diversify(emb, nbr, sim)
    keep &= np.cumsum(keep, axis=1) <= cap[:, None]
    src = np.repeat(np.arange(n, dtype=np.int64), k)[keep.reshape(-1)]
    dst = nbr.reshape(-1)[keep.reshape(-1)]
    fsim = sim.reshape(-1)[keep.reshape(-1)]
    order = np.lexsort((src, -fsim, dst))          # reverse edges grouped by target, most similar first
    r_src, r_dst = src[order], dst[order]
    starts = np.searchsorted(r_dst, np.arange(n), side="left")
    ends = np.searchsorted(r_dst, np.arange(n), side="right")
    out = []
    for i in range(n):
        sel = list(nbr[i][keep[i]])
        have = set(sel)
        for v in r_src[starts[i]:ends[i]]:
            if len(sel) >= cap[i]:
                break
            if v not in have:
                sel.append(int(v))
                have.add(int(v))
        if len(sel) < low_deg:
            for v in nbr[i]:
                if len(sel) >= low_deg:
                    break
                if v not in have:
                    sel.append(int(v))
                    have.add(int(v))
        out.append(np.asarray(sel, dtype=np.int64))
    return out, hubs, indeg
