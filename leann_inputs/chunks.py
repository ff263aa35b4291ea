"""Synthetic token stores: chunks of token ids plus valid lengths (PAD = 0)."""
import numpy as np


def uniform_chunks(n, seq, tok_lo, tok_hi, len_lo, len_hi, seed):
    """Token ids uniform in [tok_lo, tok_hi), lengths uniform integers in [len_lo, len_hi].

    Positions at or beyond a chunk's length hold PAD (0).
    Returns (tokens int32 [n][seq], lengths int32 [n]).
    """
    rng = np.random.Generator(np.random.Philox(seed))
    tokens = rng.integers(tok_lo, tok_hi, size=(n, seq), dtype=np.int32)
    lengths = rng.integers(len_lo, len_hi + 1, size=n, dtype=np.int32)
    tokens[np.arange(seq)[None, :] >= lengths[:, None]] = 0
    return tokens, lengths


def _zipf_cdf(size, a):
    p = 1.0 / np.arange(1, size + 1, dtype=np.float64) ** a
    c = np.cumsum(p)
    return (c / c[-1]).astype(np.float64)


def make_topics(vocab, n_topics, topic_vocab, seed, zipf_a=1.1):
    """Topic tables for topic_chunks: each topic owns a Zipf-ranked list of token ids."""
    rng = np.random.Generator(np.random.Philox(seed))
    return {
        "vocab": vocab,
        "subsets": rng.integers(1, vocab, size=(n_topics, topic_vocab), dtype=np.int32),
        "background": (rng.permutation(vocab - 1) + 1).astype(np.int32),
        "cdf_topic": _zipf_cdf(topic_vocab, zipf_a),
        "cdf_bg": _zipf_cdf(vocab - 1, zipf_a),
    }


def topic_chunks(topics, n, seq, len_lo, len_hi, seed, topic_frac=0.7, block=32768):
    """Topic-mixture corpus standing in for a text collection.

    Each chunk draws one topic; each token comes from that topic's Zipf
    distribution with probability topic_frac, else from a global Zipf
    background.  Returns (tokens int32 [n][seq], lengths int32 [n], topic int32 [n]).
    """
    rng = np.random.Generator(np.random.Philox(seed))
    n_topics, topic_vocab = topics["subsets"].shape
    tokens = np.zeros((n, seq), dtype=np.int32)
    lengths = rng.integers(len_lo, len_hi + 1, size=n, dtype=np.int32)
    topic = rng.integers(0, n_topics, size=n, dtype=np.int32)
    for s in range(0, n, block):
        e = min(n, s + block)
        u = rng.random((e - s, seq))
        rank_t = np.minimum(np.searchsorted(topics["cdf_topic"], u), topic_vocab - 1)
        u = rng.random((e - s, seq))
        rank_b = np.minimum(np.searchsorted(topics["cdf_bg"], u), topics["vocab"] - 2)
        pick = rng.random((e - s, seq)) < topic_frac
        tk = np.where(pick, topics["subsets"][topic[s:e, None], rank_t], topics["background"][rank_b])
        tk[np.arange(seq)[None, :] >= lengths[s:e, None]] = 0
        tokens[s:e] = tk
    return tokens, lengths, topic


def _topic_draws(topics, topic, seq, rng, topic_frac):
    """One token per (row, position) from each row's topic mixture."""
    n = len(topic)
    topic_vocab = topics["subsets"].shape[1]
    rank_t = np.minimum(np.searchsorted(topics["cdf_topic"], rng.random((n, seq))), topic_vocab - 1)
    rank_b = np.minimum(np.searchsorted(topics["cdf_bg"], rng.random((n, seq))), topics["vocab"] - 2)
    pick = rng.random((n, seq)) < topic_frac
    return np.where(pick, topics["subsets"][topic[:, None], rank_t], topics["background"][rank_b]).astype(np.int32)


def family_corpus(topics, n, seq, len_lo, len_hi, seed, family_size=4, resample=0.3, topic_frac=0.7, len_jitter=4,
                  block=32768):
    """Topic-mixture corpus with near-duplicate families, standing in for a text collection in which several
    passages cover the same material.

    ceil(n / family_size) base chunks are drawn from the topic mixture; every corpus chunk is a variant of one
    base: a copy with a fraction `resample` of its positions redrawn from the same topic mixture and its own
    length.  Family membership is spread over the id range by a seeded permutation.
    A variant's length is its base's length (uniform in [len_lo, len_hi]) plus a jitter of at most len_jitter.
    Returns dict(tokens int32 [n][seq], lengths int32 [n], family int32 [n], base int32 [n_fam][seq],
    base_topic int32 [n_fam], base_len int32 [n_fam]).
    """
    rng = np.random.Generator(np.random.Philox(seed))
    n_topics = topics["subsets"].shape[0]
    n_fam = -(-n // family_size)
    base_topic = rng.integers(0, n_topics, size=n_fam, dtype=np.int32)
    base = np.empty((n_fam, seq), dtype=np.int32)
    for s in range(0, n_fam, block):
        e = min(n_fam, s + block)
        base[s:e] = _topic_draws(topics, base_topic[s:e], seq, rng, topic_frac)
    base_len = rng.integers(len_lo, len_hi + 1, size=n_fam, dtype=np.int32)
    family = (rng.permutation(n_fam * family_size)[:n] // family_size).astype(np.int32)
    corpus = dict(base=base, base_topic=base_topic, base_len=base_len, len_lo=len_lo, len_hi=len_hi,
                  len_jitter=len_jitter)
    tokens, lengths = variants_of(topics, corpus, family, seq, rng, resample, topic_frac, block)
    corpus.update(tokens=tokens, lengths=lengths, family=family)
    return corpus


def variants_of(topics, corpus, family, seq, rng, resample, topic_frac, block=32768):
    base, base_topic = corpus["base"], corpus["base_topic"]
    n = len(family)
    tokens = np.empty((n, seq), dtype=np.int32)
    j = corpus["len_jitter"]
    lengths = np.clip(corpus["base_len"][family] + rng.integers(-j, j + 1, size=n), corpus["len_lo"],
                      corpus["len_hi"]).astype(np.int32)
    for s in range(0, n, block):
        e = min(n, s + block)
        fresh = _topic_draws(topics, base_topic[family[s:e]], seq, rng, topic_frac)
        redo = rng.random((e - s, seq)) < resample
        tk = np.where(redo, fresh, base[family[s:e]])
        tk[np.arange(seq)[None, :] >= lengths[s:e, None]] = 0
        tokens[s:e] = tk
    return tokens, lengths


def family_queries(topics, corpus, nq, seq, seed, resample=0.3, topic_frac=0.7):
    """Queries = fresh variants (not in the corpus) of randomly chosen families of a family_corpus."""
    rng = np.random.Generator(np.random.Philox(seed))
    fam = rng.integers(0, corpus["base"].shape[0], size=nq).astype(np.int32)
    tokens, lengths = variants_of(topics, corpus, fam, seq, rng, resample, topic_frac)
    return tokens, lengths, fam


# ---------------------------------------------------------------------------------------------------------
# Latent-position corpus: multi-scale, continuous similarity structure (what a trained text encoder gives a real
# collection, and what a proximity graph needs in order to be navigable).

def make_latent_space(vocab, seed, layers=((4, 16), (16, 8), (64, 4)), zipf_a=1.1):
    """Token tables of a 2-D torus of "subject matter".  Layer (g, m): the torus is cut into g x g cells and each
    cell owns m token ids; coarse layers make far-apart chunks faintly similar, fine layers make close chunks
    very similar.  The remaining token ids form a global Zipf background."""
    rng = np.random.Generator(np.random.Philox(seed))
    ids = (rng.permutation(vocab - 1) + 1).astype(np.int32)
    tables, o = [], 0
    for g, m in layers:
        cnt = g * g * m
        tables.append(ids[o:o + cnt].reshape(g * g, m))
        o += cnt
    assert o < vocab - 1, "vocabulary too small for these layers"
    bg = ids[o:]
    return {"layers": tuple(layers), "tables": tables, "background": bg, "cdf_bg": _zipf_cdf(len(bg), zipf_a)}


def _latent_draws(space, z, seq, rng, bg_frac, jitter):
    """One token per (row, position): background with probability bg_frac, else a uniformly chosen layer; within a
    layer the cell of (z + Gaussian jitter of `jitter` cell widths) and one of that cell's tokens."""
    n = z.shape[0]
    n_layers = len(space["layers"])
    src = rng.random((n, seq))
    layer = np.minimum((rng.random((n, seq)) * n_layers).astype(np.int64), n_layers - 1)
    bg_rank = np.minimum(np.searchsorted(space["cdf_bg"], rng.random((n, seq))), len(space["background"]) - 1)
    out = space["background"][bg_rank].astype(np.int32)
    noise = rng.standard_normal((n, seq, 2))
    which = rng.random((n, seq))
    for li_, ((g, m), table) in enumerate(zip(space["layers"], space["tables"])):
        u = (z[:, None, :] + noise * (jitter / g)) % 1.0
        cell = (np.minimum((u[..., 0] * g).astype(np.int64), g - 1) * g +
                np.minimum((u[..., 1] * g).astype(np.int64), g - 1))
        tok = table[cell, np.minimum((which * m).astype(np.int64), m - 1)]
        sel = (src >= bg_frac) & (layer == li_)
        out[sel] = tok[sel]
    return out


def latent_corpus(space, n, seq, len_lo, len_hi, seed, family_size=4, resample=0.3, bg_frac=0.25, jitter=0.7,
                  len_jitter=4, block=16384, progress=None):
    """Corpus of near-duplicate families placed uniformly on the latent torus.

    Each family has a position z and a base chunk drawn at z; every corpus chunk is a variant of its family's
    base: `resample` of the positions redrawn at the same z, length = base length +- len_jitter.
    Returns dict(tokens, lengths, family, base, base_len, z, ...)."""
    rng = np.random.Generator(np.random.Philox(seed))
    n_fam = -(-n // family_size)
    z = rng.random((n_fam, 2))
    base = np.empty((n_fam, seq), dtype=np.int32)
    for s in range(0, n_fam, block):
        e = min(n_fam, s + block)
        base[s:e] = _latent_draws(space, z[s:e], seq, rng, bg_frac, jitter)
    base_len = rng.integers(len_lo, len_hi + 1, size=n_fam, dtype=np.int32)
    family = (rng.permutation(n_fam * family_size)[:n] // family_size).astype(np.int32)
    corpus = dict(base=base, z=z, base_len=base_len, len_lo=len_lo, len_hi=len_hi, len_jitter=len_jitter,
                  resample=resample, bg_frac=bg_frac, jitter=jitter, seq=seq)
    tokens, lengths = latent_variants(space, corpus, family, rng, block, progress)
    corpus.update(tokens=tokens, lengths=lengths, family=family)
    return corpus


def latent_variants(space, corpus, family, rng, block=16384, progress=None):
    n, seq = len(family), corpus["seq"]
    tokens = np.empty((n, seq), dtype=np.int32)
    j = corpus["len_jitter"]
    lengths = np.clip(corpus["base_len"][family] + rng.integers(-j, j + 1, size=n), corpus["len_lo"],
                      corpus["len_hi"]).astype(np.int32)
    for s in range(0, n, block):
        e = min(n, s + block)
        fresh = _latent_draws(space, corpus["z"][family[s:e]], seq, rng, corpus["bg_frac"], corpus["jitter"])
        redo = rng.random((e - s, seq)) < corpus["resample"]
        tk = np.where(redo, fresh, corpus["base"][family[s:e]])
        tk[np.arange(seq)[None, :] >= lengths[s:e, None]] = 0
        tokens[s:e] = tk
        if progress is not None:
            progress(e, n)
    return tokens, lengths


def latent_queries(space, corpus, nq, seed):
    """Queries = fresh variants (not in the corpus) of randomly chosen families."""
    rng = np.random.Generator(np.random.Philox(seed))
    fam = rng.integers(0, corpus["base"].shape[0], size=nq).astype(np.int32)
    tokens, lengths = latent_variants(space, corpus, fam, rng)
    return tokens, lengths, fam
