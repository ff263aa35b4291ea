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
