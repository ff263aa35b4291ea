"""Pins for the encoder oracle (CPU only).

The paper prints no encoder values, so the oracle is pinned by: a hand-derived
worked example (tests/golden/encoder_zero_layer.txt), a structurally different
whole-matrix fp64 formulation on padded inputs, closed-form special cases and
invariants.  Numeric parity with the paper's trained encoder is unpinned
(its weights are not available).
"""
import math
import os

import numpy as np
import pytest

import leann_inputs as li

GOLD = os.path.join(os.path.dirname(__file__), "golden")

SMALL = dict(layers=2, hidden=16, heads=2, ffn=32, vocab=50, max_pos=12, ln_eps=1e-12)


def split(cfg, packed):
    out, o = {}, 0
    for name, shape, _ in li.weight_layout(cfg):
        n = int(np.prod(shape))
        out[name] = packed[o:o + n].reshape(shape).astype(np.float64)
        o += n
    assert o == packed.size
    return out


def pack(cfg, named):
    return np.concatenate([np.asarray(named[n], np.float32).reshape(-1) for n, _, _ in li.weight_layout(cfg)])


def matrix_encoder(cfg, W, tokens, lengths):
    """Whole-batch fp64 formulation on the padded [n][S] grid with additive -inf key masks."""
    d, H = cfg["hidden"], cfg["heads"]
    dh = d // H
    n, S = tokens.shape

    def ln(x, g, b):
        mu = x.mean(-1, keepdims=True)
        var = ((x - mu) ** 2).mean(-1, keepdims=True)
        return (x - mu) / np.sqrt(var + cfg["ln_eps"]) * g + b

    valid = np.arange(S)[None, :] < lengths[:, None]
    x = W["tok_emb"][tokens] + W["pos_emb"][None, :S] + W["seg_emb"]
    x = ln(x, W["emb_ln_g"], W["emb_ln_b"])
    erf = np.vectorize(math.erf)
    for l in range(cfg["layers"]):
        qkv = x @ W[f"l{l}.wqkv"].T + W[f"l{l}.bqkv"]
        q, k, v = [t.reshape(n, S, H, dh).transpose(0, 2, 1, 3) for t in np.split(qkv, 3, axis=-1)]
        s = np.einsum("nhid,nhjd->nhij", q, k) / math.sqrt(dh)
        s = np.where(valid[:, None, None, :], s, -np.inf)
        s = s - s.max(-1, keepdims=True)
        p = np.exp(s)
        p /= p.sum(-1, keepdims=True)
        a = np.einsum("nhij,nhjd->nhid", p, v).transpose(0, 2, 1, 3).reshape(n, S, d)
        x = ln(x + a @ W[f"l{l}.wo"].T + W[f"l{l}.bo"], W[f"l{l}.ln1_g"], W[f"l{l}.ln1_b"])
        h = x @ W[f"l{l}.w1"].T + W[f"l{l}.b1"]
        h = 0.5 * h * (1.0 + erf(h / math.sqrt(2.0)))
        x = ln(x + h @ W[f"l{l}.w2"].T + W[f"l{l}.b2"], W[f"l{l}.ln2_g"], W[f"l{l}.ln2_b"])
    e = (x * valid[:, :, None]).sum(1) / lengths[:, None]
    return e / np.linalg.norm(e, axis=1, keepdims=True)


def small_inputs(seed, n=6, seq=12, cfg=SMALL):
    w = li.encoder_weights(cfg, seed, std=0.3, perturb=True)
    tokens, lengths = li.uniform_chunks(n, seq, 1, cfg["vocab"], 1, seq, seed + 1)
    lengths[0], lengths[1] = 1, seq  # always cover the shortest and the full-length chunk
    tokens[0, 1:] = 0
    return w, tokens, lengths


def test_worked_example_zero_layers(orc):
    """Hand-derived values: embedding = normalise(mean(LN(emb)))."""
    want = np.loadtxt(os.path.join(GOLD, "encoder_zero_layer.txt"))
    cfg = dict(layers=0, hidden=4, heads=1, ffn=4, vocab=3, max_pos=2, ln_eps=0.0)
    named = {n: np.zeros(s, np.float32) for n, s, _ in li.weight_layout(cfg)}
    named["tok_emb"][1] = [0.5, 1.5, 2.0, 3.0]
    named["tok_emb"][2] = [3.0, -1.0, -0.5, 0.0]
    named["pos_emb"][0] = [0.25, 0.25, 0.5, 0.5]     # a = tok1 + pos0 + seg = [1,2,3,4]
    named["pos_emb"][1] = [0.75, 0.75, 0.0, -0.5]    # b = tok2 + pos1 + seg = [4,0,0,0]
    named["seg_emb"][:] = [0.25, 0.25, 0.5, 0.5]
    named["emb_ln_g"][:] = 1.0
    got = orc.embed(orc.desc(**cfg), pack(cfg, named), np.array([[1, 2]], np.int32), np.array([2], np.int32))
    np.testing.assert_allclose(got[0], want, atol=2e-7)


def test_matches_whole_matrix_formulation(orc):
    """Per-token scalar loops == padded whole-matrix fp64 products, incl. biases, LN scales and masks."""
    w, tokens, lengths = small_inputs(11)
    got = orc.embed(orc.desc(**SMALL), w, tokens, lengths)
    want = matrix_encoder(SMALL, split(SMALL, w), tokens, lengths)
    assert np.abs(got - want).max() < 1e-5
    # the comparison is sensitive: dropping one bias moves the result far more than the tolerance
    named = split(SMALL, w)
    named["l1.b2"] = np.zeros_like(named["l1.b2"])
    assert np.abs(got - matrix_encoder(SMALL, named, tokens, lengths)).max() > 1e-3


def test_unit_norm_and_batch_invariance(orc):
    w, tokens, lengths = small_inputs(5, n=9)
    e = orc.desc(**SMALL)
    full = orc.embed(e, w, tokens, lengths)
    np.testing.assert_allclose(np.linalg.norm(full, axis=1), 1.0, atol=1e-6)
    ids = np.array([7, 2, 2, 5], np.int64)
    sub = orc.embed(e, w, tokens, lengths, ids=ids)
    assert np.array_equal(sub, full[ids])  # bit-identical whatever it is batched with


def test_padding_invariance_bit_exact(orc):
    w, tokens, lengths = small_inputs(9)
    e = orc.desc(**SMALL)
    base = orc.embed(e, w, tokens, lengths)
    junk = tokens.copy()
    junk[np.arange(tokens.shape[1])[None, :] >= lengths[:, None]] = 7
    assert np.array_equal(orc.embed(e, w, junk, lengths), base)
    short = np.ascontiguousarray(tokens[:, :int(lengths.max())])
    wider = np.zeros((tokens.shape[0], SMALL["max_pos"]), np.int32)
    wider[:, :tokens.shape[1]] = tokens
    assert np.array_equal(orc.embed(e, w, short, lengths), base)
    assert np.array_equal(orc.embed(e, w, wider, lengths), base)


def test_single_token_attention_is_value(orc):
    """L = 1: softmax over one key is 1, so the attention output is v; checked through a closed form."""
    cfg = dict(layers=1, hidden=4, heads=2, ffn=4, vocab=4, max_pos=2, ln_eps=1e-12)
    w = li.encoder_weights(cfg, 3, std=0.5, perturb=True)
    W = split(cfg, w)

    def ln(x, g, b):
        return (x - x.mean()) / math.sqrt(((x - x.mean()) ** 2).mean() + cfg["ln_eps"]) * g + b

    x = ln(W["tok_emb"][2] + W["pos_emb"][0] + W["seg_emb"], W["emb_ln_g"], W["emb_ln_b"])
    v = (W["l0.wqkv"] @ x + W["l0.bqkv"])[8:12]
    x = ln(x + W["l0.wo"] @ v + W["l0.bo"], W["l0.ln1_g"], W["l0.ln1_b"])
    h = W["l0.w1"] @ x + W["l0.b1"]
    h = np.array([0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in h])
    x = ln(x + W["l0.w2"] @ h + W["l0.b2"], W["l0.ln2_g"], W["l0.ln2_b"])
    want = x / np.linalg.norm(x)
    got = orc.embed(orc.desc(**cfg), w, np.array([[2, 0]], np.int32), np.array([1], np.int32))
    np.testing.assert_allclose(got[0], want, atol=2e-6)


def test_zero_query_projection_gives_uniform_attention(orc):
    """W_q = 0, b_q = 0: all scores are 0, attention = plain mean of the value rows."""
    cfg = dict(SMALL, layers=1)
    w, tokens, lengths = small_inputs(21, cfg=cfg)
    W = split(cfg, w)
    d = cfg["hidden"]
    W["l0.wqkv"][:d] = 0
    W["l0.bqkv"][:d] = 0
    got = orc.embed(orc.desc(**cfg), pack(cfg, W), tokens, lengths)

    def ln(x, g, b):
        mu = x.mean(-1, keepdims=True)
        return (x - mu) / np.sqrt(((x - mu) ** 2).mean(-1, keepdims=True) + cfg["ln_eps"]) * g + b

    erf = np.vectorize(math.erf)
    for c in range(tokens.shape[0]):
        L = int(lengths[c])
        x = ln(W["tok_emb"][tokens[c, :L]] + W["pos_emb"][:L] + W["seg_emb"], W["emb_ln_g"], W["emb_ln_b"])
        v = x @ W["l0.wqkv"][2 * d:].T + W["l0.bqkv"][2 * d:]
        a = np.repeat(v.mean(0, keepdims=True), L, axis=0)
        x = ln(x + a @ W["l0.wo"].T + W["l0.bo"], W["l0.ln1_g"], W["l0.ln1_b"])
        h = x @ W["l0.w1"].T + W["l0.b1"]
        h = 0.5 * h * (1 + erf(h / math.sqrt(2)))
        x = ln(x + h @ W["l0.w2"].T + W["l0.b2"], W["l0.ln2_g"], W["l0.ln2_b"])
        e = x.mean(0)
        np.testing.assert_allclose(got[c], e / np.linalg.norm(e), atol=1e-5)


def test_token_order_invariance_without_positions(orc):
    """With pos_emb = 0 the mean-pooled encoder cannot see token order."""
    w, tokens, lengths = small_inputs(31)
    W = split(SMALL, w)
    W["pos_emb"][:] = 0
    wp = pack(SMALL, W)
    e = orc.desc(**SMALL)
    base = orc.embed(e, wp, tokens, lengths)
    rng = np.random.default_rng(0)
    shuf = tokens.copy()
    for c in range(tokens.shape[0]):
        L = int(lengths[c])
        shuf[c, :L] = rng.permutation(tokens[c, :L])
    np.testing.assert_allclose(orc.embed(e, wp, shuf, lengths), base, atol=2e-6)
    # and positions do matter once pos_emb is restored (the invariance test is not vacuous)
    assert np.abs(orc.embed(e, w, shuf, lengths) - orc.embed(e, w, tokens, lengths)).max() > 1e-4


def test_head_split_matters_and_heads_concatenate(orc):
    """Zeroing W_o columns of head 1 must equal removing head 1's contribution (concat order h*dh + c)."""
    cfg = dict(SMALL, layers=1)
    w, tokens, lengths = small_inputs(41, cfg=cfg)
    W = split(cfg, w)
    d, dh = cfg["hidden"], cfg["hidden"] // cfg["heads"]
    Wa = {k: v.copy() for k, v in W.items()}
    Wa["l0.wo"][:, dh:] = 0                      # ignore head 1's output
    Wb = {k: v.copy() for k, v in W.items()}
    Wb["l0.wqkv"][2 * d + dh:] = 0               # head 1's values are zero
    Wb["l0.bqkv"][2 * d + dh:] = 0
    e = orc.desc(**cfg)
    np.testing.assert_allclose(orc.embed(e, pack(cfg, Wa), tokens, lengths),
                               orc.embed(e, pack(cfg, Wb), tokens, lengths), atol=2e-6)


def test_bf16_emulation_mode_is_close_and_input_checks(orc):
    w, tokens, lengths = small_inputs(51)
    e = orc.desc(**SMALL)
    a = orc.embed(e, w, tokens, lengths, precision=0)
    b = orc.embed(e, w, tokens, lengths, precision=1)
    assert 0 < np.abs(a - b).max() < 2e-2
    bad = tokens.copy()
    bad[1, 0] = SMALL["vocab"]
    with pytest.raises(RuntimeError):
        orc.embed(e, w, bad, lengths)
    with pytest.raises(RuntimeError):
        orc.embed(e, w, tokens, np.zeros_like(lengths))


def test_tiny_config_embeddings_are_unit_and_distinct(orc):
    """Config 1 shape: unit-norm rows; distinct chunks give distinct embeddings."""
    cfg = li.TINY
    w = li.encoder_weights(cfg, li.config_seed(1))
    tokens, lengths = li.uniform_chunks(64, 32, 1, 1000, 32, 32, li.config_seed(1) + 1)
    emb = orc.embed(orc.desc(**cfg), w, tokens, lengths)
    np.testing.assert_allclose(np.linalg.norm(emb, axis=1), 1.0, atol=1e-6)
    s = emb @ emb.T
    np.fill_diagonal(s, 0)
    assert s.max() < 1 - 1e-4
