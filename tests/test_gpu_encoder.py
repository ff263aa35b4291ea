"""GPU parity: leann_embed against the encoder oracle (bound from the benchmark spec: max-abs 2e-2, bf16 GPU vs
fp32 oracle; a tighter 3e-3 against the oracle's bf16-storage mode)."""
import numpy as np
import pytest

import leann_inputs as li
from gpu_util import say, to_dev

pytestmark = pytest.mark.gpu

TOL_FP32 = 2e-2
TOL_BF16_MODE = 3e-3


@pytest.fixture(scope="module")
def L():
    import paper_2506_08276_amd as L
    L.load_library()
    return L


@pytest.fixture(scope="module")
def tiny(L, orc):
    import torch
    cfg = li.TINY
    w = li.encoder_weights(cfg, 7, perturb=True)
    tokens, lengths = li.uniform_chunks(700, 32, 1, 1000, 1, 32, 8)
    lengths[:3] = [1, 32, 31]
    ctx = L.leann_create(cfg, to_dev(w))
    yield dict(cfg=cfg, w=w, tokens=tokens, lengths=lengths, ctx=ctx, t=to_dev(tokens), l=to_dev(lengths))
    L.leann_destroy(ctx)


def test_tiny_ragged_matches_oracle(L, orc, tiny):
    """700 ragged chunks (about 11.5k packed tokens: ~90 row tiles of 128 and a ragged tail)."""
    say("tiny ragged embed, seed 7/8, n=700")
    got = L.leann_embed(tiny["ctx"], tiny["t"], tiny["l"], hidden=128).cpu().numpy()
    e = orc.desc(**tiny["cfg"])
    want = orc.embed(e, tiny["w"], tiny["tokens"], tiny["lengths"])
    want_bf = orc.embed(e, tiny["w"], tiny["tokens"], tiny["lengths"], precision=1)
    assert np.isfinite(got).all()
    assert np.abs(got - want).max() <= TOL_FP32
    assert np.abs(got - want_bf).max() <= TOL_BF16_MODE
    np.testing.assert_allclose(np.linalg.norm(got, axis=1), 1.0, atol=1e-5)


def test_batch_composition_and_pass_invariance(L, tiny):
    """A chunk's embedding is bit-identical whatever shares its batch or its pass."""
    import torch
    say("batch composition invariance")
    full = L.leann_embed(tiny["ctx"], tiny["t"], tiny["l"], hidden=128)
    ids = torch.tensor([5, 699, 0, 5, 123, 77], dtype=torch.int64, device="cuda:0")
    sub = L.leann_embed(tiny["ctx"], tiny["t"], tiny["l"], ids=ids, hidden=128)
    assert torch.equal(sub, full[ids])
    say("pass slicing invariance (64-token passes)")
    L.leann_set_limits(tiny["ctx"], max_tokens_per_pass=64)
    try:
        sliced = L.leann_embed(tiny["ctx"], tiny["t"], tiny["l"], hidden=128)
    finally:
        L.leann_set_limits(tiny["ctx"], max_tokens_per_pass=262144)
    assert torch.equal(sliced, full)
    first = L.leann_embed(tiny["ctx"], tiny["t"], tiny["l"], n_ids=10, hidden=128)
    assert torch.equal(first, full[:10])


def test_padding_content_is_ignored(L, tiny):
    import torch
    say("padding invariance")
    full = L.leann_embed(tiny["ctx"], tiny["t"], tiny["l"], hidden=128)
    junk = tiny["tokens"].copy()
    junk[np.arange(32)[None, :] >= tiny["lengths"][:, None]] = 999
    got = L.leann_embed(tiny["ctx"], to_dev(junk), tiny["l"], hidden=128)
    assert torch.equal(got, full)


def test_empty_and_errors(L, tiny):
    import torch
    say("empty request and invalid inputs")
    out = L.leann_embed(tiny["ctx"], tiny["t"], tiny["l"], n_ids=0, hidden=128)
    assert out.shape == (0, 128)
    bad_tok = tiny["tokens"].copy()
    bad_tok[3, 0] = 1000
    with pytest.raises(L.LeannError) as ei:
        L.leann_embed(tiny["ctx"], to_dev(bad_tok), tiny["l"], hidden=128)
    assert ei.value.status == -1
    bad_len = tiny["lengths"].copy()
    bad_len[4] = 33
    with pytest.raises(L.LeannError):
        L.leann_embed(tiny["ctx"], tiny["t"], to_dev(bad_len), hidden=128)
    with pytest.raises(L.LeannError):
        L.leann_embed(tiny["ctx"], tiny["t"], tiny["l"], ids=torch.tensor([700], dtype=torch.int64, device="cuda:0"),
                      hidden=128)
    with pytest.raises(L.LeannError) as ei:
        L.leann_create(dict(li.TINY, hidden=96, heads=2), to_dev(np.zeros(10, np.float32)))
    assert ei.value.status == -4
    # the context still works after the rejected calls
    ok = L.leann_embed(tiny["ctx"], tiny["t"], tiny["l"], n_ids=4, hidden=128)
    assert torch.isfinite(ok).all()


def test_base_shape_sample_matches_oracle(L, orc):
    """BERT-base shape at seq 256, bf16-exact random weights (config 2); a few chunks the oracle can afford."""
    import torch
    cfg = li.BASE
    say("base-shape sample, seed cfg2")
    w = li.encoder_weights(cfg, li.config_seed(2), bf16_exact=True)
    tokens, lengths = li.uniform_chunks(40, 256, 1, cfg["vocab"], 64, 256, li.config_seed(2) + 1)
    lengths[:5] = [1, 33, 64, 200, 256]
    ctx = L.leann_create(cfg, to_dev(w).to(torch.bfloat16))  # bf16 weight upload path
    try:
        got = L.leann_embed(ctx, to_dev(tokens), to_dev(lengths), hidden=768).cpu().numpy()  # 10240 padded rows: 256 x 256 tiles
        L.leann_set_gemm_tiles(ctx, 128, 0)  # the same pass through 128 x 128 tiles: the same bits
        assert np.array_equal(L.leann_embed(ctx, to_dev(tokens), to_dev(lengths), hidden=768).cpu().numpy(), got)
        with pytest.raises(L.LeannError):
            L.leann_set_gemm_tiles(ctx, 192, 0)
    finally:
        L.leann_destroy(ctx)
    ids = np.array([0, 1, 2, 3, 4, 17], np.int64)
    e = orc.desc(**cfg)
    want = orc.embed(e, w, tokens, lengths, ids=ids)
    want_bf = orc.embed(e, w, tokens, lengths, ids=ids, precision=1)
    assert np.isfinite(got).all()
    assert np.abs(got[ids] - want).max() <= TOL_FP32
    assert np.abs(got[ids] - want_bf).max() <= TOL_BF16_MODE
    print("base sample max-abs vs fp32 oracle %.3e, vs bf16-mode oracle %.3e" %
          (np.abs(got[ids] - want).max(), np.abs(got[ids] - want_bf).max()))


def test_small_shape_sample_matches_oracle(L, orc):
    """The 12 x 384 encoder (second throughput point; widths that are not multiples of 256 take the 128-wide GEMM
    tile) at seq 256; a few chunks against the oracle."""
    import torch
    cfg = li.SMALL
    say("small-shape sample (12 x 384)")
    w = li.encoder_weights(cfg, li.config_seed(2) + 7, bf16_exact=True)
    tokens, lengths = li.uniform_chunks(300, 256, 1, cfg["vocab"], 64, 256, li.config_seed(2) + 8)
    lengths[:4] = [1, 47, 129, 256]
    ctx = L.leann_create(cfg, to_dev(w).to(torch.bfloat16))
    try:
        got = L.leann_embed(ctx, to_dev(tokens), to_dev(lengths), hidden=384).cpu().numpy()
    finally:
        L.leann_destroy(ctx)
    ids = np.array([0, 1, 2, 3, 150, 299], np.int64)
    e = orc.desc(**cfg)
    want = orc.embed(e, w, tokens, lengths, ids=ids)
    want_bf = orc.embed(e, w, tokens, lengths, ids=ids, precision=1)
    assert np.isfinite(got).all()
    assert np.abs(got[ids] - want).max() <= TOL_FP32
    assert np.abs(got[ids] - want_bf).max() <= TOL_BF16_MODE
    print("small sample max-abs vs fp32 oracle %.3e, vs bf16-mode oracle %.3e" %
          (np.abs(got[ids] - want).max(), np.abs(got[ids] - want_bf).max()))


def test_width_256_all_three_gemm_tiles(L, orc):
    """hidden = 256: the 256 x 256 GEMM tile with K = 256 (eight K-slabs, the fewest it is launched for: no
    full group of four before the tail) and K = 1024; ragged rows; against the oracle.  The same chunks embedded in
    passes small enough for the 128 x 128 and the 64 x 64 tile give the same bits (all tiles add the K-slabs in one
    order)."""
    import torch
    cfg = dict(layers=3, hidden=256, heads=4, ffn=1024, vocab=2000, max_pos=128, ln_eps=1e-12)
    say("width-256 encoder, large and small GEMM tile")
    w = li.encoder_weights(cfg, li.config_seed(2) + 21, bf16_exact=True)
    tokens, lengths = li.uniform_chunks(100, 128, 1, cfg["vocab"], 16, 128, li.config_seed(2) + 22)
    lengths[:4] = [1, 31, 77, 128]
    ctx = L.leann_create(cfg, to_dev(w).to(torch.bfloat16))
    try:
        t, l = to_dev(tokens), to_dev(lengths)
        got = L.leann_embed(ctx, t, l, hidden=256).cpu().numpy()            # 12800 padded rows: large tile
        some = L.leann_embed(ctx, t, l, n_ids=48, hidden=256).cpu().numpy()  # 6144 padded rows: 128 x 128 tile
        few = L.leann_embed(ctx, t, l, n_ids=16, hidden=256).cpu().numpy()   # 2048 padded rows: 64 x 64 tile
    finally:
        L.leann_destroy(ctx)
    assert np.array_equal(got[:48], some)
    assert np.array_equal(got[:16], few)
    ids = np.array([0, 1, 2, 3, 50, 99], np.int64)
    e = orc.desc(**cfg)
    want = orc.embed(e, w, tokens, lengths, ids=ids)
    want_bf = orc.embed(e, w, tokens, lengths, ids=ids, precision=1)
    assert np.isfinite(got).all()
    assert np.abs(got[ids] - want).max() <= TOL_FP32
    assert np.abs(got[ids] - want_bf).max() <= TOL_BF16_MODE
    print("width-256 sample max-abs vs fp32 oracle %.3e, vs bf16-mode oracle %.3e" %
          (np.abs(got[ids] - want).max(), np.abs(got[ids] - want_bf).max()))
