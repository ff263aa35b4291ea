"""Encoder shapes and seeds of the benchmark configurations."""

SEED0 = 20250608


def config_seed(index):
    """One documented 64-bit seed per configuration: SEED0 + configuration index."""
    return SEED0 + int(index)


# layers, hidden, heads, ffn, vocab, max_pos, ln_eps
TINY = dict(layers=2, hidden=128, heads=2, ffn=512, vocab=1000, max_pos=64, ln_eps=1e-12)
BASE = dict(layers=12, hidden=768, heads=12, ffn=3072, vocab=30522, max_pos=512, ln_eps=1e-12)
# second throughput point: a 34 M-parameter encoder (App. D, the ablation with a lightweight embedding model); the paper gives
# only the parameter count, the 12 x 384 split is this repository's choice
SMALL = dict(layers=12, hidden=384, heads=6, ffn=1536, vocab=30522, max_pos=512, ln_eps=1e-12)
BASE_S128 = dict(BASE)
