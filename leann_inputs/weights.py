"""Random-init encoder weights in the packed order both sides accept.

Packed order (fp32, row-major, linear maps stored [out][in]):
  tok_emb[vocab][d], pos_emb[max_pos][d], seg_emb[d], emb_ln_g[d], emb_ln_b[d],
  per layer: Wqkv[3d][d], bqkv[3d], Wo[d][d], bo[d], ln1_g[d], ln1_b[d],
             W1[F][d], b1[F], W2[d][F], b2[d], ln2_g[d], ln2_b[d].
"""
import numpy as np


def weight_layout(cfg):
    """List of (name, shape, kind) in packed order; kind in {matrix, bias, gamma, beta}."""
    d, F = cfg["hidden"], cfg["ffn"]
    out = [("tok_emb", (cfg["vocab"], d), "matrix"), ("pos_emb", (cfg["max_pos"], d), "matrix"),
           ("seg_emb", (d,), "matrix"), ("emb_ln_g", (d,), "gamma"), ("emb_ln_b", (d,), "beta")]
    for l in range(cfg["layers"]):
        out += [(f"l{l}.wqkv", (3 * d, d), "matrix"), (f"l{l}.bqkv", (3 * d,), "bias"),
                (f"l{l}.wo", (d, d), "matrix"), (f"l{l}.bo", (d,), "bias"),
                (f"l{l}.ln1_g", (d,), "gamma"), (f"l{l}.ln1_b", (d,), "beta"),
                (f"l{l}.w1", (F, d), "matrix"), (f"l{l}.b1", (F,), "bias"),
                (f"l{l}.w2", (d, F), "matrix"), (f"l{l}.b2", (d,), "bias"),
                (f"l{l}.ln2_g", (d,), "gamma"), (f"l{l}.ln2_b", (d,), "beta")]
    return out


def to_bf16_exact(a):
    """Round fp32 values to the nearest bf16-representable fp32 (ties to even)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def encoder_weights(cfg, seed, std=0.02, perturb=False, bf16_exact=False, as_dict=False):
    """N(0, std) matrices and embeddings; biases 0, gamma 1, beta 0.

    perturb=True draws non-trivial biases / LayerNorm parameters instead, so
    that a dropped bias or scale shows up in a comparison.  bf16_exact=True
    rounds matrices and embedding tables to bf16-representable values (the
    "random-init bf16 weights" of the encoder-throughput configuration).
    """
    rng = np.random.Generator(np.random.Philox(seed))
    parts, named = [], {}
    for name, shape, kind in weight_layout(cfg):
        if kind == "matrix":
            w = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
            if bf16_exact:
                w = to_bf16_exact(w)
        elif kind == "bias" or kind == "beta":
            w = (rng.standard_normal(shape, dtype=np.float32) * np.float32(std)) if perturb \
                else np.zeros(shape, np.float32)
        else:
            w = (1.0 + 0.1 * rng.standard_normal(shape, dtype=np.float32)).astype(np.float32) if perturb \
                else np.ones(shape, np.float32)
        named[name] = w
        parts.append(w.reshape(-1))
    packed = np.concatenate(parts).astype(np.float32)
    return (packed, named) if as_dict else packed
