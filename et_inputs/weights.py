"""Random-init encoder weights: N(0, 0.02) everywhere, LayerNorm gain 1 + N(0, 0.02)."""
import numpy as np

from .bf16 import round_to_bf16


def make_weights(shape, seed, bf16=False, n_layers=None):
    """Return a dict of float32 arrays in the layout the C boundary documents.

    Linear layers are stored out-features major (y = x @ W.T + b).
    With bf16=True every value is rounded once to a bfloat16-representable
    float32, so a bf16 engine and an fp64 oracle start from identical numbers.
    """
    rng = np.random.default_rng(seed)
    nl = shape.n_layers if n_layers is None else n_layers
    D, Mh, L, Kp = shape.d_model, shape.d_mlp, shape.tokens_per_frame, shape.patch_dim
    std = 0.02

    def normal(*s):
        a = rng.standard_normal(s, dtype=np.float32) * np.float32(std)
        return round_to_bf16(a) if bf16 else a

    def gain(*s):
        a = np.float32(1.0) + rng.standard_normal(s, dtype=np.float32) * np.float32(std)
        return round_to_bf16(a) if bf16 else a

    w = {
        "patch_w": normal(D, Kp),
        "patch_b": normal(D),
        "pos_emb": normal(L, D),
        "layers": [],
    }
    for _ in range(nl):
        w["layers"].append({
            "ln1_g": gain(D), "ln1_b": normal(D),
            "wqkv": normal(3 * D, D), "bqkv": normal(3 * D),
            "wo": normal(D, D), "bo": normal(D),
            "ln2_g": gain(D), "ln2_b": normal(D),
            "w1": normal(Mh, D), "b1": normal(Mh),
            "w2": normal(D, Mh), "b2": normal(D),
        })
    w["final_ln_g"] = gain(D)
    w["final_ln_b"] = normal(D)
    return w
