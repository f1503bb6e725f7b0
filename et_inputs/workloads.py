"""The five named synthetic workloads (stand-ins for the paper's benchmark videos)."""
import numpy as np

from .shapes import TINY, SIGLIP
from .weights import make_weights
from .clips import (make_clip, make_hidden_states, scene_lengths_fixed,
                    scene_lengths_uniform, scene_lengths_geometric)

# name -> recipe.  "variant" shifts the seed: seed = 1000 * config + variant.
WORKLOADS = {
    "c1_tiny": dict(config=1, shape=TINY, bf16=False, T=8, base="uniform", sigma=0.02,
                    lengths=("fixed", 4), merge_layer=2, sim_threshold=0.9, keep_ratio=0.5),
    "c2_siglip_t8": dict(config=2, shape=SIGLIP, bf16=True, T=8, base="smooth", sigma=0.02,
                         lengths=("uniform", 1, 4), merge_layer=8, sim_threshold=0.9,
                         keep_ratio=0.5),
    "c3_siglip_t32": dict(config=3, shape=SIGLIP, bf16=True, T=32, base="smooth", sigma=0.02,
                          lengths=("geometric", 4, 0.0), merge_layer=8, sim_threshold=0.9,
                          keep_ratio=0.5),
    "c4_siglip_t64": dict(config=4, shape=SIGLIP, bf16=True, T=64, base="smooth", sigma=0.05,
                          lengths=("geometric", 8, 0.10), merge_layer=4, sim_threshold=0.85,
                          keep_ratio=0.25),
    "c5_merge_only": dict(config=5, shape=SIGLIP, T=64, sigma=0.1,
                          lengths=("geometric", 8, 0.0), sim_threshold=0.9, keep_ratio=0.3),
}


def _lengths(rng, spec, T):
    if spec[0] == "fixed":
        return scene_lengths_fixed(T, spec[1])
    if spec[0] == "uniform":
        return scene_lengths_uniform(rng, T, spec[1], spec[2])
    if spec[0] == "geometric":
        return scene_lengths_geometric(rng, T, spec[1], spec[2])
    raise ValueError(spec)


def build_workload(name, variant=0, T=None, with_weights=True, n_layers=None):
    """Materialise one workload.  Returns a dict with the recipe plus the arrays.

    Encoder workloads: "weights" (see make_weights), "frames" float32 [T,C,H,W],
    "lengths" (ground-truth scene lengths).  c5: "x_bits" uint16 [T,L,D].
    """
    rec = dict(WORKLOADS[name])
    seed = 1000 * rec["config"] + variant
    rng = np.random.default_rng(seed)
    if T is not None:
        rec["T"] = T
    lengths = _lengths(rng, rec["lengths"], rec["T"])
    rec["lengths"] = lengths
    rec["seed"] = seed
    shape = rec["shape"]
    if name == "c5_merge_only":
        rec["x_bits"] = make_hidden_states(rec["T"], shape.tokens_per_frame, shape.d_model,
                                           lengths, seed + 500, sigma=rec["sigma"])
        return rec
    if with_weights:
        rec["weights"] = make_weights(shape, seed + 100, bf16=rec["bf16"], n_layers=n_layers)
    rec["frames"] = make_clip(shape, lengths, seed + 200, base=rec["base"], sigma=rec["sigma"])
    return rec
