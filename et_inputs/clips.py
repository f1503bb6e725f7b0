"""Synthetic video clips: runs of near-identical frames ("scenes") plus per-frame noise."""
import numpy as np
from scipy import ndimage

from .bf16 import f32_to_bf16_bits


def scene_lengths_fixed(T, length):
    out, left = [], T
    while left > 0:
        n = min(length, left)
        out.append(n)
        left -= n
    return out


def scene_lengths_uniform(rng, T, lo, hi):
    """Scene lengths i.i.d. uniform on {lo..hi} until T frames are filled (last one cut)."""
    out, left = [], T
    while left > 0:
        n = min(int(rng.integers(lo, hi + 1)), left)
        out.append(n)
        left -= n
    return out


def scene_lengths_geometric(rng, T, mean, cut_prob=0.0):
    """Scene lengths Geometric(1/mean) on {1,2,..}; an extra per-frame chance of an abrupt cut."""
    p = 1.0 / float(mean)
    out, left = [], T
    while left > 0:
        n = int(rng.geometric(p))
        if cut_prob > 0.0:
            for j in range(1, n):
                if rng.random() < cut_prob:
                    n = j
                    break
        n = min(n, left)
        out.append(n)
        left -= n
    return out


def _base_image(rng, kind, C, H, W):
    if kind == "uniform":
        return rng.random((C, H, W), dtype=np.float64)
    if kind == "smooth":
        img = rng.standard_normal((C, H, W))
        img = ndimage.gaussian_filter(img, sigma=(0.0, 3.0, 3.0), mode="wrap")
        img -= img.mean()
        img /= img.std()
        return img
    raise ValueError(kind)


def make_clip(shape, lengths, seed, base="smooth", sigma=0.02):
    """Frames float32 [T, C, H, W]; scene j spans lengths[j] frames = base_j + N(0, sigma^2)."""
    rng = np.random.default_rng(seed)
    C, H, W = shape.channels, shape.image_h, shape.image_w
    frames = []
    for n in lengths:
        b = _base_image(rng, base, C, H, W)
        for _ in range(n):
            frames.append(b + sigma * rng.standard_normal((C, H, W)))
    return np.ascontiguousarray(np.stack(frames), dtype=np.float32)


def make_hidden_states(T, L, D, lengths, seed, sigma=0.1, dup_rows=0):
    """bf16 hidden states [T, L, D] as uint16 bit patterns: scene embedding N(0,1) + noise.

    dup_rows > 0 copies, in every scene embedding, row 0 onto that many further
    rows (before noise is skipped for them), which yields exactly tied token
    scores inside a frame for tie-break tests.
    """
    rng = np.random.default_rng(seed)
    out = np.empty((T, L, D), dtype=np.float32)
    t = 0
    for n in lengths:
        emb = rng.standard_normal((L, D))
        for _ in range(n):
            fr = emb + sigma * rng.standard_normal((L, D))
            if dup_rows > 0:
                idx = np.arange(1, 1 + dup_rows) * max(1, L // (dup_rows + 1))
                fr[idx % L] = fr[0]
            out[t] = fr
            t += 1
    assert t == T
    return f32_to_bf16_bits(out)
