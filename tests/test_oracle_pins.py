"""Pins for the CPU oracle: closed forms, hand cases, brute force and library routines.

None of these re-types the oracle's own formula: each expected value comes from
a closed form, a hand-worked case file, a brute-force search or an independent
library routine (torch CPU ops in float64).
"""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from et_inputs import TINY, EncoderShape, make_weights, make_clip
from oracle import earlytom_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _cases(name):
    out = []
    for line in open(os.path.join(GOLD, name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        parts = [p.strip() for p in line.split("|")]
        out.append([p.split() for p in parts])
    return out


# ---------------------------------------------------------------- encoder pieces

def test_layer_norm_textbook_values():
    x = np.array([[1.0, 2.0, 3.0, 4.0]])
    # mean 2.5, biased variance 1.25
    y = O.layer_norm(x, np.ones(4), np.zeros(4), 0.0)
    expect = np.array([-1.5, -0.5, 0.5, 1.5]) / math.sqrt(1.25)
    np.testing.assert_allclose(y[0], expect, rtol=1e-14)
    # constant row -> beta exactly (numerator is 0), eps keeps it finite
    y = O.layer_norm(np.full((1, 4), 7.0), np.array([1., 2., 3., 4.]), np.array([.1, .2, .3, .4]), 1e-6)
    np.testing.assert_allclose(y[0], [.1, .2, .3, .4], rtol=0, atol=1e-15)
    # gain and bias act per feature after normalisation
    y = O.layer_norm(x, np.array([2., 2., 2., 2.]), np.array([1., 1., 1., 1.]), 0.0)
    np.testing.assert_allclose(y[0], 2 * expect + 1, rtol=1e-14)


def test_layer_norm_matches_library():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 7, 48))
    g, b = rng.standard_normal(48), rng.standard_normal(48)
    ref = F.layer_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), torch.from_numpy(b), 1e-6)
    np.testing.assert_allclose(O.layer_norm(x, g, b, 1e-6), ref.numpy(), rtol=1e-12, atol=1e-12)


def test_softmax_closed_forms():
    np.testing.assert_allclose(O.softmax_rows(np.zeros((2, 5))), np.full((2, 5), 0.2), rtol=1e-15)
    np.testing.assert_allclose(O.softmax_rows(np.array([[0.0, math.log(2.0)]])), [[1 / 3, 2 / 3]],
                               rtol=1e-15)
    # shift invariance and no overflow for huge logits
    np.testing.assert_allclose(O.softmax_rows(np.array([[1000.0, 1000.0 + math.log(3.0)]])),
                               [[0.25, 0.75]], rtol=1e-12)


def test_gelu_tanh_special_values_and_library():
    assert O.gelu_tanh(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(O.gelu_tanh(np.array([30.0, -30.0])), [30.0, 0.0], atol=1e-12)
    # value worked by hand: sqrt(2/pi)*1.044715 = 0.8335633; tanh = 0.6823844; 0.5*1.6823844
    np.testing.assert_allclose(O.gelu_tanh(np.array([1.0]))[0], 0.8411920, atol=2e-7)
    u = np.linspace(-6, 6, 241)
    ref = F.gelu(torch.from_numpy(u), approximate="tanh").numpy()
    np.testing.assert_allclose(O.gelu_tanh(u), ref, rtol=1e-12, atol=1e-14)
    # it is the tanh form, not the erf form
    assert abs(O.gelu_tanh(np.array([1.0]))[0] - 0.5 * (1 + math.erf(1 / math.sqrt(2)))) > 1e-4


def test_patch_embed_equals_strided_convolution():
    """Patch embedding == conv2d with kernel = stride = patch (library routine); 30x33 images
    with patch 7 leave trailing pixels that must be ignored."""
    rng = np.random.default_rng(1)
    shape = EncoderShape(n_layers=1, d_model=10, n_heads=2, d_mlp=12, patch=7, image_h=30, image_w=33)
    w = make_weights(shape, 3)
    frames = rng.standard_normal((3, 3, 30, 33))
    x = O.patch_embed(frames, w, 7)
    conv = F.conv2d(torch.from_numpy(frames),
                    torch.from_numpy(w["patch_w"].astype(np.float64)).reshape(10, 3, 7, 7),
                    torch.from_numpy(w["patch_b"].astype(np.float64)), stride=7)
    assert conv.shape == (3, 10, 4, 4)
    ref = conv.flatten(2).transpose(1, 2).numpy() + w["pos_emb"].astype(np.float64)[None]
    assert x.shape == (3, 16, 10)
    np.testing.assert_allclose(x, ref, rtol=1e-12, atol=1e-12)


def _torch_block(x, lw, n_heads, eps):
    """One pre-LN ViT block from torch library routines only (float64)."""
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    x = t(x)
    Fn, n, D = x.shape
    hd = D // n_heads
    h = F.layer_norm(x, (D,), t(lw["ln1_g"]), t(lw["ln1_b"]), eps)
    qkv = F.linear(h, t(lw["wqkv"]), t(lw["bqkv"]))
    q, k, v = qkv.split(D, dim=-1)
    sp = lambda a: a.reshape(Fn, n, n_heads, hd).transpose(1, 2)
    o = F.scaled_dot_product_attention(sp(q), sp(k), sp(v))
    o = o.transpose(1, 2).reshape(Fn, n, D)
    x = x + F.linear(o, t(lw["wo"]), t(lw["bo"]))
    h = F.layer_norm(x, (D,), t(lw["ln2_g"]), t(lw["ln2_b"]), eps)
    h = F.gelu(F.linear(h, t(lw["w1"]), t(lw["b1"])), approximate="tanh")
    return (x + F.linear(h, t(lw["w2"]), t(lw["b2"]))).numpy()


def test_encoder_block_matches_library_block():
    rng = np.random.default_rng(2)
    shape = EncoderShape(n_layers=2, d_model=24, n_heads=3, d_mlp=40, patch=14, image_h=28, image_w=28)
    w = make_weights(shape, 5)
    # larger weights so attention is far from uniform and a transposed operand shows
    for lw in w["layers"]:
        for k_ in lw:
            lw[k_] = lw[k_] * (1.0 if k_.startswith("ln") else 12.0)
    x = rng.standard_normal((3, 11, 24))
    got = O.encoder_block(x, w["layers"][0], 3, 1e-6)
    ref = _torch_block(x, w["layers"][0], 3, 1e-6)
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-10)
    # frames do not interact: block on one frame == that frame's slice
    one = O.encoder_block(x[1:2], w["layers"][0], 3, 1e-6)
    np.testing.assert_allclose(one[0], got[1], rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- similarity (Sec. 3.2)

def test_similarity_closed_forms():
    rng = np.random.default_rng(3)
    L, D = 9, 16
    f0 = rng.standard_normal((L, D))
    # identical frames -> 1 ; negated -> -1 ; positive per-row rescale -> 1
    x = np.stack([f0, f0, -f0, -f0 * rng.uniform(0.5, 3.0, (L, 1))])
    c, s = O.frame_similarity(x)
    assert c.shape == (3, L) and s.shape == (3,)
    np.testing.assert_allclose(s, [1.0, -1.0, 1.0], atol=1e-14)
    # x and x + n with n orthogonal to x and |n|^2 = rho |x|^2  ->  1/sqrt(1+rho) exactly
    rho = 0.44
    n = rng.standard_normal((L, D))
    n -= (n * f0).sum(-1, keepdims=True) / (f0 * f0).sum(-1, keepdims=True) * f0
    n *= np.sqrt(rho * (f0 * f0).sum(-1, keepdims=True) / (n * n).sum(-1, keepdims=True))
    c, s = O.frame_similarity(np.stack([f0, f0 + n]))
    np.testing.assert_allclose(c[0], np.full(L, 1 / math.sqrt(1 + rho)), rtol=1e-12)
    np.testing.assert_allclose(s[0], 1 / math.sqrt(1.44), rtol=1e-12)


def test_similarity_is_mean_of_per_position_cosines_not_cosine_of_flattened():
    # two positions: one aligned (cos 1), one orthogonal (cos 0), very different norms
    x = np.zeros((2, 2, 2))
    x[0, 0] = [10, 0]; x[1, 0] = [5, 0]
    x[0, 1] = [0, 1];  x[1, 1] = [1, 0]
    c, s = O.frame_similarity(x)
    np.testing.assert_allclose(c[0], [1.0, 0.0], atol=1e-15)
    assert abs(s[0] - 0.5) < 1e-15          # flattened cosine would be ~0.98
    # pairs are (t, t-1): entry t-1 of s compares frames t and t-1
    y = np.stack([x[0], x[0], x[1]])
    _, s2 = O.frame_similarity(y)
    np.testing.assert_allclose(s2, [1.0, 0.5], atol=1e-15)


def test_similarity_zero_rows_use_eps_floor():
    x = np.zeros((2, 1, 4))
    c, s = O.frame_similarity(x)
    assert c[0, 0] == 0.0 and s[0] == 0.0


# ---------------------------------------------------------------- boundary scan (Eq. 1)

@pytest.mark.parametrize("case", _cases("segment_scan_cases.txt"))
def test_segment_scan_hand_cases(case):
    tau = float(case[0][0])
    s = np.array([float(v) for v in case[1]])
    expect = [int(v) for v in case[2]]
    got = O.segment_starts(s, tau, len(s) + 1)
    assert got.dtype == np.int32
    assert got.tolist() == expect


def test_segment_scan_properties():
    rng = np.random.default_rng(4)
    for _ in range(50):
        T = int(rng.integers(1, 40))
        s = rng.random(T - 1)
        seg = O.segment_starts(s, 0.5, T)
        assert seg[0] == 0 and seg[-1] == T and np.all(np.diff(seg) >= 1)
        assert len(seg) - 1 == 1 + int((s < 0.5).sum())
        inner = set(seg[1:-1].tolist())
        assert inner == {t for t in range(1, T) if s[t - 1] < 0.5}


# ---------------------------------------------------------------- segment mean

def test_segment_mean_special_cases():
    rng = np.random.default_rng(5)
    f = rng.standard_normal((6, 5, 8))
    # length-1 segments are copies
    np.testing.assert_array_equal(O.segment_mean(f, np.arange(7)), f)
    # identical frames -> the frame (exact for power-of-two lengths)
    x = np.stack([f[0]] * 4 + [f[1]] * 2)
    m = O.segment_mean(x, np.array([0, 4, 6]))
    np.testing.assert_array_equal(m[0], f[0])
    np.testing.assert_array_equal(m[1], f[1])
    # hand case: frames 1,2,6 -> mean 3 ; segments are contiguous frame ranges, per position
    x = np.array([1.0, 2.0, 6.0, 10.0]).reshape(4, 1, 1) * np.ones((1, 2, 3))
    m = O.segment_mean(x, np.array([0, 3, 4]))
    np.testing.assert_allclose(m[:, 0, 0], [3.0, 10.0], rtol=1e-15)
    # linearity: sum over segments of len * mean == sum of all frames
    seg = np.array([0, 2, 3, 6])
    m = O.segment_mean(f, seg)
    np.testing.assert_allclose((m * np.diff(seg)[:, None, None]).sum(0), f.sum(0), rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- selection (Eq. 4, 7)

def _brute_topk(z, k):
    """Repeatedly take the largest remaining score, lowest position first."""
    z = [(-math.inf if (isinstance(v, float) and math.isnan(v)) else v) for v in z]
    left = list(range(len(z)))
    kept = []
    for _ in range(k):
        best = left[0]
        for j in left:
            if z[j] > z[best]:
                best = j
        kept.append(best)
        left.remove(best)
    return sorted(kept)


@pytest.mark.parametrize("case", _cases("topk_cases.txt"))
def test_topk_hand_cases(case):
    k = int(case[0][0])
    z = np.array([float(v) for v in case[1]])
    assert O.topk_positions(z, k).tolist() == [int(v) for v in case[2]]


def test_topk_matches_brute_force_with_heavy_ties():
    rng = np.random.default_rng(6)
    for trial in range(300):
        n = int(rng.integers(1, 65))
        levels = int(rng.integers(1, 6))
        z = rng.integers(0, levels, n).astype(np.float64) if trial % 2 else rng.random(n)
        k = int(rng.integers(1, n + 1))
        got = O.topk_positions(z, k)
        assert got.dtype == np.int32
        assert got.tolist() == _brute_topk(z.tolist(), k)
    # k = L is the identity ; NaN ranks last
    assert O.topk_positions(np.array([2., 1., 3.]), 3).tolist() == [0, 1, 2]
    assert O.topk_positions(np.array([np.nan, 0.0, 1.0]), 2).tolist() == [1, 2]


def test_keep_count_rule():
    assert O.keep_count(64, 0.5) == 32
    assert O.keep_count(729, 0.5) == 364
    assert O.keep_count(729, 0.25) == 182
    assert O.keep_count(729, 0.3) == 218
    assert O.keep_count(10, np.float32(0.7)) == 7     # 0.7f * 10 = 6.9999999
    assert O.keep_count(729, 1.0) == 729
    assert O.keep_count(729, 1e-9) == 1


def test_compact_and_merge_select_bookkeeping():
    rng = np.random.default_rng(7)
    T, L, D = 6, 10, 8
    scenes = rng.standard_normal((2, L, D))
    x = np.concatenate([np.repeat(scenes[:1], 4, 0), np.repeat(scenes[1:], 2, 0)])
    x = x + 0.01 * rng.standard_normal(x.shape)
    r = O.merge_select(x, 0.9, 0.3)
    assert r["seg_start"].tolist() == [0, 4, 6] and r["k"] == 3
    assert r["cu_tokens"].tolist() == [0, 3, 6]
    assert r["tokens"].shape == (6, D)
    for n in range(2):
        kept = r["kept_idx"][n]
        assert np.all(np.diff(kept) > 0)
        # kept rows are the merged rows at those positions, in ascending position order
        np.testing.assert_array_equal(r["tokens"][3 * n:3 * n + 3], r["merged"][n][kept])
        # every kept score >= every dropped score
        z = r["score"][n]
        dropped = np.setdiff1d(np.arange(L), kept)
        assert z[kept].min() >= z[dropped].max()
    # the score is the squared L2 norm: scaling a token by 2 scales it by 4
    np.testing.assert_allclose(O.token_score(2 * r["merged"]), 4 * r["score"], rtol=1e-13)
    # keep_ratio = 1 with a threshold above 1 is the identity
    r = O.merge_select(x, math.inf, 1.0)
    assert r["seg_start"].tolist() == list(range(T + 1))
    np.testing.assert_array_equal(r["tokens"], x.reshape(T * L, D))
    assert r["kept_idx"].tolist() == [list(range(L))] * T


# ---------------------------------------------------------------- end-to-end invariants

@pytest.fixture(scope="module")
def tiny():
    w = make_weights(TINY, 11)
    frames = make_clip(TINY, [4, 4], 12, base="uniform", sigma=0.02)
    return w, frames


def test_disabled_compression_equals_plain_encoder(tiny):
    w, frames = tiny
    plain = O.encode_clip(TINY, w, frames, -1, 0.9, 0.5)
    assert plain["tokens"].shape == (8 * 64, 64)
    for m in (0, 2, 4):
        off = O.encode_clip(TINY, w, frames, m, math.inf, 1.0)
        np.testing.assert_allclose(off["tokens"], plain["tokens"], rtol=1e-12, atol=1e-12)
        assert off["seg_start"].tolist() == list(range(9))
        assert off["kept_idx"].tolist() == list(range(64)) * 8
    # frames are independent in the plain encoder
    for t in (0, 5):
        one = O.encode_clip(TINY, w, frames[t:t + 1], -1, 0.9, 0.5)
        np.testing.assert_allclose(one["tokens"], plain["tokens"][64 * t:64 * (t + 1)],
                                   rtol=1e-12, atol=1e-12)


def test_plain_encoder_matches_library_blocks(tiny):
    w, frames = tiny
    x = O.patch_embed(frames[:2], w, TINY.patch)
    for lw in w["layers"]:
        x = _torch_block(x, lw, TINY.n_heads, TINY.ln_eps)
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    ref = F.layer_norm(t(x), (64,), t(w["final_ln_g"]), t(w["final_ln_b"]), TINY.ln_eps).numpy()
    got = O.encode_clip(TINY, w, frames[:2], -1, 0.9, 0.5)["tokens"]
    np.testing.assert_allclose(got, ref.reshape(128, 64), rtol=1e-10, atol=1e-10)


def test_identical_frames_merge_to_the_single_frame_result(tiny):
    w, frames = tiny
    clip = np.repeat(frames[:1], 8, axis=0)
    for keep in (0.5, 1.0):
        many = O.encode_clip(TINY, w, clip, 2, 0.9, keep)
        one = O.encode_clip(TINY, w, frames[:1], 2, 0.9, keep)
        assert many["n_frames_out"] == 1 and many["seg_start"].tolist() == [0, 8]
        np.testing.assert_allclose(many["frame_sim"], np.ones(7), atol=1e-12)
        assert many["kept_idx"].tolist() == one["kept_idx"].tolist()
        np.testing.assert_allclose(many["tokens"], one["tokens"], rtol=1e-11, atol=1e-11)
    plain = O.encode_clip(TINY, w, frames[:1], -1, 0.9, 0.5)
    np.testing.assert_allclose(many["tokens"], plain["tokens"], rtol=1e-11, atol=1e-11)


def test_config1_compresses_as_designed(tiny):
    """Two static scenes of four frames: two segments, 32 of 64 tokens kept per merged frame,
    every similarity at least 1e-2 away from the threshold."""
    w, frames = tiny
    r = O.encode_clip(TINY, w, frames, 2, 0.9, 0.5)
    assert r["seg_start"].tolist() == [0, 4, 8]
    assert r["cu_tokens"].tolist() == [0, 32, 64]
    assert r["tokens"].shape == (64, 64)
    assert np.all(np.abs(r["frame_sim"] - 0.9) >= 1e-2)
    # compression sits after `merge_layer` blocks: hidden state there equals the plain
    # encoder truncated to two blocks (before its final LayerNorm)
    w2 = dict(w, layers=w["layers"][:2])
    x2 = O.patch_embed(frames, w, TINY.patch)
    for lw in w2["layers"]:
        x2 = _torch_block(x2, lw, TINY.n_heads, TINY.ln_eps)
    np.testing.assert_allclose(r["hidden_at_merge"], x2, rtol=1e-10, atol=1e-10)


def test_blocks_after_compression_run_on_the_packed_tokens(tiny):
    """After the merge layer each output frame attends only over its own kept tokens."""
    w, frames = tiny
    r = O.encode_clip(TINY, w, frames, 2, 0.9, 0.5)
    st = O.merge_select(r["hidden_at_merge"], 0.9, 0.5)
    x = st["tokens"].reshape(2, 32, 64)
    for lw in w["layers"][2:]:
        x = _torch_block(x, lw, TINY.n_heads, TINY.ln_eps)
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    ref = F.layer_norm(t(x), (64,), t(w["final_ln_g"]), t(w["final_ln_b"]), TINY.ln_eps).numpy()
    np.testing.assert_allclose(r["tokens"], ref.reshape(64, 64), rtol=1e-10, atol=1e-10)
    assert r["kept_idx"].tolist() == st["kept_idx"].reshape(-1).tolist()
    # forcing the decisions reproduces the same result; forcing others changes it
    f = O.encode_clip(TINY, w, frames, 2, 0.9, 0.5, force_seg_start=[0, 4, 8],
                      force_kept=st["kept_idx"])
    np.testing.assert_array_equal(f["tokens"], r["tokens"])


def test_projector_equals_library_linear_gelu_linear():
    """The projector (Sec. 3.1) is linear -> GELU-tanh -> linear: against torch's library routines, and a
    dropped bias or a transposed weight shows."""
    import torch
    rng = np.random.default_rng(12)
    n, D, Dh, Do = 7, 16, 24, 10
    x, w1, b1 = rng.standard_normal((n, D)), rng.standard_normal((Dh, D)) * 0.3, rng.standard_normal(Dh)
    w2, b2 = rng.standard_normal((Do, Dh)) * 0.3, rng.standard_normal(Do)
    got = O.project_tokens(x, w1, b1, w2, b2)
    t = lambda a: torch.from_numpy(a)
    want = torch.nn.functional.linear(torch.nn.functional.gelu(torch.nn.functional.linear(t(x), t(w1), t(b1)),
                                                               approximate="tanh"), t(w2), t(b2)).numpy()
    assert got.shape == (n, Do)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    assert np.max(np.abs(O.project_tokens(x, w1, 0 * b1, w2, b2) - want)) > 1e-2
    # zero input: only the biases act
    np.testing.assert_allclose(O.project_tokens(np.zeros((1, D)), w1, b1, w2, b2)[0], O.gelu_tanh(b1) @ w2.T + b2, rtol=1e-13)
