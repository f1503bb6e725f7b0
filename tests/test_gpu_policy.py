"""GPU parity of the paper-exact compression forms (Eq. 1 with smoothing, Alg. 1, Alg. 2) against
the oracle's *_policy functions, through the C boundary.  Same bars as the simple path: integer
outputs bit-exact on inputs with safe decision margins, merged tokens within one bf16 step,
encoder tokens within relative L2 2e-2."""
import math

import numpy as np
import pytest
import torch

import paper_2605_30010_amd as et
from et_inputs import (TINY, SIGLIP, bf16_bits_to_f32, build_workload, make_clip, make_hidden_states,
                       scene_lengths_geometric)
from oracle import earlytom_oracle as O
from tests._util import bits_to_dev, dev_to_bits, dev_to_f64, bf16_ulp_distance, f64_to_bits, rel_l2

pytestmark = pytest.mark.gpu

POLICIES = [
    dict(merge_mode="alg1", select_mode="decoupled", alpha=0.9, tau_seg=0.8, tau_merge=0.8, ratio=0.2),
    dict(merge_mode="alg1", select_mode="uniform", alpha=0.9, tau_seg=0.8, tau_merge=0.8, ratio=0.3),
    dict(merge_mode="mean", select_mode="decoupled", alpha=1.0, tau_seg=0.9, tau_merge=0.9, ratio=0.1),
    dict(merge_mode="mean", select_mode="uniform", alpha=1.0, tau_seg=0.9, tau_merge=0.9, ratio=0.3),
    dict(merge_mode="alg1", select_mode="decoupled", alpha=0.5, tau_seg=0.9, tau_merge=0.995, ratio=0.6),
]


def _f32_policy(p):
    q = dict(p)
    for k in ("alpha", "tau_seg", "tau_merge", "ratio"):
        q[k] = float(np.float32(p[k]))
    return q


def _margins_ok(ref, pol, L):
    """Decisions are only promised bit-exact away from ties: smoothed similarities 1e-2 from tau_seg,
    Alg. 1 comparisons s_i vs s_{i+1} 1e-6 apart (float32 similarities agree to ~1e-7), selection gaps (k-th vs next score; best vs second in a window)
    2e-6 relative, ten times the float32 rounding of a 1152-term sum of squares."""
    if len(ref["s_hat"]) and np.min(np.abs(ref["s_hat"] - pol["tau_seg"])) < 1e-2:
        return False
    s = ref["frame_sim"]
    if pol["merge_mode"] == "alg1" and len(s) > 1:
        if np.min(np.abs(np.diff(s))) < 1e-6 or np.min(np.abs(s - pol["tau_merge"])) < 1e-5:
            return False
    cu = ref["cu_tokens"]
    for n, z in enumerate(ref["score"]):
        k = int(cu[n + 1] - cu[n])
        if ref["frame_dynamic"][n] or pol["select_mode"] == "uniform":
            zs = np.sort(z)[::-1]
            if k < L and (zs[k - 1] - zs[k]) < 2e-6 * zs[k - 1]:
                return False
        else:                                          # static frame: top-2 gap inside every window
            w = -(-L // k) if k > 0 else L
            w = L // O.rescaled_count(pol["ratio"], len(ref["frame_sim"]) + 1, L, len(ref["plan"]))
            for lo in range(0, L, w):
                win = np.sort(z[lo:lo + w])[::-1]
                if len(win) > 1 and (win[0] - win[1]) < 2e-6 * win[0]:
                    return False
    return True


def _check_stage(r, ref, exact_tokens=False):
    assert r["n_frames_out"] == len(ref["plan"])
    assert r["n_segments"] == len(ref["seg_start"]) - 1
    assert r["seg_start"].tolist() == ref["seg_start"].tolist()
    assert r["frame_first"].tolist() == ref["frame_first"].tolist()
    assert r["frame_count"].tolist() == ref["frame_count"].tolist()
    assert r["frame_dynamic"].tolist() == ref["frame_dynamic"].tolist()
    assert r["cu_tokens"].tolist() == ref["cu_tokens"].tolist()
    assert r["n_tokens"] == int(ref["cu_tokens"][-1])
    assert np.array_equal(r["kept_idx"].cpu().numpy(), ref["kept_idx"])
    got_bits = dev_to_bits(r["tokens"])
    dist = bf16_ulp_distance(got_bits, f64_to_bits(ref["tokens"]))
    if exact_tokens:
        assert dist.max() == 0
    else:
        # one bf16 step at most, except where a fused pair cancels to almost nothing: there the float32
        # rounding of w0 x0 + w1 x1 (about 1e-8 absolute) is no longer small against the result
        got = bf16_bits_to_f32(got_bits).astype(np.float64)
        assert np.all((dist <= 1) | (np.abs(got - ref["tokens"]) <= 1e-7))
        # Fused pairs have weights within 1e-5 of 1/2, so (x0 + x1) / 2 of two bf16 values lands on or
        # next to a bf16 rounding tie for a large share of elements; which way those round depends on
        # the last float32 bits of the weights.  Hence a looser bound on how many differ (by one step).
        assert (dist > 0).mean() < 0.05


@pytest.mark.parametrize("pi", range(len(POLICIES)))
@pytest.mark.parametrize("T,L,D,mean_len", [(14, 100, 256, 4), (40, 729, 1152, 6), (33, 64, 64, 5)])
def test_merge_select_policy_matches_oracle(pi, T, L, D, mean_len):
    pol = _f32_policy(POLICIES[pi])
    for variant in range(80):
        rng = np.random.default_rng(1000 * pi + 10 * T + variant)
        lengths = scene_lengths_geometric(rng, T, mean_len)
        bits = make_hidden_states(T, L, D, lengths, 31 * T + variant, sigma=0.1)
        ref = O.merge_select_policy(bf16_bits_to_f32(bits).astype(np.float64), pol)
        if _margins_ok(ref, pol, L):
            break
    else:
        pytest.fail("no seed with safe margins")
    r = et.et_merge_select_policy(bits_to_dev(bits), pol)
    _check_stage(r, ref)
    if pol["merge_mode"] == "alg1":
        assert r["n_frames_out"] >= r["n_segments"]
    # the default policy is the simple entry point, bit for bit
    if pol["merge_mode"] == "mean" and pol["select_mode"] == "uniform":
        simple = et.et_merge_select(bits_to_dev(bits), pol["tau_seg"], pol["ratio"])
        assert torch.equal(simple["tokens"], r["tokens"]) and torch.equal(simple["kept_idx"], r["kept_idx"])
        assert simple["cu_tokens"].tolist() == r["cu_tokens"].tolist()


def _alg1_golden_cases():
    import os
    out = []
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "alg1_cases.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        p = [q.strip() for q in line.split("|")]
        if len(p) > 4 and p[4] == "exact":
            continue                      # sits on an equality: only meaningful for exactly given similarities
        alpha, tau_seg, tau_merge = [float(v) for v in p[0].split()]
        frames = [(int(t.split(":")[0]), int(t.split(":")[1].split("(")[0])) for t in p[3].split()]
        out.append((alpha, tau_seg, tau_merge, [float(v) for v in p[1].split()], [int(v) for v in p[2].split()], frames))
    return out


@pytest.mark.parametrize("case", _alg1_golden_cases())
def test_device_plan_on_the_hand_worked_alg1_cases(case):
    """The hand-worked cases of Eq. 1 / Alg. 1 (tests/golden/alg1_cases.txt) against the DEVICE plan, not via the
    oracle: hidden states are built so that every position's cosine between frames t and t-1 is the case's s_t
    (x_t = s_t x_{t-1} + sqrt(1 - s_t^2) w_t with w_t a fresh unit vector orthogonal to x_{t-1}); the bfloat16
    rounding moves a similarity by < 1e-3, the cases keep every comparison at least 5e-3 apart."""
    alpha, tau_seg, tau_merge, s, seg, frames = case
    T, L, D = len(s) + 1, 8, 256
    rng = np.random.default_rng(T * 7 + len(frames))
    x = np.empty((T, L, D))
    x[0] = rng.standard_normal((L, D))
    x[0] /= np.linalg.norm(x[0], axis=-1, keepdims=True)
    for t in range(1, T):
        w = rng.standard_normal((L, D))
        w -= (w * x[t - 1]).sum(-1, keepdims=True) * x[t - 1]
        w /= np.linalg.norm(w, axis=-1, keepdims=True)
        x[t] = s[t - 1] * x[t - 1] + math.sqrt(1.0 - s[t - 1] ** 2) * w
    bits = f64_to_bits(x * 3.0)
    pol = _f32_policy(dict(merge_mode="alg1", select_mode="uniform", alpha=alpha, tau_seg=tau_seg, tau_merge=tau_merge,
                           ratio=1.0))
    r = et.et_merge_select_policy(bits_to_dev(bits), pol)
    np.testing.assert_allclose(r["frame_sim"].cpu().numpy(), s, atol=1.5e-3)
    assert r["seg_start"].tolist() == seg
    assert list(zip(r["frame_first"].tolist(), r["frame_count"].tolist())) == frames
    dyn = r["frame_dynamic"].tolist()
    for n in range(len(seg) - 1):                    # head and tail of every segment are the dynamic frames
        idx = [i for i, (f, c) in enumerate(frames) if seg[n] <= f < seg[n + 1]]
        assert [dyn[i] for i in idx] == [1 if i in (idx[0], idx[-1]) else 0 for i in idx]


def test_policy_degenerate_cases():
    rng = np.random.default_rng(5)
    from et_inputs import f32_to_bf16_bits
    L, D = 48, 128
    one = f32_to_bf16_bits(rng.standard_normal((1, L, D)).astype(np.float32))
    pol = _f32_policy(POLICIES[0])
    ref = O.merge_select_policy(bf16_bits_to_f32(one).astype(np.float64), pol)
    _check_stage(et.et_merge_select_policy(bits_to_dev(one), pol), ref, exact_tokens=True)
    # identical frames: similarities tie at 1, the strict rule of Eq. 2 fuses nothing
    same = np.repeat(one, 7, axis=0)
    r = et.et_merge_select_policy(bits_to_dev(same), dict(pol, ratio=1.0))
    assert r["n_segments"] == 1 and r["n_frames_out"] == 7 and r["frame_count"].tolist() == [1] * 7
    assert r["frame_dynamic"].tolist() == [1, 0, 0, 0, 0, 0, 1]
    # ratio 1 with nothing merged keeps everything in order
    many = f32_to_bf16_bits(rng.standard_normal((5, L, D)).astype(np.float32))
    r = et.et_merge_select_policy(bits_to_dev(many), dict(pol, tau_seg=math.inf, ratio=1.0))
    assert r["n_frames_out"] == 5 and r["n_tokens"] == 5 * L
    assert np.array_equal(dev_to_bits(r["tokens"]), many.reshape(5 * L, D))
    lib = et.load_library()
    with pytest.raises(et.EtError):
        et.et_merge_select_policy(bits_to_dev(many), dict(pol, alpha=0.0))
    with pytest.raises(et.EtError):
        et.et_merge_select_policy(bits_to_dev(many), dict(pol, ratio=1.5))


def _encode_check(shape, w, frames, m, pol, tol=2e-2):
    T = frames.shape[0]
    L, D = shape.tokens_per_frame, shape.d_model
    from dataclasses import replace
    trunc = et.Encoder(replace(shape, n_layers=m, has_final_ln=0), dict(w, layers=w["layers"][:m]), T)
    xm = trunc.encode(torch.from_numpy(frames).cuda(), -1, 0.0, 1.0)["tokens"].clone()
    trunc.close()
    x_gpu = bf16_bits_to_f32(dev_to_bits(xm)).astype(np.float64).reshape(T, L, D)
    enc = et.Encoder(shape, w, T)
    got = enc.encode_policy(torch.from_numpy(frames).cuda(), m, pol)
    got = {k: (v.clone() if isinstance(v, torch.Tensor) else v) for k, v in got.items()}
    enc.close()
    ref = O.encode_clip_policy(shape, w, frames, m, pol, x_at_merge=x_gpu)
    assert got["seg_start"].tolist() == ref["seg_start"].tolist()
    assert got["frame_first"].tolist() == ref["frame_first"].tolist()
    assert got["frame_count"].tolist() == ref["frame_count"].tolist()
    assert got["cu_tokens"].tolist() == ref["cu_tokens"].tolist()
    same = np.array_equal(got["kept_idx"].cpu().numpy(), ref["kept_idx"])
    if not same:      # near-tied scores: separate arithmetic error from rank flips
        cu = ref["cu_tokens"]
        kept = got["kept_idx"].cpu().numpy()
        ref = O.encode_clip_policy(shape, w, frames, m, pol, x_at_merge=x_gpu,
                                   force_kept=[kept[cu[n]:cu[n + 1]] for n in range(len(cu) - 1)])
    err = rel_l2(dev_to_f64(got["tokens"]), ref["tokens"])
    assert err <= tol, err
    return got, ref, err, same


def test_tiny_encoder_with_paper_policy():
    rec = build_workload("c1_tiny")
    w = rec["weights"]
    frames = make_clip(TINY, [6, 1, 5], 21, base="uniform", sigma=0.02)
    pol = _f32_policy(dict(merge_mode="alg1", select_mode="decoupled", alpha=0.9, tau_seg=0.9, tau_merge=0.9,
                           ratio=0.25))
    got, ref, err, same = _encode_check(TINY, w, frames, 2, pol)
    assert got["seg_start"].tolist() == [0, 6, 7, 12]
    assert same
    counts = np.diff(got["cu_tokens"].cpu().numpy())
    assert len(set(counts.tolist())) == 2                     # ragged: dynamic and static counts differ
    # the default policy equals the simple entry point bit for bit
    enc = et.Encoder(TINY, w, 12)
    a = enc.encode(torch.from_numpy(frames).cuda(), 2, 0.9, 0.5)
    a = {k: (v.clone() if isinstance(v, torch.Tensor) else v) for k, v in a.items()}
    b = enc.encode_policy(torch.from_numpy(frames).cuda(), 2,
                          dict(merge_mode="mean", select_mode="uniform", alpha=1.0, tau_seg=0.9, tau_merge=0.9,
                               ratio=0.5))
    assert torch.equal(a["tokens"], b["tokens"]) and torch.equal(a["kept_idx"], b["kept_idx"])
    enc.close()


def test_siglip_32_frames_with_paper_policy():
    """32-frame SigLIP-shaped clip under the paper's settings (alpha 0.9, three-frame-plus segments
    fused by Alg. 1, 20 % overall retention with decoupled selection)."""
    rec = build_workload("c3_siglip_t32")
    pol = _f32_policy(dict(merge_mode="alg1", select_mode="decoupled", alpha=0.9, tau_seg=0.8, tau_merge=0.8,
                           ratio=0.2))
    got, ref, err, same = _encode_check(SIGLIP, rec["weights"], rec["frames"], 8, pol)
    truth = np.concatenate([[0], np.cumsum(rec["lengths"])]).tolist()
    assert got["seg_start"].tolist() == truth
    total_in = 32 * 729
    assert abs(got["n_tokens"] / total_in - 0.2) < 0.03
    print("paper policy, 32 frames: N=%d tokens=%d (%.1f%%) rel-L2 %.4g, indices identical: %s"
          % (got["n_frames_out"], got["n_tokens"], 100.0 * got["n_tokens"] / total_in, err, same))


# ---- Stage I at several layers, Stage II once (Table 8) ---------------------------------------

ALL_TOKENS = dict(merge_mode="mean", select_mode="uniform", alpha=1.0, tau_seg=0.9, tau_merge=0.9, ratio=1.0)


def _gpu_hidden_at(shape, w, frames, merge_layers, layer, pol, as_device=False):
    """bf16 hidden states the device path sees at `layer`, given the merges at `merge_layers` (all
    <= layer; those before `layer` have run, and if `layer` itself is listed, so has its own merge): an
    encoder cut after `layer` blocks that keeps every token."""
    from dataclasses import replace
    T = frames.shape[0]
    L, D = shape.tokens_per_frame, shape.d_model
    enc = et.Encoder(replace(shape, n_layers=layer, has_final_ln=0), dict(w, layers=w["layers"][:layer]), T)
    fr = torch.from_numpy(frames).cuda()
    if merge_layers:
        keep_all = dict(pol, select_mode="uniform", ratio=1.0, score_mode="l2")
        r = enc.encode_multi(fr, merge_layers, layer, keep_all)
        assert r["n_tokens"] == r["n_frames_out"] * L
        assert np.array_equal(r["kept_idx"].cpu().numpy(), np.tile(np.arange(L), r["n_frames_out"]))
    else:
        r = enc.encode(fr, -1, 0.0, 1.0)
    if as_device:
        x = r["tokens"].clone()
    else:
        x = bf16_bits_to_f32(dev_to_bits(r["tokens"])).astype(np.float64).reshape(-1, L, D)
    enc.close()
    return x


def _stage_margins_ok(ref, pol):
    for st in ref["stages"].values():
        if len(st["s_hat"]) and np.min(np.abs(st["s_hat"] - pol["tau_seg"])) < 1e-2:
            return False
        s = st["frame_sim"]
        if pol["merge_mode"] == "alg1" and len(s) > 1:
            if np.min(np.abs(np.diff(s))) < 1e-6 or np.min(np.abs(s - pol["tau_merge"])) < 1e-5:
                return False
    return True


def _selection_margins_ok(ref, pol, L, T):
    cu = ref["cu_tokens"]
    for n, z in enumerate(ref["score"]):
        k = int(cu[n + 1] - cu[n])
        if ref["frame_dynamic"][n] or pol["select_mode"] == "uniform":
            zs = np.sort(z)[::-1]
            if k < L and (zs[k - 1] - zs[k]) < 2e-6 * zs[k - 1]:
                return False
        else:
            w = L // O.rescaled_count(pol["ratio"], T, L, len(ref["score"]))
            for lo in range(0, L, w):
                win = np.sort(z[lo:lo + w])[::-1]
                if len(win) > 1 and (win[0] - win[1]) < 2e-6 * win[0]:
                    return False
    return True


def _multi_check(shape, w, frames, merge_layers, select_layer, pol, tol=2e-2, strict_selection=True):
    """Device path against the oracle fed the device's own bf16 hidden states at every stage layer, so
    that each stage is compared on identical inputs; the tokens are compared end to end."""
    T = frames.shape[0]
    L = shape.tokens_per_frame
    x_at = {}
    by_attention = pol.get("score_mode", "l2") == "attention"
    for layer in sorted(set(merge_layers) | {select_layer} | ({select_layer - 1} if by_attention else set())):
        x_at[layer] = _gpu_hidden_at(shape, w, frames, [m for m in merge_layers if m < layer], layer, pol)
    # decisions are promised away from ties only: look at every merge layer's similarities first (a
    # tie there may already have given the next stage a different number of frames)
    for layer in merge_layers:
        s_l = O.frame_similarity(x_at[layer])[1]
        _, s_hat = O.ema_segment_starts(s_l, pol["alpha"], pol["tau_seg"], x_at[layer].shape[0])
        if not _stage_margins_ok(dict(stages={layer: dict(frame_sim=s_l, s_hat=s_hat)}), pol):
            return None
    enc = et.Encoder(shape, w, T)
    got = enc.encode_multi(torch.from_numpy(frames).cuda(), merge_layers, select_layer, pol)
    got = {k: (v.clone() if isinstance(v, torch.Tensor) else v) for k, v in got.items()}
    qk = None
    if by_attention:
        # The ranking is compared on identical inputs, like every other stage: the device's own bf16 q | k of
        # the scoring block (its first two launches, on the frames that block sees) go into the oracle's
        # plain softmax / column-mean arithmetic.
        sl = select_layer - 1
        x_dev = _gpu_hidden_at(shape, w, frames, [m for m in merge_layers if m <= sl], sl, pol, as_device=True)
        qkv, _ = et.et_encoder_block_qkv(enc.handle, sl, x_dev)
        D = shape.d_model
        qk = bf16_bits_to_f32(dev_to_bits(qkv[:, :2 * D].contiguous())).astype(np.float64).reshape(-1, L, 2 * D)
    enc.close()
    ref = O.encode_clip_multi(shape, w, frames, merge_layers, select_layer, pol, x_at_layers=x_at,
                              qk_at_score_layer=qk)
    if not _stage_margins_ok(ref, pol) or (strict_selection and not _selection_margins_ok(ref, pol, L, T)):
        return None
    for layer, st in ref["stages"].items():          # every stage saw the frame count the oracle derives
        later = [j for j in x_at if j > layer]
        if later:
            assert x_at[min(later)].shape[0] == st["n_frames"]
    assert got["n_frames_out"] == ref["n_frames_out"]
    assert got["seg_start"].tolist() == ref["seg_start"].tolist()
    assert got["frame_first"].tolist() == ref["frame_first"].tolist()
    assert got["frame_count"].tolist() == ref["frame_count"].tolist()
    assert got["frame_dynamic"].tolist() == ref["frame_dynamic"].tolist()
    assert got["cu_tokens"].tolist() == ref["cu_tokens"].tolist()
    kept = got["kept_idx"].cpu().numpy()
    same = np.array_equal(kept, ref["kept_idx"])
    if by_attention:
        # Same q and k on both sides: what is left is the float32 rounding of the device's softmax sums
        # (~2e-5 relative on a score).  The device's choice must be a correct selection for the oracle's
        # scores within 1e-4, and the positions where it differs from the oracle's own choice are few.
        r_hat = O.rescaled_count(pol["ratio"], T, L, ref["n_frames_out"])
        assert _selection_valid(kept, ref["cu_tokens"], ref["score"], ref["frame_dynamic"],
                                pol["select_mode"] == "uniform", r_hat, L, 1e-4)
        cu = ref["cu_tokens"]
        swapped = sum(len(np.setdiff1d(kept[cu[n]:cu[n + 1]], ref["kept_idx"][cu[n]:cu[n + 1]])) for n in range(len(cu) - 1))
        assert swapped <= 0.005 * len(kept) + 1
        # Against the oracle's scores computed from the hidden states in float64 all the way (no device q, k):
        # the device stores q and k in bfloat16 (relative step 2^-8), which moves a logit by ~|s| 2^-8 and a
        # score by a few 1e-3 relative; the device's selection must still be valid for those scores within 2e-2.
        plain = O.encode_clip_multi(shape, w, frames, merge_layers, select_layer, pol, x_at_layers=x_at)
        assert np.max(np.abs(plain["score"] - ref["score"]) / plain["score"]) < 2e-2
        assert _selection_valid(kept, plain["cu_tokens"], plain["score"], plain["frame_dynamic"],
                                pol["select_mode"] == "uniform", r_hat, L, 2e-2)
    if strict_selection:
        assert same
    elif not same and not by_attention:      # near-tied scores somewhere: few flips, and the tokens compared on the device's choice
        assert (kept != ref["kept_idx"]).mean() < 2e-3
    if not same:
        cu = ref["cu_tokens"]
        ref = O.encode_clip_multi(shape, w, frames, merge_layers, select_layer, pol, x_at_layers=x_at,
                                  force_kept=[kept[cu[n]:cu[n + 1]] for n in range(len(cu) - 1)])
    err = rel_l2(dev_to_f64(got["tokens"]), ref["tokens"])
    assert err <= tol, err
    return got, ref, err


@pytest.mark.gpu
@pytest.mark.parametrize("merge_layers,select_layer,pi", [([1, 2], 3, 0), ([0, 2, 3], 4, 2), ([], 2, 0),
                                                          ([1, 3], 3, 4), ([2], 2, 1)])
def test_tiny_encoder_multi_layer_merging(merge_layers, select_layer, pi):
    rec = build_workload("c1_tiny")
    w = rec["weights"]
    pol = _f32_policy(dict(POLICIES[pi], tau_seg=0.9, tau_merge=0.9))
    for seed in range(40):
        frames = make_clip(TINY, [7, 2, 6, 1], 300 + seed, base="uniform", sigma=0.02)
        res = _multi_check(TINY, w, frames, merge_layers, select_layer, pol)
        if res is not None:
            break
    else:
        pytest.fail("no clip with clear margins in 40 seeds")
    got, ref, err = res
    if merge_layers:
        assert got["n_frames_out"] < 16
    first, count = got["frame_first"].cpu().numpy(), got["frame_count"].cpu().numpy()
    assert first[0] == 0 and np.array_equal(first[1:], (first + count)[:-1]) and first[-1] + count[-1] == 16


@pytest.mark.gpu
def test_multi_equals_single_layer_entry_point():
    rec = build_workload("c1_tiny")
    w = rec["weights"]
    frames = torch.from_numpy(make_clip(TINY, [6, 1, 5], 21, base="uniform", sigma=0.02)).cuda()
    enc = et.Encoder(TINY, w, 12)
    for pol in POLICIES:
        a = enc.encode_policy(frames, 2, pol)
        a = {k: (v.clone() if isinstance(v, torch.Tensor) else v) for k, v in a.items()}
        b = enc.encode_multi(frames, [2], 2, pol)
        for key in ("tokens", "kept_idx", "cu_tokens", "seg_start", "frame_first", "frame_count", "frame_dynamic"):
            assert torch.equal(a[key], b[key]), key
    enc.close()


@pytest.mark.gpu
def test_siglip_multi_layer_merging_stagewise():
    """SigLIP-sized layers (6 of them), merges after blocks 2 and 4, selection after block 5."""
    from dataclasses import replace
    shape = replace(SIGLIP, n_layers=6)
    pol = _f32_policy(dict(merge_mode="alg1", select_mode="decoupled", alpha=0.9, tau_seg=0.8, tau_merge=0.8,
                           ratio=0.25))
    rec = build_workload("c2_siglip_t8", n_layers=6)
    rec["lengths"] = [6, 1, 5]
    for seed in range(10):
        # frame noise 0.2: in-scene similarities near 0.96 whose differences (about 1e-4) decide Alg. 1
        # well clear of float32 rounding
        frames = make_clip(SIGLIP, rec["lengths"], 700 + seed, base=rec["base"], sigma=0.2)
        res = _multi_check(shape, rec["weights"], frames, [2, 4], 5, pol, strict_selection=False)
        if res is not None:
            break
    else:
        pytest.fail("no clip with clear margins")
    got, ref, err = res
    print("multi-layer SigLIP-size: scenes %s, N = %d, tokens = %d, rel-L2 = %.4f"
          % (rec["lengths"], got["n_frames_out"], got["n_tokens"], err))
    assert got["n_frames_out"] < 12


@pytest.mark.gpu
def test_siglip_32_frames_three_merge_layers_selection_after_encoder():
    """The paper's layer choice at full size: Stage I after blocks 6, 14 and 20, Stage II on the
    encoder output (27 blocks), 32 frames, 20 % retention."""
    rec = build_workload("c3_siglip_t32")
    pol = _f32_policy(dict(merge_mode="alg1", select_mode="decoupled", alpha=0.9, tau_seg=0.8, tau_merge=0.8,
                           ratio=0.2))
    for seed in range(4):
        frames = make_clip(SIGLIP, rec["lengths"], 900 + seed, base=rec["base"], sigma=0.2)
        res = _multi_check(SIGLIP, rec["weights"], frames, [6, 14, 20], 27, pol, strict_selection=False)
        if res is not None:
            break
    else:
        pytest.fail("no clip with clear margins")
    got, ref, err = res
    counts = [st["n_frames"] for _, st in sorted(ref["stages"].items())]
    print("layers 6/14/20 + selection at 27: scenes %s, frames 32 -> %s, tokens = %d (%.1f %%), rel-L2 = %.4f"
          % (rec["lengths"], counts, got["n_tokens"], 100.0 * got["n_tokens"] / (32 * 729), err))
    assert counts[0] <= 32 and counts[1] <= counts[0] and counts[2] <= counts[1]
    assert abs(got["n_tokens"] / (32 * 729) - 0.2) < 0.03


# ---- attention-received scores (Sec. 3.3; reading stated in the header and the oracle) ---------------

def _selection_valid(kept, cu, z, dyn, uniform, r_hat, L, delta):
    """The kept set of every frame is a correct answer for the oracle's scores z up to a relative band
    delta: top-k frames keep nothing below the k-th largest score and drop nothing above it; window frames
    keep, per window, a token within delta of the window maximum."""
    for n in range(len(cu) - 1):
        K = kept[cu[n]:cu[n + 1]]
        if uniform or dyn[n]:
            k = len(K)
            thr = np.sort(z[n])[::-1][k - 1]
            rest = np.setdiff1d(np.arange(L), K)
            if z[n][K].min() < thr * (1 - delta) or (len(rest) and z[n][rest].max() > thr * (1 + delta)):
                return False
        else:
            w = L // r_hat
            if len(K) != -(-L // w):
                return False
            for i, lo in enumerate(range(0, L, w)):
                if not (lo <= K[i] < lo + w) or z[n][K[i]] < z[n][lo:lo + w].max() * (1 - delta):
                    return False
    return True


@pytest.mark.gpu
@pytest.mark.parametrize("F,n,H,hd", [(3, 100, 4, 16), (2, 729, 16, 72), (1, 33, 2, 72), (2, 64, 1, 128)])
def test_attention_scores_match_oracle(F, n, H, hd):
    """LayerNorm -> q, k projection -> attention received, each step through its own entry point.  Against
    the oracle from x in float64 the bfloat16 storage of the LayerNorm output and of q, k shows (logits of
    standard deviation ~4 here, so a relative step of 2^-8 moves a probability by ~1 %); with the device's
    own q, k taken as given the two sides agree to float32 rounding."""
    rng = np.random.default_rng(F * 1000 + n)
    D = H * hd
    x_bits = f64_to_bits(rng.standard_normal((F * n, D)))
    x = bf16_bits_to_f32(x_bits).astype(np.float64)
    lw = dict(ln1_g=(1.0 + 0.1 * rng.standard_normal(D)).astype(np.float32),
              ln1_b=(0.1 * rng.standard_normal(D)).astype(np.float32),
              bqkv=(0.1 * rng.standard_normal(3 * D)).astype(np.float32))
    w_bits = f64_to_bits(rng.standard_normal((3 * D, D)) * (2.0 / math.sqrt(D)))
    lw["wqkv"] = bf16_bits_to_f32(w_bits)
    xn = et.et_layernorm(bits_to_dev(x_bits), torch.from_numpy(lw["ln1_g"]).cuda(), torch.from_numpy(lw["ln1_b"]).cuda(),
                         1e-6)
    qkv = et.et_gemm_bf16(xn, bits_to_dev(w_bits), torch.from_numpy(lw["bqkv"]).cuda(), 0)
    got = et.et_attention_scores(qkv, F, n, H, hd).cpu().numpy().astype(np.float64)
    ref = O.attention_received(x.reshape(F, n, D), lw, H, 1e-6)
    assert np.allclose(got.sum(axis=1), 1.0, atol=1e-5)
    assert rel_l2(got, ref) < 2e-2
    # the device's own q, k taken as given: agreement to float32 rounding
    qk = bf16_bits_to_f32(dev_to_bits(qkv)).astype(np.float64).reshape(F, n, 3 * D)
    want = O.attention_received_from_qk(qk[..., :D], qk[..., D:2 * D], H)
    assert np.max(np.abs(got - want) / want) < 2e-5


@pytest.mark.gpu
@pytest.mark.parametrize("merge_layers,select_layer,pi", [([1], 3, 0), ([0, 1], 2, 2), ([], 4, 1), ([1, 2], 4, 4)])
def test_tiny_encoder_selection_by_attention_scores(merge_layers, select_layer, pi):
    rec = build_workload("c1_tiny")
    w = rec["weights"]
    pol = _f32_policy(dict(POLICIES[pi], tau_seg=0.9, tau_merge=0.9, score_mode="attention"))
    for seed in range(40):
        frames = make_clip(TINY, [7, 2, 6, 1], 400 + seed, base="uniform", sigma=0.02)
        res = _multi_check(TINY, w, frames, merge_layers, select_layer, pol, strict_selection=False)
        if res is not None:
            break
    else:
        pytest.fail("no clip with clear margins in 40 seeds")
    got, ref, err = res
    assert np.allclose(ref["score"].sum(axis=1), 1.0)


@pytest.mark.gpu
def test_attention_score_mode_argument_errors():
    rec = build_workload("c1_tiny")
    frames = torch.from_numpy(rec["frames"]).cuda()
    enc = et.Encoder(TINY, rec["weights"], frames.shape[0])
    pol = dict(POLICIES[0], score_mode="attention")
    with pytest.raises(et.EtError, match="block before"):
        enc.encode_multi(frames, [], 0, pol)
    with pytest.raises(et.EtError, match="between the last merge"):
        enc.encode_multi(frames, [1, 2], 2, pol)
    with pytest.raises(et.EtError, match="needs the encoder"):
        et.et_merge_select_policy(torch.zeros((4, 16, 64), dtype=torch.bfloat16, device="cuda"), pol)
    enc.close()


@pytest.mark.gpu
def test_siglip_32_frames_attention_scores_after_encoder():
    """The paper's placement with attention scores: Stage I after blocks 6, 14, 20; Stage II on the encoder
    output ranked by the attention received in the last block."""
    rec = build_workload("c3_siglip_t32")
    pol = _f32_policy(dict(merge_mode="alg1", select_mode="decoupled", alpha=0.9, tau_seg=0.8, tau_merge=0.8,
                           ratio=0.2, score_mode="attention"))
    for seed in range(4):
        frames = make_clip(SIGLIP, rec["lengths"], 900 + seed, base=rec["base"], sigma=0.2)
        res = _multi_check(SIGLIP, rec["weights"], frames, [6, 14, 20], 27, pol, strict_selection=False)
        if res is not None:
            break
    else:
        pytest.fail("no clip with clear margins")
    got, ref, err = res
    z = ref["score"]
    print("attention scores, layers 6/14/20 + selection at 27: N = %d, tokens = %d, rel-L2 = %.4f, largest score x L = %.1f"
          % (got["n_frames_out"], got["n_tokens"], err, z.max() * 729))


@pytest.mark.gpu
@pytest.mark.parametrize("score_mode", ["l2", "attention"])
def test_multi_layer_degenerate_clips(score_mode):
    """One frame; identical frames that collapse to a single frame at the first merge layer and stay one
    frame at the later ones; every frame its own scene (nothing merges at any layer)."""
    rec = build_workload("c1_tiny")
    w = rec["weights"]
    L = TINY.tokens_per_frame
    base = dict(alpha=0.9, tau_seg=0.9, tau_merge=0.9, ratio=0.25, score_mode=score_mode)
    one = make_clip(TINY, [1], 5, base="uniform", sigma=0.02)
    same = np.repeat(one, 6, axis=0)
    scenes = make_clip(TINY, [1] * 5, 6, base="smooth", sigma=0.02)
    enc = et.Encoder(TINY, w, 6)
    for frames, merge_mode, want_n in ((one, "alg1", 1), (same, "mean", 1), (same, "alg1", 6), (scenes, "alg1", 5)):
        pol = _f32_policy(dict(base, merge_mode=merge_mode, select_mode="decoupled"))
        got = enc.encode_multi(torch.from_numpy(frames).cuda(), [1, 2], 3, pol)
        got = {k: (v.clone() if isinstance(v, torch.Tensor) else v) for k, v in got.items()}
        T = frames.shape[0]
        assert got["n_frames_out"] == want_n
        first, count = got["frame_first"].cpu().numpy(), got["frame_count"].cpu().numpy()
        assert first[0] == 0 and first[-1] + count[-1] == T and np.array_equal(first[1:], (first + count)[:-1])
        res = _multi_check(TINY, w, frames, [1, 2], 3, pol, strict_selection=False)
        if res is not None:                         # (identical frames sit exactly on Alg. 1's ties: plan checked above)
            assert res[0]["n_frames_out"] == want_n
    enc.close()
