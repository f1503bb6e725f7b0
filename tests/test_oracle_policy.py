"""Pins for the oracle's paper-exact Stage I / Stage II functions (Eq. 1-7, Alg. 1-2).

The paper prints no worked example, so these are hand cases derived from the algorithm text
under the readings stated in the oracle, reductions to the already pinned simple forms,
brute force, and invariants.  Parity of these forms beyond that is unpinned (documented).
"""
import math
import os

import numpy as np
import pytest

from et_inputs import TINY, make_clip, make_weights
from oracle import earlytom_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _alg1_cases():
    out = []
    for line in open(os.path.join(GOLD, "alg1_cases.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        p = [q.strip() for q in line.split("|")]        # (a fifth field, "exact", is for the device test)
        alpha, tau_seg, tau_merge = [float(v) for v in p[0].split()]
        s = [float(v) for v in p[1].split()]
        seg = [int(v) for v in p[2].split()]
        frames = []
        for tok in p[3].split():
            first, rest = tok.split(":")
            if "(" in rest:
                cnt, ws = rest.split("(")
                frames.append((int(first), int(cnt), [float(v) for v in ws.rstrip(")").split(",")]))
            else:
                frames.append((int(first), int(rest), None))
        out.append((alpha, tau_seg, tau_merge, s, seg, frames))
    return out


def _plan_by_runs(s, seg_start, tau_merge):
    """Alg. 1's result characterised without walking the frames: inside a segment with frames F_0 .. F_k,
    index i (1 <= i <= k - 2) is 'eligible' iff s_i > tau_merge and s_i > s_{i+1}; in every maximal run
    a .. b of consecutive eligible indices the fused pairs start at a, a + 2, a + 4, ... <= b.  Everything
    not covered by a pair is a frame of its own.  Returns [(first, count)]."""
    out = []
    for n in range(len(seg_start) - 1):
        a0, k = int(seg_start[n]), int(seg_start[n + 1]) - int(seg_start[n]) - 1
        elig = [1 <= i <= k - 2 and s[a0 + i] > tau_merge and s[a0 + i] > s[a0 + i + 1] for i in range(k + 1)]
        starts, i = set(), 0
        while i <= k:
            if elig[i]:
                j = i
                while j + 1 <= k and elig[j + 1]:
                    j += 1
                starts.update(range(i, j + 1, 2))
                i = j + 1
            else:
                i += 1
        covered = {p + 1 for p in starts}
        out += [(a0 + i, 2 if i in starts else 1) for i in range(k + 1) if i not in covered]
    return out


def test_alg1_walk_equals_the_run_characterisation():
    """The oracle walks the middle frames left to right as Alg. 1 does; the same plan follows from the
    maximal runs of eligible indices.  Random similarities on a coarse grid, so that ties s_i = s_{i+1} and
    s_i = tau_merge occur often."""
    rng = np.random.default_rng(4)
    for _ in range(300):
        T = int(rng.integers(1, 25))
        s = rng.integers(0, 8, T - 1) / 8.0 + 0.125          # {0.125, 0.25, .. 1.0}
        seg = O.segment_starts(s, 0.375, T)
        for tau_merge in (0.5, 0.625, 0.0):
            plan = O.merge_plan(s, seg, tau_merge, "alg1")
            assert [(p["first"], p["count"]) for p in plan] == _plan_by_runs(s, seg, tau_merge)


@pytest.mark.parametrize("case", _alg1_cases())
def test_alg1_hand_cases(case):
    alpha, tau_seg, tau_merge, s, seg, frames = case
    T = len(s) + 1
    got_seg, _ = O.ema_segment_starts(np.array(s), alpha, tau_seg, T)
    assert got_seg.tolist() == seg
    plan = O.merge_plan(np.array(s), got_seg, tau_merge, "alg1")
    assert [(p["first"], p["count"]) for p in plan] == [(f, c) for f, c, _ in frames]
    for p, (_, c, ws) in zip(plan, frames):
        assert abs(sum(p["weights"]) - 1.0) < 1e-12
        if ws is not None:
            np.testing.assert_allclose(p["weights"], ws, atol=6e-5)
    # frames are covered exactly once, in order
    covered = [t for p in plan for t in range(p["first"], p["first"] + p["count"])]
    assert covered == list(range(T))
    # head and tail of every segment are dynamic, everything else static
    for n in range(len(seg) - 1):
        mine = [p for p in plan if p["segment"] == n]
        assert mine[0]["dynamic"] and mine[-1]["dynamic"]
        assert all(not p["dynamic"] for p in mine[1:-1])
        assert mine[0]["first"] == seg[n] and mine[-1]["first"] + mine[-1]["count"] == seg[n + 1]


def test_ema_reduces_to_plain_threshold_and_smooths():
    rng = np.random.default_rng(0)
    for _ in range(40):
        T = int(rng.integers(1, 30))
        s = rng.random(T - 1)
        seg, s_hat = O.ema_segment_starts(s, 1.0, 0.5, T)
        assert seg.tolist() == O.segment_starts(s, 0.5, T).tolist()
        np.testing.assert_array_equal(s_hat, s)
    # hand-worked recursion: 0.9*0.97 + 0.1*0.95 = 0.968 ; 0.9*0.5 + 0.1*0.968 = 0.5468
    seg, s_hat = O.ema_segment_starts(np.array([0.95, 0.97, 0.5, 0.6]), 0.9, 0.8, 5)
    np.testing.assert_allclose(s_hat, [0.95, 0.968, 0.5468, 0.6], atol=1e-12)
    assert seg.tolist() == [0, 3, 4, 5]          # the recursion restarts after the break at frame 3
    # smoothing can keep a segment together across one dip (the alpha = 0.5 case of the golden file) and NaN breaks
    assert O.ema_segment_starts(np.array([0.99, np.nan, 0.99]), 0.9, 0.5, 4)[0].tolist() == [0, 2, 4]


def test_identical_frames_never_merge_under_the_strict_rule():
    s = np.ones(7)
    seg, _ = O.ema_segment_starts(s, 0.9, 0.8, 8)
    plan = O.merge_plan(s, seg, 0.8, "alg1")
    assert seg.tolist() == [0, 8] and len(plan) == 8 and all(p["count"] == 1 for p in plan)


def test_plan_mean_mode_is_the_segment_mean_and_weighted_pairs_are_convex():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((9, 4, 6))
    seg = np.array([0, 3, 4, 9], dtype=np.int32)
    plan = O.merge_plan(np.zeros(8), seg, 0.0, "mean")
    np.testing.assert_array_equal(O.apply_plan(x, plan), O.segment_mean(x, seg))
    # a fused pair is s_i F_i + s_{i+1} F_{i+1} over their sum (Eq. 3): check one by hand
    s = np.array([0.9, 0.8, 0.6, 0.9])
    plan = O.merge_plan(s, np.array([0, 5]), 0.5, "alg1")
    assert [(p["first"], p["count"]) for p in plan] == [(0, 1), (1, 2), (3, 1), (4, 1)]
    y = O.apply_plan(x[:5], plan)
    np.testing.assert_allclose(y[1], (0.8 * x[1] + 0.6 * x[2]) / 1.4, rtol=1e-13)
    np.testing.assert_array_equal(y[0], x[0])
    np.testing.assert_array_equal(y[3], x[4])
    # fusing two identical frames returns the frame
    xx = x.copy(); xx[2] = xx[1]
    np.testing.assert_allclose(O.apply_plan(xx[:5], plan)[1], xx[1], rtol=1e-14)


def test_rescaled_count_keeps_the_overall_ratio():
    assert O.rescaled_count(0.25, 32, 729, 32) == 182          # nothing merged: r * L = 182.25
    assert O.rescaled_count(0.2, 32, 729, 8) == 583            # 0.2 * 32 * 729 / 8 = 583.2
    assert O.rescaled_count(0.5, 32, 729, 8) == 729            # clamps at L
    assert O.rescaled_count(1e-6, 32, 729, 8) == 1
    for B, L, r in [(32, 729, 0.1), (64, 729, 0.15), (8, 64, 0.3)]:
        for N in range(max(1, int(B * r) + 1), B + 1):
            rh = O.rescaled_count(r, B, L, N)
            assert abs(N * rh - r * B * L) <= 0.5 * N + 1e-9


def _brute_windows(z, r_hat):
    L = len(z)
    w = L // r_hat
    kept, lo = [], 0
    while lo < L:
        hi = min(lo + w, L)
        best = lo
        for j in range(lo, hi):
            zj, zb = z[j], z[best]
            if (not math.isnan(zj)) and (math.isnan(zb) or zj > zb):
                best = j
        kept.append(best)
        lo = hi
    return kept


def test_window_selection_hand_and_brute_force():
    assert O.window_positions(np.array([1, 5, 2, 7, 7, 0, 3.]), 3).tolist() == [1, 3, 4, 6]
    assert O.window_positions(np.array([4., 4., 4., 4.]), 2).tolist() == [0, 2]        # ties: lowest position
    assert O.window_positions(np.array([1., 2., 3.]), 3).tolist() == [0, 1, 2]         # w = 1: identity
    rng = np.random.default_rng(2)
    for trial in range(200):
        L = int(rng.integers(1, 80))
        z = rng.integers(0, 4, L).astype(np.float64) if trial % 2 else rng.random(L)
        r_hat = int(rng.integers(1, L + 1))
        got = O.window_positions(z, r_hat)
        assert got.tolist() == _brute_windows(z.tolist(), r_hat)
        w = L // r_hat
        assert len(got) == -(-L // w)
    # L = 729: r_hat 182 -> w = 4 -> 183 windows ; r_hat 400 -> w = 1 -> all 729 positions
    assert len(O.window_positions(rng.random(729), 182)) == 183
    assert len(O.window_positions(rng.random(729), 400)) == 729


@pytest.fixture(scope="module")
def tiny():
    return make_weights(TINY, 11), make_clip(TINY, [4, 4], 12, base="uniform", sigma=0.02)


def test_default_policy_reproduces_the_simple_path(tiny):
    w, frames = tiny
    pol = dict(alpha=1.0, tau_seg=0.9, tau_merge=0.9, merge_mode="mean", select_mode="uniform", ratio=0.5)
    a = O.encode_clip(TINY, w, frames, 2, 0.9, 0.5)
    b = O.encode_clip_policy(TINY, w, frames, 2, pol)
    assert b["seg_start"].tolist() == a["seg_start"].tolist()
    assert b["cu_tokens"].tolist() == a["cu_tokens"].tolist()
    assert b["kept_idx"].tolist() == a["kept_idx"].tolist()
    np.testing.assert_allclose(b["tokens"], a["tokens"], rtol=1e-12, atol=1e-12)


def test_paper_policy_end_to_end_bookkeeping(tiny):
    w, _ = tiny
    frames = make_clip(TINY, [6, 1, 5], 21, base="uniform", sigma=0.02)
    pol = dict(alpha=0.9, tau_seg=0.9, tau_merge=0.9, merge_mode="alg1", select_mode="decoupled", ratio=0.25)
    r = O.encode_clip_policy(TINY, w, frames, 2, pol)
    assert r["seg_start"].tolist() == [0, 6, 7, 12]
    N = r["n_frames_out"]
    assert N == len(r["plan"]) and N <= 12 and N >= 3 * 2 - 1
    r_hat = O.rescaled_count(0.25, 12, 64, N)
    w_ = 64 // r_hat
    M = -(-64 // w_)
    counts = np.diff(r["cu_tokens"])
    assert all(c == (r_hat if d else M) for c, d in zip(counts, r["frame_dynamic"]))
    assert r["tokens"].shape == (int(r["cu_tokens"][-1]), 64)
    for n in range(N):
        kept = r["kept_idx"][r["cu_tokens"][n]:r["cu_tokens"][n + 1]]
        assert np.all(np.diff(kept) > 0)
    # an output frame's tokens depend only on its own source frames and kept positions:
    # re-encoding the single-frame middle segment alone gives the same tokens for that frame
    n_mid = [i for i, p in enumerate(r["plan"]) if p["segment"] == 1][0]
    kept_mid = r["kept_idx"][r["cu_tokens"][n_mid]:r["cu_tokens"][n_mid + 1]]
    solo = O.encode_clip_policy(TINY, w, frames[6:7], 2, pol, force_kept=[kept_mid])
    np.testing.assert_allclose(solo["tokens"], r["tokens"][r["cu_tokens"][n_mid]:r["cu_tokens"][n_mid + 1]],
                               rtol=1e-10, atol=1e-10)


def test_multi_layer_merging_reductions_and_bookkeeping(tiny):
    w, _ = tiny
    frames = make_clip(TINY, [6, 1, 5], 21, base="uniform", sigma=0.02)
    pol = dict(alpha=0.9, tau_seg=0.9, tau_merge=0.9, merge_mode="alg1", select_mode="decoupled", ratio=0.25)
    # one merge layer that is also the select layer == the single-layer policy path
    a = O.encode_clip_policy(TINY, w, frames, 2, pol)
    b = O.encode_clip_multi(TINY, w, frames, [2], 2, pol)
    assert b["cu_tokens"].tolist() == a["cu_tokens"].tolist() and b["kept_idx"].tolist() == a["kept_idx"].tolist()
    np.testing.assert_allclose(b["tokens"], a["tokens"], rtol=1e-12, atol=1e-12)
    assert b["frame_first"].tolist() == a["frame_first"].tolist()
    assert b["frame_count"].tolist() == a["frame_count"].tolist()
    assert b["seg_start"].tolist() == a["seg_start"].tolist()
    # no merge layer, selection after the last block == plain encoder, then selection on its output
    c = O.encode_clip_multi(TINY, w, frames, [], 4, dict(pol, select_mode="uniform", ratio=0.5))
    d = O.encode_clip_policy(TINY, w, frames, 4, dict(pol, tau_seg=math.inf, merge_mode="mean",
                                                      select_mode="uniform", ratio=0.5))
    assert c["kept_idx"].tolist() == d["kept_idx"].tolist()
    np.testing.assert_allclose(c["tokens"], d["tokens"], rtol=1e-12, atol=1e-12)
    assert c["frame_dynamic"].tolist() == [1] * 12
    # three merge layers: output frames are contiguous, disjoint ranges of the original frames, and
    # frame counts never grow from layer to layer
    e = O.encode_clip_multi(TINY, w, frames, [1, 2, 3], 4, pol)
    covered = [t for f, c_ in zip(e["frame_first"], e["frame_count"]) for t in range(f, f + c_)]
    assert covered == list(range(12))
    sizes = [e["hidden"][i].shape[0] for i in (1, 2, 3, 4)]
    assert sizes[0] == 12 and all(x >= y for x, y in zip(sizes, sizes[1:])) and sizes[-1] == e["n_frames_out"]
    assert e["n_frames_out"] < 12                         # the six-frame scene fuses at least one pair
    # mean mode collapses each scene at the first layer; later layers find nothing more to merge
    pm = dict(pol, merge_mode="mean", alpha=1.0)
    f1 = O.encode_clip_multi(TINY, w, frames, [1], 3, pm)
    f3 = O.encode_clip_multi(TINY, w, frames, [1, 2, 3], 3, pm)
    assert f1["n_frames_out"] == f3["n_frames_out"] == 3
    assert f3["frame_first"].tolist() == [0, 6, 7] and f3["frame_count"].tolist() == [6, 1, 5]
    np.testing.assert_allclose(f3["tokens"], f1["tokens"], rtol=1e-12, atol=1e-12)


# ---- attention-received scores (Sec. 3.3 "per-token attention scores"; reading stated in the oracle) ----

def _tiny_layer(rng, D, H):
    return dict(ln1_g=1.0 + 0.1 * rng.standard_normal(D), ln1_b=0.1 * rng.standard_normal(D),
                wqkv=0.4 * rng.standard_normal((3 * D, D)), bqkv=0.1 * rng.standard_normal(3 * D))


def test_attention_received_matches_explicit_loops():
    """Written out with scalar loops: softmax row by row, then the column mean over queries and heads."""
    rng = np.random.default_rng(0)
    F, n, D, H, eps = 2, 7, 8, 2, 1e-6
    lw = _tiny_layer(rng, D, H)
    x = rng.standard_normal((F, n, D))
    got = O.attention_received(x, lw, H, eps)
    hd = D // H
    want = np.zeros((F, n))
    for f in range(F):
        xn = np.zeros((n, D))
        for i in range(n):
            mu = sum(x[f, i]) / D
            var = sum((v - mu) ** 2 for v in x[f, i]) / D
            xn[i] = [(v - mu) / math.sqrt(var + eps) * g + b for v, g, b in zip(x[f, i], lw["ln1_g"], lw["ln1_b"])]
        q = [[sum(lw["wqkv"][c, d] * xn[i, d] for d in range(D)) + lw["bqkv"][c] for c in range(D)] for i in range(n)]
        k = [[sum(lw["wqkv"][D + c, d] * xn[i, d] for d in range(D)) + lw["bqkv"][D + c] for c in range(D)]
             for i in range(n)]
        for h in range(H):
            for i in range(n):
                logit = [sum(q[i][h * hd + c] * k[j][h * hd + c] for c in range(hd)) / math.sqrt(hd) for j in range(n)]
                mx = max(logit)
                e = [math.exp(v - mx) for v in logit]
                tot = sum(e)
                for j in range(n):
                    want[f, j] += e[j] / tot / (n * H)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-15)
    assert np.allclose(got.sum(axis=1), 1.0)


def test_attention_received_closed_form_two_token_types():
    """One head, identity LayerNorm (rows already have mean 0, variance 1), q = k = c x: the logits take
    two values +-t, so every softmax row is known in closed form.  m tokens of type (1,-1), n-m of type
    (-1,1): a column of the larger group receives more than 1/n - a row mean would give exactly 1/n."""
    n, m, c = 7, 5, 0.8
    D = 2
    x = np.array([[1.0, -1.0]] * m + [[-1.0, 1.0]] * (n - m))[None]
    lw = dict(ln1_g=np.ones(D), ln1_b=np.zeros(D), wqkv=np.concatenate([c * np.eye(D), c * np.eye(D), np.eye(D)]),
              bqkv=np.zeros(3 * D))
    got = O.attention_received(x, lw, 1, 0.0)[0]
    t = 2 * c * c / math.sqrt(2.0)
    row_a = m * math.exp(t) + (n - m) * math.exp(-t)         # normaliser of a type-A query
    row_b = (n - m) * math.exp(t) + m * math.exp(-t)
    col_a = (m * math.exp(t) / row_a + (n - m) * math.exp(-t) / row_b) / n
    col_b = (m * math.exp(-t) / row_a + (n - m) * math.exp(t) / row_b) / n
    assert np.allclose(got[:m], col_a, rtol=1e-13) and np.allclose(got[m:], col_b, rtol=1e-13)
    assert col_a > 1.0 / n > col_b


def test_attention_received_special_cases():
    rng = np.random.default_rng(3)
    D, H = 8, 2
    lw = _tiny_layer(rng, D, H)
    same = np.tile(rng.standard_normal((1, 1, D)), (1, 9, 1))
    assert np.allclose(O.attention_received(same, lw, H, 1e-6), 1.0 / 9)       # identical tokens: uniform
    x = rng.standard_normal((3, 6, D))
    perm = rng.permutation(6)
    a = O.attention_received(x, lw, H, 1e-6)
    assert np.allclose(O.attention_received(x[:, perm], lw, H, 1e-6), a[:, perm])   # equivariant to token order


def test_multi_layer_selection_by_attention_scores(tiny):
    w, frames = tiny
    pol = dict(merge_mode="alg1", select_mode="decoupled", alpha=0.9, tau_seg=0.9, tau_merge=0.9, ratio=0.25,
               score_mode="attention")
    r = O.encode_clip_multi(TINY, w, frames, [1], 3, pol)
    # the scores are those of block 2 on the frames it sees, and the kept tokens are their top-k / window maxima
    z = O.attention_received(r["hidden"][2], w["layers"][2], TINY.n_heads, TINY.ln_eps)
    assert np.array_equal(r["score"], z)
    L = TINY.tokens_per_frame
    r_hat = O.rescaled_count(pol["ratio"], frames.shape[0], L, r["n_frames_out"])
    cu = r["cu_tokens"]
    for n in range(r["n_frames_out"]):
        kept = r["kept_idx"][cu[n]:cu[n + 1]]
        want = O.topk_positions(z[n], r_hat) if r["frame_dynamic"][n] else O.window_positions(z[n], r_hat)
        assert np.array_equal(kept, want)
    with pytest.raises(AssertionError):
        O.encode_clip_multi(TINY, w, frames, [1, 3], 3, pol)       # a merge between the scoring block and the selection


def test_layernorm_folded_into_a_linear_layer_is_an_identity():
    """LN(x) W^T + b = (x Wf^T) / sqrt(var + eps) + c with Wf[n, k] = W[n, k] gamma[k] - mean_k(W[n, :] gamma)
    and c = W beta + b (every row of Wf sums to zero, so the row mean of x drops out).  The folded form is
    written out here, in the test, against the oracle's separate LayerNorm and linear layer: it is the form
    a device may compute in, and the oracle itself never does."""
    rng = np.random.default_rng(7)
    D, N = 48, 20
    x = rng.standard_normal((3, 5, D)) * rng.uniform(0.5, 3.0, (3, 5, 1)) + rng.uniform(-20.0, 20.0, (3, 5, 1))
    g, b = 1.0 + 0.2 * rng.standard_normal(D), 0.3 * rng.standard_normal(D)
    W, bias = rng.standard_normal((N, D)), rng.standard_normal(N)
    want = O.layer_norm(x, g, b, 1e-6) @ W.T + bias
    Wg = W * g[None, :]
    Wf = Wg - Wg.mean(axis=1, keepdims=True)
    got = (x @ Wf.T) / np.sqrt(x.var(axis=-1, keepdims=True) + 1e-6) + W @ b + bias
    assert np.max(np.abs(got - want)) < 1e-10
    # a mistake in any term shows: dropping the centring leaves the mean term, dropping W beta the shift
    no_centre = (x @ Wg.T) / np.sqrt(x.var(axis=-1, keepdims=True) + 1e-6) + W @ b + bias
    assert np.max(np.abs(no_centre - want)) > 1.0


def test_attention_received_from_given_queries_and_keys():
    """attention_received is LayerNorm -> q, k projection -> attention_received_from_qk; the second half on
    its own against scalar loops, and encode_clip_multi with qk_at_score_layer set to the oracle's own
    q | k reproduces the run without it."""
    rng = np.random.default_rng(8)
    F, n, H, hd = 2, 9, 2, 8
    D = H * hd
    x = rng.standard_normal((F, n, D))
    lw = dict(ln1_g=1.0 + 0.1 * rng.standard_normal(D), ln1_b=0.1 * rng.standard_normal(D),
              wqkv=rng.standard_normal((3 * D, D)) * 0.3, bqkv=0.1 * rng.standard_normal(3 * D))
    xn = O.layer_norm(x, lw["ln1_g"], lw["ln1_b"], 1e-6)
    qk = xn @ lw["wqkv"][:2 * D].T + lw["bqkv"][:2 * D]
    got = O.attention_received_from_qk(qk[..., :D], qk[..., D:], H)
    assert np.array_equal(got, O.attention_received(x, lw, H, 1e-6))
    want = np.zeros((F, n))
    for f in range(F):
        for h in range(H):
            for i in range(n):
                logit = [sum(qk[f, i, h * hd + c] * qk[f, j, D + h * hd + c] for c in range(hd)) / math.sqrt(hd)
                         for j in range(n)]
                e = [math.exp(v - max(logit)) for v in logit]
                for j in range(n):
                    want[f, j] += e[j] / sum(e) / (n * H)
    assert np.allclose(got, want, rtol=1e-12, atol=1e-15)
    # swapping the roles of q and k is a different quantity (a transposed operand shows)
    assert np.max(np.abs(O.attention_received_from_qk(qk[..., D:], qk[..., :D], H) - got)) > 1e-3


def test_multi_layer_scores_from_injected_queries_and_keys(tiny):
    w, frames = tiny
    pol = dict(merge_mode="alg1", select_mode="decoupled", alpha=0.9, tau_seg=0.9, tau_merge=0.9, ratio=0.25,
               score_mode="attention")
    r = O.encode_clip_multi(TINY, w, frames, [1], 3, pol)
    D = TINY.d_model
    lw = w["layers"][2]
    xn = O.layer_norm(r["hidden"][2], lw["ln1_g"].astype(np.float64), lw["ln1_b"].astype(np.float64), TINY.ln_eps)
    qk = xn @ lw["wqkv"].astype(np.float64)[:2 * D].T + lw["bqkv"].astype(np.float64)[:2 * D]
    r2 = O.encode_clip_multi(TINY, w, frames, [1], 3, pol, qk_at_score_layer=qk)
    assert np.array_equal(r2["kept_idx"], r["kept_idx"]) and np.allclose(r2["score"], r["score"], rtol=1e-13)
    # other queries and keys, other scores: the injected ones are really what is ranked
    r3 = O.encode_clip_multi(TINY, w, frames, [1], 3, pol, qk_at_score_layer=qk[:, ::-1])
    assert not np.allclose(r3["score"], r["score"])
    with pytest.raises(ValueError):
        O.encode_clip_multi(TINY, w, frames, [1], 3, pol, qk_at_score_layer=qk[:1])
