"""CPU oracle for EarlyTom's in-encoder token compression.  TEST INFRASTRUCTURE ONLY.

A plain, slow, step-by-step numpy implementation of what the HIP library
computes: a pre-LayerNorm ViT encoder (SigLIP layout) over the frames of a video
clip, with the paper's early token compression applied once inside the encoder:

  Sec. 3.2  frame similarity s_t = mean over spatial positions of the cosine
            similarity of co-located tokens of frames t and t-1;
  Eq. 1     a segment boundary is placed before frame t when the (smoothed)
            similarity drops below the threshold (alpha = 1 here: no smoothing);
  Sec. 3.2  frames of a segment are merged (here: the whole segment is averaged
            per spatial position, the simplified form this build's task names;
            Eq. 2-3 pairwise weighted merging is not part of this file);
  Eq. 4     per frame, the top-k tokens by score are kept (score = squared L2
            norm of the merged token; ties go to the lower position);
  Eq. 7     kept tokens are gathered in their original order and the remaining
            encoder blocks run on the shorter sequence.
The paper-exact forms (Eq. 1 with smoothing, Alg. 1's head/tail + weighted middle
pairs, Alg. 2's dynamic top-k / static local windows with the re-scaled count of
Eq. 5) are the *_policy functions further down.

Everything is float64 unless `dtype` says otherwise; matmul/einsum are the only
library primitives; nothing is blocked, fused or reordered.  Only tests,
`__graft_entry__.smoke()` and `bench.py`'s cpu_baseline leg may import this
file; the product path never does, and this file imports nothing of the product.

Parity pins (tests/test_oracle_pins.py): closed forms for the similarity, hand
cases for the boundary scan, brute-force selection for the top-k, textbook
special cases for LayerNorm / softmax / GELU, one encoder block assembled from
torch library routines, patch embedding as a strided convolution, and the
end-to-end invariants (compression disabled == plain encoder; identical frames
== single frame).
"""
import math

import numpy as np


# --------------------------------------------------------------------------
# Encoder pieces (SigLIP layout; the paper names the model only, Sec. 4.1)
# --------------------------------------------------------------------------

def patchify(frames, patch):
    """[T,C,H,W] -> [T, L, C*P*P]; non-overlapping patches, trailing pixels dropped.

    Token l = gy * grid_w + gx; the patch vector is flattened in (c, py, px) order.
    """
    T, C, H, W = frames.shape
    gy, gx = H // patch, W // patch
    f = frames[:, :, :gy * patch, :gx * patch]
    f = f.reshape(T, C, gy, patch, gx, patch)
    f = f.transpose(0, 2, 4, 1, 3, 5)                    # T, gy, gx, C, py, px
    return f.reshape(T, gy * gx, C * patch * patch)


def patch_embed(frames, w, patch, dtype=np.float64):
    """x[t,l,:] = patch(t,l) @ patch_w.T + patch_b + pos_emb[l]."""
    p = patchify(np.asarray(frames, dtype=dtype), patch)
    x = p @ np.asarray(w["patch_w"], dtype=dtype).T
    x = x + np.asarray(w["patch_b"], dtype=dtype) + np.asarray(w["pos_emb"], dtype=dtype)[None]
    return x


def layer_norm(x, g, b, eps):
    """(x - mean) / sqrt(biased variance + eps) * g + b over the last axis."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * g + b


def gelu_tanh(u):
    """0.5 u (1 + tanh( sqrt(2/pi) (u + 0.044715 u^3) ))."""
    return 0.5 * u * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (u + 0.044715 * u ** 3)))


def softmax_rows(s):
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=-1, keepdims=True)


def attention(xn, lw, n_heads):
    """Bidirectional multi-head self-attention inside each frame.  xn: [F, n, D]."""
    F, n, D = xn.shape
    hd = D // n_heads
    dt = xn.dtype
    qkv = xn @ np.asarray(lw["wqkv"], dtype=dt).T + np.asarray(lw["bqkv"], dtype=dt)
    q, k, v = qkv[..., :D], qkv[..., D:2 * D], qkv[..., 2 * D:]
    q = q.reshape(F, n, n_heads, hd).transpose(0, 2, 1, 3)      # F, H, n, hd
    k = k.reshape(F, n, n_heads, hd).transpose(0, 2, 1, 3)
    v = v.reshape(F, n, n_heads, hd).transpose(0, 2, 1, 3)
    s = (q @ k.transpose(0, 1, 3, 2)) / math.sqrt(hd)
    p = softmax_rows(s)
    o = (p @ v).transpose(0, 2, 1, 3).reshape(F, n, D)
    return o @ np.asarray(lw["wo"], dtype=dt).T + np.asarray(lw["bo"], dtype=dt)


def attention_received_from_qk(q, k, n_heads):
    """Column means of the softmax matrices: q, k [F, n, D] (head h = columns h*hd ..) -> [F, n],
    entry [f, j] = mean over heads and over the queries i of frame f of softmax_j(q_i . k_j / sqrt(hd))."""
    F, n, D = q.shape
    hd = D // n_heads
    qh = q.reshape(F, n, n_heads, hd).transpose(0, 2, 1, 3)
    kh = k.reshape(F, n, n_heads, hd).transpose(0, 2, 1, 3)
    p = softmax_rows((qh @ kh.transpose(0, 1, 3, 2)) / math.sqrt(hd))        # F, H, query, key
    return p.mean(axis=(1, 2))


def attention_received(x, lw, n_heads, eps):
    """Per-token attention score for Sec. 3.3 / Alg. 2 (input A, the encoder's attentions).

    The paper does not say how one score per token is taken from the attention maps; the reading
    here: the attention a token RECEIVES in the block with weights `lw`, i.e. the column mean of the
    softmax matrix over all queries of its frame, averaged over the heads.  x: [F, n, D] is the
    input of that block.  Returns [F, n]; every row sums to 1."""
    F, n, D = x.shape
    dt = x.dtype
    xn = layer_norm(x, np.asarray(lw["ln1_g"], dt), np.asarray(lw["ln1_b"], dt), eps)
    qk = xn @ np.asarray(lw["wqkv"], dtype=dt)[:2 * D].T + np.asarray(lw["bqkv"], dtype=dt)[:2 * D]
    return attention_received_from_qk(qk[..., :D], qk[..., D:], n_heads)


def mlp(xn, lw):
    dt = xn.dtype
    h = gelu_tanh(xn @ np.asarray(lw["w1"], dtype=dt).T + np.asarray(lw["b1"], dtype=dt))
    return h @ np.asarray(lw["w2"], dtype=dt).T + np.asarray(lw["b2"], dtype=dt)


def project_tokens(x, w1, b1, w2, b2):
    """The projector between encoder and language model (Sec. 3.1 names it, the paper gives no formula;
    reading: a two-layer MLP with GELU-tanh): [n, D] -> [n, D_out] = gelu_tanh(x W1^T + b1) W2^T + b2."""
    dt = x.dtype
    h = gelu_tanh(x @ np.asarray(w1, dtype=dt).T + np.asarray(b1, dtype=dt))
    return h @ np.asarray(w2, dtype=dt).T + np.asarray(b2, dtype=dt)


def encoder_block(x, lw, n_heads, eps):
    """Pre-LN block: x += Attn(LN1(x)); x += MLP(LN2(x)).  x: [F, n, D]."""
    dt = x.dtype
    x = x + attention(layer_norm(x, np.asarray(lw["ln1_g"], dt), np.asarray(lw["ln1_b"], dt), eps),
                      lw, n_heads)
    x = x + mlp(layer_norm(x, np.asarray(lw["ln2_g"], dt), np.asarray(lw["ln2_b"], dt), eps), lw)
    return x


# --------------------------------------------------------------------------
# Compression pieces
# --------------------------------------------------------------------------

COS_EPS = 1e-8


def frame_similarity(x):
    """Sec. 3.2.  x: [T, L, D] -> (c [T-1, L], s [T-1]).

    c[t-1, l] = <x[t,l], x[t-1,l]> / max(|x[t,l]| |x[t-1,l]|, 1e-8); s = mean over l.
    """
    a, b = x[1:], x[:-1]
    dot = (a * b).sum(axis=-1)
    na = np.sqrt((a * a).sum(axis=-1))
    nb = np.sqrt((b * b).sum(axis=-1))
    c = dot / np.maximum(na * nb, COS_EPS)
    return c, c.mean(axis=-1)


def segment_starts(s, tau, T):
    """Eq. 1 with alpha = 1: frame t opens a new segment iff s_t < tau (strict).

    Returns seg_start [N+1] (int32): first input frame of each segment, last entry T.
    """
    starts = [0]
    for t in range(1, T):
        sim = float(s[t - 1])
        if sim < tau or math.isnan(sim):
            starts.append(t)
    starts.append(T)
    return np.asarray(starts, dtype=np.int32)


def segment_mean(x, seg_start):
    """x: [T, L, D] -> [N, L, D]: per spatial position, the mean over the segment's frames."""
    N = len(seg_start) - 1
    out = np.empty((N,) + x.shape[1:], dtype=x.dtype)
    for n in range(N):
        a, b = int(seg_start[n]), int(seg_start[n + 1])
        acc = np.zeros(x.shape[1:], dtype=x.dtype)
        for t in range(a, b):
            acc = acc + x[t]
        out[n] = acc / (b - a)
    return out


def token_score(xm):
    """Score of a merged token = its squared L2 norm.  [N, L, D] -> [N, L]."""
    return (xm * xm).sum(axis=-1)


def keep_count(L, keep_ratio):
    """k = clamp(floor(keep_ratio * L + 1e-4), 1, L)."""
    k = int(math.floor(float(keep_ratio) * L + 1e-4))
    return max(1, min(L, k))


def topk_positions(z, k):
    """Eq. 4 with a total order: rank by (score descending, position ascending), keep the
    first k, return those positions in ascending order (the order Eq. 7 restores).

    The ranking is decided on float32 scores (the precision the kernel ranks in);
    NaN ranks below everything.
    """
    z32 = np.asarray(z, dtype=np.float32)
    key = np.where(np.isnan(z32), -np.inf, z32.astype(np.float64))
    pos = np.arange(len(key))
    order = np.lexsort((pos, -key))          # primary: -key ascending, secondary: pos ascending
    return np.sort(order[:k]).astype(np.int32)


def compact(xm, kept):
    """Eq. 7.  xm: [N, L, D], kept: [N, k] -> packed [N*k, D], frame-major."""
    N, k = kept.shape
    return np.concatenate([xm[n][kept[n]] for n in range(N)], axis=0)


def merge_select(x, sim_threshold, keep_ratio, force_seg_start=None, force_kept=None):
    """The whole compression stage on hidden states x [T, L, D].

    Returns a dict: frame_sim [T-1], cos [T-1, L], seg_start [N+1], merged [N, L, D],
    score [N, L], k, kept_idx [N, k], cu_tokens [N+1], tokens [N*k, D].
    `force_*` replace the decisions (used to separate arithmetic error from rank flips).
    """
    T, L, D = x.shape
    if T > 1:
        c, s = frame_similarity(x)
    else:
        c, s = np.zeros((0, L), x.dtype), np.zeros((0,), x.dtype)
    seg = segment_starts(s, sim_threshold, T) if force_seg_start is None \
        else np.asarray(force_seg_start, dtype=np.int32)
    xm = segment_mean(x, seg)
    z = token_score(xm)
    k = keep_count(L, keep_ratio)
    N = xm.shape[0]
    if force_kept is None:
        kept = np.stack([topk_positions(z[n], k) for n in range(N)])
    else:
        kept = np.asarray(force_kept, dtype=np.int32).reshape(N, k)
    cu = (np.arange(N + 1) * k).astype(np.int32)
    return dict(frame_sim=s, cos=c, seg_start=seg, merged=xm, score=z, k=k,
                kept_idx=kept, cu_tokens=cu, tokens=compact(xm, kept))


# --------------------------------------------------------------------------
# Paper-exact Stage I (Alg. 1) and Stage II (Alg. 2)
#
# Readings where the paper is silent or inconsistent (also listed in the design notes):
#  - Eq. 1: the smoothed similarity restarts at every segment start (the first pair of a segment
#    uses its raw similarity); the paper gives no initial value.
#  - Alg. 1: a pair (F_i, F_{i+1}) of middle frames is eligible only if both are middle frames
#    (i + 1 <= k - 1); as printed the loop would read past the segment and merge the tail frame
#    that it appends afterwards.  tau_merge has no value in the paper; callers pass one.
#  - Eq. 3: frame-level scalar weights, F_i by s_i = Sim(F_i, F_{i+1}), F_{i+1} by s_{i+1}.
#  - Eq. 5 as printed is not a count and divides by zero when nothing merges; here
#    r_hat = clamp(floor(r * B * L / N + 0.5), 1, L): per-frame count that keeps about r of the
#    original B * L tokens.
#  - Eq. 6: windows are contiguous ranges of the flattened position index; the last one may be short.
# No worked example exists in the paper: beyond hand cases derived from the text, parity of these
# functions is UNPINNED.
# --------------------------------------------------------------------------

def ema_segment_starts(s, alpha, tau, T):
    """Eq. 1: s_hat_t = alpha s_t + (1 - alpha) s_hat_{t-1}; frame t opens a segment iff s_hat_t < tau.
    The recursion restarts after every break.  Returns (seg_start [n_seg+1], s_hat [T-1])."""
    starts, s_hat = [0], np.zeros(max(T - 1, 0), dtype=np.float64)
    prev, fresh = 0.0, True
    for t in range(1, T):
        st = float(s[t - 1])
        cur = st if fresh else alpha * st + (1.0 - alpha) * prev
        s_hat[t - 1] = cur
        if cur < tau or math.isnan(cur):
            starts.append(t)
            fresh = True
        else:
            prev, fresh = cur, False
    starts.append(T)
    return np.asarray(starts, dtype=np.int32), s_hat


def merge_plan(s, seg_start, tau_merge, mode):
    """Output-frame plan: list of dicts {first, count, weights, dynamic, segment}.

    mode "mean": one output frame per segment, uniform weights 1/len.
    mode "alg1": Alg. 1 — head and tail of a segment are kept; middle frames are walked left to
    right and (F_i, F_{i+1}) are fused with weights (s_i, s_{i+1}) / (s_i + s_{i+1}) iff
    s_i > tau_merge and s_i > s_{i+1} (Eq. 2-3), where s_i = Sim(F_i, F_{i+1}).
    `dynamic` marks head and tail frames (Sec. 3.3)."""
    plan = []
    for n in range(len(seg_start) - 1):
        a, b = int(seg_start[n]), int(seg_start[n + 1])
        if mode == "mean":
            plan.append(dict(first=a, count=b - a, weights=[1.0 / (b - a)] * (b - a), dynamic=True, segment=n))
            continue
        k = b - a - 1                                  # frames F_0 .. F_k
        sim = lambda i: float(s[a + i])                # Sim(F_i, F_{i+1}): pair of global frames a+i, a+i+1
        plan.append(dict(first=a, count=1, weights=[1.0], dynamic=True, segment=n))
        i = 1
        while i < k:
            if i + 1 <= k - 1 and sim(i) > tau_merge and sim(i) > sim(i + 1):
                si, sj = sim(i), sim(i + 1)
                plan.append(dict(first=a + i, count=2, weights=[si / (si + sj), sj / (si + sj)],
                                 dynamic=False, segment=n))
                i += 2
            else:
                plan.append(dict(first=a + i, count=1, weights=[1.0], dynamic=False, segment=n))
                i += 1
        if k >= 1:
            plan.append(dict(first=a + k, count=1, weights=[1.0], dynamic=True, segment=n))
    return plan


def apply_plan(x, plan):
    """[T, L, D] -> [N, L, D]: each output frame is the weighted sum of its source frames (a plain
    mean, summed in ascending frame order and divided by the length, for uniform plans)."""
    out = np.empty((len(plan),) + x.shape[1:], dtype=x.dtype)
    for n, p in enumerate(plan):
        a, c = p["first"], p["count"]
        if all(w == p["weights"][0] for w in p["weights"]):
            acc = np.zeros(x.shape[1:], dtype=x.dtype)
            for t in range(a, a + c):
                acc = acc + x[t]
            out[n] = acc / c
        else:
            acc = np.zeros(x.shape[1:], dtype=x.dtype)
            for j in range(c):
                acc = acc + p["weights"][j] * x[a + j]
            out[n] = acc
    return out


def rescaled_count(r, B, L, N):
    """Reading of Eq. 5: tokens kept per dynamic frame so that N frames keep about r * B * L."""
    v = int(math.floor(float(r) * B * L / N + 0.5))
    return max(1, min(L, v))


def window_positions(z, r_hat):
    """Eq. 6: w = floor(L / r_hat), M = ceil(L / w) windows of consecutive positions; keep the
    arg-max score of each window (lowest position on ties; NaN ranks last; float32 ranking)."""
    L = len(z)
    w = L // r_hat
    M = -(-L // w)
    z32 = np.asarray(z, dtype=np.float32)
    key = np.where(np.isnan(z32), -np.inf, z32.astype(np.float64))
    kept = []
    for j in range(M):
        lo, hi = j * w, min((j + 1) * w, L)
        kept.append(lo + int(np.argmax(key[lo:hi])))      # argmax returns the first maximum
    return np.asarray(kept, dtype=np.int32)


def merge_select_policy(x, policy, force_kept=None):
    """Compression stage under a policy dict: alpha, tau_seg, tau_merge, merge_mode ("mean" | "alg1"),
    select_mode ("uniform" | "decoupled"), ratio.  Returns the fields of merge_select plus `plan`,
    `s_hat`, `frame_dynamic`; kept_idx is a flat list (frames may keep different counts)."""
    T, L, D = x.shape
    if T > 1:
        c, s = frame_similarity(x)
    else:
        c, s = np.zeros((0, L), x.dtype), np.zeros((0,), x.dtype)
    seg, s_hat = ema_segment_starts(s, policy["alpha"], policy["tau_seg"], T)
    plan = merge_plan(s, seg, policy["tau_merge"], policy["merge_mode"])
    xm = apply_plan(x, plan)
    z = token_score(xm)
    N = len(plan)
    if policy["select_mode"] == "uniform":
        k = keep_count(L, policy["ratio"])
        per_frame = [topk_positions(z[n], k) for n in range(N)]
    else:
        r_hat = rescaled_count(policy["ratio"], T, L, N)
        per_frame = [topk_positions(z[n], r_hat) if plan[n]["dynamic"] else window_positions(z[n], r_hat)
                     for n in range(N)]
    if force_kept is not None:                        # one array of positions per output frame
        per_frame = [np.asarray(p, dtype=np.int32) for p in force_kept]
        assert len(per_frame) == N
    counts = [len(p) for p in per_frame]
    cu = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    kept = np.concatenate(per_frame).astype(np.int32)
    tokens = np.concatenate([xm[n][per_frame[n]] for n in range(N)], axis=0)
    return dict(frame_sim=s, s_hat=s_hat, cos=c, seg_start=seg, plan=plan, merged=xm, score=z,
                kept_idx=kept, cu_tokens=cu, tokens=tokens,
                frame_dynamic=np.asarray([p["dynamic"] for p in plan], dtype=np.int32),
                frame_first=np.asarray([p["first"] for p in plan], dtype=np.int32),
                frame_count=np.asarray([p["count"] for p in plan], dtype=np.int32))


def encode_clip_policy(shape, w, frames, merge_layer, policy, dtype=np.float64, x_at_merge=None,
                       force_kept=None):
    """Encoder forward with the policy-driven compression after `merge_layer` blocks; the blocks
    after it attend inside each output frame over that frame's kept tokens (ragged lengths)."""
    n_layers = len(w["layers"])
    x = patch_embed(frames, w, shape.patch, dtype)
    info, cu = None, None
    for i in range(n_layers + 1):
        if i == merge_layer:
            if x_at_merge is not None:
                x = np.asarray(x_at_merge, dtype=dtype)
            info = merge_select_policy(x, policy, force_kept)
            info["hidden_at_merge"] = x
            cu = info["cu_tokens"]
            rows = info["tokens"]
        if i < n_layers:
            if info is None:
                if x_at_merge is not None and i < merge_layer:
                    continue
                x = encoder_block(x, w["layers"][i], shape.n_heads, shape.ln_eps)
            else:                                          # ragged frames: block by block per frame
                rows = np.concatenate([encoder_block(rows[cu[n]:cu[n + 1]][None], w["layers"][i],
                                                     shape.n_heads, shape.ln_eps)[0]
                                       for n in range(len(cu) - 1)], axis=0)
    out_rows = rows
    if shape.has_final_ln:
        out_rows = layer_norm(out_rows, np.asarray(w["final_ln_g"], dtype), np.asarray(w["final_ln_b"], dtype),
                              shape.ln_eps)
    info = dict(info)
    info["tokens"] = out_rows
    info["n_frames_out"] = len(cu) - 1
    return info


# --------------------------------------------------------------------------
# Whole path
# --------------------------------------------------------------------------

def encode_clip(shape, w, frames, merge_layer, sim_threshold, keep_ratio,
                dtype=np.float64, force_seg_start=None, force_kept=None, x_at_merge=None):
    """Encoder forward with the compression applied after `merge_layer` blocks.

    merge_layer < 0 disables compression (plain encoder).  merge_layer == n_layers
    compresses after the last block, before the final LayerNorm.
    `x_at_merge` (optional [T, L, D]) replaces the hidden states the compression
    stage sees and the blocks after it continue from; used for stage-wise parity.
    Returns a dict with tokens [n_tokens, D], kept_idx [n_tokens], cu_tokens,
    seg_start, frame_sim, hidden_at_merge, n_frames_out.
    """
    n_layers = len(w["layers"])
    T = frames.shape[0]
    L = shape.tokens_per_frame
    x = patch_embed(frames, w, shape.patch, dtype)
    info = None
    for i in range(n_layers + 1):
        if i == merge_layer:
            if x_at_merge is not None:
                x = np.asarray(x_at_merge, dtype=dtype)
            info = merge_select(x, sim_threshold, keep_ratio, force_seg_start, force_kept)
            info["hidden_at_merge"] = x
            N, k = info["kept_idx"].shape
            x = info["tokens"].reshape(N, k, -1)
        if i < n_layers:
            if x_at_merge is not None and 0 <= merge_layer and i < merge_layer:
                continue                      # replaced at the merge layer anyway
            x = encoder_block(x, w["layers"][i], shape.n_heads, shape.ln_eps)
    if shape.has_final_ln:
        x = layer_norm(x, np.asarray(w["final_ln_g"], dtype), np.asarray(w["final_ln_b"], dtype),
                       shape.ln_eps)
    F, n, D = x.shape
    out = dict(tokens=x.reshape(F * n, D), n_frames_out=F)
    if info is None:
        out.update(kept_idx=np.tile(np.arange(L, dtype=np.int32), T),
                   cu_tokens=(np.arange(T + 1) * L).astype(np.int32),
                   seg_start=np.arange(T + 1, dtype=np.int32),
                   frame_sim=np.zeros((max(T - 1, 0),), dtype), hidden_at_merge=None)
    else:
        out.update(kept_idx=info["kept_idx"].reshape(-1), cu_tokens=info["cu_tokens"],
                   seg_start=info["seg_start"], frame_sim=info["frame_sim"],
                   hidden_at_merge=info["hidden_at_merge"], score=info["score"])
    return out


def encode_clip_multi(shape, w, frames, merge_layers, select_layer, policy, dtype=np.float64,
                      x_at_layers=None, force_kept=None, qk_at_score_layer=None):
    """Stage I at several encoder layers, Stage II once (the paper merges at three layers, e.g.
    [6, 14, 20], and selects after the encoder).

    At every layer in `merge_layers` (ascending) the adjacent-frame similarity of the CURRENT frames
    drives Eq. 1 and the merge of `policy["merge_mode"]`; frames keep all L tokens.  At `select_layer`
    (>= the last merge layer; after that layer's merge if they coincide) the selection of
    `policy["select_mode"]` runs once: dynamic flags come from the most recent merge (every frame is
    dynamic if there was none), the re-scaled count uses the ORIGINAL frame count.
    `x_at_layers` (optional dict layer -> [frames, L, D]) replaces the hidden states seen at a merge /
    select layer (stage-wise parity); a block whose output would be replaced that way is not evaluated.
    `qk_at_score_layer` (optional [frames, L, 2 D], attention scores only) replaces the queries and keys
    of the scoring block in the same way: the scores are then the column means of the softmax of THOSE
    q . k / sqrt(hd) (stage-wise parity of the ranking on identical inputs).
    Returns tokens, kept_idx, cu_tokens, frame_first / frame_count (ranges of original frames),
    frame_dynamic, seg_start (original frame index of each segment start of the last merge),
    n_frames_out, hidden (dict of the states seen at each layer), stages (per merge layer: frame_sim,
    s_hat, n_frames) and score (the selection scores)."""
    n_layers = len(w["layers"])
    T0 = frames.shape[0]
    L = shape.tokens_per_frame
    x = patch_embed(frames, w, shape.patch, dtype)
    first = np.arange(T0, dtype=np.int64)
    count = np.ones(T0, dtype=np.int64)
    dyn = np.ones(T0, dtype=np.int32)
    seg_orig = np.arange(T0 + 1, dtype=np.int64)
    hidden, rows, cu, kept = {}, None, None, None
    merge_layers = list(merge_layers)
    stage_layers = sorted(set(merge_layers) | {select_layer})
    stages, score = {}, None
    by_attention = policy.get("score_mode", "l2") == "attention"
    z_att = None
    if by_attention:
        # the scores are the attention received in the block just before the selection, which has to
        # see the frames the selection sees: no merge may sit between that block and the selection
        assert select_layer >= 1 and select_layer not in merge_layers, \
            "attention scores need a block between the last merge and the selection"
        stage_layers = sorted(set(stage_layers) | {select_layer - 1})

    def replaced_later(i):
        nxt = [j for j in stage_layers if j > i]
        return bool(nxt) and x_at_layers is not None and nxt[0] in x_at_layers
    for i in range(n_layers + 1):
        if by_attention and i == select_layer - 1 and i not in merge_layers:
            if x_at_layers is not None and i in x_at_layers:
                x = np.asarray(x_at_layers[i], dtype=dtype)
                if x.shape[0] != len(first):
                    raise ValueError("x_at_layers[%d] holds %d frames, the plan so far gives %d"
                                     % (i, x.shape[0], len(first)))
            hidden[i] = x
        if rows is None and (i in merge_layers or i == select_layer):
            if x_at_layers is not None and i in x_at_layers:
                x = np.asarray(x_at_layers[i], dtype=dtype)
                if x.shape[0] != len(first):
                    raise ValueError("x_at_layers[%d] holds %d frames, the plan so far gives %d"
                                     % (i, x.shape[0], len(first)))
            hidden[i] = x
            z = None
            if i in merge_layers:
                Tc = x.shape[0]
                s = frame_similarity(x)[1] if Tc > 1 else np.zeros((0,), dtype)
                seg, s_hat = ema_segment_starts(s, policy["alpha"], policy["tau_seg"], Tc)
                plan = merge_plan(s, seg, policy["tau_merge"], policy["merge_mode"])
                x = apply_plan(x, plan)
                z = token_score(x)
                stages[i] = dict(frame_sim=s, s_hat=s_hat, n_frames=len(plan), merged=x)
                ends = first + count
                seg_orig = np.asarray([first[a] for a in seg[:-1]] + [T0], dtype=np.int64)
                nf = np.asarray([first[p["first"]] for p in plan], dtype=np.int64)
                ne = np.asarray([ends[p["first"] + p["count"] - 1] for p in plan], dtype=np.int64)
                first, count = nf, ne - nf
                dyn = np.asarray([p["dynamic"] for p in plan], dtype=np.int32)
            if i == select_layer:
                if by_attention:
                    z = z_att
                elif z is None:
                    z = token_score(x)
                N = x.shape[0]
                score = z
                if force_kept is not None:
                    per_frame = [np.asarray(p, dtype=np.int32) for p in force_kept]
                elif policy["select_mode"] == "uniform":
                    k = keep_count(L, policy["ratio"])
                    per_frame = [topk_positions(z[n], k) for n in range(N)]
                else:
                    r_hat = rescaled_count(policy["ratio"], T0, L, N)
                    per_frame = [topk_positions(z[n], r_hat) if dyn[n] else window_positions(z[n], r_hat)
                                 for n in range(N)]
                cu = np.concatenate([[0], np.cumsum([len(p) for p in per_frame])]).astype(np.int32)
                kept = np.concatenate(per_frame).astype(np.int32)
                rows = np.concatenate([x[n][per_frame[n]] for n in range(N)], axis=0)
        if by_attention and i == select_layer - 1:
            # (after this layer's own merge, if it has one: the block runs on the merged frames)
            if qk_at_score_layer is not None:
                qk = np.asarray(qk_at_score_layer, dtype=dtype)
                if qk.shape != (x.shape[0], L, 2 * shape.d_model):
                    raise ValueError("qk_at_score_layer has shape %s, the scoring block sees %d frames"
                                     % (qk.shape, x.shape[0]))
                z_att = attention_received_from_qk(qk[..., :shape.d_model], qk[..., shape.d_model:], shape.n_heads)
            else:
                z_att = attention_received(x, w["layers"][i], shape.n_heads, shape.ln_eps)
        if i < n_layers:
            if rows is None:
                if not replaced_later(i):
                    x = encoder_block(x, w["layers"][i], shape.n_heads, shape.ln_eps)
            else:
                rows = np.concatenate([encoder_block(rows[cu[n]:cu[n + 1]][None], w["layers"][i],
                                                     shape.n_heads, shape.ln_eps)[0]
                                       for n in range(len(cu) - 1)], axis=0)
    assert rows is not None, "select_layer must lie in [0, n_layers]"
    if shape.has_final_ln:
        rows = layer_norm(rows, np.asarray(w["final_ln_g"], dtype), np.asarray(w["final_ln_b"], dtype),
                          shape.ln_eps)
    return dict(tokens=rows, kept_idx=kept, cu_tokens=cu, frame_first=first.astype(np.int32),
                frame_count=count.astype(np.int32), frame_dynamic=dyn, seg_start=seg_orig.astype(np.int32),
                n_frames_out=len(cu) - 1, hidden=hidden, stages=stages, score=score)

