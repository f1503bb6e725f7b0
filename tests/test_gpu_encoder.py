"""GPU parity of the whole hot path (et_encode_clip) against the CPU oracle.

Decisions (segments, kept positions) are compared bit-exactly under the protocol the
oracle's float64 and the kernels' bf16 arithmetic allow: the hidden states at the merge
layer are taken from the GPU (an encoder truncated to `merge_layer` blocks, same kernels,
so bit-identical to what the full run sees), the oracle continues from them, and seeds are
chosen so that every similarity is >= 1e-2 from the threshold and the k-th / (k+1)-th score
gap is >= 1e-5 relative.  Output tokens: relative L2 error <= 2e-2.
"""
import math

import numpy as np
import pytest
import torch

import paper_2605_30010_amd as et
from et_inputs import TINY, SIGLIP, build_workload, make_clip, make_weights, bf16_bits_to_f32
from oracle import earlytom_oracle as O
from tests._util import dev_to_bits, dev_to_f64, rel_l2

pytestmark = pytest.mark.gpu
TOL = 2e-2


def _encode(enc, frames, m, tau, keep):
    r = enc.encode(torch.from_numpy(frames).cuda(), m, tau, keep)
    return {k: (v.clone() if isinstance(v, torch.Tensor) else v) for k, v in r.items()}


def _truncated(shape, w, m, max_frames):
    """Encoder with only the first m blocks and no final LayerNorm: its plain output is the
    residual stream the compression stage sees."""
    from dataclasses import replace
    sh = replace(shape, n_layers=m, has_final_ln=0)
    return et.Encoder(sh, dict(w, layers=w["layers"][:m]), max_frames)


def _stagewise_check(shape, w, frames, m, tau, keep, enc=None):
    T = frames.shape[0]
    L, D = shape.tokens_per_frame, shape.d_model
    enc = enc or et.Encoder(shape, w, T)
    got = _encode(enc, frames, m, tau, keep)
    trunc = _truncated(shape, w, m, T)
    xm = _encode(trunc, frames, -1, 0.0, 1.0)["tokens"]
    trunc.close()
    x_gpu = bf16_bits_to_f32(dev_to_bits(xm)).astype(np.float64).reshape(T, L, D)
    ref = O.encode_clip(shape, w, frames, m, tau, np.float32(keep), x_at_merge=x_gpu)
    # margins: only then are bit-exact decisions promised
    assert np.min(np.abs(ref["frame_sim"] - tau)) >= 1e-2
    k = O.keep_count(L, np.float32(keep))
    safe = all((np.sort(z)[::-1][k - 1] - np.sort(z)[::-1][k]) >= 1e-5 * np.sort(z)[::-1][k - 1]
               for z in ref["score"]) if k < L else True
    assert got["seg_start"].tolist() == ref["seg_start"].tolist()
    assert got["cu_tokens"].tolist() == ref["cu_tokens"].tolist()
    np.testing.assert_allclose(got["frame_sim"].cpu().numpy(), ref["frame_sim"], atol=5e-6, rtol=0)
    same_idx = np.array_equal(got["kept_idx"].cpu().numpy(), ref["kept_idx"])
    if safe:
        assert same_idx, "kept positions differ although the score gaps are safe"
    if not same_idx:       # separate arithmetic error from rank flips of near-tied scores
        ref = O.encode_clip(shape, w, frames, m, tau, np.float32(keep), x_at_merge=x_gpu,
                            force_kept=got["kept_idx"].cpu().numpy())
    err = rel_l2(dev_to_f64(got["tokens"]), ref["tokens"])
    assert err <= TOL, err
    return got, ref, err, safe


@pytest.fixture(scope="module")
def tiny():
    rec = build_workload("c1_tiny")
    return rec["weights"], rec["frames"]


def test_tiny_plain_encoder_matches_oracle(tiny):
    w, frames = tiny
    enc = et.Encoder(TINY, w, 8)
    got = _encode(enc, frames, -1, 0.9, 0.5)
    ref = O.encode_clip(TINY, w, frames, -1, 0.9, 0.5)
    assert got["n_frames_out"] == 8 and got["n_tokens"] == 512
    assert got["kept_idx"].tolist() == ref["kept_idx"].tolist()
    assert got["cu_tokens"].tolist() == ref["cu_tokens"].tolist()
    assert got["seg_start"].tolist() == ref["seg_start"].tolist()
    assert rel_l2(dev_to_f64(got["tokens"]), ref["tokens"]) <= TOL
    # disabled by arguments instead of merge_layer < 0: identical bits
    for m in (0, 2, 4):
        off = _encode(enc, frames, m, math.inf, 1.0)
        assert torch.equal(off["tokens"], got["tokens"])
        assert off["seg_start"].tolist() == list(range(9))
    # frames are independent
    one = _encode(enc, frames[3:4], -1, 0.9, 0.5)
    assert torch.equal(one["tokens"], got["tokens"][3 * 64:4 * 64])
    enc.close()


@pytest.mark.parametrize("offset", [1.0, -1.0])
def test_rows_with_a_large_mean(tiny, offset):
    """The block LayerNorms are folded into the GEMMs that follow them; the row mean then cancels only
    because every folded weight row sums to (almost) zero.  A constant added to the patch-embedding bias
    gives every row of the residual stream a mean of several standard deviations (more than that and the
    bfloat16 residual stream itself no longer resolves the signal: at |x| = 4 its step is 0.03, and a
    float64 model of the bfloat16 storage points alone, LayerNorm unfolded, is then 7 % away from the oracle): the output
    must still match the oracle, which keeps LayerNorm and linear layer apart.  Without the centring of the
    folded weights the error would be of the order of the mean."""
    w, frames = tiny
    w2 = dict(w)
    w2["patch_b"] = (np.asarray(w["patch_b"], dtype=np.float32) + np.float32(offset)).astype(np.float32)
    enc = et.Encoder(TINY, w2, 8)
    got = _encode(enc, frames, -1, 0.9, 0.5)
    ref = O.encode_clip(TINY, w2, frames, -1, 0.9, 0.5)
    x0 = O.patch_embed(frames, w2, TINY.patch)
    assert np.mean(np.abs(x0.mean(-1)) / x0.std(-1)) > 3.0           # the premise: |mean| well above the standard deviation
    err = rel_l2(dev_to_f64(got["tokens"]), ref["tokens"])
    assert err <= TOL, err
    enc.close()


def test_tiny_config_end_to_end(tiny):
    """Config 1: two scenes of four frames -> two segments, 32 of 64 tokens each."""
    w, frames = tiny
    enc = et.Encoder(TINY, w, 8)
    got, ref, err, safe = _stagewise_check(TINY, w, frames, 2, 0.9, 0.5, enc)
    assert got["n_frames_out"] == 2 and got["n_tokens"] == 64
    assert got["seg_start"].tolist() == [0, 4, 8]
    # fully end-to-end against the float64 oracle (no hidden-state injection)
    e2e = O.encode_clip(TINY, w, frames, 2, 0.9, 0.5)
    assert got["seg_start"].tolist() == e2e["seg_start"].tolist()
    if np.array_equal(got["kept_idx"].cpu().numpy(), e2e["kept_idx"]):
        assert rel_l2(dev_to_f64(got["tokens"]), e2e["tokens"]) <= TOL
    for m in (0, 1, 3, 4):
        _stagewise_check(TINY, w, frames, m, 0.9, 0.5, enc)
    # two runs are bit-identical
    again = _encode(enc, frames, 2, 0.9, 0.5)
    assert torch.equal(again["tokens"], got["tokens"]) and torch.equal(again["kept_idx"], got["kept_idx"])
    enc.close()


def test_identical_frames_collapse_to_the_single_frame_result(tiny):
    w, frames = tiny
    enc = et.Encoder(TINY, w, 8)
    clip = np.repeat(frames[:1], 8, axis=0)
    for keep in (0.5, 1.0):
        many = _encode(enc, clip, 2, 0.9, keep)
        one = _encode(enc, frames[:1], 2, 0.9, keep)
        assert many["n_frames_out"] == 1 and many["seg_start"].tolist() == [0, 8]
        assert torch.equal(many["kept_idx"], one["kept_idx"])
        assert torch.equal(many["tokens"], one["tokens"])
    plain = _encode(enc, frames[:1], -1, 0.9, 0.5)
    assert torch.equal(many["tokens"], plain["tokens"])
    enc.close()


def test_ragged_clip_lengths_and_merge_at_the_ends(tiny):
    w, _ = tiny
    enc = et.Encoder(TINY, w, 11)
    frames = make_clip(TINY, [1, 5, 2, 3], 77, base="uniform", sigma=0.02)
    for m in (0, 4):
        got, ref, err, safe = _stagewise_check(TINY, w, frames, m, 0.9, 0.3, enc)
        assert got["seg_start"].tolist() == [0, 1, 6, 8, 11]
    with pytest.raises(et.EtError):
        enc.encode(torch.zeros((12, 3, 112, 112), device="cuda"), 2, 0.9, 0.5)
    with pytest.raises(et.EtError):
        enc.encode(torch.from_numpy(frames).cuda(), 5, 0.9, 0.5)
    enc.close()


def test_both_patch_extraction_kernels_agree_bit_for_bit(tiny):
    """Frames that are not 16-byte aligned take the element-wise patch extraction, aligned ones the one that goes
    through LDS a row of patches at a time: same patches, so the whole encoder output is identical."""
    w, frames = tiny
    enc = et.Encoder(TINY, w, 8)
    x = torch.from_numpy(frames).cuda()
    assert x.data_ptr() % 16 == 0
    shifted = torch.empty(x.numel() + 1, dtype=torch.float32, device="cuda")[1:].view_as(x)
    shifted.copy_(x)
    assert shifted.data_ptr() % 16 == 4
    a = {k: (v.clone() if isinstance(v, torch.Tensor) else v) for k, v in enc.encode(x, 2, 0.9, 0.5).items()}
    b = enc.encode(shifted, 2, 0.9, 0.5)
    for key in ("tokens", "kept_idx", "seg_start", "cu_tokens", "frame_sim"):
        assert torch.equal(a[key], b[key]), key
    enc.close()


def test_two_encoders_on_two_streams_from_two_host_threads(tiny):
    """Encoders share no state: two of them driven at the same time, each from a host thread and a
    stream of its own, give what each gives alone (bit for bit)."""
    import threading
    w, frames = tiny
    clips = [frames, make_clip(TINY, [3, 1, 4], 5, base="uniform", sigma=0.02)]
    settings = [(2, 0.9, 0.5), (1, 0.9, 0.3)]
    alone = []
    for clip, (m, tau, keep) in zip(clips, settings):
        enc = et.Encoder(TINY, w, 8)
        alone.append(_encode(enc, clip, m, tau, keep))
        enc.close()
    results, errors = [None, None], []

    def worker(i):
        try:
            enc = et.Encoder(TINY, w, 8)
            stream = torch.cuda.Stream()
            x = torch.from_numpy(clips[i]).cuda()
            torch.cuda.synchronize()
            m, tau, keep = settings[i]
            for _ in range(25):
                r = enc.encode(x, m, tau, keep, stream=stream)
                stream.synchronize()
                for key in ("tokens", "kept_idx", "seg_start", "cu_tokens"):
                    assert torch.equal(r[key], alone[i][key]), key
            results[i] = True
            enc.close()
        except Exception as e:      # noqa: BLE001 - reported by the parent thread
            errors.append(repr(e))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(120)
    assert not errors, errors
    assert results == [True, True]


@pytest.fixture(scope="module")
def siglip8():
    rec = build_workload("c2_siglip_t8")
    return rec


def test_siglip_shape_8_frames_stagewise(siglip8):
    """Config 2 (27 layers, d = 1152, 16 heads of 72, 8 frames of 384 x 384, merge after 8 blocks)."""
    rec = siglip8
    enc = et.Encoder(SIGLIP, rec["weights"], 8)
    got, ref, err, safe = _stagewise_check(SIGLIP, rec["weights"], rec["frames"], rec["merge_layer"],
                                           rec["sim_threshold"], rec["keep_ratio"], enc)
    assert got["seg_start"].tolist() == np.concatenate([[0], np.cumsum(rec["lengths"])]).tolist()
    assert got["n_tokens"] == got["n_frames_out"] * 364
    print("config 2: rel-L2 %.4g, safe margins %s" % (err, safe))
    enc.close()


# ------------------------------------------------------------------ full-size workloads

@pytest.fixture(scope="module")
def siglip_weights(siglip8):
    # one set of SigLIP-shaped weights serves every full-size case (generating 415 M values takes ~15 s)
    return siglip8["weights"]


def _full_size_check(name, w, variant_range, keep=None, m=None):
    """Whole-clip decisions bit-exact (oracle fed the GPU's hidden states at the merge layer); the tokens
    of EVERY output frame against the oracle continued from those states (whole output and worst single
    row); one short segment end to end from pixels."""
    for variant in variant_range:
        rec = build_workload(name, variant=variant, with_weights=False)
        shape, frames, T = rec["shape"], rec["frames"], rec["T"]
        m_ = rec["merge_layer"] if m is None else m
        keep_ = rec["keep_ratio"] if keep is None else keep
        tau = rec["sim_threshold"]
        L, D = shape.tokens_per_frame, shape.d_model
        trunc = _truncated(shape, w, m_, T)
        xm = _encode(trunc, frames, -1, 0.0, 1.0)["tokens"]
        trunc.close()
        x_gpu = bf16_bits_to_f32(dev_to_bits(xm)).astype(np.float64).reshape(T, L, D)
        st = O.merge_select(x_gpu, tau, np.float32(keep_))
        k = st["k"]
        gaps_ok = all((np.sort(z)[::-1][k - 1] - np.sort(z)[::-1][k]) >= 1e-5 * np.sort(z)[::-1][k - 1]
                      for z in st["score"])
        if np.min(np.abs(st["frame_sim"] - tau)) >= 1e-2 and gaps_ok:
            break
    else:
        pytest.fail("no variant with safe decision margins")
    enc = et.Encoder(shape, w, T)
    got = _encode(enc, frames, m_, tau, keep_)
    enc.close()
    truth = np.concatenate([[0], np.cumsum(rec["lengths"])]).tolist()
    assert st["seg_start"].tolist() == truth
    assert got["seg_start"].tolist() == truth
    assert got["cu_tokens"].tolist() == st["cu_tokens"].tolist()
    assert np.array_equal(got["kept_idx"].cpu().numpy(), st["kept_idx"].reshape(-1))
    np.testing.assert_allclose(got["frame_sim"].cpu().numpy(), st["frame_sim"], atol=5e-6, rtol=0)
    N = got["n_frames_out"]
    tok = dev_to_f64(got["tokens"]).reshape(N, k, D)
    assert np.all(np.isfinite(tok))
    # every output frame: remaining blocks + final LayerNorm on the oracle side
    x = st["tokens"].reshape(N, k, D)
    for lw in w["layers"][m_:]:
        x = O.encoder_block(x, lw, shape.n_heads, shape.ln_eps)
    x = O.layer_norm(x, w["final_ln_g"].astype(np.float64), w["final_ln_b"].astype(np.float64), shape.ln_eps)
    err = rel_l2(tok, x)
    per_frame = [rel_l2(tok[n], x[n]) for n in range(N)]
    row_err = np.linalg.norm(tok - x, axis=-1) / np.linalg.norm(x, axis=-1)
    assert err <= TOL, err
    assert max(per_frame) <= TOL, per_frame
    # one short segment fully end to end (pixels -> tokens) with the decisions forced to the GPU's
    lens = np.diff(st["seg_start"])
    n = int(np.argmin(lens))
    a, b = int(st["seg_start"][n]), int(st["seg_start"][n + 1])
    ref = O.encode_clip(shape, w, frames[a:b], m_, -np.inf, np.float32(keep_),
                        force_kept=st["kept_idx"][n:n + 1])
    e2e = rel_l2(tok[n], ref["tokens"])
    assert e2e <= TOL, e2e
    print("%s variant %d m=%d keep=%.2f: N=%d k=%d, rel-L2 all %d tokens %.4g (worst frame %.4g, worst single row %.4g), "
          "end-to-end segment rel-L2 %.4g" % (name, variant, m_, keep_, N, k, N * k, err, max(per_frame),
                                                float(row_err.max()), e2e))
    return err, float(row_err.max())


@pytest.mark.parametrize("m", [4, 8, 13])
@pytest.mark.parametrize("keep", [0.25, 0.5])
def test_full_size_32_frame_clip(siglip_weights, m, keep):
    """Config 3 at the size and launch configuration bench.py times (32 x 729 tokens), over the whole
    sweep of merge layers and keep ratios (Table 3 varies the first merge layer for this trade-off)."""
    _full_size_check("c3_siglip_t32", siglip_weights, range(0, 6), keep=keep, m=m)


def test_full_size_64_frame_clip(siglip_weights):
    """Config 4: 64 frames, noisier scenes with abrupt cuts, merge after 4 blocks, keep 0.25."""
    _full_size_check("c4_siglip_t64", siglip_weights, range(0, 6))
