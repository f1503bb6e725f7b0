"""GPU parity of the compression-stage kernels against the CPU oracle, through the C boundary.

Integer outputs (segment starts, kept positions, offsets) must be bit-exact; merged tokens
are compared as bf16 bit patterns (at most one step apart, where the oracle's float64 mean
rounds across a bf16 tie differently from the kernel's float32 mean); float32 scores and
similarities to a few float32 ulps.
"""
import math
import os

import numpy as np
import pytest
import torch

import paper_2605_30010_amd as et
from et_inputs import (bf16_bits_to_f32, build_workload, make_hidden_states,
                       scene_lengths_geometric)
from oracle import earlytom_oracle as O
from tests._util import bits_to_dev, dev_to_bits, bf16_ulp_distance, f64_to_bits

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rand_bits(rng, shape, scale=1.0):
    from et_inputs import f32_to_bf16_bits
    return f32_to_bf16_bits((rng.standard_normal(shape) * scale).astype(np.float32))


@pytest.mark.parametrize("T,L,D", [(2, 1, 8), (9, 70, 64), (5, 729, 1152), (17, 33, 1160),
                                   (3, 5, 4096), (26, 130, 520)])
def test_similarity_matches_oracle(T, L, D):
    rng = np.random.default_rng(T * 1000 + L)
    bits = _rand_bits(rng, (T, L, D))
    # make some adjacent frames nearly equal so that similarities span [-1, 1]
    x = bf16_bits_to_f32(bits)
    for t in range(1, T, 2):
        x[t] = x[t - 1] * rng.uniform(0.5, 2.0) + 0.05 * x[t]
    if T > 3:
        x[3] = -x[2]
    bits = f64_to_bits(x)
    c_ref, s_ref = O.frame_similarity(bf16_bits_to_f32(bits).astype(np.float64))
    cos, sim = et.et_frame_similarity(bits_to_dev(bits))
    torch.cuda.synchronize()
    np.testing.assert_allclose(cos.cpu().numpy(), c_ref, rtol=0, atol=3e-6)
    np.testing.assert_allclose(sim.cpu().numpy(), s_ref, rtol=0, atol=2e-6)


def test_similarity_zero_rows_hit_the_eps_floor():
    bits = np.zeros((3, 4, 64), dtype=np.uint16)
    cos, sim = et.et_frame_similarity(bits_to_dev(bits))
    assert torch.all(cos == 0) and torch.all(sim == 0)


def _scan_cases():
    out = []
    for line in open(os.path.join(GOLD, "segment_scan_cases.txt")):
        line = line.strip()
        if line and not line.startswith("#"):
            p = [q.strip() for q in line.split("|")]
            out.append((float(p[0]), [float(v) for v in p[1].split()], [int(v) for v in p[2].split()]))
    return out


def _gpu_scan(s32, T, tau):
    dev = torch.from_numpy(np.ascontiguousarray(s32, dtype=np.float32)).cuda() if T > 1 else \
        torch.zeros(1, dtype=torch.float32, device="cuda")
    seg, n = et.et_segment_scan(dev, T, tau)
    n = int(n.item())
    return seg[:n + 1].cpu().numpy()


def test_segment_scan_hand_cases_and_random():
    for tau, s, expect in _scan_cases():
        got = _gpu_scan(np.array(s, dtype=np.float32), len(s) + 1, tau)
        # the kernel compares in float32, like np.float32(s) < np.float32(tau)
        ref = O.segment_starts(np.array(s, dtype=np.float32), float(np.float32(tau)), len(s) + 1)
        assert got.tolist() == ref.tolist()
        if not any(abs(v - tau) < 1e-6 for v in s):
            assert got.tolist() == expect
    rng = np.random.default_rng(0)
    for T in (1, 2, 63, 64, 65, 66, 129, 300, 1000):
        s = rng.random(max(T - 1, 0)).astype(np.float32)
        if T > 10:
            s[4] = np.nan                                   # NaN similarity opens a segment
        for tau in (0.5, 0.05, 0.999, math.inf, -1.0):
            ref = O.segment_starts(s, float(np.float32(tau)), T)
            assert _gpu_scan(s, T, tau).tolist() == ref.tolist()


@pytest.mark.parametrize("T,L,D", [(7, 19, 64), (12, 100, 1152), (40, 9, 520)])
def test_segment_mean_and_score_match_oracle(T, L, D):
    rng = np.random.default_rng(T)
    bits = _rand_bits(rng, (T, L, D))
    cuts = sorted(set(rng.integers(1, T, size=max(1, T // 4)).tolist()))
    seg = np.array([0] + cuts + [T], dtype=np.int32)
    N = len(seg) - 1
    x64 = bf16_bits_to_f32(bits).astype(np.float64)
    m_ref = O.segment_mean(x64, seg)
    z_ref = O.token_score(m_ref)
    seg_dev = torch.zeros(T + 1, dtype=torch.int32, device="cuda")
    seg_dev[:N + 1] = torch.from_numpy(seg).cuda()
    n_dev = torch.tensor([N], dtype=torch.int32, device="cuda")
    merged, score = et.et_segment_mean(bits_to_dev(bits), seg_dev, n_dev)
    torch.cuda.synchronize()
    got_bits = dev_to_bits(merged[:N])
    dist = bf16_ulp_distance(got_bits, f64_to_bits(m_ref))
    assert dist.max() <= 1
    assert (dist > 0).mean() < 2e-3
    np.testing.assert_allclose(score[:N].cpu().numpy(), z_ref, rtol=2e-6)
    # length-1 segments are bit copies
    for n in range(N):
        if seg[n + 1] - seg[n] == 1:
            assert np.array_equal(got_bits[n], bits[seg[n]])


def _check_topk(z32, k):
    got = et.et_topk_select(torch.from_numpy(z32).cuda(), k).cpu().numpy()
    for n in range(z32.shape[0]):
        assert got[n].tolist() == O.topk_positions(z32[n], k).tolist(), (n, k)


def test_topk_matches_oracle_bit_exactly():
    rng = np.random.default_rng(1)
    for n_rows, L in [(7, 729), (3, 1000), (2, 64), (1, 1), (5, 4097), (4, 255), (4, 257), (2, 15360)]:
        z = (rng.random((n_rows, L)) * 1000).astype(np.float32)
        for k in sorted({1, max(1, L // 4), max(1, L // 2), L}):
            _check_topk(z, k)
        # heavy ties: few distinct levels, all-equal rows, zeros
        zt = rng.integers(0, 4, (n_rows, L)).astype(np.float32)
        zt[0] = 5.0
        for k in sorted({1, max(1, L // 3), max(1, L - 1), L}):
            _check_topk(zt, k)
    # ties that differ only in the low radix digits, infinities and NaN
    z = np.full((2, 729), 1.0, dtype=np.float32)
    z[0, ::3] = np.nextafter(np.float32(1.0), np.float32(2.0))
    z[0, 5] = np.inf
    z[0, 9] = np.nan
    z[1, 100:300] = np.float32(1.0) + np.arange(200, dtype=np.float32) * np.float32(2 ** -20)
    for k in (1, 2, 100, 243, 244, 364, 728, 729):
        _check_topk(z, k)


def test_topk_rejects_frames_longer_than_its_limit():
    z = torch.zeros((1, 15361), dtype=torch.float32, device="cuda")
    with pytest.raises(et.EtError) as e:
        et.et_topk_select(z, 4)
    assert e.value.code == -5 and "15360" in str(e.value)


def test_topk_hand_cases():
    for line in open(os.path.join(GOLD, "topk_cases.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, z, kept = [p.split() for p in line.split("|")]
        got = et.et_topk_select(torch.tensor([[float(v) for v in z]], dtype=torch.float32, device="cuda"),
                                int(k[0]))
        assert got[0].tolist() == [int(v) for v in kept]


def test_compact_is_an_exact_gather():
    rng = np.random.default_rng(2)
    n, L, D, k = 5, 60, 264, 17
    bits = _rand_bits(rng, (n, L, D))
    kept = np.stack([np.sort(rng.choice(L, k, replace=False)) for _ in range(n)]).astype(np.int32)
    out = et.et_compact_tokens(bits_to_dev(bits), torch.from_numpy(kept).cuda())
    ref = np.concatenate([bits[i][kept[i]] for i in range(n)])
    assert np.array_equal(dev_to_bits(out), ref)


def _margins_ok(ref, tau, rel_gap=1e-5):
    if len(ref["frame_sim"]) and np.min(np.abs(ref["frame_sim"] - tau)) < 1e-2:
        return False
    k = ref["k"]
    for z in ref["score"]:
        zs = np.sort(z)[::-1]
        if k < len(zs) and (zs[k - 1] - zs[k]) < rel_gap * zs[k - 1]:
            return False
    return True


def _run_merge_select(bits, tau, keep):
    r = et.et_merge_select(bits_to_dev(bits), tau, keep)
    return {k: (v.clone() if isinstance(v, torch.Tensor) else v) for k, v in r.items()}


def _assert_stage_equal(r, ref, exact_tokens=False):
    assert r["n_frames_out"] == len(ref["seg_start"]) - 1
    assert r["seg_start"].cpu().numpy().tolist() == ref["seg_start"].tolist()
    assert r["cu_tokens"].cpu().numpy().tolist() == ref["cu_tokens"].tolist()
    assert r["n_tokens"] == ref["tokens"].shape[0]
    assert np.array_equal(r["kept_idx"].cpu().numpy(), ref["kept_idx"].reshape(-1))
    np.testing.assert_allclose(r["frame_sim"].cpu().numpy(), ref["frame_sim"], atol=2e-6, rtol=0)
    dist = bf16_ulp_distance(dev_to_bits(r["tokens"]), f64_to_bits(ref["tokens"]))
    assert dist.max() <= (0 if exact_tokens else 1)
    assert (dist > 0).mean() < 2e-3


@pytest.mark.parametrize("T,L,D,keep,mean_len", [(12, 100, 256, 0.3, 3), (16, 729, 1152, 0.5, 4),
                                                 (33, 64, 64, 0.25, 5), (70, 40, 128, 0.6, 6),
                                                 # long clips (many pairs per workgroup of the mean / scan launch)
                                                 (1025, 16, 64, 0.5, 6), (1100, 12, 64, 0.5, 6),
                                                 (300, 400, 64, 0.25, 8),
                                                 # frames longer than the fused selection + gather launch holds:
                                                 # selection and gather as launches of their own
                                                 (3, 8000, 64, 0.1, 2)])
def test_merge_select_matches_oracle(T, L, D, keep, mean_len):
    tau = 0.9
    for variant in range(20):                     # re-seed until the decision margins hold
        rng = np.random.default_rng(100 * T + variant)
        lengths = scene_lengths_geometric(rng, T, mean_len)
        bits = make_hidden_states(T, L, D, lengths, 7 * T + variant, sigma=0.1)
        ref = O.merge_select(bf16_bits_to_f32(bits).astype(np.float64), tau, np.float32(keep))
        if _margins_ok(ref, tau):
            break
    else:
        pytest.fail("no seed with safe margins")
    assert ref["seg_start"].tolist() == np.concatenate([[0], np.cumsum(lengths)]).tolist()
    r = _run_merge_select(bits, tau, keep)
    _assert_stage_equal(r, ref)
    # bit-reproducible run to run
    r2 = _run_merge_select(bits, tau, keep)
    for key in ("tokens", "kept_idx", "seg_start", "cu_tokens", "frame_sim"):
        assert torch.equal(r[key], r2[key])


def test_merge_select_exact_ties_go_to_the_lower_position():
    T, L, D = 6, 96, 128
    bits = make_hidden_states(T, L, D, [1, 1, 1, 1, 1, 1], 5, sigma=0.1, dup_rows=40)
    ref = O.merge_select(bf16_bits_to_f32(bits).astype(np.float64), 0.9, 0.2)
    z = ref["score"].astype(np.float32)
    assert all(len(np.unique(z[n])) < L - 30 for n in range(T))      # ties really are there
    r = _run_merge_select(bits, 0.9, 0.2)
    _assert_stage_equal(r, ref, exact_tokens=True)                   # length-1 segments: bit copies


def test_merge_select_degenerate_cases():
    rng = np.random.default_rng(3)
    L, D = 50, 192
    one = _rand_bits(rng, (1, L, D))
    # a single frame
    ref = O.merge_select(bf16_bits_to_f32(one).astype(np.float64), 0.9, 0.5)
    _assert_stage_equal(_run_merge_select(one, 0.9, 0.5), ref, exact_tokens=True)
    # identical frames -> one segment equal to the frame
    same = np.repeat(one, 8, axis=0)
    r = _run_merge_select(same, 0.9, 1.0)
    assert r["n_frames_out"] == 1 and r["seg_start"].tolist() == [0, 8]
    assert np.array_equal(dev_to_bits(r["tokens"]), one[0])
    assert r["kept_idx"].tolist() == list(range(L))
    # threshold +inf and keep_ratio 1 -> identity
    many = _rand_bits(rng, (5, L, D))
    r = _run_merge_select(many, math.inf, 1.0)
    assert r["n_frames_out"] == 5 and r["seg_start"].tolist() == list(range(6))
    assert np.array_equal(dev_to_bits(r["tokens"]), many.reshape(5 * L, D))
    assert r["cu_tokens"].tolist() == [0, 50, 100, 150, 200, 250]
    # threshold -inf -> everything merges
    r = _run_merge_select(many, -math.inf, 0.1)
    assert r["n_frames_out"] == 1 and r["n_tokens"] == 5


def test_merge_select_full_size_microbench_workload():
    """The 64-frame [64, 729, 1152] workload, complete comparison (the oracle takes seconds)."""
    for variant in range(10):
        rec = build_workload("c5_merge_only", variant=variant)
        bits = rec["x_bits"]
        ref = O.merge_select(bf16_bits_to_f32(bits).astype(np.float64), rec["sim_threshold"],
                             np.float32(rec["keep_ratio"]))
        if _margins_ok(ref, rec["sim_threshold"]):
            break
    else:
        pytest.fail("no variant with safe margins")
    assert ref["k"] == 218
    assert ref["seg_start"].tolist() == np.concatenate([[0], np.cumsum(rec["lengths"])]).tolist()
    r = _run_merge_select(bits, rec["sim_threshold"], rec["keep_ratio"])
    _assert_stage_equal(r, ref)
