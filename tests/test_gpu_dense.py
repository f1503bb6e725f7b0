"""GPU parity of the dense encoder kernels (LayerNorm, MFMA GEMM + epilogues, attention)
against the CPU oracle's definitions, on bf16-representable inputs.

Tolerances: the kernels accumulate in float32 and round the result once to bf16
(relative step 2^-8), so element errors are bounded by about 2^-8 of the result's
magnitude plus float32 accumulation noise; relative L2 errors stay below 4e-3.
"""
import math

import numpy as np
import pytest
import torch

import paper_2605_30010_amd as et
from et_inputs import bf16_bits_to_f32, f32_to_bf16_bits
from oracle import earlytom_oracle as O
from tests._util import bits_to_dev, dev_to_bits, dev_to_f64, rel_l2

pytestmark = pytest.mark.gpu


def _bf(rng, shape, scale=1.0, shift=0.0):
    bits = f32_to_bf16_bits((rng.standard_normal(shape) * scale + shift).astype(np.float32))
    return bits, bf16_bits_to_f32(bits).astype(np.float64)


@pytest.mark.parametrize("rows,D", [(1, 64), (37, 64), (1000, 1152), (5, 4096), (9, 520)])
def test_layernorm_matches_oracle(rows, D):
    rng = np.random.default_rng(rows + D)
    bits, x = _bf(rng, (rows, D), scale=3.0, shift=1.5)
    g = (1 + 0.1 * rng.standard_normal(D)).astype(np.float32)
    b = (0.1 * rng.standard_normal(D)).astype(np.float32)
    ref = O.layer_norm(x, g.astype(np.float64), b.astype(np.float64), 1e-6)
    y = et.et_layernorm(bits_to_dev(bits), torch.from_numpy(g).cuda(), torch.from_numpy(b).cuda(), 1e-6)
    got = dev_to_f64(y)
    assert np.max(np.abs(got - ref) - 2 ** -8 * np.abs(ref)) < 2e-5
    assert rel_l2(got, ref) < 3e-3


@pytest.mark.parametrize("M,N,K", [(64, 64, 64), (300, 192, 128), (1000, 1152, 1152), (257, 4304, 1152),
                                   (513, 1152, 4304), (5, 8, 8), (2050, 3456, 1152), (700, 1152, 592)])
@pytest.mark.parametrize("epi", [0, 1, 2])
def test_gemm_matches_oracle(M, N, K, epi):
    rng = np.random.default_rng(M + N + K + epi)
    a_bits, a = _bf(rng, (M, K))
    w_bits, w = _bf(rng, (N, K), scale=0.05)
    bias = (0.1 * rng.standard_normal(N)).astype(np.float32)
    r_bits, r = _bf(rng, (M, N))
    ref = a @ w.T + bias.astype(np.float64)
    if epi == 1:
        ref = O.gelu_tanh(ref)
    if epi == 2:
        ref = ref + r
    c = et.et_gemm_bf16(bits_to_dev(a_bits), bits_to_dev(w_bits), torch.from_numpy(bias).cuda(), epi,
                        residual=bits_to_dev(r_bits) if epi == 2 else None)
    got = dev_to_f64(c)
    scale = np.sqrt(K) * 0.05 + 1.0
    assert np.max(np.abs(got - ref) - 2 ** -8 * np.abs(ref)) < 2e-4 * scale
    assert rel_l2(got, ref) < 4e-3


@pytest.mark.parametrize("cfg", [0, 1, 2])
def test_gemm_every_tile_configuration(cfg):
    """Each workgroup tiling, on a shape with ragged M, several k-tiles and a partial N tile."""
    rng = np.random.default_rng(cfg)
    M, N, K = 777, 1160, 448
    a_bits, a = _bf(rng, (M, K))
    w_bits, w = _bf(rng, (N, K), scale=0.05)
    bias = (0.1 * rng.standard_normal(N)).astype(np.float32)
    r_bits, r = _bf(rng, (M, N))
    ref = O.gelu_tanh(a @ w.T + bias.astype(np.float64))
    c = et.et_gemm_bf16(bits_to_dev(a_bits), bits_to_dev(w_bits), torch.from_numpy(bias).cuda(), 1,
                        tile_config=cfg)
    got = dev_to_f64(c)
    assert np.max(np.abs(got - ref) - 2 ** -8 * np.abs(ref)) < 5e-4
    assert rel_l2(got, ref) < 4e-3
    ref2 = a @ w.T + bias.astype(np.float64) + r
    c2 = et.et_gemm_bf16(bits_to_dev(a_bits), bits_to_dev(w_bits), torch.from_numpy(bias).cuda(), 2,
                         residual=bits_to_dev(r_bits), tile_config=cfg)
    assert rel_l2(dev_to_f64(c2), ref2) < 4e-3


def test_gemm_residual_in_place():
    rng = np.random.default_rng(5)
    M, N, K = 333, 128, 64
    a_bits, a = _bf(rng, (M, K))
    w_bits, w = _bf(rng, (N, K), scale=0.1)
    r_bits, r = _bf(rng, (M, N))
    bias = torch.zeros(N, dtype=torch.float32, device="cuda")
    res = bits_to_dev(r_bits)
    lib = et.load_library()
    import ctypes as C
    a_d, w_d = bits_to_dev(a_bits), bits_to_dev(w_bits)
    rc = lib.et_gemm_bf16(C.c_void_p(a_d.data_ptr()), C.c_void_p(w_d.data_ptr()), C.c_void_p(bias.data_ptr()),
                          C.c_void_p(res.data_ptr()), M, N, K, 2, -1, C.c_void_p(res.data_ptr()),
                          C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, et.et_last_error()
    assert rel_l2(dev_to_f64(res), a @ w.T + r) < 4e-3


def _attention_ref(qkv, cu, n_heads, hd):
    D = n_heads * hd
    out = np.zeros((qkv.shape[0], D))
    for f in range(len(cu) - 1):
        a, b = cu[f], cu[f + 1]
        if b == a:
            continue
        q = qkv[a:b, :D].reshape(b - a, n_heads, hd).transpose(1, 0, 2)
        k = qkv[a:b, D:2 * D].reshape(b - a, n_heads, hd).transpose(1, 0, 2)
        v = qkv[a:b, 2 * D:].reshape(b - a, n_heads, hd).transpose(1, 0, 2)
        p = O.softmax_rows(q @ k.transpose(0, 2, 1) / math.sqrt(hd))
        out[a:b] = (p @ v).transpose(1, 0, 2).reshape(b - a, D)
    return out


@pytest.mark.parametrize("n_heads,hd", [(4, 16), (16, 72), (2, 64), (2, 128), (3, 32), (2, 80), (2, 96)])
def test_attention_matches_oracle(n_heads, hd):
    rng = np.random.default_rng(n_heads * hd)
    lens = [5, 64, 131, 729, 1, 128, 364, 182] if hd in (16, 72) else [5, 130, 64, 1]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    rows, D = int(cu[-1]), n_heads * hd
    # logits with a spread of several units so that the softmax is far from uniform
    bits, qkv = _bf(rng, (rows, 3 * D), scale=1.0)
    qkv_s = qkv.copy()
    qkv_s[:, :D] *= 2.0
    bits = f32_to_bf16_bits(qkv_s.astype(np.float32))
    qkv_s = bf16_bits_to_f32(bits).astype(np.float64)
    ref = _attention_ref(qkv_s, cu, n_heads, hd)
    out = et.et_attention(bits_to_dev(bits), torch.from_numpy(cu).cuda(), max(lens), n_heads, hd)
    got = dev_to_f64(out)
    assert rel_l2(got, ref) < 6e-3
    assert np.max(np.abs(got - ref)) < 0.05
    # a one-token frame attends to itself only: output = its own v, exactly
    one = int(cu[lens.index(1)])
    assert np.array_equal(got[one], qkv_s[one, 2 * D:])


@pytest.mark.parametrize("n_heads,hd,n_frames,length", [(16, 72, 3, 729), (16, 72, 5, 364), (16, 72, 2, 182),
                                                        (4, 16, 8, 64), (4, 16, 2, 32), (2, 64, 3, 130),
                                                        (2, 128, 2, 70), (3, 32, 2, 1), (2, 80, 2, 129),
                                                        (2, 96, 2, 65), (16, 72, 1, 218),
                                                        # enough workgroups for two query blocks per wavefront
                                                        (16, 72, 11, 729), (4, 16, 130, 70), (2, 80, 90, 300)])
def test_attention_uniform_matches_oracle(n_heads, hd, n_frames, length):
    rng = np.random.default_rng(n_heads * hd + length)
    D, rows = n_heads * hd, n_frames * length
    _, qkv = _bf(rng, (rows, 3 * D))
    qkv[:, :D] *= 2.0
    bits = f32_to_bf16_bits(qkv.astype(np.float32))
    qkv = bf16_bits_to_f32(bits).astype(np.float64)
    cu = (np.arange(n_frames + 1) * length).astype(np.int32)
    ref = _attention_ref(qkv, cu, n_heads, hd)
    out = et.et_attention_uniform(bits_to_dev(bits), n_frames, length, n_heads, hd)
    got = dev_to_f64(out)
    assert np.all(np.isfinite(got))
    assert rel_l2(got, ref) < 6e-3
    assert np.max(np.abs(got - ref)) < 0.05
    # the ragged entry point (row ranges from cu_tokens) agrees on the same input
    gen = et.et_attention(bits_to_dev(bits), torch.from_numpy(cu).cuda(), length, n_heads, hd)
    assert rel_l2(dev_to_f64(gen), got) < 6e-3


@pytest.mark.parametrize("order", ["rising", "falling", "negative_first", "spike_last"])
def test_attention_uniform_moving_maxima(order):
    """The online softmax keeps a reference maximum that it moves only when a 64-key tile exceeds it by
    2^8; these inputs make the row maxima climb by far more than that from tile to tile (rising), never
    move after the first tile (falling), start far below zero (negative_first), or jump in the last,
    partly filled tile (spike_last)."""
    n_heads, hd, length = 16, 72, 729
    n_frames = 11 if order in ("rising", "spike_last") else 2    # 11 frames: two query blocks per wavefront
    rng = np.random.default_rng({"rising": 1, "falling": 2, "negative_first": 3, "spike_last": 4}[order])
    D, rows = n_heads * hd, n_frames * length
    _, qkv = _bf(rng, (rows, 3 * D))
    pos = np.tile(np.arange(length), n_frames).astype(np.float64)
    # logits = q . k / sqrt(72): a shared direction u with |u| = 1 gives q.k ~ a_q * a_k
    u = np.zeros(D)
    u.reshape(n_heads, hd)[:, 0] = 1.0
    ramp = {"rising": pos / 64.0 * 3.0, "falling": (length - pos) / 64.0 * 3.0,
            "negative_first": np.where(pos < 64, -40.0, 0.0), "spike_last": np.where(pos >= 720, 30.0, 0.0)}[order]
    qkv[:, :D] = qkv[:, :D] * 0.5 + 8.0 * u                      # q . u = 8 per head
    qkv[:, D:2 * D] = qkv[:, D:2 * D] * 0.5 + ramp[:, None] * u  # k . u = ramp -> logit shift 8 ramp / sqrt(72)
    bits = f32_to_bf16_bits(qkv.astype(np.float32))
    qkv = bf16_bits_to_f32(bits).astype(np.float64)
    cu = (np.arange(n_frames + 1) * length).astype(np.int32)
    ref = _attention_ref(qkv, cu, n_heads, hd)
    got = dev_to_f64(et.et_attention_uniform(bits_to_dev(bits), n_frames, length, n_heads, hd))
    assert np.all(np.isfinite(got))
    assert rel_l2(got, ref) < 1e-2
    assert np.max(np.abs(got - ref)) < 0.05


@pytest.mark.parametrize("cfg", [0, 1, 2])
def test_gemm_persistent_configs_walk_several_tiles_per_workgroup(cfg):
    """More output tiles than compute units, so each persistent workgroup finishes a tile, clears its
    accumulators and goes on; ragged last tile row and column; all three epilogues."""
    rng = np.random.default_rng(100 + cfg)
    M, N, K = 4500, 4304, 320                       # 18 x 17 = 306 tiles of 256 x 256
    a_bits, a = _bf(rng, (M, K))
    w_bits, w = _bf(rng, (N, K), scale=0.05)
    bias = (0.1 * rng.standard_normal(N)).astype(np.float32)
    r_bits, r = _bf(rng, (M, N))
    lin = a @ w.T + bias.astype(np.float64)
    a_d, w_d, b_d = bits_to_dev(a_bits), bits_to_dev(w_bits), torch.from_numpy(bias).cuda()
    for epi, ref in ((0, lin), (1, O.gelu_tanh(lin)), (2, lin + r)):
        c = et.et_gemm_bf16(a_d, w_d, b_d, epi, residual=bits_to_dev(r_bits) if epi == 2 else None,
                            tile_config=cfg)
        got = dev_to_f64(c)
        assert np.max(np.abs(got - ref) - 2 ** -8 * np.abs(ref)) < 5e-4, epi
        assert rel_l2(got, ref) < 4e-3, epi


def test_gemm_fc2_shape_with_residual_at_encoder_row_counts():
    """The fc2 step as the encoder runs it (K = 4304, bias + residual) on the kept-token and the all-token
    row counts: every element against exact products summed in float64."""
    rng = np.random.default_rng(4304)
    N, K = 1152, 4304
    w_bits, w = _bf(rng, (N, K), scale=0.02)
    bias = (0.1 * rng.standard_normal(N)).astype(np.float32)
    w_d, b_d = bits_to_dev(w_bits), torch.from_numpy(bias).cuda()
    for M in (2912, 23328):
        a_bits, a = _bf(rng, (M, K))
        r_bits, r = _bf(rng, (M, N))
        ref = a @ w.T + bias.astype(np.float64) + r
        c = et.et_gemm_bf16(bits_to_dev(a_bits), w_d, b_d, 2, residual=bits_to_dev(r_bits))
        got = dev_to_f64(c)
        assert np.max(np.abs(got - ref) - 2 ** -8 * np.abs(ref)) < 5e-4, M
        assert rel_l2(got, ref) < 4e-3, M


@pytest.mark.parametrize("N,epi", [(3456, 0), (4304, 1), (4304, 2), (1152, 2)])
def test_gemm_library_choice_at_encoder_row_count(N, epi):
    """32 x 729 rows with the library's own tiling, which splits a nearly empty last tile row or a partly
    filled last tile column off into launches of their own: every output element against the oracle."""
    rng = np.random.default_rng(N + epi)
    M, K = 23328, 128
    a_bits, a = _bf(rng, (M, K))
    w_bits, w = _bf(rng, (N, K), scale=0.1)
    bias = (0.1 * rng.standard_normal(N)).astype(np.float32)
    ref = a.astype(np.float32) @ w.astype(np.float32).T + bias            # exact products, float32 sums of 128 terms
    res = None
    if epi == 1:
        ref = O.gelu_tanh(ref.astype(np.float64))
    if epi == 2:
        r_bits, r = _bf(rng, (M, N))
        ref = ref + r.astype(np.float32)
        res = bits_to_dev(r_bits)
    c = et.et_gemm_bf16(bits_to_dev(a_bits), bits_to_dev(w_bits), torch.from_numpy(bias).cuda(), epi, residual=res)
    got = bf16_bits_to_f32(dev_to_bits(c))
    assert np.max(np.abs(got - ref) - 2 ** -8 * np.abs(ref)) < 5e-4
    assert rel_l2(got.astype(np.float64), ref.astype(np.float64)) < 4e-3


@pytest.mark.parametrize("rows,d_in,d_hidden,d_out", [(4949, 1152, 3584, 3584), (300, 64, 104, 72), (1, 128, 8, 8)])
def test_projector_matches_oracle(rows, d_in, d_hidden, d_out):
    """The two-layer projector (Sec. 3.1) on as many tokens as the paper's layout keeps of a 32-frame clip,
    at the widths of a 7B language model, and on small ragged widths; the hidden activation passes through
    bfloat16 once, hence 1e-2."""
    rng = np.random.default_rng(rows + d_out)
    x_bits, x = _bf(rng, (rows, d_in))
    w1_bits, w1 = _bf(rng, (d_hidden, d_in), scale=1.0 / math.sqrt(d_in))
    w2_bits, w2 = _bf(rng, (d_out, d_hidden), scale=1.0 / math.sqrt(d_hidden))
    b1 = (0.1 * rng.standard_normal(d_hidden)).astype(np.float32)
    b2 = (0.1 * rng.standard_normal(d_out)).astype(np.float32)
    proj = et.Projector(w1, b1, w2, b2)
    got = dev_to_f64(proj.project(bits_to_dev(x_bits)))
    proj.close()
    ref = O.project_tokens(x, w1, b1.astype(np.float64), w2, b2.astype(np.float64))
    assert got.shape == ref.shape
    assert rel_l2(got, ref) < 1e-2
    assert np.max(np.abs(got - ref)) < 0.05 * max(1.0, np.abs(ref).max())
