"""ctypes binding of include/earlytom.h.  Argument marshalling only."""
import ctypes as C
import math
import os

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libearlytom.so")
_lib = None

ET_OK = 0
ET_K_COUNT = 15
KERNEL_KINDS = ["im2col", "gemm_patch", "layernorm", "gemm_qkv", "attention", "gemm_out",
                "gemm_fc1", "gemm_fc2", "similarity", "scan", "merge", "select", "compact", "misc", "score"]


class EtError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("earlytom error %d: %s" % (code, msg))
        self.code = code


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_heads", "d_mlp", "patch",
                                          "image_h", "image_w", "channels")] + \
               [("ln_eps", C.c_float), ("has_final_ln", C.c_int32)]


_FP = C.POINTER(C.c_float)
_FPP = C.POINTER(_FP)
_LAYER_FIELDS = ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")


class _Weights(C.Structure):
    _fields_ = [("patch_w", _FP), ("patch_b", _FP), ("pos_emb", _FP)] + \
               [(n, _FPP) for n in _LAYER_FIELDS] + [("final_ln_g", _FP), ("final_ln_b", _FP)]


class _Output(C.Structure):
    _fields_ = [("tokens_dev", C.c_void_p), ("kept_idx_dev", C.c_void_p), ("cu_tokens_dev", C.c_void_p),
                ("seg_start_dev", C.c_void_p), ("frame_sim_dev", C.c_void_p),
                ("n_frames_out", C.c_int32), ("n_tokens", C.c_int32)]


class _Policy(C.Structure):
    _fields_ = [("merge_mode", C.c_int32), ("select_mode", C.c_int32), ("alpha", C.c_float),
                ("tau_seg", C.c_float), ("tau_merge", C.c_float), ("ratio", C.c_float),
                ("score_mode", C.c_int32)]


class _PlanOut(C.Structure):
    _fields_ = [("frame_first_dev", C.c_void_p), ("frame_count_dev", C.c_void_p),
                ("frame_dynamic_dev", C.c_void_p), ("n_segments", C.c_int32)]


ET_MERGE_MEAN, ET_MERGE_ALG1 = 0, 1
ET_SELECT_UNIFORM, ET_SELECT_DECOUPLED = 0, 1
ET_SCORE_L2NORM, ET_SCORE_ATTENTION = 0, 1


def library_path():
    return _LIB_PATH


def load_library():
    """Load libearlytom.so; raises (never falls back) when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libearlytom.so is not built: run `python -c 'import __graft_entry__ as g; "
                          "g.build()'` (or python paper_2605_30010_amd/build.py) first")
    lib = C.CDLL(_LIB_PATH)
    i32, f32, vp, sz = C.c_int32, C.c_float, C.c_void_p, C.c_size_t
    sig = {
        "et_last_error": (C.c_char_p, []),
        "et_keep_count": (i32, [i32, f32]),
        "et_merge_workspace_bytes": (sz, [i32, i32, i32]),
        "et_merge_select": (C.c_int, [vp, i32, i32, i32, f32, f32, vp, sz, vp, C.POINTER(_Output)]),
        "et_merge_select_policy": (C.c_int, [vp, i32, i32, i32, C.POINTER(_Policy), vp, sz, vp,
                                            C.POINTER(_Output), C.POINTER(_PlanOut)]),
        "et_encode_clip_policy": (C.c_int, [vp, vp, i32, i32, C.POINTER(_Policy), vp, sz, vp,
                                           C.POINTER(_Output), C.POINTER(_PlanOut)]),
        "et_encode_clip_multi": (C.c_int, [vp, vp, i32, C.POINTER(i32), i32, i32, C.POINTER(_Policy), vp, sz, vp,
                                          C.POINTER(_Output), C.POINTER(_PlanOut)]),
        "et_attention_scores_scratch_bytes": (C.c_size_t, [i32, i32, i32]),
        "et_attention_scores": (C.c_int, [vp, i32, i32, i32, i32, vp, vp, vp]),
        "et_frame_similarity": (C.c_int, [vp, i32, i32, i32, vp, vp, vp]),
        "et_segment_scan": (C.c_int, [vp, i32, f32, vp, vp, vp]),
        "et_segment_mean": (C.c_int, [vp, i32, i32, i32, vp, vp, vp, vp, vp]),
        "et_topk_select": (C.c_int, [vp, i32, i32, i32, vp, vp]),
        "et_compact_tokens": (C.c_int, [vp, vp, i32, i32, i32, i32, vp, vp]),
        "et_layernorm": (C.c_int, [vp, vp, vp, f32, i32, i32, vp, vp]),
        "et_gemm_bf16": (C.c_int, [vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, vp]),
        "et_attention": (C.c_int, [vp, vp, i32, i32, i32, i32, vp, vp]),
        "et_attention_uniform": (C.c_int, [vp, i32, i32, i32, i32, vp, vp]),
        "et_encoder_block_qkv": (C.c_int, [vp, i32, vp, i32, vp, vp, vp]),
        "et_merge_select_static": (C.c_int, [vp, i32, i32, i32, f32, f32, vp, C.POINTER(_Output)]),
        "et_encoder_create": (C.c_int, [C.POINTER(_Config), C.POINTER(_Weights), i32, C.POINTER(vp)]),
        "et_encoder_destroy": (None, [vp]),
        "et_workspace_bytes": (sz, [vp, i32]),
        "et_encode_clip": (C.c_int, [vp, vp, i32, i32, f32, f32, vp, sz, vp, C.POINTER(_Output)]),
        "et_profile_enable": (C.c_int, [vp, i32]),
        "et_profile_read": (C.c_int, [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64), i32]),
        "et_kernel_name": (C.c_char_p, [i32]),
        "et_projector_create": (C.c_int, [i32, i32, i32, _FP, _FP, _FP, _FP, C.POINTER(vp)]),
        "et_projector_destroy": (None, [vp]),
        "et_projector_workspace_bytes": (sz, [vp, i32]),
        "et_project_tokens": (C.c_int, [vp, vp, i32, vp, sz, vp, vp]),
        "et_merge_profile_enable": (C.c_int, [i32]),
        "et_merge_profile_read": (C.c_int, [C.POINTER(C.c_double), C.POINTER(C.c_int64), C.POINTER(C.c_double),
                                           C.POINTER(C.c_int64), i32]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def _check(rc):
    if rc != ET_OK:
        raise EtError(rc, load_library().et_last_error().decode())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _dev(t, dtype, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError("%s must be a contiguous CUDA tensor of dtype %s" % (name, dtype))
    return t


def et_last_error():
    return load_library().et_last_error().decode()


def et_keep_count(L, keep_ratio):
    return int(load_library().et_keep_count(int(L), float(keep_ratio)))


def et_merge_workspace_bytes(T, L, D):
    return int(load_library().et_merge_workspace_bytes(T, L, D))


def _alloc_outputs(T, L, D, device, with_sim=True):
    return dict(
        tokens=torch.empty((T * L, D), dtype=torch.bfloat16, device=device),
        kept_idx=torch.empty((T * L,), dtype=torch.int32, device=device),
        cu_tokens=torch.empty((T + 1,), dtype=torch.int32, device=device),
        seg_start=torch.empty((T + 1,), dtype=torch.int32, device=device),
        frame_sim=torch.empty((max(T - 1, 1),), dtype=torch.float32, device=device) if with_sim else None,
    )


def _out_struct(bufs):
    o = _Output()
    o.tokens_dev = bufs["tokens"].data_ptr()
    o.kept_idx_dev = bufs["kept_idx"].data_ptr()
    o.cu_tokens_dev = bufs["cu_tokens"].data_ptr()
    o.seg_start_dev = bufs["seg_start"].data_ptr()
    o.frame_sim_dev = bufs["frame_sim"].data_ptr() if bufs.get("frame_sim") is not None else None
    return o


def _trim(bufs, o, T):
    n, nt = int(o.n_frames_out), int(o.n_tokens)
    res = dict(n_frames_out=n, n_tokens=nt, tokens=bufs["tokens"][:nt], kept_idx=bufs["kept_idx"][:nt],
               cu_tokens=bufs["cu_tokens"][:n + 1], seg_start=bufs["seg_start"][:n + 1])
    if bufs.get("frame_sim") is not None:
        res["frame_sim"] = bufs["frame_sim"][:max(T - 1, 0)]
    return res


def et_merge_select(x, sim_threshold, keep_ratio, workspace=None, outputs=None, stream=None):
    """x: bf16 CUDA tensor [T, L, D].  Returns a dict of (views of) output tensors."""
    lib = load_library()
    _dev(x, torch.bfloat16, "x")
    T, L, D = x.shape
    if workspace is None:
        workspace = torch.empty((max(et_merge_workspace_bytes(T, L, D), 1),), dtype=torch.uint8, device=x.device)
    bufs = outputs if outputs is not None else _alloc_outputs(T, L, D, x.device)
    o = _out_struct(bufs)
    _check(lib.et_merge_select(_ptr(x), T, L, D, float(sim_threshold), float(keep_ratio), _ptr(workspace),
                               workspace.numel(), _stream(stream), C.byref(o)))
    return _trim(bufs, o, T)


def et_merge_select_static(x, sim_threshold, keep_ratio, outputs=None, stream=None):
    """et_merge_select on the library's static scratch buffer (no workspace argument)."""
    lib = load_library()
    _dev(x, torch.bfloat16, "x")
    T, L, D = x.shape
    bufs = outputs if outputs is not None else _alloc_outputs(T, L, D, x.device)
    o = _out_struct(bufs)
    _check(lib.et_merge_select_static(_ptr(x), T, L, D, float(sim_threshold), float(keep_ratio), _stream(stream),
                                      C.byref(o)))
    return _trim(bufs, o, T)


def _policy_struct(policy):
    """policy: dict with merge_mode ("mean" | "alg1"), select_mode ("uniform" | "decoupled"), alpha,
    tau_seg, tau_merge, ratio."""
    p = _Policy()
    p.merge_mode = {"mean": ET_MERGE_MEAN, "alg1": ET_MERGE_ALG1}[policy["merge_mode"]]
    p.select_mode = {"uniform": ET_SELECT_UNIFORM, "decoupled": ET_SELECT_DECOUPLED}[policy["select_mode"]]
    p.alpha, p.tau_seg = float(policy["alpha"]), float(policy["tau_seg"])
    p.tau_merge, p.ratio = float(policy["tau_merge"]), float(policy["ratio"])
    p.score_mode = {"l2": ET_SCORE_L2NORM, "attention": ET_SCORE_ATTENTION}[policy.get("score_mode", "l2")]
    return p


def _plan_bufs(T, device):
    bufs = {k: torch.empty((T,), dtype=torch.int32, device=device)
            for k in ("frame_first", "frame_count", "frame_dynamic")}
    po = _PlanOut()
    po.frame_first_dev = bufs["frame_first"].data_ptr()
    po.frame_count_dev = bufs["frame_count"].data_ptr()
    po.frame_dynamic_dev = bufs["frame_dynamic"].data_ptr()
    return bufs, po


def _trim_policy(bufs, o, plan_bufs, po, T):
    n, nt, ns = int(o.n_frames_out), int(o.n_tokens), int(po.n_segments)
    res = dict(n_frames_out=n, n_tokens=nt, n_segments=ns, tokens=bufs["tokens"][:nt],
               kept_idx=bufs["kept_idx"][:nt], cu_tokens=bufs["cu_tokens"][:n + 1],
               seg_start=bufs["seg_start"][:ns + 1], frame_sim=bufs["frame_sim"][:max(T - 1, 0)])
    for k, v in plan_bufs.items():
        res[k] = v[:n]
    return res


def et_merge_select_policy(x, policy, workspace=None, stream=None):
    """Paper-exact compression stage on x (bf16 CUDA [T, L, D]) under `policy` (see _policy_struct)."""
    lib = load_library()
    _dev(x, torch.bfloat16, "x")
    T, L, D = x.shape
    if workspace is None:
        workspace = torch.empty((max(et_merge_workspace_bytes(T, L, D), 1),), dtype=torch.uint8, device=x.device)
    bufs = _alloc_outputs(T, L, D, x.device)
    o = _out_struct(bufs)
    plan_bufs, po = _plan_bufs(T, x.device)
    pol = _policy_struct(policy)
    _check(lib.et_merge_select_policy(_ptr(x), T, L, D, C.byref(pol), _ptr(workspace), workspace.numel(),
                                      _stream(stream), C.byref(o), C.byref(po)))
    return _trim_policy(bufs, o, plan_bufs, po, T)


def et_encode_clip_policy(handle, frames, merge_layer, policy, L, D, workspace=None, stream=None):
    lib = load_library()
    _dev(frames, torch.float32, "frames")
    T = frames.shape[0]
    if workspace is None:
        workspace = torch.empty((max(et_workspace_bytes(handle, T), 1),), dtype=torch.uint8,
                                device=frames.device)
    bufs = _alloc_outputs(T, L, D, frames.device)
    o = _out_struct(bufs)
    plan_bufs, po = _plan_bufs(T, frames.device)
    pol = _policy_struct(policy)
    _check(lib.et_encode_clip_policy(handle, _ptr(frames), T, int(merge_layer), C.byref(pol), _ptr(workspace),
                                     workspace.numel(), _stream(stream), C.byref(o), C.byref(po)))
    return _trim_policy(bufs, o, plan_bufs, po, T)


def et_encode_clip_multi(handle, frames, merge_layers, select_layer, policy, L, D, workspace=None, stream=None):
    lib = load_library()
    _dev(frames, torch.float32, "frames")
    T = frames.shape[0]
    if workspace is None:
        workspace = torch.empty((max(et_workspace_bytes(handle, T), 1),), dtype=torch.uint8,
                                device=frames.device)
    bufs = _alloc_outputs(T, L, D, frames.device)
    o = _out_struct(bufs)
    plan_bufs, po = _plan_bufs(T, frames.device)
    pol = _policy_struct(policy)
    layers = (C.c_int32 * max(len(merge_layers), 1))(*[int(v) for v in merge_layers])
    _check(lib.et_encode_clip_multi(handle, _ptr(frames), T, layers, len(merge_layers), int(select_layer),
                                    C.byref(pol), _ptr(workspace), workspace.numel(), _stream(stream),
                                    C.byref(o), C.byref(po)))
    return _trim_policy(bufs, o, plan_bufs, po, T)


def et_attention_scores(qkv, n_frames, L, n_heads, head_dim, stream=None):
    """Attention received per token: float32 [n_frames, L] from qkv bf16 [n_frames * L, 3 * n_heads * head_dim]."""
    lib = load_library()
    _dev(qkv, torch.bfloat16, "qkv")
    scratch = torch.empty((max(lib.et_attention_scores_scratch_bytes(n_frames, L, n_heads), 1),), dtype=torch.uint8,
                          device=qkv.device)
    score = torch.empty((n_frames, L), dtype=torch.float32, device=qkv.device)
    _check(lib.et_attention_scores(_ptr(qkv), n_frames, L, n_heads, head_dim, _ptr(scratch), _ptr(score),
                                   _stream(stream)))
    return score


def et_frame_similarity(x, stream=None):
    lib = load_library()
    _dev(x, torch.bfloat16, "x")
    T, L, D = x.shape
    cos = torch.empty((max(T - 1, 1), L), dtype=torch.float32, device=x.device)
    sim = torch.empty((max(T - 1, 1),), dtype=torch.float32, device=x.device)
    _check(lib.et_frame_similarity(_ptr(x), T, L, D, _ptr(cos), _ptr(sim), _stream(stream)))
    return cos[:T - 1], sim[:T - 1]


def et_segment_scan(sim, T, sim_threshold, stream=None):
    lib = load_library()
    _dev(sim, torch.float32, "sim")
    seg = torch.empty((T + 1,), dtype=torch.int32, device=sim.device)
    n = torch.zeros((1,), dtype=torch.int32, device=sim.device)
    _check(lib.et_segment_scan(_ptr(sim), T, float(sim_threshold), _ptr(seg), _ptr(n), _stream(stream)))
    return seg, n


def et_segment_mean(x, seg_start, n_seg, stream=None):
    lib = load_library()
    _dev(x, torch.bfloat16, "x")
    _dev(seg_start, torch.int32, "seg_start")
    _dev(n_seg, torch.int32, "n_seg")
    T, L, D = x.shape
    merged = torch.empty((T, L, D), dtype=torch.bfloat16, device=x.device)
    score = torch.empty((T, L), dtype=torch.float32, device=x.device)
    _check(lib.et_segment_mean(_ptr(x), T, L, D, _ptr(seg_start), _ptr(n_seg), _ptr(merged), _ptr(score),
                               _stream(stream)))
    return merged, score


def et_topk_select(score, k, stream=None):
    lib = load_library()
    _dev(score, torch.float32, "score")
    n, L = score.shape
    kept = torch.empty((n, k), dtype=torch.int32, device=score.device)
    _check(lib.et_topk_select(_ptr(score), n, L, int(k), _ptr(kept), _stream(stream)))
    return kept


def et_compact_tokens(merged, kept, stream=None):
    lib = load_library()
    _dev(merged, torch.bfloat16, "merged")
    _dev(kept, torch.int32, "kept")
    n, L, D = merged.shape
    k = kept.shape[1]
    out = torch.empty((n * k, D), dtype=torch.bfloat16, device=merged.device)
    _check(lib.et_compact_tokens(_ptr(merged), _ptr(kept), n, L, D, k, _ptr(out), _stream(stream)))
    return out


def et_layernorm(x, gamma, beta, eps, stream=None):
    lib = load_library()
    _dev(x, torch.bfloat16, "x")
    _dev(gamma, torch.float32, "gamma")
    _dev(beta, torch.float32, "beta")
    rows, D = x.shape
    y = torch.empty_like(x)
    _check(lib.et_layernorm(_ptr(x), _ptr(gamma), _ptr(beta), float(eps), rows, D, _ptr(y), _stream(stream)))
    return y


def et_gemm_bf16(a, w, bias, epilogue=0, residual=None, tile_config=-1, stream=None):
    """C = A @ W.T + bias (+GELU-tanh | +residual).  a [M,K], w [N,K] bf16; bias fp32 [N]."""
    lib = load_library()
    _dev(a, torch.bfloat16, "a")
    _dev(w, torch.bfloat16, "w")
    _dev(bias, torch.float32, "bias")
    if residual is not None:
        _dev(residual, torch.bfloat16, "residual")
    M, K = a.shape
    N = w.shape[0]
    c = torch.empty((M, N), dtype=torch.bfloat16, device=a.device)
    _check(lib.et_gemm_bf16(_ptr(a), _ptr(w), _ptr(bias), _ptr(residual), M, N, K, int(epilogue), int(tile_config), _ptr(c),
                            _stream(stream)))
    return c


def et_attention(qkv, cu_tokens, max_len, n_heads, head_dim, stream=None):
    lib = load_library()
    _dev(qkv, torch.bfloat16, "qkv")
    _dev(cu_tokens, torch.int32, "cu_tokens")
    rows = qkv.shape[0]
    out = torch.empty((rows, n_heads * head_dim), dtype=torch.bfloat16, device=qkv.device)
    _check(lib.et_attention(_ptr(qkv), _ptr(cu_tokens), cu_tokens.numel() - 1, int(max_len), n_heads,
                            head_dim, _ptr(out), _stream(stream)))
    return out


def et_attention_uniform(qkv, n_frames, length, n_heads, head_dim, stream=None):
    lib = load_library()
    _dev(qkv, torch.bfloat16, "qkv")
    out = torch.empty((qkv.shape[0], n_heads * head_dim), dtype=torch.bfloat16, device=qkv.device)
    _check(lib.et_attention_uniform(_ptr(qkv), n_frames, int(length), n_heads, head_dim, _ptr(out), _stream(stream)))
    return out


# ---------------------------------------------------------------- encoder

def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def et_encoder_create(shape, weights, max_frames):
    """shape: object with the et_config fields (e.g. et_inputs.EncoderShape) or a dict;
    weights: dict of host float32 arrays (layout of et_weights).  Returns an opaque handle."""
    lib = load_library()
    get = (lambda n: shape[n]) if isinstance(shape, dict) else (lambda n: getattr(shape, n))
    cfg = _Config()
    for n in ("n_layers", "d_model", "n_heads", "d_mlp", "patch", "image_h", "image_w", "channels",
              "has_final_ln"):
        setattr(cfg, n, int(get(n)))
    cfg.ln_eps = float(get("ln_eps"))
    keep = []                                     # keeps the host arrays alive during the call

    def fp(a):
        a = _f32(a)
        keep.append(a)
        return a.ctypes.data_as(_FP)

    w = _Weights()
    w.patch_w, w.patch_b, w.pos_emb = fp(weights["patch_w"]), fp(weights["patch_b"]), fp(weights["pos_emb"])
    nl = len(weights["layers"])
    for name in _LAYER_FIELDS:
        arr = (_FP * nl)(*[fp(lw[name]) for lw in weights["layers"]])
        keep.append(arr)
        setattr(w, name, C.cast(arr, _FPP))
    if weights.get("final_ln_g") is not None:
        w.final_ln_g, w.final_ln_b = fp(weights["final_ln_g"]), fp(weights["final_ln_b"])
    handle = C.c_void_p()
    _check(lib.et_encoder_create(C.byref(cfg), C.byref(w), int(max_frames), C.byref(handle)))
    return handle


def et_encoder_destroy(handle):
    load_library().et_encoder_destroy(handle)


def et_workspace_bytes(handle, T):
    return int(load_library().et_workspace_bytes(handle, int(T)))


def et_encode_clip(handle, frames, merge_layer, sim_threshold, keep_ratio, L, D, workspace=None,
                   outputs=None, stream=None):
    """frames: float32 CUDA tensor [T, C, H, W].  Returns a dict of output tensors."""
    lib = load_library()
    _dev(frames, torch.float32, "frames")
    T = frames.shape[0]
    if workspace is None:
        workspace = torch.empty((max(et_workspace_bytes(handle, T), 1),), dtype=torch.uint8,
                                device=frames.device)
    bufs = outputs if outputs is not None else _alloc_outputs(T, L, D, frames.device)
    o = _out_struct(bufs)
    _check(lib.et_encode_clip(handle, _ptr(frames), T, int(merge_layer), float(sim_threshold),
                              float(keep_ratio), _ptr(workspace), workspace.numel(), _stream(stream),
                              C.byref(o)))
    return _trim(bufs, o, T)


def et_encoder_block_qkv(handle, layer, x, stream=None):
    """Row scales and fused q | k | v projection of encoder block `layer` on x (bf16 CUDA [rows, D]),
    as the encode calls launch them.  Returns (qkv bf16 [rows, 3D], rstd float32 [rows])."""
    lib = load_library()
    _dev(x, torch.bfloat16, "x")
    rows, D = x.shape
    qkv = torch.empty((rows, 3 * D), dtype=torch.bfloat16, device=x.device)
    rstd = torch.empty((max(rows, 1),), dtype=torch.float32, device=x.device)
    _check(lib.et_encoder_block_qkv(handle, int(layer), _ptr(x), rows, _ptr(rstd), _ptr(qkv), _stream(stream)))
    return qkv, rstd[:rows]


def et_profile_enable(handle, on):
    _check(load_library().et_profile_enable(handle, int(bool(on))))


def et_profile_read(handle, reset=True):
    """Returns {(kind, phase): (milliseconds, launches)}; phase 0 = on all tokens, 1 = on kept tokens."""
    ms = (C.c_double * (2 * ET_K_COUNT))()
    cnt = (C.c_int64 * (2 * ET_K_COUNT))()
    _check(load_library().et_profile_read(handle, ms, cnt, int(bool(reset))))
    return {(KERNEL_KINDS[i % ET_K_COUNT], i // ET_K_COUNT): (float(ms[i]), int(cnt[i]))
            for i in range(2 * ET_K_COUNT)}


def et_merge_profile_enable(on):
    """0 = off, 1 = time the whole launch sequence, 2 = also every launch."""
    _check(load_library().et_merge_profile_enable(int(on)))


def et_merge_profile_read(reset=True):
    """Returns ({kind: (milliseconds, launches)}, total milliseconds, calls) of the stand-alone stage."""
    ms = (C.c_double * ET_K_COUNT)()
    cnt = (C.c_int64 * ET_K_COUNT)()
    tot, calls = C.c_double(0.0), C.c_int64(0)
    _check(load_library().et_merge_profile_read(ms, cnt, C.byref(tot), C.byref(calls), int(bool(reset))))
    return ({KERNEL_KINDS[i]: (float(ms[i]), int(cnt[i])) for i in range(ET_K_COUNT) if cnt[i]},
            float(tot.value), int(calls.value))


def et_kernel_name(kind):
    return load_library().et_kernel_name(int(kind)).decode()


class Projector:
    """Owns an et_projector handle (two-layer MLP: w1 [d_hidden, d_in], b1, w2 [d_out, d_hidden], b2; host float32)."""

    def __init__(self, w1, b1, w2, b2, device="cuda:0"):
        self.device = torch.device(device)
        w1, b1, w2, b2 = _f32(w1), _f32(b1), _f32(w2), _f32(b2)
        self.d_hidden, self.d_in = w1.shape
        self.d_out = w2.shape[0]
        handle = C.c_void_p()
        with torch.cuda.device(self.device):
            _check(load_library().et_projector_create(self.d_in, self.d_hidden, self.d_out, w1.ctypes.data_as(_FP),
                                                      b1.ctypes.data_as(_FP), w2.ctypes.data_as(_FP),
                                                      b2.ctypes.data_as(_FP), C.byref(handle)))
        self.handle = handle
        self._ws = None

    def project(self, tokens, out=None, stream=None):
        """tokens bf16 CUDA [rows, d_in] -> bf16 [rows, d_out] (asynchronous on the stream)."""
        lib = load_library()
        _dev(tokens, torch.bfloat16, "tokens")
        rows = tokens.shape[0]
        need = int(lib.et_projector_workspace_bytes(self.handle, rows))
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty((max(need, 1),), dtype=torch.uint8, device=self.device)
        if out is None:
            out = torch.empty((rows, self.d_out), dtype=torch.bfloat16, device=self.device)
        _check(lib.et_project_tokens(self.handle, _ptr(tokens), rows, _ptr(self._ws), self._ws.numel(), _ptr(out),
                                     _stream(stream)))
        return out

    def close(self):
        if self.handle is not None:
            load_library().et_projector_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Encoder:
    """Owns an et_encoder handle plus reusable workspace/output buffers for one clip length."""

    def __init__(self, shape, weights, max_frames, device="cuda:0"):
        self.shape = shape
        self.device = torch.device(device)
        with torch.cuda.device(self.device):
            self.handle = et_encoder_create(shape, weights, max_frames)
        self.max_frames = max_frames
        self._ws = None
        self._bufs = {}

    def encode(self, frames, merge_layer, sim_threshold, keep_ratio, stream=None):
        T = frames.shape[0]
        L, D = self.shape.tokens_per_frame, self.shape.d_model
        need = et_workspace_bytes(self.handle, T)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty((need,), dtype=torch.uint8, device=self.device)
        if T not in self._bufs:
            self._bufs[T] = _alloc_outputs(T, L, D, self.device)
        return et_encode_clip(self.handle, frames, merge_layer, sim_threshold, keep_ratio, L, D,
                              workspace=self._ws, outputs=self._bufs[T], stream=stream)

    def encode_policy(self, frames, merge_layer, policy, stream=None):
        T = frames.shape[0]
        need = et_workspace_bytes(self.handle, T)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty((need,), dtype=torch.uint8, device=self.device)
        return et_encode_clip_policy(self.handle, frames, merge_layer, policy, self.shape.tokens_per_frame,
                                     self.shape.d_model, workspace=self._ws, stream=stream)

    def encode_multi(self, frames, merge_layers, select_layer, policy, stream=None):
        T = frames.shape[0]
        need = et_workspace_bytes(self.handle, T)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty((need,), dtype=torch.uint8, device=self.device)
        return et_encode_clip_multi(self.handle, frames, merge_layers, select_layer, policy,
                                    self.shape.tokens_per_frame, self.shape.d_model, workspace=self._ws,
                                    stream=stream)

    def close(self):
        if self.handle is not None:
            et_encoder_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
