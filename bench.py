#!/usr/bin/env python3
"""Benchmark of the EarlyTom hot path on one MI355X.

A step = one pass of the whole path (patch embedding, 27 encoder blocks, the in-encoder
compression stage after `merge_layer` blocks, final LayerNorm) over one synthetic 32-frame
384x384 clip that is already resident in device memory.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3_siglip_t32]
                  [--merge-layer M] [--keep-ratio R] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published


def flops_tables(shape, T, N, k, merge_layer):
    """Algorithmic FLOPs (2 m n k convention, unpadded sizes) per launch of each kernel kind,
    for launches on all T*L tokens (phase 0) and on the N*k kept tokens (phase 1)."""
    D, Mh, H, hd, L = shape.d_model, shape.d_mlp, shape.n_heads, shape.head_dim, shape.tokens_per_frame
    out = {}
    for phase, (frames, n) in enumerate(((T, L), (N, k))):
        R = frames * n
        out[("gemm_qkv", phase)] = 2.0 * R * D * 3 * D
        out[("gemm_out", phase)] = 2.0 * R * D * D
        out[("gemm_fc1", phase)] = 2.0 * R * D * Mh
        out[("gemm_fc2", phase)] = 2.0 * R * D * Mh
        out[("attention", phase)] = 4.0 * frames * H * n * n * hd
    out[("gemm_patch", 0)] = 2.0 * T * L * shape.patch_dim * D
    return out


def bytes_tables(shape, T, N, k):
    """Algorithmic HBM bytes per launch of the bandwidth-bound kernels."""
    D, L = shape.d_model, shape.tokens_per_frame
    X = T * L * D * 2
    return {
        ("similarity", 0): X + (T - 1) * L * 4,
        ("scan", 0): (T - 1) * L * 4 + (T - 1) * 4 + (T + 1) * 4,
        ("merge", 0): X + N * L * D * 2 + N * L * 4,
        ("select", 0): N * L * 4 + N * k * 4,
        ("compact", 0): 2 * N * k * D * 2 + N * k * 4,
        # row statistics of the LayerNorms folded into the QKV / fc1 GEMMs: the rows are read, one float per row
        # is written (phase 1 also holds the one real LayerNorm, the final one: slightly under-counted)
        ("layernorm", 0): T * L * D * 2 + T * L * 4,
        ("layernorm", 1): N * k * D * 2 + N * k * 4,
        ("im2col", 0): T * shape.channels * shape.image_h * shape.image_w * 4
                       + T * L * ((shape.patch_dim + 63) // 64 * 64) * 2,
    }


def measured_traffic(kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary, or None."""
    path = os.path.join(ROOT, "profiles", "gemm_fc1_c3_siglip_t32_hbm_traffic.md")
    if kernel != "gemm_fc1@all" or not os.path.exists(path):
        return None
    for line in open(path):
        if line.strip().startswith("traffic_bytes_per_launch"):
            return float(line.split("=")[1])
    return None


def cpu_baseline(rec, sample_frames):
    """The oracle, as it is, on the first `sample_frames` frames of the same clip."""
    import numpy as np
    from oracle import earlytom_oracle as O
    try:
        import threadpoolctl
        threads = max(i["num_threads"] for i in threadpoolctl.threadpool_info() if i.get("num_threads"))
    except Exception:
        threads = os.cpu_count()
    frames = rec["frames"][:sample_frames]
    t0 = time.perf_counter()
    out = O.encode_clip(rec["shape"], rec["weights"], frames, rec["merge_layer"], rec["sim_threshold"],
                        np.float32(rec["keep_ratio"]))
    dt = time.perf_counter() - t0
    return {"value": sample_frames / dt, "unit": "frames/s", "cores": int(threads), "kind": "oracle",
            "sample": "first %d frames of the same clip (float64 numpy oracle, %d segment(s), %.1f s)"
                      % (sample_frames, out["n_frames_out"], dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3_siglip_t32")
    ap.add_argument("--merge-layer", type=int, default=None)
    ap.add_argument("--keep-ratio", type=float, default=None)
    ap.add_argument("--variant", type=int, default=0)
    ap.add_argument("--cpu-frames", type=int, default=8)
    ap.add_argument("--groups", type=int, default=1,
                    help="frame groups run on streams of their own (et_encoder_set_frame_groups)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile-pass", action="store_true")
    ap.add_argument("--no-paper-policy", action="store_true",
                    help="skip the extra timing of the paper's own configuration (reported beside the headline)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy first (reference for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import numpy as np
    import torch
    import paper_2605_30010_amd as et
    from et_inputs import build_workload

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    rec = build_workload(args.workload, variant=args.variant)
    if args.merge_layer is not None:
        rec["merge_layer"] = args.merge_layer
    if args.keep_ratio is not None:
        rec["keep_ratio"] = args.keep_ratio
    shape, T = rec["shape"], rec["T"]
    m, tau, keep = rec["merge_layer"], rec["sim_threshold"], rec["keep_ratio"]

    enc = et.Encoder(shape, rec["weights"], T, device=dev)
    enc.set_frame_groups(args.groups)
    frames = torch.from_numpy(rec["frames"]).to(dev)
    stream = torch.cuda.current_stream()

    if args.copy_calibration:
        src = torch.empty(256 * 1024 * 1024, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        out = enc.encode(frames, m, tau, keep, stream=stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        out = enc.encode(frames, m, tau, keep, stream=stream)
    torch.cuda.synchronize()
    total = time.perf_counter() - t0
    ms_per_step = 1e3 * total / args.steps
    N, n_tokens = out["n_frames_out"], out["n_tokens"]
    k = n_tokens // max(N, 1)

    # per-kernel pass: same steps with HIP events around every launch on the same stream
    kernels, roofline = {}, None
    if not args.no_profile_pass:
        et.et_profile_enable(enc.handle, True)
        et.et_profile_read(enc.handle, reset=True)
        for _ in range(args.steps):
            enc.encode(frames, m, tau, keep, stream=stream)
        prof = et.et_profile_read(enc.handle, reset=True)
        et.et_profile_enable(enc.handle, False)
        fl = flops_tables(shape, T, N, k, m)
        by = bytes_tables(shape, T, N, k)
        tot_ms = sum(v[0] for v in prof.values())
        for (kind, phase), (ms, cnt) in sorted(prof.items()):
            if cnt == 0:
                continue
            avg_us = 1e3 * ms / cnt
            e = {"launches_per_step": cnt / args.steps, "avg_us": round(avg_us, 2),
                 "share": round(ms / tot_ms, 4)}
            if (kind, phase) in fl:
                e["tflops"] = round(fl[(kind, phase)] / (avg_us * 1e-6) / 1e12, 1)
                e["mfma_util"] = round(e["tflops"] / PEAK_BF16_TFLOPS, 4)
            if (kind, phase) in by:
                e["gbs"] = round(by[(kind, phase)] / (avg_us * 1e-6) / 1e9, 1)
                e["hbm_frac"] = round(e["gbs"] / PEAK_HBM_GBS, 4)
            kernels["%s@%s" % (kind, "all" if phase == 0 else "kept")] = e
        # dominant kernel = largest share of device time
        dom = max((x for x in kernels.items() if "tflops" in x[1]), key=lambda x: x[1]["share"])
        roofline = {"kernel": dom[0], "bound": "mfma", "achieved": dom[1]["tflops"], "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(dom[1]["tflops"] / PEAK_BF16_TFLOPS, 4),
                    "traffic": measured_traffic(dom[0]) if args.workload == "c3_siglip_t32" else None,
                    "avg_us": dom[1]["avg_us"]}
        # the compression stage as one bandwidth figure: 2 reads of X + merged write + gather
        stage_ms = sum(prof[(kk, 0)][0] for kk in ("similarity", "scan", "merge", "select", "compact"))
        stage_cnt = max(prof[("similarity", 0)][1], 1)
        D, L = shape.d_model, shape.tokens_per_frame
        stage_bytes = 2 * T * L * D * 2 + N * L * D * 2 + 2 * N * k * D * 2 + 2 * T * L * 4
        kernels["merge_stage"] = {"avg_us": round(1e3 * stage_ms / stage_cnt, 2),
                                  "gbs": round(stage_bytes / (stage_ms / stage_cnt * 1e-3) / 1e9, 1)}
        kernels["merge_stage"]["hbm_frac"] = round(kernels["merge_stage"]["gbs"] / PEAK_HBM_GBS, 4)

    # Extra, not the headline: the paper's own layout (Table 8 / Alg. 1-2) on the same clip - Stage I after
    # blocks 6, 14, 20 with EMA segmentation and the weighted middle-pair merge, Stage II once on the encoder
    # output (decoupled top-k / local windows, overall retention 20 %, attention-received scores).
    paper = None
    if not args.no_paper_policy and shape.n_layers >= 21:
        pol = dict(merge_mode="alg1", select_mode="decoupled", alpha=0.9, tau_seg=0.8, tau_merge=0.8, ratio=0.2,
                   score_mode="attention")
        layers, sel = [6, 14, 20], shape.n_layers
        for _ in range(max(args.warmup, 1)):
            po = enc.encode_multi(frames, layers, sel, pol, stream=stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            po = enc.encode_multi(frames, layers, sel, pol, stream=stream)
        torch.cuda.synchronize()
        pt = time.perf_counter() - t1
        paper = {"merge_layers": layers, "select_layer": sel, "policy": pol, "ms_per_step": round(1e3 * pt / args.steps, 3),
                 "frames_per_s": round(T * args.steps / pt, 2), "n_frames_out": po["n_frames_out"],
                 "n_tokens_out": po["n_tokens"], "retention": round(po["n_tokens"] / (T * shape.tokens_per_frame), 4)}

    fl = flops_tables(shape, T, N, k, m)
    total_flops = fl[("gemm_patch", 0)]
    for kind in ("gemm_qkv", "gemm_out", "gemm_fc1", "gemm_fc2", "attention"):
        total_flops += max(m, 0) * fl[(kind, 0)] if m >= 0 else shape.n_layers * fl[(kind, 0)]
        if m >= 0:
            total_flops += (shape.n_layers - m) * fl[(kind, 1)]

    res = {
        "metric": "frames/s, SigLIP-shaped encoder + in-encoder merge/select, 32-frame 384x384 clip",
        "value": round(T * args.steps / total, 2), "unit": "frames/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": args.workload, "frames": T, "tokens_in": T * shape.tokens_per_frame,
                   "merge_layer": m, "sim_threshold": tau, "keep_ratio": keep,
                   "n_frames_out": N, "n_tokens_out": n_tokens, "scene_lengths": rec["lengths"]},
        "algorithmic_tflop_per_clip": round(total_flops / 1e12, 3),
        "effective_tflops": round(total_flops / (ms_per_step * 1e-3) / 1e12, 1),
        "roofline": roofline,
        "kernels": kernels,
        "paper_policy": paper,
    }
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(rec, min(args.cpu_frames, T))
    enc.close()
    print(json.dumps(res))


if __name__ == "__main__":
    main()
