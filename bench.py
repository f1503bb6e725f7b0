#!/usr/bin/env python3
"""Benchmark of the EarlyTom hot path on one MI355X.

A step = one pass of the whole path (patch embedding, 27 encoder blocks, the in-encoder
compression stage after `merge_layer` blocks, final LayerNorm) over one synthetic 32-frame
384x384 clip that is already resident in device memory.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3_siglip_t32 | c5_merge_only]
                  [--merge-layer M] [--keep-ratio R] [--no-cpu-baseline] [--no-sweep] [--no-merge-microbench]

Beside the headline (frames/s of the 32-frame clip, merge layer 8, keep 0.5) the line carries:
  kernels       per-kernel averages from HIP events around every launch (a second pass of the same steps)
  roofline      the kernel kind with the largest share of device time against the bf16 MFMA peak
  sweep         the other settings of the 32-frame workload (merge layer 4 / 8 / 13, keep 0.25 / 0.5), the
                8-frame and the 64-frame clip (same encoder weights: only shapes matter for timing)
  merge_stage_c5  the compression stage alone on a [64, 729, 1152] tensor that starts cold in HBM
  paper_policy  the paper's own layout (Stage I at layers 6 / 14 / 20, Stage II after the encoder)
  power         board power, shader clock and junction temperature while the headline step runs back to back
  cpu_baseline  the oracle on the same clip on the host cores
With --workload c5_merge_only the compression stage alone is the step and its GB/s the value.
"""
import argparse
import glob
import json
import os
import sys
import threading
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


def clip_flops(shape, T, N, k, m):
    fl = flops_tables(shape, T, N, k, m)
    total = fl[("gemm_patch", 0)]
    for kind in ("gemm_qkv", "gemm_out", "gemm_fc1", "gemm_fc2", "attention"):
        total += (max(m, 0) if m >= 0 else shape.n_layers) * fl[(kind, 0)]
        if m >= 0:
            total += (shape.n_layers - m) * fl[(kind, 1)]
    return total


def stage_bytes(T, L, D, N, k):
    """Algorithmic HBM bytes of the compression stage: X is read twice (every position's similarity must be
    known before any frame can be merged), the merged frames are written, the kept rows are read and written,
    plus the per-position cosines and scores."""
    return 2 * T * L * D * 2 + N * L * D * 2 + 2 * N * k * D * 2 + 2 * T * L * 4


def bytes_tables(shape, T, N, k):
    """Algorithmic HBM bytes per launch of the bandwidth-bound kernels."""
    D, L = shape.d_model, shape.tokens_per_frame
    X = T * L * D * 2
    return {
        ("similarity", 0): X + (T - 1) * L * 4,
        ("scan", 0): (T - 1) * ((L + 3) // 4) * 4 + (T - 1) * 4 + (T + 1) * 4,
        ("merge", 0): X + N * L * D * 2 + N * L * 4,
        ("select", 0): N * L * 4 + N * k * 4 + 2 * N * k * D * 2,      # selection and gather are one launch
        # row statistics of the LayerNorms folded into the QKV / fc1 GEMMs: the rows are read, one float per row
        # is written (phase 1 also holds the one real LayerNorm, the final one: slightly under-counted)
        ("layernorm", 0): T * L * D * 2 + T * L * 4,
        ("layernorm", 1): N * k * D * 2 + N * k * 4,
        ("im2col", 0): T * shape.channels * shape.image_h * shape.image_w * 4
                       + T * L * ((shape.patch_dim + 63) // 64 * 64) * 2,
    }


def measured_traffic(kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary (not from this run), or
    None when no summary names that kernel."""
    path = os.path.join(ROOT, "profiles", "gemm_fc1_c3_siglip_t32_hbm_traffic.md")
    if not os.path.exists(path):
        return None, None
    keys = {}
    for line in open(path):
        if "=" in line and not line.startswith(("#", " ", "|")):
            a, b = line.split("=", 1)
            keys[a.strip()] = b.strip()
    if keys.get("kernel") != kernel or "traffic_bytes_per_launch" not in keys:
        return None, None
    return float(keys["traffic_bytes_per_launch"]), "profiles/gemm_fc1_c3_siglip_t32_hbm_traffic.md"


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
    what = "the whole clip" if sample_frames == rec["T"] else "the first %d frames of the same clip" % sample_frames
    return {"value": round(sample_frames / dt, 4), "unit": "frames/s", "cores": int(threads), "kind": "oracle",
            "sample": "%s (%d frames, float64 numpy oracle, %d segment(s), %.1f s)"
                      % (what, sample_frames, out["n_frames_out"], dt)}


def cpu_baseline_stage(x_bits, tau, keep):
    import numpy as np
    from oracle import earlytom_oracle as O
    from et_inputs import bf16_bits_to_f32
    try:
        import threadpoolctl
        threads = max(i["num_threads"] for i in threadpoolctl.threadpool_info() if i.get("num_threads"))
    except Exception:
        threads = os.cpu_count()
    x = bf16_bits_to_f32(x_bits).astype(np.float64)
    t0 = time.perf_counter()
    st = O.merge_select(x, tau, np.float32(keep))
    dt = time.perf_counter() - t0
    T, L, D = x.shape
    N, k = st["kept_idx"].shape
    return {"value": round(stage_bytes(T, L, D, N, k) / dt / 1e9, 3), "unit": "GB/s", "cores": int(threads),
            "kind": "oracle", "sample": "the whole [%d, %d, %d] tensor, float64 numpy oracle, %.1f s" % (T, L, D, dt)}


class PowerSampler(threading.Thread):
    """Board power, shader clock and junction temperature read from the amdgpu driver's sysfs files every 20 ms
    (power1_input in microwatts, the starred line of pp_dpm_sclk, temp2_input in millidegrees)."""

    def __init__(self, period=0.02):
        super().__init__(daemon=True)
        self.period, self.stop_flag, self.rows = period, False, []
        self.dev = self.hwmon = None
        for d in sorted(glob.glob("/sys/class/drm/card*/device")):
            h = glob.glob(os.path.join(d, "hwmon/hwmon*/power1_input"))
            if h:
                self.dev, self.hwmon = d, os.path.dirname(h[0])
                break

    @staticmethod
    def _read(path):
        try:
            with open(path) as f:
                return f.read()
        except OSError:
            return ""

    def available(self):
        return self.hwmon is not None and self._read(os.path.join(self.hwmon, "power1_input")).strip() != ""

    def cap_w(self):
        v = self._read(os.path.join(self.hwmon, "power1_cap")).strip()
        return float(v) / 1e6 if v else None

    def sample(self):
        p = self._read(os.path.join(self.hwmon, "power1_input")).strip()
        t = self._read(os.path.join(self.hwmon, "temp2_input")).strip()
        clk = None
        for ln in self._read(os.path.join(self.dev, "pp_dpm_sclk")).splitlines():
            if "*" in ln:
                clk = float(ln.split(":")[1].lower().replace("mhz", "").replace("*", "").strip())
        return (time.perf_counter(), float(p) / 1e6 if p else None, clk, float(t) / 1e3 if t else None)

    def run(self):
        while not self.stop_flag:
            self.rows.append(self.sample())
            time.sleep(self.period)


def power_under_load(fn, torch, seconds, settle=0.7):
    """Runs fn back to back for `seconds` and returns the mean board power / shader clock over the samples taken
    after the first `settle` seconds (the driver's power reading is itself an average over a short window)."""
    s = PowerSampler()
    if not s.available():
        return None
    fn()
    torch.cuda.synchronize()
    s.start()
    t0 = time.perf_counter()
    n = 0
    while time.perf_counter() - t0 < seconds:
        for _ in range(10):
            fn()
        n += 10
        torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    s.stop_flag = True
    s.join()
    rows = [r for r in s.rows if r[0] - t0 >= settle and r[1] is not None]
    if not rows:
        return None
    mean = lambda v: sum(v) / len(v)
    clk = [r[2] for r in rows if r[2] is not None]
    tj = [r[3] for r in rows if r[3] is not None]
    return {"avg_w": round(mean([r[1] for r in rows]), 1), "max_w": round(max(r[1] for r in rows), 1),
            "sclk_mhz": round(mean(clk), 0) if clk else None, "junction_c": round(mean(tj), 1) if tj else None,
            "samples": len(rows), "us_per_call": round(1e6 * dt / n, 1)}


def time_steps(fn, steps, warmup, torch):
    for _ in range(warmup):
        out = fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        out = fn()
    torch.cuda.synchronize()
    return time.perf_counter() - t0, out


def merge_microbench(et, torch, steps, warmup, variant=0):
    """The compression stage alone (et_merge_select) on the [64, 729, 1152] bf16 tensor of the merge-only
    workload.  Before every timed call a 1 GiB buffer is READ (a reduction: the caches are left full of clean
    lines of another buffer, with nothing to write back), so the tensor starts out of the 256 MiB last-level
    cache: the stage's first pass comes from HBM, as it would behind a real encoder whose activations do not fit.  Times come from HIP events that the library records on the launch stream around
    every launch and around the whole sequence (et_merge_profile_*)."""
    import numpy as np
    from et_inputs import build_workload, bf16_bits_to_f32
    from oracle import earlytom_oracle as O
    from paper_2605_30010_amd import binding as B
    rec = build_workload("c5_merge_only", variant=variant)
    bits, tau, keep = rec["x_bits"], rec["sim_threshold"], rec["keep_ratio"]
    T, L, D = bits.shape
    x = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()
    ws = torch.empty((et.et_merge_workspace_bytes(T, L, D),), dtype=torch.uint8, device="cuda")
    bufs = B._alloc_outputs(T, L, D, x.device)
    flush = torch.ones((256 << 20,), dtype=torch.float32, device="cuda")     # 1 GiB
    stream = torch.cuda.current_stream()
    run = lambda: et.et_merge_select(x, tau, keep, workspace=ws, outputs=bufs, stream=stream)
    for _ in range(warmup):
        out = run()
    N, k = out["n_frames_out"], out["n_tokens"] // out["n_frames_out"]
    # decisions against the oracle on the same bits (margins as in the tests)
    st = O.merge_select(bf16_bits_to_f32(bits).astype(np.float64), tau, np.float32(keep))
    assert np.min(np.abs(st["frame_sim"] - tau)) >= 1e-2, "similarity margin"
    assert out["seg_start"].tolist() == st["seg_start"].tolist()
    assert np.array_equal(out["kept_idx"].cpu().numpy(), st["kept_idx"].reshape(-1))
    b_alg = stage_bytes(T, L, D, N, k)
    alg = {"similarity": T * L * D * 2 + (T - 1) * L * 4, "scan": (T - 1) * ((L + 3) // 4) * 4 + 2 * T * 4,
           "merge": T * L * D * 2 + N * L * D * 2 + N * L * 4,
           "select": N * L * 4 + N * k * 4 + 2 * N * k * D * 2}          # selection and gather are one launch

    def timed(cold, level):
        et.et_merge_profile_enable(level)
        et.et_merge_profile_read(reset=True)
        for _ in range(steps):
            if cold:
                flush.sum()
            run()
        per, total_ms, calls = et.et_merge_profile_read(reset=True)
        et.et_merge_profile_enable(0)
        us = 1e3 * total_ms / calls
        kernels = {}
        for kind, (ms, cnt) in per.items():
            kus = 1e3 * ms / cnt
            kernels[kind] = {"avg_us": round(kus, 2), "gbs": round(alg[kind] / kus / 1e3, 1),
                             "hbm_frac": round(alg[kind] / kus / 1e3 / PEAK_HBM_GBS, 4)}
        return us, kernels
    us_cold, _ = timed(True, 1)              # the sequence as it runs, two events around it
    _, k_cold = timed(True, 2)               # again with events around every launch
    us_warm, _ = timed(False, 1)
    _, k_warm = timed(False, 2)
    res = {"workload": "c5_merge_only", "shape": [T, L, D], "n_frames_out": N, "k": k, "steps": steps,
           "algorithmic_bytes": b_alg, "avg_us": round(us_cold, 2), "gbs": round(b_alg / us_cold / 1e3, 1),
           "hbm_frac": round(b_alg / us_cold / 1e3 / PEAK_HBM_GBS, 4),
           "kernels": k_cold,
           "cache_resident": {"avg_us": round(us_warm, 2), "gbs": round(b_alg / us_warm / 1e3, 1),
                              "kernels": {n_: e["avg_us"] for n_, e in k_warm.items()}},
           "timed": "first launch's start to last launch's end on the launch stream (4 launches, gaps included)",
           "decisions_match_oracle": True}
    return res, rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3_siglip_t32")
    ap.add_argument("--merge-layer", type=int, default=None)
    ap.add_argument("--keep-ratio", type=float, default=None)
    ap.add_argument("--variant", type=int, default=0)
    ap.add_argument("--cpu-frames", type=int, default=None, help="frames the oracle is timed on (default: all)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile-pass", action="store_true")
    ap.add_argument("--no-paper-policy", action="store_true",
                    help="skip the extra timing of the paper's own configuration (reported beside the headline)")
    ap.add_argument("--no-sweep", action="store_true", help="skip the other merge layers / keep ratios / clip lengths")
    ap.add_argument("--no-merge-microbench", action="store_true", help="skip the compression stage on its own")
    ap.add_argument("--no-power", action="store_true", help="skip the board power / clock reading under load")
    ap.add_argument("--power-kernels", action="store_true",
                    help="also read power / clock under the MLP GEMM pair and under attention run alone")
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

    idle_sampler = PowerSampler()
    idle_w = idle_sampler.sample()[1] if idle_sampler.available() else None      # before anything runs on the device
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")

    if args.copy_calibration:
        src = torch.empty(256 * 1024 * 1024, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.workload == "c5_merge_only":
        res, rec = merge_microbench(et, torch, args.steps, args.warmup, args.variant)
        line = {"metric": "HBM GB/s of the merge / select / repack stage alone, [64, 729, 1152] bf16",
                "value": res["gbs"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                "ms_per_step": round(res["avg_us"] / 1e3, 5), "higher_is_better": True, "scaling": "weak",
                "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                "config": {"workload": "c5_merge_only", "frames": rec["T"], "sim_threshold": rec["sim_threshold"],
                           "keep_ratio": rec["keep_ratio"], "scene_lengths": rec["lengths"]},
                "roofline": {"kernel": "merge_stage", "bound": "hbm", "achieved": res["gbs"], "peak": PEAK_HBM_GBS,
                             "unit": "GB/s", "frac": res["hbm_frac"], "traffic": None},
                "merge_stage_c5": res}
        if not args.no_cpu_baseline:
            line["cpu_baseline"] = cpu_baseline_stage(rec["x_bits"], rec["sim_threshold"], rec["keep_ratio"])
        print(json.dumps(line))
        return

    rec = build_workload(args.workload, variant=args.variant)
    if args.merge_layer is not None:
        rec["merge_layer"] = args.merge_layer
    if args.keep_ratio is not None:
        rec["keep_ratio"] = args.keep_ratio
    shape, T = rec["shape"], rec["T"]
    m, tau, keep = rec["merge_layer"], rec["sim_threshold"], rec["keep_ratio"]
    do_sweep = not args.no_sweep and args.workload == "c3_siglip_t32"

    enc = et.Encoder(shape, rec["weights"], max(T, 64) if do_sweep else T, device=dev)
    frames = torch.from_numpy(rec["frames"]).to(dev)
    stream = torch.cuda.current_stream()

    total, out = time_steps(lambda: enc.encode(frames, m, tau, keep, stream=stream), args.steps, args.warmup, torch)
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
        traffic, source = measured_traffic(dom[0]) if args.workload == "c3_siglip_t32" else (None, None)
        roofline = {"kernel": dom[0], "bound": "mfma", "achieved": dom[1]["tflops"], "peak": PEAK_BF16_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(dom[1]["tflops"] / PEAK_BF16_TFLOPS, 4),
                    "traffic": traffic, "traffic_source": source, "avg_us": dom[1]["avg_us"],
                    "algorithmic_bytes": 2 * (T * shape.tokens_per_frame * shape.d_model + shape.d_model * shape.d_mlp
                                              + T * shape.tokens_per_frame * shape.d_mlp)
                    if dom[0].startswith("gemm_fc") else None}
        kept_share = sum(e["share"] for n_, e in kernels.items() if n_.endswith("@kept"))
        kernels["share_kept_blocks"] = round(kept_share, 4)
        # the compression stage inside the clip, as one bandwidth figure (its tensor is cache-resident here:
        # block m - 1 has just written it; the cold figure is merge_stage_c5)
        stage_ms = sum(prof[(kk, 0)][0] for kk in ("similarity", "scan", "merge", "select"))
        stage_cnt = max(prof[("similarity", 0)][1], 1)
        D, L = shape.d_model, shape.tokens_per_frame
        sb = stage_bytes(T, L, D, N, k)
        kernels["merge_stage"] = {"avg_us": round(1e3 * stage_ms / stage_cnt, 2),
                                  "gbs": round(sb / (stage_ms / stage_cnt * 1e-3) / 1e9, 1)}
        kernels["merge_stage"]["hbm_frac"] = round(kernels["merge_stage"]["gbs"] / PEAK_HBM_GBS, 4)

    # Board power and shader clock while the headline step runs back to back (sysfs; the published peaks assume
    # 2.4 GHz, the clock the chip actually holds under this load is what the roofline fractions run against).
    power = None
    if not args.no_power:
        ps = PowerSampler()
        if ps.available():
            power = {"cap_w": ps.cap_w(), "idle_w": idle_w, "peak_clock_mhz": 2400,
                     "whole_clip": power_under_load(lambda: enc.encode(frames, m, tau, keep, stream=stream), torch, 2.5)}
            if args.power_kernels:
                rngw = np.random.default_rng(11)
                mlp = et.Projector(rngw.standard_normal((shape.d_mlp, shape.d_model), dtype=np.float32) * 0.02,
                                   np.zeros(shape.d_mlp, np.float32),
                                   rngw.standard_normal((shape.d_model, shape.d_mlp), dtype=np.float32) * 0.02,
                                   np.zeros(shape.d_model, np.float32))
                rows_all = T * shape.tokens_per_frame
                for name, rows in (("mlp_gemm_pair@all", rows_all), ("mlp_gemm_pair@kept", max(n_tokens, 1))):
                    xin = torch.randn((rows, shape.d_model), device=dev).to(torch.bfloat16)
                    xout = torch.empty_like(xin)
                    e = power_under_load(lambda: mlp.project(xin, out=xout, stream=stream), torch, 2.0)
                    if e:
                        e["tflops"] = round(4.0 * rows * shape.d_mlp * shape.d_model / e["us_per_call"] / 1e6, 1)
                    power[name] = e
                mlp.close()
                L_ = shape.tokens_per_frame
                qkv = torch.randn((rows_all, 3 * shape.d_model), device=dev).to(torch.bfloat16)
                hd = shape.d_model // shape.n_heads
                e = power_under_load(lambda: et.et_attention_uniform(qkv, T, L_, shape.n_heads, hd, stream=stream), torch, 2.0)
                if e:
                    e["tflops"] = round(4.0 * T * shape.n_heads * L_ * L_ * hd / e["us_per_call"] / 1e6, 1)
                power["attention@all"] = e
                del qkv

    # Extra, not the headline: the paper's own layout (Table 8 / Alg. 1-2) on the same clip - Stage I after
    # blocks 6, 14, 20 with EMA segmentation and the weighted middle-pair merge, Stage II once on the encoder
    # output (decoupled top-k / local windows, overall retention 20 %, attention-received scores).
    paper = None
    if not args.no_paper_policy and shape.n_layers >= 21:
        pol = dict(merge_mode="alg1", select_mode="decoupled", alpha=0.9, tau_seg=0.8, tau_merge=0.8, ratio=0.2,
                   score_mode="attention")
        layers, sel = [6, 14, 20], shape.n_layers
        pt, po = time_steps(lambda: enc.encode_multi(frames, layers, sel, pol, stream=stream), args.steps,
                            max(args.warmup, 1), torch)
        paper = {"merge_layers": layers, "select_layer": sel, "policy": pol, "ms_per_step": round(1e3 * pt / args.steps, 3),
                 "frames_per_s": round(T * args.steps / pt, 2), "n_frames_out": po["n_frames_out"],
                 "n_tokens_out": po["n_tokens"], "retention": round(po["n_tokens"] / (T * shape.tokens_per_frame), 4)}
        # "encoder + visual token processing" (Sec. 3.1: encoder -> projector -> language model): the same call
        # followed by a two-layer projector of a 7B language model's width (1152 -> 3584 -> 3584, random weights)
        rngp = np.random.default_rng(7)
        d_llm = 3584
        proj = et.Projector(rngp.standard_normal((d_llm, shape.d_model), dtype=np.float32) * 0.02, np.zeros(d_llm, np.float32),
                            rngp.standard_normal((d_llm, d_llm), dtype=np.float32) * 0.02, np.zeros(d_llm, np.float32))
        pbuf = torch.empty((T * shape.tokens_per_frame, d_llm), dtype=torch.bfloat16, device=dev)

        def enc_and_project():
            o = enc.encode_multi(frames, layers, sel, pol, stream=stream)
            proj.project(o["tokens"], out=pbuf[:o["n_tokens"]], stream=stream)
            return o
        ppt, o_last = time_steps(enc_and_project, args.steps, max(args.warmup, 1), torch)
        tok = o_last["tokens"].clone()
        pj, _ = time_steps(lambda: proj.project(tok, out=pbuf[:tok.shape[0]], stream=stream), args.steps, 2, torch)
        paper["encoder_plus_projector"] = {"projector": [shape.d_model, d_llm, d_llm],
                                           "ms_per_step": round(1e3 * ppt / args.steps, 3),
                                           "projector_alone_ms": round(1e3 * pj / args.steps, 3)}
        proj.close()
        del pbuf
        # the in-encoder decoupled policy (ragged frames after the selection) at the headline's merge layer
        pol2 = dict(pol, score_mode="l2")
        pt2, po2 = time_steps(lambda: enc.encode_policy(frames, m, pol2, stream=stream), args.steps,
                              max(args.warmup, 1), torch)
        paper["in_encoder_decoupled"] = {"merge_layer": m, "ms_per_step": round(1e3 * pt2 / args.steps, 3),
                                         "frames_per_s": round(T * args.steps / pt2, 2),
                                         "n_frames_out": po2["n_frames_out"], "n_tokens_out": po2["n_tokens"]}

    # The other points of the 32-frame workload and the other clip lengths (same weights: random-init weights
    # of one shape are interchangeable for timing), each a short timed run.
    sweep = None
    if do_sweep:
        sweep = []
        sw_steps = max(args.steps // 2, 5)

        def point(name, fr, T_, m_, tau_, keep_):
            tt, o = time_steps(lambda: enc.encode(fr, m_, tau_, keep_, stream=stream), sw_steps, 2, torch)
            N_, k_ = o["n_frames_out"], o["n_tokens"] // max(o["n_frames_out"], 1)
            fl_ = clip_flops(shape, T_, N_, k_, m_)
            sweep.append({"workload": name, "frames": T_, "merge_layer": m_, "keep_ratio": keep_,
                          "ms_per_step": round(1e3 * tt / sw_steps, 3), "frames_per_s": round(T_ * sw_steps / tt, 1),
                          "n_frames_out": N_, "n_tokens_out": o["n_tokens"],
                          "algorithmic_tflop": round(fl_ / 1e12, 3),
                          "effective_tflops": round(fl_ / (tt / sw_steps) / 1e12, 1),
                          "mfma_frac": round(fl_ / (tt / sw_steps) / 1e12 / PEAK_BF16_TFLOPS, 4)})
        for m_ in (4, 8, 13):
            for keep_ in (0.25, 0.5):
                point("c3_siglip_t32", frames, T, m_, tau, keep_)
        point("c3_siglip_t32 (no compression)", frames, T, -1, tau, 1.0)
        for name in ("c2_siglip_t8", "c4_siglip_t64"):
            r2 = build_workload(name, with_weights=False)
            fr2 = torch.from_numpy(r2["frames"]).to(dev)
            point(name, fr2, r2["T"], r2["merge_layer"], r2["sim_threshold"], r2["keep_ratio"])
            del fr2

    total_flops = clip_flops(shape, T, N, k, m)
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
        "power": power,
        "paper_policy": paper,
        "sweep": sweep,
    }
    enc.close()
    del enc, frames
    torch.cuda.empty_cache()
    if not args.no_merge_microbench:
        res["merge_stage_c5"], _ = merge_microbench(et, torch, args.steps, args.warmup)
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(rec, T if args.cpu_frames is None else min(args.cpu_frames, T))
    print(json.dumps(res))


if __name__ == "__main__":
    main()
