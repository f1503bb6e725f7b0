// C boundary of libearlytom: argument validation, error reporting, the single-step entry
// points and the compression stage (et_merge_select).  The encoder itself lives in
// encoder.hip.
#include <math.h>
#include <string.h>

#include <mutex>

#include "et_common.h"

// Scratch of et_merge_select_static: one copy per GPU that loads the library, held until the process
// ends.  In host code this name is only a handle for hipGetSymbolAddress (see static_scratch below);
// it is never passed to a kernel or a copy.
static __device__ __align__(256) unsigned char scratch[ET_STATIC_SCRATCH_BYTES];

namespace et {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

int hip_fail(hipError_t e, const char *what, const char *file, int line) {
  const char *base = strrchr(file, '/');
  set_error("HIP error %d (%s) at %s:%d in %s", (int)e, hipGetErrorString(e), base ? base + 1 : file,
            line, what);
  return ET_ERR_HIP;
}

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Device address of `scratch` on the current device, looked up once per device.
static int static_scratch(void **out) {
  constexpr int kMaxDevices = 64;
  static void *ptrs[kMaxDevices] = {};
  static std::mutex mu;
  int dev = 0;
  ET_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) {
    set_error("device index %d outside [0, %d)", dev, kMaxDevices);
    return ET_ERR_UNSUPPORTED;
  }
  std::lock_guard<std::mutex> lock(mu);
  if (!ptrs[dev]) {
    void *p = nullptr;
    ET_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) {
      set_error("hipGetSymbolAddress returned a null address for the static scratch buffer");
      return ET_ERR_HIP;
    }
    ptrs[dev] = p;
  }
  *out = ptrs[dev];
  return ET_OK;
}

// Carves a workspace into 256-byte aligned pieces.
struct Carver {
  char *base;
  size_t off = 0;
  explicit Carver(void *p) : base(static_cast<char *>(p)) {}
  template <typename T>
  T *take(size_t n) {
    T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
    off += align_up(n * sizeof(T), 256);
    return p;
  }
};

MergeWs carve_merge(void *ws, int T, int L, int D) {
  Carver c(ws);
  MergeWs m;
  m.cos = c.take<float>((size_t)(T > 1 ? T - 1 : 1) * L);
  m.sim = c.take<float>((size_t)T);
  m.part = c.take<float>((size_t)(T > 1 ? T - 1 : 1) * similarity_blocks(L));
  m.score = c.take<float>((size_t)T * L);
  m.n_seg = c.take<int32_t>(64);
  m.frame_first = c.take<int32_t>((size_t)T);
  m.frame_count = c.take<int32_t>((size_t)T);
  m.frame_dyn = c.take<int32_t>((size_t)T);
  m.frame_w = c.take<float>((size_t)2 * T);
  m.orig_first = c.take<int32_t>((size_t)T);
  m.orig_count = c.take<int32_t>((size_t)T);
  m.merged = c.take<uint16_t>((size_t)T * L * D);
  m.bytes = c.off;
  return m;
}

static int check_merge_shape(int T, int L, int D) {
  ET_REQUIRE(T >= 1, "T = %d: a clip needs at least one frame", T);
  ET_REQUIRE(L >= 1, "L = %d: a frame needs at least one token", L);
  ET_REQUIRE(D >= 8 && D % 8 == 0, "D = %d must be a positive multiple of 8", D);
  ET_REQUIRE((double)T * L * D < 2.0e9 * 4, "T*L*D too large");
  if (D > 4096) { set_error("D = %d above the supported 4096", D); return ET_ERR_UNSUPPORTED; }
  if (L > 15360) { set_error("L = %d above the supported 15360", L); return ET_ERR_UNSUPPORTED; }
  return ET_OK;
}

static int check_outputs(const et_output *out) {
  ET_REQUIRE(out != nullptr, "out is NULL");
  ET_REQUIRE(out->tokens_dev && out->kept_idx_dev && out->cu_tokens_dev && out->seg_start_dev,
             "an output buffer is NULL (tokens_dev, kept_idx_dev, cu_tokens_dev, seg_start_dev are required)");
  return ET_OK;
}

int enqueue_merge_stage(const uint16_t *x, int T, int L, int D, float tau, int k, const MergeWs &w,
                        float *sim_out, int32_t *seg_start, int32_t *kept, int32_t *cu_tokens,
                        uint16_t *packed, hipStream_t s, Profiler *prof, const EarlyCount *early) {
  float *sim = sim_out ? sim_out : w.sim;
  ET_TIMED_P(prof, ET_K_SIMILARITY, launch_similarity(x, T, L, D, w.cos, w.part, s));
  ET_TIMED_P(prof, ET_K_SCAN, launch_sim_mean_scan(w.part, similarity_blocks(L), T, L, tau, sim, seg_start, w.n_seg,
                                                   true, true, s));
  if (early) {
    ET_HIP(hipMemcpyAsync(early->host, w.n_seg, sizeof(int32_t), hipMemcpyDeviceToHost, s));
    ET_HIP(hipEventRecord(early->ready, s));
  }
  ET_TIMED_P(prof, ET_K_MERGE, launch_segment_mean(x, T, L, D, seg_start, w.n_seg, w.merged, w.score, s));
  if (L <= 7680) {     // selection and gather in one launch
    ET_TIMED_P(prof, ET_K_SELECT, launch_topk_gather(w.score, w.merged, T, w.n_seg, L, D, k, kept, cu_tokens, packed, s));
  } else {
    ET_TIMED_P(prof, ET_K_SELECT, launch_topk(w.score, T, w.n_seg, L, k, kept, cu_tokens, s));
    ET_TIMED_P(prof, ET_K_COMPACT, launch_compact(w.merged, kept, T, w.n_seg, L, D, k, packed, s));
  }
  return ET_OK;
}

int check_policy(const et_policy *p) {
  ET_REQUIRE(p != nullptr, "policy is NULL");
  ET_REQUIRE(p->merge_mode == ET_MERGE_MEAN || p->merge_mode == ET_MERGE_ALG1, "merge_mode = %d unknown", p->merge_mode);
  ET_REQUIRE(p->select_mode == ET_SELECT_UNIFORM || p->select_mode == ET_SELECT_DECOUPLED,
             "select_mode = %d unknown", p->select_mode);
  ET_REQUIRE(p->score_mode == ET_SCORE_L2NORM || p->score_mode == ET_SCORE_ATTENTION,
             "score_mode = %d unknown", p->score_mode);
  ET_REQUIRE(p->alpha > 0.f && p->alpha <= 1.f, "alpha = %g outside (0, 1]", (double)p->alpha);
  ET_REQUIRE(!isnan(p->tau_seg) && !isnan(p->tau_merge), "a threshold is NaN");
  ET_REQUIRE(p->ratio > 0.f && p->ratio <= 1.f, "ratio = %g outside (0, 1]", (double)p->ratio);
  return ET_OK;
}

int enqueue_policy_stage(const uint16_t *x, int T, int L, int D, const et_policy &pol, const PlanStep &step,
                         const MergeWs &w, float *sim_out, int32_t *seg_start, int32_t *kept,
                         int32_t *cu_tokens, uint16_t *packed, int32_t *info, hipStream_t s, Profiler *prof,
                         const float *score_override) {
  float *sim = sim_out ? sim_out : w.sim;
  const PolicyArgs pa{pol.merge_mode, pol.select_mode, pol.alpha, pol.tau_seg, pol.tau_merge, pol.ratio};
  const int k_uniform = et_keep_count(L, pol.ratio);
  if (step.do_plan) {
    ET_TIMED_P(prof, ET_K_SIMILARITY, launch_similarity(x, T, L, D, w.cos, w.part, s));
    ET_TIMED_P(prof, ET_K_SCAN, launch_sim_mean_scan(w.part, similarity_blocks(L), T, L, 0.f, sim, nullptr, nullptr,
                                                     true, false, s));
  }
  ET_TIMED_P(prof, ET_K_SCAN, launch_plan(sim, T, L, pa, k_uniform, step, seg_start, w.frame_first, w.frame_count,
                                          w.frame_dyn, w.frame_w, w.orig_first, w.orig_count, cu_tokens, info, s));
  ET_TIMED_P(prof, ET_K_MERGE, launch_plan_merge(x, T, L, D, info, w.frame_first, w.frame_count, w.frame_w,
                                                 step.do_plan && pol.merge_mode == ET_MERGE_MEAN, w.merged,
                                                 w.score, s));
  if (step.do_counts) {
    // (score_override: scores computed elsewhere, e.g. the attention received, instead of the L2 norms)
    ET_TIMED_P(prof, ET_K_SELECT, launch_select_policy(score_override ? score_override : w.score, T, info, w.frame_dyn, cu_tokens, L,
                                                       pol.select_mode == ET_SELECT_UNIFORM, kept, s));
    ET_TIMED_P(prof, ET_K_COMPACT, launch_compact_ragged(w.merged, kept, T, info, cu_tokens, L, D, packed, s));
  }
  return ET_OK;
}

int copy_plan_out(const MergeWs &w, int N, et_plan_out *plan, hipStream_t s) {
  if (!plan || N <= 0) return ET_OK;
  const size_t bytes = (size_t)N * sizeof(int32_t);
  if (plan->frame_first_dev) ET_HIP(hipMemcpyAsync(plan->frame_first_dev, w.orig_first, bytes, hipMemcpyDeviceToDevice, s));
  if (plan->frame_count_dev) ET_HIP(hipMemcpyAsync(plan->frame_count_dev, w.orig_count, bytes, hipMemcpyDeviceToDevice, s));
  if (plan->frame_dynamic_dev) ET_HIP(hipMemcpyAsync(plan->frame_dynamic_dev, w.frame_dyn, bytes, hipMemcpyDeviceToDevice, s));
  return ET_OK;
}

int Profiler::begin(int kind, hipStream_t s) {
  if (!on) return ET_OK;
  const size_t need = 2 * (kinds.size() + 1);
  while (pool.size() < need) {
    hipEvent_t e;
    ET_HIP(hipEventCreate(&e));
    pool.push_back(e);
  }
  kinds.push_back(kind + ET_K_COUNT * phase);
  ET_HIP(hipEventRecord(pool[2 * (kinds.size() - 1)], s));
  return ET_OK;
}

int Profiler::end(hipStream_t s) {
  if (!on) return ET_OK;
  ET_HIP(hipEventRecord(pool[2 * (kinds.size() - 1) + 1], s));
  return ET_OK;
}

int Profiler::collect() {
  if (!on) return ET_OK;
  for (size_t i = 0; i < kinds.size(); ++i) {
    float t = 0.f;
    ET_HIP(hipEventElapsedTime(&t, pool[2 * i], pool[2 * i + 1]));
    ms[kinds[i]] += t;
    launches[kinds[i]] += 1;
  }
  kinds.clear();
  return ET_OK;
}

void Profiler::destroy() {
  for (hipEvent_t e : pool) (void)hipEventDestroy(e);
  pool.clear();
}

}  // namespace et

using namespace et;

extern "C" {

const char *et_last_error(void) { return g_err; }

int32_t et_keep_count(int32_t L, float keep_ratio) {
  if (L < 1 || !(keep_ratio > 0.f) || !(keep_ratio <= 1.f)) return 0;
  double v = floor((double)keep_ratio * (double)L + 1e-4);
  int32_t k = (int32_t)v;
  if (k < 1) k = 1;
  if (k > L) k = L;
  return k;
}

size_t et_merge_workspace_bytes(int32_t T, int32_t L, int32_t D) {
  if (T < 1 || L < 1 || D < 8) return 0;
  return carve_merge(nullptr, T, L, D).bytes;
}

static int check_merge_args(const uint16_t *x_dev, int32_t T, int32_t L, int32_t D, float sim_threshold,
                            float keep_ratio, const et_output *out) {
  int rc;
  ET_REQUIRE(x_dev != nullptr, "x_dev is NULL");
  if ((rc = check_merge_shape(T, L, D))) return rc;
  if ((rc = check_outputs(out))) return rc;
  ET_REQUIRE(!isnan(sim_threshold), "sim_threshold is NaN");
  ET_REQUIRE(keep_ratio > 0.f && keep_ratio <= 1.f, "keep_ratio = %g outside (0, 1]", (double)keep_ratio);
  return ET_OK;
}

// Optional timing of the stand-alone stage (et_merge_profile_*): HIP events around every launch and
// around the whole sequence, on the caller's stream.  Process-wide; not thread-safe.
static struct StageProfile {
  Profiler p;
  bool on = false;                 // the whole-sequence bracket; p.on adds the per-launch brackets
  hipEvent_t t0 = nullptr, t1 = nullptr;
  double total_ms = 0.0;
  int64_t calls = 0;
} g_stage;

// The stage on a scratch area of at least et_merge_workspace_bytes(T, L, D) bytes; waits for the stream.
static int merge_select_on(const uint16_t *x_dev, int32_t T, int32_t L, int32_t D, float sim_threshold,
                           float keep_ratio, void *scratch_dev, hipStream_t s, et_output *out) {
  int rc;
  MergeWs w = carve_merge(scratch_dev, T, L, D);
  const int k = et_keep_count(L, keep_ratio);
  const bool timed = g_stage.on;
  if (timed) {
    g_stage.p.kinds.clear();
    ET_HIP(hipEventRecord(g_stage.t0, s));
  }
  if ((rc = enqueue_merge_stage(x_dev, T, L, D, sim_threshold, k, w, out->frame_sim_dev,
                                out->seg_start_dev, out->kept_idx_dev, out->cu_tokens_dev,
                                out->tokens_dev, s, g_stage.p.on ? &g_stage.p : nullptr)))
    return rc;
  if (timed) ET_HIP(hipEventRecord(g_stage.t1, s));
  int32_t n_seg = 0;
  ET_HIP(hipMemcpyAsync(&n_seg, w.n_seg, sizeof(int32_t), hipMemcpyDeviceToHost, s));
  ET_HIP(hipStreamSynchronize(s));
  if (timed) {
    float ms = 0.f;
    ET_HIP(hipEventElapsedTime(&ms, g_stage.t0, g_stage.t1));
    g_stage.total_ms += ms;
    g_stage.calls += 1;
    if ((rc = g_stage.p.collect())) return rc;
  }
  out->n_frames_out = n_seg;
  out->n_tokens = n_seg * k;
  return ET_OK;
}

int et_merge_profile_enable(int32_t on) {
  if (on && !g_stage.t0) {
    ET_HIP(hipEventCreate(&g_stage.t0));
    ET_HIP(hipEventCreate(&g_stage.t1));
  }
  g_stage.on = on != 0;
  g_stage.p.on = on >= 2;
  return ET_OK;
}

int et_merge_profile_read(double *ms, int64_t *launches, double *total_ms, int64_t *calls, int32_t reset) {
  ET_REQUIRE(ms && launches && total_ms && calls, "a pointer argument is NULL");
  for (int i = 0; i < ET_K_COUNT; ++i) {
    ms[i] = g_stage.p.ms[i];
    launches[i] = g_stage.p.launches[i];
    if (reset) { g_stage.p.ms[i] = 0; g_stage.p.launches[i] = 0; }
  }
  *total_ms = g_stage.total_ms;
  *calls = g_stage.calls;
  if (reset) { g_stage.total_ms = 0.0; g_stage.calls = 0; }
  return ET_OK;
}

int et_merge_select_static(const uint16_t *x_dev, int32_t T, int32_t L, int32_t D, float sim_threshold,
                           float keep_ratio, void *hip_stream, et_output *out) {
  int rc;
  if ((rc = check_merge_args(x_dev, T, L, D, sim_threshold, keep_ratio, out))) return rc;
  const size_t need = et_merge_workspace_bytes(T, L, D);
  if (need > (size_t)ET_STATIC_SCRATCH_BYTES) {
    set_error("T * L * D = %d * %d * %d needs %zu bytes of scratch, the static buffer holds %zu: "
              "use et_merge_select with a caller workspace", T, L, D, need, (size_t)ET_STATIC_SCRATCH_BYTES);
    return ET_ERR_WORKSPACE;
  }
  void *ptr = nullptr;
  if ((rc = static_scratch(&ptr))) return rc;
  return merge_select_on(x_dev, T, L, D, sim_threshold, keep_ratio, ptr, static_cast<hipStream_t>(hip_stream), out);
}

int et_merge_select(const uint16_t *x_dev, int32_t T, int32_t L, int32_t D, float sim_threshold,
                    float keep_ratio, void *workspace_dev, size_t workspace_bytes, void *hip_stream,
                    et_output *out) {
  int rc;
  if ((rc = check_merge_args(x_dev, T, L, D, sim_threshold, keep_ratio, out))) return rc;
  ET_REQUIRE(workspace_dev != nullptr, "workspace_dev is NULL");
  size_t need = et_merge_workspace_bytes(T, L, D);
  if (workspace_bytes < need) {
    set_error("workspace of %zu bytes is smaller than the %zu needed", workspace_bytes, need);
    return ET_ERR_WORKSPACE;
  }
  return merge_select_on(x_dev, T, L, D, sim_threshold, keep_ratio, workspace_dev,
                         static_cast<hipStream_t>(hip_stream), out);
}

int et_merge_select_policy(const uint16_t *x_dev, int32_t T, int32_t L, int32_t D, const et_policy *policy,
                           void *workspace_dev, size_t workspace_bytes, void *hip_stream, et_output *out,
                           et_plan_out *plan) {
  int rc;
  ET_REQUIRE(x_dev != nullptr, "x_dev is NULL");
  if ((rc = check_merge_shape(T, L, D))) return rc;
  if ((rc = check_outputs(out))) return rc;
  if ((rc = check_policy(policy))) return rc;
  ET_REQUIRE(policy->score_mode == ET_SCORE_L2NORM,
             "score_mode = ET_SCORE_ATTENTION needs the encoder (et_encode_clip_multi): there is no attention here");
  ET_REQUIRE(workspace_dev != nullptr, "workspace_dev is NULL");
  size_t need = et_merge_workspace_bytes(T, L, D);
  if (workspace_bytes < need) {
    set_error("workspace of %zu bytes is smaller than the %zu needed", workspace_bytes, need);
    return ET_ERR_WORKSPACE;
  }
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  MergeWs w = carve_merge(workspace_dev, T, L, D);
  int32_t *info = w.n_seg + 8;
  const PlanStep step{1, 1, 1, T};
  if ((rc = enqueue_policy_stage(x_dev, T, L, D, *policy, step, w, out->frame_sim_dev, out->seg_start_dev,
                                 out->kept_idx_dev, out->cu_tokens_dev, out->tokens_dev, info, s, nullptr)))
    return rc;
  int32_t host_info[5] = {0, 0, 0, 0, 0};
  ET_HIP(hipMemcpyAsync(host_info, info, sizeof(host_info), hipMemcpyDeviceToHost, s));
  ET_HIP(hipStreamSynchronize(s));
  if ((rc = copy_plan_out(w, host_info[0], plan, s))) return rc;
  if (plan) {
    plan->n_segments = host_info[1];
    ET_HIP(hipStreamSynchronize(s));
  }
  out->n_frames_out = host_info[0];
  out->n_tokens = host_info[2];
  return ET_OK;
}

int et_frame_similarity(const uint16_t *x_dev, int32_t T, int32_t L, int32_t D, float *cos_dev,
                        float *sim_dev, void *hip_stream) {
  int rc;
  ET_REQUIRE(x_dev && cos_dev && sim_dev, "a pointer argument is NULL");
  if ((rc = check_merge_shape(T, L, D))) return rc;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (T < 2) return ET_OK;
  if ((rc = launch_similarity(x_dev, T, L, D, cos_dev, nullptr, s))) return rc;
  return launch_sim_mean_scan(cos_dev, L, T, L, 0.f, sim_dev, nullptr, nullptr, true, false, s);
}

int et_segment_scan(const float *sim_dev, int32_t T, float sim_threshold, int32_t *seg_start_dev,
                    int32_t *n_seg_dev, void *hip_stream) {
  ET_REQUIRE(seg_start_dev && n_seg_dev, "a pointer argument is NULL");
  ET_REQUIRE(T >= 1, "T = %d: a clip needs at least one frame", T);
  ET_REQUIRE(T == 1 || sim_dev != nullptr, "sim_dev is NULL");
  ET_REQUIRE(!isnan(sim_threshold), "sim_threshold is NaN");
  return launch_sim_mean_scan(nullptr, 0, T, 1, sim_threshold, const_cast<float *>(sim_dev), seg_start_dev,
                              n_seg_dev, false, true, static_cast<hipStream_t>(hip_stream));
}

int et_segment_mean(const uint16_t *x_dev, int32_t T, int32_t L, int32_t D, const int32_t *seg_start_dev,
                    const int32_t *n_seg_dev, uint16_t *merged_dev, float *score_dev, void *hip_stream) {
  int rc;
  ET_REQUIRE(x_dev && seg_start_dev && n_seg_dev && merged_dev && score_dev, "a pointer argument is NULL");
  if ((rc = check_merge_shape(T, L, D))) return rc;
  return launch_segment_mean(x_dev, T, L, D, seg_start_dev, n_seg_dev, merged_dev, score_dev,
                             static_cast<hipStream_t>(hip_stream));
}

int et_topk_select(const float *score_dev, int32_t n_rows, int32_t L, int32_t k, int32_t *kept_idx_dev,
                   void *hip_stream) {
  ET_REQUIRE(score_dev && kept_idx_dev, "a pointer argument is NULL");
  ET_REQUIRE(n_rows >= 0 && L >= 1, "n_rows = %d, L = %d out of range", n_rows, L);
  ET_REQUIRE(k >= 1 && k <= L, "k = %d outside [1, L = %d]", k, L);
  if (n_rows == 0) return ET_OK;
  return launch_topk(score_dev, n_rows, nullptr, L, k, kept_idx_dev, nullptr,
                     static_cast<hipStream_t>(hip_stream));
}

int et_compact_tokens(const uint16_t *merged_dev, const int32_t *kept_idx_dev, int32_t n_rows, int32_t L,
                      int32_t D, int32_t k, uint16_t *out_dev, void *hip_stream) {
  ET_REQUIRE(merged_dev && kept_idx_dev && out_dev, "a pointer argument is NULL");
  ET_REQUIRE(n_rows >= 0 && L >= 1 && D >= 8 && D % 8 == 0, "n_rows = %d, L = %d, D = %d out of range",
             n_rows, L, D);
  ET_REQUIRE(k >= 1 && k <= L, "k = %d outside [1, L = %d]", k, L);
  if (n_rows == 0) return ET_OK;
  return launch_compact(merged_dev, kept_idx_dev, n_rows, nullptr, L, D, k, out_dev,
                        static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
