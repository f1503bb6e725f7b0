// Internal helpers shared by the HIP translation units of libearlytom (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>

#include <vector>

#include "earlytom.h"

namespace et {

constexpr int kWave = 64;

void set_error(const char *fmt, ...);
int hip_fail(hipError_t e, const char *what, const char *file, int line);

#define ET_HIP(call)                                                       \
  do {                                                                     \
    hipError_t e__ = (call);                                               \
    if (e__ != hipSuccess) return et::hip_fail(e__, #call, __FILE__, __LINE__); \
  } while (0)

// Checks the launch that was just issued.
#define ET_LAUNCH_CHECK() ET_HIP(hipGetLastError())

#define ET_REQUIRE(cond, ...)          \
  do {                                 \
    if (!(cond)) {                     \
      et::set_error(__VA_ARGS__);      \
      return ET_ERR_INVALID_ARG;       \
    }                                  \
  } while (0)

// ---- device-side bf16 <-> fp32 (bit-level, round to nearest even) ----
__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}
__device__ __forceinline__ float bf16lo_to_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;  // NaN stays a quiet NaN
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}


// ---- one token row held across the 64 lanes of a wavefront: NV 16-byte vectors per lane ----
template <int NV>
struct Row {
  float v[NV * 8];
};

// Loads one bf16 row of length D into per-lane registers (zeros past D).
template <int NV>
__device__ __forceinline__ void load_row(const uint16_t *__restrict__ p, int D, int lane, uint4 (&raw)[NV]) {
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    int c = (j * kWave + lane) * 8;
    if (c < D) raw[j] = *reinterpret_cast<const uint4 *>(p + c);
    else raw[j] = make_uint4(0, 0, 0, 0);
  }
}

template <int NV>
__device__ __forceinline__ void unpack_row(const uint4 (&raw)[NV], Row<NV> &r) {
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    r.v[j * 8 + 0] = bf16lo_to_f32(raw[j].x); r.v[j * 8 + 1] = bf16hi_to_f32(raw[j].x);
    r.v[j * 8 + 2] = bf16lo_to_f32(raw[j].y); r.v[j * 8 + 3] = bf16hi_to_f32(raw[j].y);
    r.v[j * 8 + 4] = bf16lo_to_f32(raw[j].z); r.v[j * 8 + 5] = bf16hi_to_f32(raw[j].z);
    r.v[j * 8 + 6] = bf16lo_to_f32(raw[j].w); r.v[j * 8 + 7] = bf16hi_to_f32(raw[j].w);
  }
}

inline int nv_for(int D) { return (D + 511) / 512; }

#define ET_DISPATCH_NV(D, ...)                                              \
  switch (et::nv_for(D)) {                                                  \
    case 1: { constexpr int NV = 1; __VA_ARGS__; } break;                   \
    case 2: { constexpr int NV = 2; __VA_ARGS__; } break;                   \
    case 3: { constexpr int NV = 3; __VA_ARGS__; } break;                   \
    case 4: { constexpr int NV = 4; __VA_ARGS__; } break;                   \
    case 5: case 6: { constexpr int NV = 6; __VA_ARGS__; } break;           \
    case 7: case 8: { constexpr int NV = 8; __VA_ARGS__; } break;           \
    default: et::set_error("d_model %d above the supported 4096", D); return ET_ERR_UNSUPPORTED; \
  }


// Brackets kernel launches with HIP events when enabled; sums elapsed time per kernel kind.
struct Profiler {
  bool on = false;
  std::vector<hipEvent_t> pool;
  std::vector<int> kinds;          // slot of the i-th bracket; its events are pool[2i], pool[2i+1]
  int phase = 0;                   // 0: before the compression stage (and the stage itself), 1: after
  double ms[2 * ET_K_COUNT] = {0}; // slot = kind + ET_K_COUNT * phase
  int64_t launches[2 * ET_K_COUNT] = {0};

  int begin(int kind, hipStream_t s);
  int end(hipStream_t s);
  int collect();                   // call after the stream has been synchronised
  void destroy();
};

// Runs `call` (an int-returning launcher) between a profiler bracket; returns on error.
#define ET_TIMED_P(prof, kind, call)                          \
  do {                                                        \
    int rc__;                                                 \
    if ((prof) && (rc__ = (prof)->begin(kind, s))) return rc__; \
    if ((rc__ = (call))) return rc__;                         \
    if ((prof) && (rc__ = (prof)->end(s))) return rc__;       \
  } while (0)

// Scratch of the compression stage, carved from a caller workspace.
struct MergeWs {
  float *cos, *sim, *score;
  float *part;                    // [T-1, similarity_blocks(L)]: per-workgroup sums of cosines
  uint16_t *merged;
  int32_t *n_seg;                 // 64 ints: [0] segment count of the simple path; [8..12] policy info
  int32_t *frame_first, *frame_count, *frame_dyn;   // [T] each: output-frame plan (policy path)
  float *frame_w;                 // [2T]
  int32_t *orig_first, *orig_count;   // [T] each: range of original frames behind each current frame
  size_t bytes;
};

// Policy of the paper-exact stage as the kernels take it (mirrors et_policy).
struct PolicyArgs {
  int merge_mode, select_mode;
  float alpha, tau_seg, tau_merge, ratio;
};
// One application of the plan kernel: build a plan from similarities or take the identity plan;
// compute the selection's token counts or not; first stage (frame ranges start as identity) or not.
struct PlanStep {
  int do_plan, do_counts, init_orig, t_orig;
};
int check_policy(const et_policy *p);
// Enqueues similarity -> plan -> weighted merge -> selection -> ragged gather; no host sync.
// info (device, >= 5 ints) receives N, segments, total tokens, tokens per dynamic / static frame.
// `step` says which parts run: with do_counts the selection and the gather into `packed` follow the
// merge; without, only `w.merged` (all L tokens per frame) and `w.score` are produced.
int enqueue_policy_stage(const uint16_t *x, int T, int L, int D, const et_policy &pol, const PlanStep &step,
                         const MergeWs &w, float *sim_out, int32_t *seg_start, int32_t *kept,
                         int32_t *cu_tokens, uint16_t *packed, int32_t *info, hipStream_t s,
                         struct Profiler *prof, const float *score_override = nullptr);
int copy_plan_out(const MergeWs &w, int N, et_plan_out *plan, hipStream_t s);
MergeWs carve_merge(void *ws, int T, int L, int D);
// Where the host learns the segment count while the stage is still running: right after the scan
// kernel the count is copied to `host` (pinned memory) and `ready` is recorded, so the host waits
// for that event only and enqueues the following blocks under the merge, selection and compaction.
struct EarlyCount {
  int32_t *host;
  hipEvent_t ready;
};
// Enqueues similarity -> scan -> segment mean (+score) -> top-k -> compaction; no host sync.
int enqueue_merge_stage(const uint16_t *x, int T, int L, int D, float tau, int k, const MergeWs &w,
                        float *sim_out, int32_t *seg_start, int32_t *kept, int32_t *cu_tokens,
                        uint16_t *packed, hipStream_t s, Profiler *prof, const EarlyCount *early = nullptr);

// ---- launchers implemented in merge_kernels.hip ----
// part [T-1, similarity_blocks(L)]: per pair and workgroup, the sum of the workgroup's cosines
int similarity_blocks(int L);
int launch_similarity(const uint16_t *x, int T, int L, int D, float *cos_out, float *part, hipStream_t s);
// sim[t] = (sum of src[t, 0..n_src)) / L (do_mean), then the boundary scan (do_scan)
int launch_sim_mean_scan(const float *src, int n_src, int T, int L, float tau, float *sim_out,
                         int32_t *seg_start, int32_t *n_seg, bool do_mean, bool do_scan,
                         hipStream_t s);
int launch_segment_mean(const uint16_t *x, int T, int L, int D, const int32_t *seg_start,
                        const int32_t *n_seg, uint16_t *merged, float *score, hipStream_t s);
int launch_topk(const float *score, int n_rows_max, const int32_t *n_rows_dev, int L, int k,
                int32_t *kept, int32_t *cu_tokens, hipStream_t s);
// selection and gather of the kept rows in one launch (n_rows_dev must not be NULL; L <= 7680)
int launch_topk_gather(const float *score, const uint16_t *merged, int n_rows_max, const int32_t *n_rows_dev, int L,
                       int D, int k, int32_t *kept, int32_t *cu_tokens, uint16_t *out, hipStream_t s);
int launch_compact(const uint16_t *merged, const int32_t *kept, int n_rows_max,
                   const int32_t *n_rows_dev, int L, int D, int k, uint16_t *out, hipStream_t s);
int launch_identity_maps(int T, int L, int32_t *kept, int32_t *cu_tokens, int32_t *seg_start,
                         hipStream_t s);
int launch_cu_uniform(int n, int step, int32_t *cu, hipStream_t s);

// ---- launchers implemented in policy_kernels.hip ----
int launch_plan(const float *sim, int T, int L, const PolicyArgs &p, int k_uniform, const PlanStep &st,
                int32_t *seg_start, int32_t *frame_first, int32_t *frame_count, int32_t *frame_dyn,
                float *frame_w, int32_t *orig_first, int32_t *orig_count, int32_t *cu_tokens, int32_t *info,
                hipStream_t s);
int launch_plan_merge(const uint16_t *x, int T, int L, int D, const int32_t *info, const int32_t *frame_first,
                      const int32_t *frame_count, const float *frame_w, bool uniform_mean, uint16_t *merged,
                      float *score, hipStream_t s);
int launch_select_policy(const float *score, int T, const int32_t *info, const int32_t *frame_dyn,
                         const int32_t *cu_tokens, int L, bool all_topk, int32_t *kept, hipStream_t s);
int launch_compact_ragged(const uint16_t *merged, const int32_t *kept, int T, const int32_t *info,
                          const int32_t *cu_tokens, int L, int D, uint16_t *out, hipStream_t s);

// ---- launchers implemented in dense_kernels.hip ----
int launch_layernorm(const uint16_t *x, const float *g, const float *b, float eps, int rows, int D,
                     uint16_t *y, hipStream_t s);
int launch_im2col(const float *frames, int T, int C, int H, int W, int P, int Kpad, uint16_t *out,
                  hipStream_t s);
enum { EPI_BIAS = 0, EPI_BIAS_GELU = 1, EPI_BIAS_RES = 2 };
// A [M, lda] bf16 (K <= lda, K % 64 == 0, pad columns readable), W [Npad, K] bf16 with
// Npad % 256 == 0 (pad rows zero), bias [Npad] fp32, C [M, ldc], residual rows indexed
// (m % res_mod) with leading dimension ldr.  Columns n < n_store are written.
// row_scale (optional, [M] fp32): the accumulator of row m is multiplied by row_scale[m] before the
// bias is added (LayerNorm folded into the GEMM: see fold_layernorm in encoder.hip).
struct GemmArgs {
  const uint16_t *A; int lda;
  const uint16_t *W; const float *bias;
  const uint16_t *res; int ldr; int res_mod;
  uint16_t *C; int ldc;
  int M, n_store, K, epilogue;
  const float *row_scale = nullptr;
};
// 1 / sqrt(var + eps) of every row of x [rows, D] bf16 (biased variance, fp32 two-pass like layernorm_kernel).
int launch_rowstats(const uint16_t *x, float eps, int rows, int D, float *rstd, hipStream_t s);
int launch_gemm(const GemmArgs &g, hipStream_t s, int force_cfg = -1);
int gemm_config_count();
int launch_attention(const uint16_t *qkv, const int32_t *cu, int n_frames, int max_len, int n_heads,
                     int head_dim, uint16_t *out, hipStream_t s);
bool head_dim_supported(int hd);
int launch_touch(const void *const *p, const size_t *bytes, int n, hipStream_t s);   // n <= 4 buffers, one launch
// Equal-length frames (frame f = rows f * len .. f * len + len - 1).
int launch_attention_uniform(const uint16_t *qkv, int n_frames, int len, int n_heads, int head_dim,
                             uint16_t *out, hipStream_t s);

// score_kernels.hip: attention received per token, equal-length frames
size_t attention_scores_workspace_bytes(int n_frames, int L, int n_heads);
int launch_attention_scores(const uint16_t *qkv, int n_frames, int L, int n_heads, int head_dim, void *stats_ws,
                            float *score, hipStream_t s);

}  // namespace et
