// The encoder object and et_encode_clip: weight packing, workspace layout, the layer loop with
// the compression stage spliced in after `merge_layer` blocks, and optional per-kernel timing.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "et_common.h"

namespace et {

static inline int round_up(int v, int a) { return (v + a - 1) / a * a; }
static inline size_t align256(size_t v) { return (v + 255) / 256 * 256; }

static uint16_t host_f32_to_bf16(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0;
  return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

struct LayerDev {
  uint16_t *wqkv, *wo, *w1, *w2;
  float *bqkv, *bo, *b1, *b2;
};

}  // namespace et

struct et_encoder {
  et_config cfg;
  int L, D, hd, Mhp, Kp, Kp_pad, max_frames;
  std::vector<void *> allocs;
  uint16_t *patch_w = nullptr, *pos_emb = nullptr;
  float *patch_b = nullptr, *final_g = nullptr, *final_b = nullptr;
  std::vector<et::LayerDev> layers;
  et::Profiler prof;
  // weight warm-up (see warm_weights): a stream and two events of its own
  hipStream_t warm_stream = nullptr;
  hipEvent_t warm_go = nullptr, warm_done = nullptr;
  int32_t *count_host = nullptr;        // pinned: segment count read back in the middle of the compression stage
  hipEvent_t count_ready = nullptr;
};

namespace et {

// LayerNorm folded into the linear layer that follows it.  With mu, rstd the row statistics,
//   LN(x) W^T + b = rstd (x - mu) (W . gamma)^T + (W beta + b) = rstd * (x Wf^T) + c,
//   Wf[n][k] = W[n][k] gamma[k] - mean_k(W[n][:] gamma),   c[n] = sum_k W[n][k] beta[k] + b[n]:
// subtracting each folded row's mean makes the mu term vanish (sum_k (x_k - mu) w_k = sum_k x_k (w_k - mean w)),
// so the GEMM reads the residual stream itself and its epilogue multiplies by the row's rstd.
// The folded weights are rounded to bfloat16 here, along each row with the rounding error carried
// into the next element (first-order error diffusion, k ascending, every step through the nearest
// float32): a row of rounded weights then still sums to zero within one step of one element, where
// independent rounding would leave ~sqrt(K) half-steps that a row's mean multiplies.
static void fold_layernorm(const float *W, const float *bias, const float *gamma, const float *beta, int N, int K,
                           std::vector<float> &Wf, std::vector<float> &c) {
  Wf.resize((size_t)N * K);
  c.resize(N);
  std::vector<double> row(K);
  for (int n = 0; n < N; ++n) {
    double mean = 0.0, cb = bias[n];
    for (int k = 0; k < K; ++k) {
      row[k] = (double)W[(size_t)n * K + k] * gamma[k];
      mean += row[k];
      cb += (double)W[(size_t)n * K + k] * beta[k];
    }
    mean /= K;
    double carry = 0.0;
    for (int k = 0; k < K; ++k) {
      const double t = row[k] - mean + carry;
      const uint32_t bits = (uint32_t)host_f32_to_bf16((float)t) << 16;
      float y;
      memcpy(&y, &bits, 4);
      Wf[(size_t)n * K + k] = y;
      carry = t - (double)y;
    }
    c[n] = (float)cb;
  }
}

// Uploads a host fp32 matrix [rows, cols] as bf16 [rows_pad, cols_pad], zero padded.
static int upload_bf16(et_encoder *e, const float *src, int rows, int cols, int rows_pad, int cols_pad,
                       uint16_t **out) {
  std::vector<uint16_t> h((size_t)rows_pad * cols_pad, 0);
  for (int r = 0; r < rows; ++r)
    for (int c = 0; c < cols; ++c) h[(size_t)r * cols_pad + c] = host_f32_to_bf16(src[(size_t)r * cols + c]);
  void *d = nullptr;
  if (hipMalloc(&d, h.size() * sizeof(uint16_t)) != hipSuccess) {
    (void)hipGetLastError();
    set_error("device allocation of %zu bytes failed", h.size() * sizeof(uint16_t));
    return ET_ERR_ALLOC;
  }
  e->allocs.push_back(d);
  ET_HIP(hipMemcpy(d, h.data(), h.size() * sizeof(uint16_t), hipMemcpyHostToDevice));
  *out = static_cast<uint16_t *>(d);
  return ET_OK;
}

static int upload_f32(et_encoder *e, const float *src, int n, int n_pad, float **out) {
  std::vector<float> h((size_t)n_pad, 0.f);
  memcpy(h.data(), src, (size_t)n * sizeof(float));
  void *d = nullptr;
  if (hipMalloc(&d, h.size() * sizeof(float)) != hipSuccess) {
    (void)hipGetLastError();
    set_error("device allocation of %zu bytes failed", h.size() * sizeof(float));
    return ET_ERR_ALLOC;
  }
  e->allocs.push_back(d);
  ET_HIP(hipMemcpy(d, h.data(), h.size() * sizeof(float), hipMemcpyHostToDevice));
  *out = static_cast<float *>(d);
  return ET_OK;
}

struct EncWs {
  uint16_t *x, *qkv, *att, *hid;
  float *rstd;         // [R]: 1 / sqrt(var + eps) of the rows of x (LayerNorm folded into the next GEMM)
  int32_t *cu_full;
  void *merge;
  void *score_ws;      // row statistics and per-head column sums of the attention-received scores
  float *att_score;    // [T, L]
  size_t bytes;
};

static EncWs carve_encoder(const et_encoder *e, void *ws, int T) {
  char *base = static_cast<char *>(ws);
  size_t off = 0;
  auto take = [&](size_t bytes) -> void * {
    void *p = base ? base + off : nullptr;
    off += align256(bytes);
    return p;
  };
  const size_t R = (size_t)T * e->L;
  EncWs w;
  w.x = static_cast<uint16_t *>(take(R * e->D * 2));
  w.rstd = static_cast<float *>(take(R * sizeof(float)));
  w.qkv = static_cast<uint16_t *>(take(R * 3 * e->D * 2));
  w.att = static_cast<uint16_t *>(take(R * e->D * 2));
  const size_t hid_cols = (size_t)(e->Mhp > e->Kp_pad ? e->Mhp : e->Kp_pad);
  w.hid = static_cast<uint16_t *>(take(R * hid_cols * 2));
  w.cu_full = static_cast<int32_t *>(take((size_t)(T + 1) * 4));
  w.merge = take(carve_merge(nullptr, T, e->L, e->D).bytes);
  w.score_ws = take(attention_scores_workspace_bytes(T, e->L, e->cfg.n_heads));
  w.att_score = static_cast<float *>(take(R * sizeof(float)));
  w.bytes = off;
  return w;
}

#define ET_TIMED(kind, call) ET_TIMED_P(&e->prof, kind, call)

// with_scores: also leave the attention each token receives in this block in w.att_score (frames of
// equal length only).
static int run_block(et_encoder *e, const LayerDev &lw, const EncWs &w, int rows, const int32_t *cu,
                     int n_frames, int max_len, bool ragged, hipStream_t s, bool with_scores = false) {
  const et_config &c = e->cfg;
  const int D = e->D;
  // LayerNorm 1 and 2 are folded into the QKV and fc1 weights (fold_layernorm): only the row scales are computed here
  ET_TIMED(ET_K_LAYERNORM, launch_rowstats(w.x, c.ln_eps, rows, D, w.rstd, s));
  GemmArgs g;
  g = GemmArgs{w.x, D, lw.wqkv, lw.bqkv, nullptr, 0, 1, w.qkv, 3 * D, rows, 3 * D, D, EPI_BIAS, w.rstd};
  ET_TIMED(ET_K_GEMM_QKV, launch_gemm(g, s));
  if (with_scores)
    ET_TIMED(ET_K_SCORE, launch_attention_scores(w.qkv, n_frames, max_len, c.n_heads, e->hd, w.score_ws, w.att_score, s));
  if (ragged) {   // frames of different lengths (decoupled selection): row ranges from cu
    ET_TIMED(ET_K_ATTENTION, launch_attention(w.qkv, cu, n_frames, max_len, c.n_heads, e->hd, w.att, s));
  } else {        // every frame has max_len tokens
    ET_TIMED(ET_K_ATTENTION, launch_attention_uniform(w.qkv, n_frames, max_len, c.n_heads, e->hd, w.att, s));
  }
  g = GemmArgs{w.att, D, lw.wo, lw.bo, w.x, D, rows, w.x, D, rows, D, D, EPI_BIAS_RES};
  ET_TIMED(ET_K_GEMM_OUT, launch_gemm(g, s));
  ET_TIMED(ET_K_LAYERNORM, launch_rowstats(w.x, c.ln_eps, rows, D, w.rstd, s));
  g = GemmArgs{w.x, D, lw.w1, lw.b1, nullptr, 0, 1, w.hid, e->Mhp, rows, e->Mhp, D, EPI_BIAS_GELU, w.rstd};
  ET_TIMED(ET_K_GEMM_FC1, launch_gemm(g, s));
  g = GemmArgs{w.hid, e->Mhp, lw.w2, lw.b2, w.x, D, rows, w.x, D, rows, D, e->Mhp, EPI_BIAS_RES};
  ET_TIMED(ET_K_GEMM_FC2, launch_gemm(g, s));
  return ET_OK;
}

// A block that runs on few rows (after the selection) is short against the time HBM needs to
// deliver its weights: every GEMM there starts on cold weights (the 27 layers' 0.8 GB stay in no
// cache) with two stages of look-ahead per workgroup, and the compute units are not full.  When
// such a block starts, its four weight matrices are therefore pulled through the cache hierarchy by
// small kernels on a stream of the encoder's own, released by an event on the caller's stream;
// nothing waits for them but the end of the encode call.  Measured on the 32-frame clip (19 blocks
// on 2912 rows): fc2 59 -> 48 us per launch, -1.5 % per clip; on blocks with many rows, or one
// matrix at a time just before its GEMM, it costs more than it gains.
constexpr int kWarmRows = 8192;
static int warm_weights(et_encoder *e, int li, hipStream_t s) {
  if (!e->warm_stream || li < 0 || li >= (int)e->layers.size()) return ET_OK;
  const LayerDev &lw = e->layers[li];
  const size_t D = e->D, Dn = round_up(e->D, 256);
  ET_HIP(hipEventRecord(e->warm_go, s));
  ET_HIP(hipStreamWaitEvent(e->warm_stream, e->warm_go, 0));
  const void *const mats[4] = {lw.wqkv, lw.wo, lw.w1, lw.w2};
  const size_t bytes[4] = {(size_t)round_up(3 * e->D, 256) * D * 2, Dn * D * 2, (size_t)round_up(e->Mhp, 256) * D * 2,
                           Dn * e->Mhp * 2};
  int rc;
  if ((rc = launch_touch(mats, bytes, 4, e->warm_stream))) return rc;
  return ET_OK;
}

}  // namespace et

using namespace et;

extern "C" {

int et_encoder_create(const et_config *config, const et_weights *weights, int32_t max_frames,
                      et_encoder **out) {
  ET_REQUIRE(config && weights && out, "config, weights or out is NULL");
  *out = nullptr;
  const et_config &c = *config;
  ET_REQUIRE(c.n_layers >= 0 && c.n_layers <= 1024, "n_layers = %d out of range", c.n_layers);
  ET_REQUIRE(c.d_model >= 8 && c.n_heads >= 1 && c.d_mlp >= 1, "d_model/n_heads/d_mlp must be positive");
  ET_REQUIRE(c.d_model % c.n_heads == 0, "d_model %d is not a multiple of n_heads %d", c.d_model, c.n_heads);
  ET_REQUIRE(c.patch >= 1 && c.channels >= 1, "patch and channels must be positive");
  ET_REQUIRE(c.image_h >= c.patch && c.image_w >= c.patch, "image %dx%d smaller than one %d-pixel patch",
             c.image_h, c.image_w, c.patch);
  ET_REQUIRE(c.ln_eps >= 0.f && isfinite(c.ln_eps), "ln_eps must be finite and non-negative");
  ET_REQUIRE(max_frames >= 1, "max_frames = %d must be at least 1", max_frames);
  const int L = (c.image_h / c.patch) * (c.image_w / c.patch);
  ET_REQUIRE((double)max_frames * L * c.d_model * 3 < 2.0e9, "max_frames * L * 3 * d_model exceeds 2^31 elements");
  ET_REQUIRE(weights->patch_w && weights->patch_b && weights->pos_emb, "a patch-embedding weight is NULL");
  ET_REQUIRE(c.n_layers == 0 || (weights->ln1_g && weights->ln1_b && weights->wqkv && weights->bqkv &&
                                 weights->wo && weights->bo && weights->ln2_g && weights->ln2_b &&
                                 weights->w1 && weights->b1 && weights->w2 && weights->b2),
             "a per-layer weight table is NULL");
  ET_REQUIRE(!c.has_final_ln || (weights->final_ln_g && weights->final_ln_b),
             "has_final_ln is set but final_ln_g/final_ln_b is NULL");
  if (c.d_model % 64 != 0 || c.d_model > 4096) {
    set_error("d_model = %d: only multiples of 64 up to 4096 are supported", c.d_model);
    return ET_ERR_UNSUPPORTED;
  }
  if (!head_dim_supported(c.d_model / c.n_heads)) {
    set_error("head_dim = %d is not instantiated (16, 32, 64, 72, 80, 96, 128)", c.d_model / c.n_heads);
    return ET_ERR_UNSUPPORTED;
  }
  if (L > 15360) {
    set_error("tokens per frame = %d above the supported 15360", L);
    return ET_ERR_UNSUPPORTED;
  }
  for (int i = 0; i < c.n_layers; ++i) {
    ET_REQUIRE(weights->ln1_g[i] && weights->ln1_b[i] && weights->wqkv[i] && weights->bqkv[i] &&
                   weights->wo[i] && weights->bo[i] && weights->ln2_g[i] && weights->ln2_b[i] &&
                   weights->w1[i] && weights->b1[i] && weights->w2[i] && weights->b2[i],
               "a weight pointer of layer %d is NULL", i);
  }

  et_encoder *e = new (std::nothrow) et_encoder();
  if (!e) { set_error("host allocation failed"); return ET_ERR_ALLOC; }
  e->cfg = c;
  e->L = L;
  e->D = c.d_model;
  e->hd = c.d_model / c.n_heads;
  e->Mhp = round_up(c.d_mlp, 64);
  e->Kp = c.channels * c.patch * c.patch;
  e->Kp_pad = round_up(e->Kp, 64);
  e->max_frames = max_frames;
  const int D = e->D, Dn = round_up(D, 256);
  int rc = ET_OK;
#define ET_TRY(x) if ((rc = (x)) != ET_OK) { et_encoder_destroy(e); return rc; }
  ET_TRY(upload_bf16(e, weights->patch_w, D, e->Kp, Dn, e->Kp_pad, &e->patch_w));
  ET_TRY(upload_f32(e, weights->patch_b, D, Dn, &e->patch_b));
  ET_TRY(upload_bf16(e, weights->pos_emb, L, D, L, D, &e->pos_emb));
  if (c.has_final_ln) {
    ET_TRY(upload_f32(e, weights->final_ln_g, D, D, &e->final_g));
    ET_TRY(upload_f32(e, weights->final_ln_b, D, D, &e->final_b));
  }
  e->layers.resize(c.n_layers);
  for (int i = 0; i < c.n_layers; ++i) {
    LayerDev &l = e->layers[i];
    std::vector<float> wf, cf;
    fold_layernorm(weights->wqkv[i], weights->bqkv[i], weights->ln1_g[i], weights->ln1_b[i], 3 * D, D, wf, cf);
    ET_TRY(upload_bf16(e, wf.data(), 3 * D, D, round_up(3 * D, 256), D, &l.wqkv));
    ET_TRY(upload_f32(e, cf.data(), 3 * D, round_up(3 * D, 256), &l.bqkv));
    ET_TRY(upload_bf16(e, weights->wo[i], D, D, Dn, D, &l.wo));
    ET_TRY(upload_f32(e, weights->bo[i], D, Dn, &l.bo));
    // MLP width padded to a multiple of 64 with zero rows / bias (GELU(0) = 0) and zero columns
    fold_layernorm(weights->w1[i], weights->b1[i], weights->ln2_g[i], weights->ln2_b[i], c.d_mlp, D, wf, cf);
    ET_TRY(upload_bf16(e, wf.data(), c.d_mlp, D, round_up(e->Mhp, 256), D, &l.w1));
    ET_TRY(upload_f32(e, cf.data(), c.d_mlp, round_up(e->Mhp, 256), &l.b1));
    ET_TRY(upload_bf16(e, weights->w2[i], D, c.d_mlp, Dn, e->Mhp, &l.w2));
    ET_TRY(upload_f32(e, weights->b2[i], D, Dn, &l.b2));
  }
#undef ET_TRY
  if (hipStreamCreateWithFlags(&e->warm_stream, hipStreamNonBlocking) != hipSuccess ||      // (default priority)
      hipEventCreateWithFlags(&e->warm_go, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&e->warm_done, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&e->count_ready, hipEventDisableTiming) != hipSuccess ||
      hipHostMalloc(reinterpret_cast<void **>(&e->count_host), 64, hipHostMallocDefault) != hipSuccess) {
    (void)hipGetLastError();
    et_encoder_destroy(e);
    set_error("creating the warm-up stream, the read-back event or its pinned word failed");
    return ET_ERR_HIP;
  }
  *out = e;
  return ET_OK;
}

void et_encoder_destroy(et_encoder *e) {
  if (!e) return;
  if (e->warm_stream) (void)hipStreamDestroy(e->warm_stream);
  if (e->warm_go) (void)hipEventDestroy(e->warm_go);
  if (e->warm_done) (void)hipEventDestroy(e->warm_done);
  if (e->count_ready) (void)hipEventDestroy(e->count_ready);
  if (e->count_host) (void)hipHostFree(e->count_host);
  for (void *p : e->allocs) (void)hipFree(p);
  e->prof.destroy();
  delete e;
}

size_t et_workspace_bytes(const et_encoder *e, int32_t T) {
  if (!e || T < 1 || T > e->max_frames) return 0;
  return carve_encoder(e, nullptr, T).bytes;
}

}  // extern "C"

// Shared body of et_encode_clip (policy == nullptr: simple stage with sim_threshold / keep_ratio)
// and et_encode_clip_policy.
// With a policy, `merge_layers[0..n_merge)` (ascending) are the layers where Stage I runs and
// `merge_layer` is the layer of Stage II (>= the last Stage I layer).
static int encode_impl(et_encoder *e, const float *frames_dev, int32_t T, int32_t merge_layer,
                       float sim_threshold, float keep_ratio, const et_policy *policy,
                       const int32_t *merge_layers, int32_t n_merge, void *workspace_dev,
                       size_t workspace_bytes, void *hip_stream, et_output *out, et_plan_out *plan) {
  ET_REQUIRE(e != nullptr, "encoder is NULL");
  ET_REQUIRE(frames_dev != nullptr, "frames_dev is NULL");
  ET_REQUIRE(T >= 1 && T <= e->max_frames, "T = %d outside [1, max_frames = %d]", T, e->max_frames);
  ET_REQUIRE(merge_layer <= e->cfg.n_layers, "merge_layer = %d above n_layers = %d", merge_layer,
             e->cfg.n_layers);
  ET_REQUIRE(out != nullptr, "out is NULL");
  ET_REQUIRE(out->tokens_dev && out->kept_idx_dev && out->cu_tokens_dev && out->seg_start_dev,
             "an output buffer is NULL (tokens_dev, kept_idx_dev, cu_tokens_dev, seg_start_dev are required)");
  const bool compress = merge_layer >= 0;
  bool by_attention = false;
  if (compress && policy) {
    int prc = check_policy(policy);
    if (prc) return prc;
    by_attention = policy->score_mode == ET_SCORE_ATTENTION;
    if (by_attention) {
      ET_REQUIRE(merge_layer >= 1, "attention scores need an encoder block before the selection (select layer >= 1)");
      for (int i = 0; i < n_merge; ++i)
        ET_REQUIRE(merge_layers[i] != merge_layer,
                   "attention scores need a block between the last merge and the selection (both at layer %d)",
                   merge_layer);
    }
  } else if (compress) {
    ET_REQUIRE(!isnan(sim_threshold), "sim_threshold is NaN");
    ET_REQUIRE(keep_ratio > 0.f && keep_ratio <= 1.f, "keep_ratio = %g outside (0, 1]", (double)keep_ratio);
  }
  ET_REQUIRE(workspace_dev != nullptr, "workspace_dev is NULL");
  const size_t need = et_workspace_bytes(e, T);
  if (workspace_bytes < need) {
    set_error("workspace of %zu bytes is smaller than the %zu needed", workspace_bytes, need);
    return ET_ERR_WORKSPACE;
  }
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const et_config &c = e->cfg;
  const int L = e->L, D = e->D;
  const EncWs w = carve_encoder(e, workspace_dev, T);
  e->prof.kinds.clear();
  e->prof.phase = 0;

  int rows = T * L, n_frames = T, max_len = L, k = L;
  (void)k;
  const int32_t *cu = w.cu_full;
  if (!compress) {
    ET_TIMED(ET_K_MISC, launch_identity_maps(T, L, out->kept_idx_dev, out->cu_tokens_dev,
                                             out->seg_start_dev, s));
    cu = out->cu_tokens_dev;
  } else {
    ET_TIMED(ET_K_MISC, launch_cu_uniform(T, L, w.cu_full, s));
  }

  // patch embedding: x = patches * Wp^T + bp + pos_emb[l]
  ET_TIMED(ET_K_IM2COL, launch_im2col(frames_dev, T, c.channels, c.image_h, c.image_w, c.patch, e->Kp_pad, w.hid, s));
  {
    GemmArgs g{w.hid, e->Kp_pad, e->patch_w, e->patch_b, e->pos_emb, D, L, w.x, D, T * L, D, e->Kp_pad, EPI_BIAS_RES};
    ET_TIMED(ET_K_GEMM_PATCH, launch_gemm(g, s));
  }

  bool ragged = false, selected = false, first_stage = true, warmed = false;
  int n_segments = T, next_merge = 0;
  for (int i = 0; i <= c.n_layers; ++i) {
    const bool merge_here = compress && policy && !selected && next_merge < n_merge && merge_layers[next_merge] == i;
    const bool select_here = compress && !selected && i == merge_layer;
    if (policy && (merge_here || select_here)) {
      const MergeWs mw = carve_merge(w.merge, T, L, D);
      int32_t *info = mw.n_seg + 8;
      const PlanStep step{merge_here ? 1 : 0, select_here ? 1 : 0, first_stage ? 1 : 0, T};
      int rc = enqueue_policy_stage(w.x, n_frames, L, D, *policy, step, mw, first_stage ? out->frame_sim_dev : nullptr,
                                    out->seg_start_dev, out->kept_idx_dev, out->cu_tokens_dev, w.x, info, s,
                                    &e->prof, (select_here && by_attention) ? w.att_score : nullptr);
      if (rc) return rc;
      if (!select_here)      // frames keep all L tokens: the merged frames become the residual stream
        ET_HIP(hipMemcpyAsync(w.x, mw.merged, (size_t)n_frames * L * D * 2, hipMemcpyDeviceToDevice, s));
      int32_t hi[5] = {0, 0, 0, 0, 0};
      ET_HIP(hipMemcpyAsync(hi, info, sizeof(hi), hipMemcpyDeviceToHost, s));
      ET_HIP(hipStreamSynchronize(s));
      if (hi[0] < 1 || hi[0] > n_frames || hi[1] < 1 || hi[1] > T) {
        set_error("plan read back from the device is inconsistent (N = %d, segments = %d)", hi[0], hi[1]);
        return ET_ERR_HIP;
      }
      n_frames = hi[0];
      n_segments = hi[1];
      first_stage = false;
      if (merge_here) ++next_merge;
      if (select_here) {
        if (hi[2] < hi[0] || hi[2] > T * L || hi[3] < 1 || hi[3] > L || hi[4] < 1 || hi[4] > L) {
          set_error("token counts read back from the device are inconsistent (tokens = %d)", hi[2]);
          return ET_ERR_HIP;
        }
        if ((rc = copy_plan_out(mw, hi[0], plan, s))) return rc;
        rows = hi[2];
        max_len = hi[3] > hi[4] ? hi[3] : hi[4];
        ragged = policy->select_mode == ET_SELECT_DECOUPLED && hi[3] != hi[4];
        cu = out->cu_tokens_dev;
        selected = true;
        e->prof.phase = 1;
      } else {
        rows = n_frames * L;     // still L tokens per frame: the uniform offsets stay valid
      }
    } else if (select_here) {
      const MergeWs mw = carve_merge(w.merge, T, L, D);
      k = et_keep_count(L, keep_ratio);
      // The segment count is final after the scan: the host waits for that copy only and enqueues the
      // next blocks while the merge, the selection and the compaction still run.
      const EarlyCount early{e->count_host, e->count_ready};
      *e->count_host = 0;
      int rc = enqueue_merge_stage(w.x, T, L, D, sim_threshold, k, mw, out->frame_sim_dev, out->seg_start_dev,
                                   out->kept_idx_dev, out->cu_tokens_dev, w.x, s, &e->prof, &early);
      if (rc) return rc;
      ET_HIP(hipEventSynchronize(e->count_ready));
      const int32_t n_seg = *e->count_host;
      if (n_seg < 1 || n_seg > T) {
        set_error("segment count %d read back from the device is outside [1, T = %d]", n_seg, T);
        return ET_ERR_HIP;
      }
      n_frames = n_segments = n_seg;
      rows = n_seg * k;
      max_len = k;
      cu = out->cu_tokens_dev;
      selected = true;
      e->prof.phase = 1;
    }
    if (i < c.n_layers) {
      const bool with_scores = by_attention && !selected && i == merge_layer - 1;
      int rc;
      if (rows < kWarmRows) {
        if ((rc = warm_weights(e, i, s))) return rc;
        warmed = true;
      }
      if ((rc = run_block(e, e->layers[i], w, rows, cu, n_frames, max_len, ragged, s, with_scores))) return rc;
    }
  }
  if (warmed) {      // the caller's stream ends after the warm-up stream
    ET_HIP(hipEventRecord(e->warm_done, e->warm_stream));
    ET_HIP(hipStreamWaitEvent(s, e->warm_done, 0));
  }
  if (plan) plan->n_segments = n_segments;
  if (c.has_final_ln) {
    ET_TIMED(ET_K_LAYERNORM, launch_layernorm(w.x, e->final_g, e->final_b, c.ln_eps, rows, D,
                                              out->tokens_dev, s));
  } else {
    ET_HIP(hipMemcpyAsync(out->tokens_dev, w.x, (size_t)rows * D * 2, hipMemcpyDeviceToDevice, s));
  }
  ET_HIP(hipStreamSynchronize(s));
  int rc = e->prof.collect();
  if (rc) return rc;
  out->n_frames_out = n_frames;
  out->n_tokens = rows;
  return ET_OK;
}

extern "C" {

int et_encode_clip(et_encoder *e, const float *frames_dev, int32_t T, int32_t merge_layer,
                   float sim_threshold, float keep_ratio, void *workspace_dev, size_t workspace_bytes,
                   void *hip_stream, et_output *out) {
  return encode_impl(e, frames_dev, T, merge_layer, sim_threshold, keep_ratio, nullptr, nullptr, 0,
                     workspace_dev, workspace_bytes, hip_stream, out, nullptr);
}

int et_encode_clip_policy(et_encoder *e, const float *frames_dev, int32_t T, int32_t merge_layer,
                          const et_policy *policy, void *workspace_dev, size_t workspace_bytes,
                          void *hip_stream, et_output *out, et_plan_out *plan) {
  ET_REQUIRE(merge_layer < 0 || policy != nullptr, "policy is NULL");
  const int32_t layers[1] = {merge_layer};
  return encode_impl(e, frames_dev, T, merge_layer, 0.f, 1.f, policy, layers, merge_layer >= 0 ? 1 : 0,
                     workspace_dev, workspace_bytes, hip_stream, out, plan);
}

int et_encode_clip_multi(et_encoder *e, const float *frames_dev, int32_t T, const int32_t *merge_layers,
                         int32_t n_merge_layers, int32_t select_layer, const et_policy *policy,
                         void *workspace_dev, size_t workspace_bytes, void *hip_stream, et_output *out,
                         et_plan_out *plan) {
  ET_REQUIRE(e != nullptr, "encoder is NULL");
  ET_REQUIRE(policy != nullptr, "policy is NULL");
  ET_REQUIRE(n_merge_layers >= 0 && n_merge_layers <= 64, "n_merge_layers = %d outside [0, 64]", n_merge_layers);
  ET_REQUIRE(n_merge_layers == 0 || merge_layers != nullptr, "merge_layers is NULL");
  ET_REQUIRE(select_layer >= 0 && select_layer <= e->cfg.n_layers, "select_layer = %d outside [0, n_layers = %d]",
             select_layer, e->cfg.n_layers);
  for (int i = 0; i < n_merge_layers; ++i) {
    ET_REQUIRE(merge_layers[i] >= 0 && merge_layers[i] <= select_layer,
               "merge_layers[%d] = %d outside [0, select_layer = %d]", i, merge_layers[i], select_layer);
    ET_REQUIRE(i == 0 || merge_layers[i] > merge_layers[i - 1], "merge_layers must be strictly ascending");
  }
  return encode_impl(e, frames_dev, T, select_layer, 0.f, 1.f, policy, merge_layers, n_merge_layers,
                     workspace_dev, workspace_bytes, hip_stream, out, plan);
}

int et_profile_enable(et_encoder *e, int32_t on) {
  ET_REQUIRE(e != nullptr, "encoder is NULL");
  e->prof.on = on != 0;
  return ET_OK;
}

int et_profile_read(et_encoder *e, double *ms, int64_t *launches, int32_t reset) {
  ET_REQUIRE(e && ms && launches, "a pointer argument is NULL");
  for (int i = 0; i < 2 * ET_K_COUNT; ++i) {
    ms[i] = e->prof.ms[i];
    launches[i] = e->prof.launches[i];
    if (reset) { e->prof.ms[i] = 0; e->prof.launches[i] = 0; }
  }
  return ET_OK;
}

const char *et_kernel_name(int32_t kind) {
  static const char *names[ET_K_COUNT] = {"im2col", "gemm_patch", "layernorm", "gemm_qkv", "attention",
                                          "gemm_out", "gemm_fc1", "gemm_fc2", "similarity", "scan",
                                          "merge", "select", "compact", "misc", "score"};
  return (kind >= 0 && kind < ET_K_COUNT) ? names[kind] : "?";
}

size_t et_attention_scores_scratch_bytes(int32_t n_frames, int32_t L, int32_t n_heads) {
  if (n_frames < 0 || L < 0 || n_heads < 1) return 0;
  return attention_scores_workspace_bytes(n_frames, L, n_heads);
}

int et_attention_scores(const uint16_t *qkv_dev, int32_t n_frames, int32_t L, int32_t n_heads, int32_t head_dim,
                        void *scratch_dev, float *score_dev, void *hip_stream) {
  ET_REQUIRE(qkv_dev && scratch_dev && score_dev, "a pointer argument is NULL");
  ET_REQUIRE(n_frames >= 0 && L >= 1 && n_heads >= 1 && (int64_t)n_frames * L <= (1 << 24),
             "n_frames = %d, L = %d, n_heads = %d out of range", n_frames, L, n_heads);
  return launch_attention_scores(qkv_dev, n_frames, L, n_heads, head_dim, scratch_dev, score_dev,
                                 static_cast<hipStream_t>(hip_stream));
}

int et_encoder_block_qkv(et_encoder *e, int32_t layer, const uint16_t *x_dev, int32_t rows, float *rstd_dev,
                         uint16_t *qkv_dev, void *hip_stream) {
  ET_REQUIRE(e != nullptr, "encoder is NULL");
  ET_REQUIRE(layer >= 0 && layer < e->cfg.n_layers, "layer = %d outside [0, n_layers = %d)", layer, e->cfg.n_layers);
  ET_REQUIRE(x_dev && rstd_dev && qkv_dev, "a pointer argument is NULL");
  ET_REQUIRE(rows >= 0 && (double)rows * e->D * 3 < 2.0e9, "rows = %d out of range", rows);
  if (rows == 0) return ET_OK;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int D = e->D;
  const LayerDev &lw = e->layers[layer];
  int rc;
  if ((rc = launch_rowstats(x_dev, e->cfg.ln_eps, rows, D, rstd_dev, s))) return rc;
  const GemmArgs g{x_dev, D, lw.wqkv, lw.bqkv, nullptr, 0, 1, qkv_dev, 3 * D, rows, 3 * D, D, EPI_BIAS, rstd_dev};
  return launch_gemm(g, s);
}

int et_layernorm(const uint16_t *x_dev, const float *gamma_dev, const float *beta_dev, float eps,
                 int32_t rows, int32_t D, uint16_t *y_dev, void *hip_stream) {
  ET_REQUIRE(x_dev && gamma_dev && beta_dev && y_dev, "a pointer argument is NULL");
  ET_REQUIRE(rows >= 0 && D >= 8 && D % 8 == 0, "rows = %d, D = %d out of range", rows, D);
  return launch_layernorm(x_dev, gamma_dev, beta_dev, eps, rows, D, y_dev, static_cast<hipStream_t>(hip_stream));
}

int et_attention(const uint16_t *qkv_dev, const int32_t *cu_tokens_dev, int32_t n_frames, int32_t max_len,
                 int32_t n_heads, int32_t head_dim, uint16_t *out_dev, void *hip_stream) {
  ET_REQUIRE(qkv_dev && cu_tokens_dev && out_dev, "a pointer argument is NULL");
  ET_REQUIRE(n_frames >= 0 && max_len >= 0 && n_heads >= 1, "n_frames/max_len/n_heads out of range");
  if (!head_dim_supported(head_dim)) {
    set_error("head_dim = %d is not instantiated (16, 32, 64, 72, 80, 96, 128)", head_dim);
    return ET_ERR_UNSUPPORTED;
  }
  return launch_attention(qkv_dev, cu_tokens_dev, n_frames, max_len, n_heads, head_dim, out_dev,
                          static_cast<hipStream_t>(hip_stream));
}

int et_attention_uniform(const uint16_t *qkv_dev, int32_t n_frames, int32_t len, int32_t n_heads,
                         int32_t head_dim, uint16_t *out_dev, void *hip_stream) {
  ET_REQUIRE(qkv_dev && out_dev, "a pointer argument is NULL");
  ET_REQUIRE(n_frames >= 0 && len >= 0 && n_heads >= 1, "n_frames/len/n_heads out of range");
  if (!head_dim_supported(head_dim)) {
    set_error("head_dim = %d is not instantiated (16, 32, 64, 72, 80, 96, 128)", head_dim);
    return ET_ERR_UNSUPPORTED;
  }
  ET_REQUIRE((double)n_frames * len * n_heads * head_dim * 3 < 2.0e9, "qkv exceeds 2^31 elements");
  if (n_frames == 0 || len == 0) return ET_OK;
  return launch_attention_uniform(qkv_dev, n_frames, len, n_heads, head_dim, out_dev,
                                  static_cast<hipStream_t>(hip_stream));
}

int et_gemm_bf16(const uint16_t *a_dev, const uint16_t *w_dev, const float *bias_dev, const uint16_t *res_dev,
                 int32_t M, int32_t N, int32_t K, int32_t epilogue, int32_t tile_config, uint16_t *c_dev,
                 void *hip_stream) {
  ET_REQUIRE(tile_config >= -1 && tile_config < gemm_config_count(), "tile_config = %d unknown", tile_config);
  ET_REQUIRE(a_dev && w_dev && bias_dev && c_dev, "a pointer argument is NULL");
  ET_REQUIRE(M >= 1 && N >= 8 && K >= 8 && N % 8 == 0 && K % 8 == 0, "M = %d, N = %d, K = %d out of range", M, N, K);
  ET_REQUIRE(epilogue >= 0 && epilogue <= 2, "epilogue = %d unknown", epilogue);
  ET_REQUIRE(epilogue != EPI_BIAS_RES || res_dev, "res_dev is NULL for the residual epilogue");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int Kp = round_up(K, 64), Np = round_up(N, 256);
  uint16_t *a = nullptr, *w = nullptr;
  float *b = nullptr;
  int rc = ET_OK;
  hipError_t he;
  if ((he = hipMalloc((void **)&a, (size_t)M * Kp * 2)) != hipSuccess ||
      (he = hipMalloc((void **)&w, (size_t)Np * Kp * 2)) != hipSuccess ||
      (he = hipMalloc((void **)&b, (size_t)Np * 4)) != hipSuccess) {
    (void)hipGetLastError();
    set_error("device allocation failed in et_gemm_bf16");
    rc = ET_ERR_ALLOC;
  }
  auto step = [&](hipError_t err, const char *what) {
    if (rc == ET_OK && err != hipSuccess) rc = hip_fail(err, what, __FILE__, __LINE__);
  };
  if (rc == ET_OK) {
    step(hipMemsetAsync(a, 0, (size_t)M * Kp * 2, s), "memset a");
    step(hipMemsetAsync(w, 0, (size_t)Np * Kp * 2, s), "memset w");
    step(hipMemsetAsync(b, 0, (size_t)Np * 4, s), "memset bias");
    step(hipMemcpy2DAsync(a, (size_t)Kp * 2, a_dev, (size_t)K * 2, (size_t)K * 2, M, hipMemcpyDeviceToDevice, s), "copy a");
    step(hipMemcpy2DAsync(w, (size_t)Kp * 2, w_dev, (size_t)K * 2, (size_t)K * 2, N, hipMemcpyDeviceToDevice, s), "copy w");
    step(hipMemcpyAsync(b, bias_dev, (size_t)N * 4, hipMemcpyDeviceToDevice, s), "copy bias");
  }
  if (rc == ET_OK) {
    GemmArgs g{a, Kp, w, b, res_dev, N, M, c_dev, N, M, N, Kp, epilogue};
    rc = launch_gemm(g, s, tile_config);
  }
  hipError_t se = hipStreamSynchronize(s);
  if (rc == ET_OK && se != hipSuccess) rc = hip_fail(se, "hipStreamSynchronize", __FILE__, __LINE__);
  if (a) (void)hipFree(a);
  if (w) (void)hipFree(w);
  if (b) (void)hipFree(b);
  return rc;
}

}  // extern "C"
