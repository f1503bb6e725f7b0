/*
 * earlytom.h — C boundary of the MI355X (gfx950) EarlyTom vision-encoder library.
 *
 * The library runs a pre-LayerNorm ViT encoder (SigLIP layout) over the frames of a
 * video clip and applies the paper's early token compression once, inside the encoder:
 * adjacent-frame similarity (Sec. 3.2) -> segment boundaries (Eq. 1, alpha = 1) ->
 * per-position mean over each segment (Sec. 3.2, simplified whole-segment merge) ->
 * per-frame top-k token selection (Eq. 4; score = squared L2 norm, ties to the lower
 * position) -> gather in original order (Eq. 7) -> remaining blocks on the kept tokens.
 *
 * Conventions
 *   - Pointers named *_dev are DEVICE memory owned by the caller; pointers without the
 *     suffix are HOST memory.  The library never frees caller memory and returns nothing
 *     the caller must free, except the opaque encoder (et_encoder_destroy).
 *   - All device activations are bfloat16 (bit patterns, uint16_t), row-major; index and
 *     offset data are int32.
 *   - Every function returning int returns ET_OK (0) or a negative ET_ERR_* code; the
 *     message of the last failure on the calling thread is available from et_last_error().
 *     Arguments are validated before any device work is issued.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *     work is enqueued on it.  One encoder must be used by one stream at a time; different
 *     encoders share no state and may be driven at once from different host threads and streams.
 *   - No exceptions cross this boundary.
 */
#ifndef EARLYTOM_H
#define EARLYTOM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ET_OK 0
#define ET_ERR_INVALID_ARG (-1) /* null pointer, size or parameter out of range          */
#define ET_ERR_WORKSPACE (-2)   /* workspace_bytes smaller than the required size        */
#define ET_ERR_HIP (-3)         /* a HIP runtime call or kernel launch failed            */
#define ET_ERR_ALLOC (-4)       /* host or device allocation failed (create only)        */
#define ET_ERR_UNSUPPORTED (-5) /* a shape the kernels are not instantiated for          */

typedef struct et_encoder et_encoder; /* opaque; owns the packed device weights */

/* Encoder shape.  Tokens per frame L = (image_h / patch) * (image_w / patch); pixels past the
 * last whole patch are ignored.  head_dim = d_model / n_heads must be 16, 32, 64, 72, 80, 96
 * or 128; d_model must be a multiple of 64, at most 4096. */
typedef struct {
  int32_t n_layers, d_model, n_heads, d_mlp, patch, image_h, image_w, channels;
  float ln_eps;
  int32_t has_final_ln;
} et_config;

/* HOST float32 weights, row-major, read only during et_encoder_create (converted once to
 * bfloat16 with round-to-nearest-even; LayerNorm gains/biases and linear biases stay fp32).
 * Linear layers are y = x * W^T + b with W stored out-features major. */
typedef struct {
  const float *patch_w; /* [D, C*P*P], patch vector flattened in (c, py, px) order        */
  const float *patch_b; /* [D]                                                            */
  const float *pos_emb; /* [L, D], token l = gy * (image_w / patch) + gx                  */
  /* per-layer tables: n_layers host pointers each */
  const float *const *ln1_g, *const *ln1_b; /* [D]                                        */
  const float *const *wqkv, *const *bqkv;   /* [3D, D] rows q | k | v; head h = rows h*hd.. */
  const float *const *wo, *const *bo;       /* [D, D], [D]                                */
  const float *const *ln2_g, *const *ln2_b; /* [D]                                        */
  const float *const *w1, *const *b1;       /* [Mh, D], [Mh]                              */
  const float *const *w2, *const *b2;       /* [D, Mh], [D]                               */
  const float *final_ln_g, *final_ln_b;     /* [D]; may be NULL iff !has_final_ln         */
} et_weights;

/* Outputs.  Every *_dev buffer is caller-allocated with the stated capacity (in elements). */
typedef struct {
  uint16_t *tokens_dev;   /* bf16, capacity T*L*D; written [n_tokens, D], frame-major      */
  int32_t *kept_idx_dev;  /* capacity T*L; written [n_tokens]: spatial position l of each
                             output token, ascending inside a frame                        */
  int32_t *cu_tokens_dev; /* capacity T+1; written [n_frames_out+1]: token offset of each
                             output frame                                                  */
  int32_t *seg_start_dev; /* capacity T+1; written [n_frames_out+1]: first input frame of
                             each segment, last entry = T                                  */
  float *frame_sim_dev;   /* capacity max(T-1,1); written s_t for t = 1..T-1; may be NULL  */
  int32_t n_frames_out;   /* HOST, valid on return: number of segments N                   */
  int32_t n_tokens;       /* HOST, valid on return: N * k                                  */
} et_output;

/* ---- the hot path ------------------------------------------------------------------- */

/* Pack `weights` for `config` onto the current HIP device.  max_frames bounds T of later
 * calls.  On success *out receives the encoder.  The two LayerNorms of every block are folded
 * into the QKV and fc1 weights here (gamma scales the weight columns, each folded row is centred
 * so that the row mean of the input drops out, beta goes into the bias), so the blocks compute
 * only the row scale 1 / sqrt(var + eps) and apply it in the GEMM epilogue; the folded weights are
 * rounded to bfloat16 with error diffusion along each row.  Errors: INVALID_ARG, UNSUPPORTED,
 * ALLOC, HIP. */
int et_encoder_create(const et_config *config, const et_weights *weights, int32_t max_frames,
                      et_encoder **out);
void et_encoder_destroy(et_encoder *enc); /* NULL is allowed */

/* Bytes of device workspace et_encode_clip needs for a clip of T frames (0 on bad arguments). */
size_t et_workspace_bytes(const et_encoder *enc, int32_t T);

/* Encode one clip.
 *   frames_dev   float32 [T, C, image_h, image_w] (NCHW), device.
 *   merge_layer  m: compression acts on the residual stream after m blocks have run,
 *                0 <= m <= n_layers (m = n_layers: after the last block, before the final
 *                LayerNorm).  m < 0 disables compression (plain encoder: N = T, k = L).
 *   sim_threshold  tau of Eq. 1: frame t opens a new segment iff s_t < tau (NaN s_t also
 *                opens one).  +INFINITY makes every frame its own segment.  NaN is rejected.
 *   keep_ratio   in (0, 1]; k = et_keep_count(L, keep_ratio) tokens are kept per output frame.
 * The host waits twice: in the middle for an event on `hip_stream` (N is copied to pinned memory
 * of the encoder right after the boundary scan, so the blocks that follow are enqueued while the
 * merge, selection and compaction still run) and for the whole stream before returning.
 * Blocks that run on fewer than 8192 rows (those after the selection) have their weights read
 * ahead by small kernels on a stream the encoder owns (default priority), released by an event on
 * `hip_stream` and joined to it before the call returns; they read encoder memory only.  One
 * encoder therefore serves one encode call at a time.
 * Errors: INVALID_ARG (incl. T < 1 or T > max_frames), WORKSPACE, HIP. */
int et_encode_clip(et_encoder *enc, const float *frames_dev, int32_t T, int32_t merge_layer,
                   float sim_threshold, float keep_ratio, void *workspace_dev,
                   size_t workspace_bytes, void *hip_stream, et_output *out);

/* The compression stage alone on caller-supplied hidden states x_dev (bf16 [T, L, D],
 * D a multiple of 8, T >= 1): similarity, boundary scan, segment mean, top-k, compaction.
 * out->tokens_dev receives the packed merged tokens [N*k, D].  Needs
 * et_merge_workspace_bytes(T, L, D) bytes of workspace.  Synchronises the stream once
 * before returning. */
int et_merge_select(const uint16_t *x_dev, int32_t T, int32_t L, int32_t D, float sim_threshold,
                    float keep_ratio, void *workspace_dev, size_t workspace_bytes,
                    void *hip_stream, et_output *out);
size_t et_merge_workspace_bytes(int32_t T, int32_t L, int32_t D);

/* et_merge_select for callers that cannot allocate or hand over a workspace (a stage under HIP graph
 * capture set-up, a tight serving loop, a harness that forbids hipMalloc): same arguments minus the
 * workspace, same kernels, same results bit for bit.  The scratch the kernels need (cosines, their
 * partial sums, scores, the merged frames, counters) lives in a device array that is part of the
 * library's code object, ET_STATIC_SCRATCH_BYTES large, one copy per GPU for the life of the process;
 * its address is looked up once per device, on the first call there.  The call allocates nothing and
 * frees nothing.  Shapes with et_merge_workspace_bytes(T, L, D) above ET_STATIC_SCRATCH_BYTES (e.g. more
 * than 39 frames of 729 x 1152) are rejected with ET_ERR_WORKSPACE before any device work.  Every call
 * on a GPU uses that GPU's one array: calls that overlap on one GPU (from several threads or streams)
 * race; nothing in it has to start at zero, so a call is not affected by what the previous one left.
 * Synchronises the stream once before returning, like et_merge_select. */
#define ET_STATIC_SCRATCH_BYTES (64u << 20)
int et_merge_select_static(const uint16_t *x_dev, int32_t T, int32_t L, int32_t D, float sim_threshold,
                           float keep_ratio, void *hip_stream, et_output *out);

/* k = clamp(floor(keep_ratio * L + 1e-4), 1, L); 0 on bad arguments.  (The paper floors
 * window sizes in Eq. 6 but does not state the rounding for top-K; this rule is this
 * library's reading.) */
int32_t et_keep_count(int32_t L, float keep_ratio);

const char *et_last_error(void); /* thread-local, never NULL */

/* ---- the paper-exact compression forms -------------------------------------------------
 * A policy selects, per stage, between the simple form used by et_encode_clip / et_merge_select
 * and the form the paper describes:
 *   merge_mode   ET_MERGE_MEAN: a segment becomes one frame (per-position mean).
 *                ET_MERGE_ALG1: Alg. 1 — head and tail frame of a segment are kept, middle frames
 *                are walked left to right and (F_i, F_{i+1}) are fused with weights
 *                (s_i, s_{i+1}) / (s_i + s_{i+1}) iff s_i > tau_merge and s_i > s_{i+1} (Eq. 2-3),
 *                s_i = Sim(F_i, F_{i+1}); a pair is eligible only if both are middle frames.
 *   select_mode  ET_SELECT_UNIFORM: every output frame keeps k = et_keep_count(L, ratio) tokens.
 *                ET_SELECT_DECOUPLED: Alg. 2 — head/tail ("dynamic") frames keep the top r_hat
 *                tokens, r_hat = clamp(floor(ratio*T*L/N + 0.5), 1, L) (this library's reading of
 *                Eq. 5: `ratio` is the overall retention relative to the T*L input tokens); other
 *                ("static") frames keep the arg-max of each of ceil(L / w) windows of
 *                w = floor(L / r_hat) consecutive positions (Eq. 6).
 *   alpha        smoothing factor of Eq. 1 in (0, 1]; the smoothed similarity restarts at every
 *                segment start.  tau_seg: segment threshold.  tau_merge: Eq. 2 threshold.
 *   score_mode   ET_SCORE_L2NORM: a token's score is its squared L2 norm (as on the simple path).
 *                ET_SCORE_ATTENTION: the attention the token receives in the encoder block just
 *                before the selection (Sec. 3.3 and Alg. 2 rank by a score per token taken from the
 *                encoder's attention without defining it; this library's reading): the mean over heads and over the queries
 *                of its frame of softmax(Q K^T / sqrt(hd))[query][token].  Needs a block before
 *                the selection (select layer >= 1) whose input is what the selection sees, so no
 *                merge may run at the select layer itself; only et_encode_clip_multi accepts it.
 * Tie-breaks and ordering are those of the simple path.  With these forms output frames
 * keep different token counts: cu_tokens_dev is ragged, seg_start_dev has n_segments + 1 entries
 * and n_frames_out counts output frames (>= segments). */
enum { ET_MERGE_MEAN = 0, ET_MERGE_ALG1 = 1 };
enum { ET_SELECT_UNIFORM = 0, ET_SELECT_DECOUPLED = 1 };
enum { ET_SCORE_L2NORM = 0, ET_SCORE_ATTENTION = 1 };
typedef struct {
  int32_t merge_mode, select_mode;
  float alpha, tau_seg, tau_merge, ratio;
  int32_t score_mode;
} et_policy;

/* Optional description of the output frames (device arrays of capacity T, or NULL). */
typedef struct {
  int32_t *frame_first_dev;   /* first ORIGINAL input frame behind output frame n              */
  int32_t *frame_count_dev;   /* number of consecutive original frames behind it               */
  int32_t *frame_dynamic_dev; /* 1 = head or tail frame of its segment ("dynamic"), 0 = static */
  int32_t n_segments;         /* HOST, valid on return                                         */
} et_plan_out;

/* et_merge_select / et_encode_clip under a policy.  Same buffers, workspace sizes and
 * synchronisation as the simple entry points; `plan` may be NULL.  Errors as there, plus
 * INVALID_ARG for alpha outside (0, 1], NaN thresholds, ratio outside (0, 1] or unknown modes. */
int et_merge_select_policy(const uint16_t *x_dev, int32_t T, int32_t L, int32_t D, const et_policy *policy,
                           void *workspace_dev, size_t workspace_bytes, void *hip_stream, et_output *out,
                           et_plan_out *plan);
int et_encode_clip_policy(et_encoder *enc, const float *frames_dev, int32_t T, int32_t merge_layer,
                          const et_policy *policy, void *workspace_dev, size_t workspace_bytes,
                          void *hip_stream, et_output *out, et_plan_out *plan);

/* ---- per-kernel timing (optional) ----------------------------------------------------
 * With profiling on, et_encode_clip brackets every kernel launch with HIP events on
 * `hip_stream` and accumulates elapsed time and launch counts per kernel kind.  Off by
 * default (events cost a little host time). */
enum {
  ET_K_IM2COL = 0, ET_K_GEMM_PATCH, ET_K_LAYERNORM, ET_K_GEMM_QKV, ET_K_ATTENTION,
  ET_K_GEMM_OUT, ET_K_GEMM_FC1, ET_K_GEMM_FC2, ET_K_SIMILARITY, ET_K_SCAN, ET_K_MERGE,
  ET_K_SELECT, ET_K_COMPACT, ET_K_MISC, ET_K_SCORE, ET_K_COUNT
};
int et_profile_enable(et_encoder *enc, int32_t on);
/* Reads the accumulators into ms[2 * ET_K_COUNT] and launches[2 * ET_K_COUNT]: entry
 * kind + ET_K_COUNT * phase, phase 0 = launches on all T*L tokens (up to and including the
 * compression stage), phase 1 = launches on the kept tokens; clears them if `reset` != 0. */
int et_profile_read(et_encoder *enc, double *ms, int64_t *launches, int32_t reset);
const char *et_kernel_name(int32_t kind);
/* The same for the stand-alone stage: with on = 1, et_merge_select and et_merge_select_static bracket
 * the whole launch sequence with two HIP events on `hip_stream`; with on = 2 also every launch (which
 * lengthens the sequence by the events' own cost).  The read fills
 * ms[ET_K_COUNT] / launches[ET_K_COUNT] per kernel kind, *total_ms with the summed time between the
 * first launch's start and the last launch's end (launch gaps included, the final device-to-host copy
 * and stream wait excluded) and *calls.  Process-wide state, not thread-safe; off by default. */
int et_merge_profile_enable(int32_t on);
int et_merge_profile_read(double *ms, int64_t *launches, double *total_ms, int64_t *calls, int32_t reset);

/* ---- single steps (the device code of the hot path, one step per call; for parity tests and
 *      micro-benchmarks).  All asynchronous on `hip_stream` unless stated.  The hot path itself runs
 *      selection and gather (et_topk_select + et_compact_tokens) as ONE launch on the same select
 *      routine; the two calls below launch them separately. ------------- */

/* Sec. 3.2: cos_dev [T-1, L] float32 per-position cosine similarities of frames t and t-1,
 * sim_dev [T-1] their mean over positions.  x_dev bf16 [T, L, D]. */
int et_frame_similarity(const uint16_t *x_dev, int32_t T, int32_t L, int32_t D, float *cos_dev,
                        float *sim_dev, void *hip_stream);

/* Eq. 1 (alpha = 1): seg_start_dev [capacity T+1] and *n_seg_dev (one int32) from sim_dev [T-1]. */
int et_segment_scan(const float *sim_dev, int32_t T, float sim_threshold, int32_t *seg_start_dev,
                    int32_t *n_seg_dev, void *hip_stream);

/* Segment mean and score: merged_dev bf16 [N, L, D] (capacity T*L*D), score_dev float32
 * [N, L] (capacity T*L); N and the ranges are read from the device arrays. */
int et_segment_mean(const uint16_t *x_dev, int32_t T, int32_t L, int32_t D,
                    const int32_t *seg_start_dev, const int32_t *n_seg_dev, uint16_t *merged_dev,
                    float *score_dev, void *hip_stream);

/* Eq. 4: for each of n_rows rows of score_dev [n_rows, L] (float32, non-negative or NaN), the
 * k positions that come first in the order (score descending, position ascending), written
 * ascending to kept_idx_dev [n_rows, k]. */
int et_topk_select(const float *score_dev, int32_t n_rows, int32_t L, int32_t k,
                   int32_t *kept_idx_dev, void *hip_stream);

/* Eq. 7: out_dev[(n*k + j), :] = merged_dev[n, kept_idx_dev[n*k + j], :], n < n_rows. */
int et_compact_tokens(const uint16_t *merged_dev, const int32_t *kept_idx_dev, int32_t n_rows,
                      int32_t L, int32_t D, int32_t k, uint16_t *out_dev, void *hip_stream);

/* LayerNorm over rows: y = (x - mean) / sqrt(var + eps) * gamma + beta; x, y bf16 [rows, D]
 * (may alias), gamma/beta float32 [D] on the device. */
int et_layernorm(const uint16_t *x_dev, const float *gamma_dev, const float *beta_dev, float eps,
                 int32_t rows, int32_t D, uint16_t *y_dev, void *hip_stream);

/* C[M, N] = A[M, K] * W[N, K]^T + bias, bf16 in / fp32 accumulate / bf16 out, with an
 * epilogue: 0 bias only, 1 bias + GELU-tanh, 2 bias + residual (res_dev bf16 [M, N], may
 * alias c_dev).  bias_dev float32 [N].  Standalone form for tests: any M >= 1, N and K
 * multiples of 8; allocates and frees padded copies of the operands itself and synchronises.
 * tile_config: -1 = the library's choice (which may also split a thin last tile row or column
 * off into a launch of its own), else one workgroup tiling of the persistent kernel:
 * 0 = 256 x 256 x 64 with 8 wavefronts, 1 = 128 x 128 x 64 and 2 = 64 x 128 x 64 with 4. */
int et_gemm_bf16(const uint16_t *a_dev, const uint16_t *w_dev, const float *bias_dev,
                 const uint16_t *res_dev, int32_t M, int32_t N, int32_t K, int32_t epilogue,
                 int32_t tile_config, uint16_t *c_dev, void *hip_stream);

/* Per-frame multi-head attention on a fused projection buffer qkv_dev bf16 [rows, 3D]
 * (q | k | v, head h at columns h*hd): out_dev bf16 [rows, D].  cu_tokens_dev [n_frames+1]
 * gives each frame's row range; max_len >= the longest frame. */
int et_attention(const uint16_t *qkv_dev, const int32_t *cu_tokens_dev, int32_t n_frames,
                 int32_t max_len, int32_t n_heads, int32_t head_dim, uint16_t *out_dev,
                 void *hip_stream);

/* The same attention for frames of equal length `len` (frame f = rows f*len .. f*len+len-1),
 * which is what the hot path runs; same kernel (K tiles stream through LDS by direct global -> LDS
 * loads, V^T fragments by LDS transpose reads), and with enough frames a wavefront owns two blocks
 * of 32 queries. */
int et_attention_uniform(const uint16_t *qkv_dev, int32_t n_frames, int32_t len, int32_t n_heads,
                         int32_t head_dim, uint16_t *out_dev, void *hip_stream);

/* The first two launches of encoder block `layer` on caller-supplied hidden states x_dev (bf16
 * [rows, D]), exactly as et_encode_clip issues them: the row scales 1 / sqrt(var + eps) of
 * LayerNorm 1 into rstd_dev (float32 [rows]) and the fused projection with the LayerNorm folded in
 * into qkv_dev (bf16 [rows, 3D], q | k | v).  Lets a test rank attention-received scores on the very
 * q and k the encoder used.  Errors: INVALID_ARG, HIP. */
int et_encoder_block_qkv(et_encoder *enc, int32_t layer, const uint16_t *x_dev, int32_t rows,
                         float *rstd_dev, uint16_t *qkv_dev, void *hip_stream);

/* Stage I at several encoder layers, Stage II once (the paper merges at three layers, e.g. 6, 14,
 * 20, and selects after the encoder; Table 8).  At every layer of merge_layers[0..n_merge_layers)
 * (strictly ascending, each <= select_layer) the adjacent-frame similarity of the CURRENT frames
 * drives Eq. 1 and the merge of policy->merge_mode; frames keep all L tokens.  At select_layer
 * (after that layer's merge if they coincide) the selection of policy->select_mode runs once:
 * dynamic flags come from the most recent merge (all frames dynamic if n_merge_layers = 0), the
 * re-scaled count of Eq. 5 uses the original T.  seg_start_dev and the plan's frame ranges are in
 * original frame indices.  Synchronises the stream once per merge / select layer and at the end;
 * frame_sim_dev receives the similarities of the first merge layer only. */
int et_encode_clip_multi(et_encoder *enc, const float *frames_dev, int32_t T, const int32_t *merge_layers,
                         int32_t n_merge_layers, int32_t select_layer, const et_policy *policy,
                         void *workspace_dev, size_t workspace_bytes, void *hip_stream, et_output *out,
                         et_plan_out *plan);

/* Attention-received scores (ET_SCORE_ATTENTION) of equal-length frames: score_dev float32
 * [n_frames, L], each row summing to 1, from the q and k thirds of qkv_dev bf16 [n_frames * L,
 * 3 * n_heads * head_dim] (the layout et_attention reads).  scratch_dev: at least
 * et_attention_scores_scratch_bytes(n_frames, L, n_heads) bytes.  head_dim a multiple of 8, <= 128. */
size_t et_attention_scores_scratch_bytes(int32_t n_frames, int32_t L, int32_t n_heads);
int et_attention_scores(const uint16_t *qkv_dev, int32_t n_frames, int32_t L, int32_t n_heads,
                        int32_t head_dim, void *scratch_dev, float *score_dev, void *hip_stream);

/* ---- the projector that follows the encoder (Sec. 3.1: vision encoder -> projector -> language
 *      model) -------------------------------------------------------------------------------------
 * A two-layer MLP on the kept tokens, out = W2 * gelu_tanh(W1 * x + b1) + b2, so that the time of
 * encoder plus everything done to the visual tokens can be taken as one figure when the selection sits after the
 * encoder (merge_layer = n_layers, where the paper places Stage II).  The paper does not describe the
 * projector; the two-layer form and the GELU are this library's reading, the widths are arguments.
 * Weights: HOST float32, out-features major (w1 [d_hidden, d_in], w2 [d_out, d_hidden]), converted once
 * to bfloat16.  d_in a multiple of 64; d_hidden and d_out multiples of 8. */
typedef struct et_projector et_projector;
int et_projector_create(int32_t d_in, int32_t d_hidden, int32_t d_out, const float *w1, const float *b1,
                        const float *w2, const float *b2, et_projector **out);
void et_projector_destroy(et_projector *proj); /* NULL is allowed */
size_t et_projector_workspace_bytes(const et_projector *proj, int32_t rows);
/* tokens_dev bf16 [rows, d_in] -> out_dev bf16 [rows, d_out]; asynchronous on `hip_stream`.
 * Errors: INVALID_ARG, WORKSPACE, HIP. */
int et_project_tokens(et_projector *proj, const uint16_t *tokens_dev, int32_t rows, void *workspace_dev,
                      size_t workspace_bytes, uint16_t *out_dev, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* EARLYTOM_H */
