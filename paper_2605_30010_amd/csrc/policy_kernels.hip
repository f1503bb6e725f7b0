// Paper-exact compression stage: Eq. 1 with smoothing, Alg. 1 (head and tail of a segment kept,
// middle frames fused pairwise with similarity weights, Eq. 2-3), Alg. 2 (dynamic frames: global
// top-k with the re-scaled count of Eq. 5; static frames: arg-max per local window, Eq. 6) and
// the gather of Eq. 7 with per-frame token counts.
//
// Readings of points the paper leaves open are stated at plan_kernel.  The similarity kernel of
// the simple path is reused; this file adds the sequential plan builder (one lane; the work is
// O(T)), a weighted-range merge, the per-frame selection with two modes and a ragged gather.
#include "select_common.h"

namespace et {

namespace {

constexpr int kRowsPerBlock = 4;

// ---------------------------------------------------------------------------------------
// Plan builder.  info[0] = N output frames, info[1] = segments, info[2] = total kept tokens,
// info[3] = tokens per dynamic frame, info[4] = tokens per static frame.
//  - Eq. 1: s_hat restarts at every segment start (first pair of a segment: s_hat = s_t); a NaN
//    value opens a segment.
//  - Alg. 1: the pair (F_i, F_{i+1}) is eligible only if both are middle frames of the segment;
//    fused with weights s_i / (s_i + s_{i+1}), s_{i+1} / (s_i + s_{i+1}), s_i = Sim(F_i, F_{i+1}).
//  - Eq. 5 (as a count): r_hat = clamp(floor(ratio * T * L / N + 0.5), 1, L).
//  - Eq. 6: w = L / r_hat (integer division), M = ceil(L / w) windows.
// ---------------------------------------------------------------------------------------
__global__ void plan_kernel(const float *__restrict__ sim, int T, int L, PolicyArgs p, int k_uniform,
                            PlanStep st, int32_t *__restrict__ seg_start, int32_t *__restrict__ frame_first,
                            int32_t *__restrict__ frame_count, int32_t *__restrict__ frame_dyn,
                            float *__restrict__ frame_w, int32_t *__restrict__ orig_first,
                            int32_t *__restrict__ orig_count, int32_t *__restrict__ cu_tokens,
                            int32_t *__restrict__ info) {
  // T = current number of frames.  st.do_plan: build segments and output frames from sim (else the
  // identity plan over the T current frames, dynamic flags left as they are).  st.do_counts: token
  // counts and offsets of the selection.  orig_first / orig_count: range of ORIGINAL frames behind
  // each current frame (st.init_orig: identity, first stage), updated in place; seg_start is
  // written in original frame indices.
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  int N = 0;
  if (st.do_plan) {
    int n_seg = 0;
    seg_start[0] = 0;
    float prev = 0.f;
    bool fresh = true;
    for (int t = 1; t < T; ++t) {
      const float sv = sim[t - 1];
      const float cur = fresh ? sv : p.alpha * sv + (1.0f - p.alpha) * prev;
      if (!(cur >= p.tau_seg)) {
        seg_start[++n_seg] = t;
        fresh = true;
      } else {
        prev = cur;
        fresh = false;
      }
    }
    seg_start[++n_seg] = T;
    auto emit = [&](int first, int count, float w0, float w1, int dyn) {
      frame_first[N] = first;
      frame_count[N] = count;
      frame_dyn[N] = dyn;
      frame_w[2 * N] = w0;
      frame_w[2 * N + 1] = w1;
      ++N;
    };
    for (int sgi = 0; sgi < n_seg; ++sgi) {
      const int a = seg_start[sgi], b = seg_start[sgi + 1];
      if (p.merge_mode == ET_MERGE_MEAN) {
        emit(a, b - a, 0.f, 0.f, 1);                 // uniform weights: handled as sum / count
        continue;
      }
      const int k = b - a - 1;
      emit(a, 1, 1.f, 0.f, 1);
      int i = 1;
      while (i < k) {
        const float si = sim[a + i];                 // Sim(F_i, F_{i+1})
        if (i + 1 <= k - 1 && si > p.tau_merge && si > sim[a + i + 1]) {
          const float sj = sim[a + i + 1];
          emit(a + i, 2, si / (si + sj), sj / (si + sj), 0);
          i += 2;
        } else {
          emit(a + i, 1, 1.f, 0.f, 0);
          i += 1;
        }
      }
      if (k >= 1) emit(a + k, 1, 1.f, 0.f, 1);
    }
    // segment starts and frame ranges in original frame indices (ascending, in place: entry n only
    // reads entries >= n)
    for (int i = 0; i < n_seg; ++i) seg_start[i] = st.init_orig ? seg_start[i] : orig_first[seg_start[i]];
    seg_start[n_seg] = st.t_orig;
    for (int n = 0; n < N; ++n) {
      const int f = frame_first[n], l = f + frame_count[n] - 1;
      const int of = st.init_orig ? f : orig_first[f];
      const int oe = st.init_orig ? l + 1 : orig_first[l] + orig_count[l];
      orig_first[n] = of;
      orig_count[n] = oe - of;
    }
    info[1] = n_seg;
  } else {
    N = T;
    for (int n = 0; n < N; ++n) {
      frame_first[n] = n;
      frame_count[n] = 1;
      frame_w[2 * n] = 1.f;
      frame_w[2 * n + 1] = 0.f;
      if (st.init_orig) {
        frame_dyn[n] = 1;
        orig_first[n] = n;
        orig_count[n] = 1;
      }
    }
    if (st.init_orig) {
      for (int i = 0; i <= T; ++i) seg_start[i] = i;
      info[1] = T;
    }
  }
  info[0] = N;
  if (!st.do_counts) return;
  int n_dyn_tok, n_sta_tok;
  if (p.select_mode == ET_SELECT_UNIFORM) {
    n_dyn_tok = n_sta_tok = k_uniform;
  } else {
    double v = floor((double)p.ratio * (double)st.t_orig * (double)L / (double)N + 0.5);
    int r_hat = v < 1.0 ? 1 : (v > (double)L ? L : (int)v);
    const int w = L / r_hat;
    n_dyn_tok = r_hat;
    n_sta_tok = (L + w - 1) / w;
  }
  int total = 0;
  for (int n = 0; n < N; ++n) {
    cu_tokens[n] = total;
    total += (p.select_mode == ET_SELECT_UNIFORM || frame_dyn[n]) ? n_dyn_tok : n_sta_tok;
  }
  cu_tokens[N] = total;
  info[2] = total;
  info[3] = n_dyn_tok;
  info[4] = n_sta_tok;
}

// ---------------------------------------------------------------------------------------
// Weighted-range merge: output frame n = sum over its source frames.  Three cases, all fp32 with
// one rounding to bf16 and the score taken from the unrounded value: a single source frame
// (bit copy), a uniform mean (ascending-t sum divided by the count, exactly the simple path's
// arithmetic), a fused pair w0 x0 + w1 x1 (Eq. 3).
// ---------------------------------------------------------------------------------------
template <int NV>
__global__ __launch_bounds__(kRowsPerBlock * kWave) void plan_merge_kernel(
    const uint16_t *__restrict__ x, int L, int D, const int32_t *__restrict__ info,
    const int32_t *__restrict__ frame_first, const int32_t *__restrict__ frame_count,
    const float *__restrict__ frame_w, int uniform_mean, uint16_t *__restrict__ merged,
    float *__restrict__ score) {
  const int n = blockIdx.y;
  if (n >= info[0]) return;
  const int lane = threadIdx.x & 63;
  const int l = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (l >= L) return;
  const int a = frame_first[n], cnt = frame_count[n];
  const size_t frame_stride = (size_t)L * D;
  const uint16_t *p = x + (size_t)a * frame_stride + (size_t)l * D;
  Row<NV> acc, r;
  uint4 raw[NV];
  if (uniform_mean || cnt == 1) {
#pragma unroll
    for (int i = 0; i < NV * 8; ++i) acc.v[i] = 0.f;
    for (int t = 0; t < cnt; ++t) {
      load_row<NV>(p + (size_t)t * frame_stride, D, lane, raw);
      unpack_row<NV>(raw, r);
#pragma unroll
      for (int i = 0; i < NV * 8; ++i) acc.v[i] += r.v[i];
    }
    const float len = (float)cnt;
#pragma unroll
    for (int i = 0; i < NV * 8; ++i) acc.v[i] = acc.v[i] / len;
  } else {                                           // cnt == 2 by construction
    const float w0 = frame_w[2 * n], w1 = frame_w[2 * n + 1];
    load_row<NV>(p, D, lane, raw);
    unpack_row<NV>(raw, r);
#pragma unroll
    for (int i = 0; i < NV * 8; ++i) acc.v[i] = w0 * r.v[i];
    load_row<NV>(p + frame_stride, D, lane, raw);
    unpack_row<NV>(raw, r);
#pragma unroll
    for (int i = 0; i < NV * 8; ++i) acc.v[i] = fmaf(w1, r.v[i], acc.v[i]);
  }
  float z = 0.f;
  uint16_t *q = merged + ((size_t)n * L + l) * D;
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const float *m = &acc.v[j * 8];
#pragma unroll
    for (int e = 0; e < 8; ++e) z = fmaf(m[e], m[e], z);
    const int c = (j * kWave + lane) * 8;
    if (c < D) {
      uint4 o;
      o.x = pack_bf16x2(m[0], m[1]); o.y = pack_bf16x2(m[2], m[3]);
      o.z = pack_bf16x2(m[4], m[5]); o.w = pack_bf16x2(m[6], m[7]);
      *reinterpret_cast<uint4 *>(q + c) = o;
    }
  }
  z = wave_sum(z);
  if (lane == 0) score[(size_t)n * L + l] = z;
}

// ---------------------------------------------------------------------------------------
// Per-frame selection with ragged output.  Dynamic frames (and every frame in uniform mode): the
// radix select of the simple path (select_common.h) with k = cu[n+1] - cu[n].  Static frames: one thread per local
// window of w consecutive positions, arg-max of the key, lowest position on ties.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSelThreads) void select_policy_kernel(
    const float *__restrict__ score, const int32_t *__restrict__ info, const int32_t *__restrict__ frame_dyn,
    const int32_t *__restrict__ cu_tokens, int L, int all_topk, int32_t *__restrict__ kept) {
  extern __shared__ uint32_t keys[];     // [L]
  __shared__ SelectShared sh;

  const int n = blockIdx.x;
  if (n >= info[0]) return;
  const int tid = threadIdx.x;
  const int out0 = cu_tokens[n], k = cu_tokens[n + 1] - out0;
  const float *row = score + (size_t)n * L;
  for (int i = tid; i < L; i += kSelThreads) keys[i] = score_key(row[i]);
  __syncthreads();
  int32_t *dst = kept + out0;

  if (!all_topk && !frame_dyn[n]) {                  // static frame: local windows (Eq. 6)
    const int r_hat = info[3], w = L / r_hat;
    for (int j = tid; j < k; j += kSelThreads) {
      const int lo = j * w, hi = min(lo + w, L);
      int best = lo;
      uint32_t kb = keys[lo];
      for (int i = lo + 1; i < hi; ++i) {
        const uint32_t ki = keys[i];
        if (ki > kb) { kb = ki; best = i; }
      }
      dst[j] = best;
    }
    return;
  }

  radix_select_emit(keys, L, k, dst, sh);
}

// Gather with per-frame counts: out[cu[n] + j, :] = merged[n, kept[cu[n] + j], :].
__global__ __launch_bounds__(kRowsPerBlock * kWave) void compact_ragged_kernel(
    const uint16_t *__restrict__ merged, const int32_t *__restrict__ kept, const int32_t *__restrict__ info,
    const int32_t *__restrict__ cu_tokens, int L, int D, uint16_t *__restrict__ out) {
  const int n = blockIdx.y;
  if (n >= info[0]) return;
  const int lane = threadIdx.x & 63;
  const int j = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  const int out0 = cu_tokens[n];
  if (j >= cu_tokens[n + 1] - out0) return;
  const size_t orow = (size_t)out0 + j;
  const int l = kept[orow];
  if (l < 0 || l >= L) return;
  const uint4 *src = reinterpret_cast<const uint4 *>(merged + ((size_t)n * L + l) * D);
  uint4 *dst = reinterpret_cast<uint4 *>(out + orow * D);
  for (int c = lane; c < D / 8; c += kWave) dst[c] = src[c];
}

}  // namespace

int launch_plan(const float *sim, int T, int L, const PolicyArgs &p, int k_uniform, const PlanStep &st,
                int32_t *seg_start, int32_t *frame_first, int32_t *frame_count, int32_t *frame_dyn,
                float *frame_w, int32_t *orig_first, int32_t *orig_count, int32_t *cu_tokens, int32_t *info,
                hipStream_t s) {
  hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(64), 0, s, sim, T, L, p, k_uniform, st, seg_start, frame_first,
                     frame_count, frame_dyn, frame_w, orig_first, orig_count, cu_tokens, info);
  ET_LAUNCH_CHECK();
  return ET_OK;
}

int launch_plan_merge(const uint16_t *x, int T, int L, int D, const int32_t *info, const int32_t *frame_first,
                      const int32_t *frame_count, const float *frame_w, bool uniform_mean, uint16_t *merged,
                      float *score, hipStream_t s) {
  dim3 grid((L + kRowsPerBlock - 1) / kRowsPerBlock, T), block(kRowsPerBlock * kWave);
  ET_DISPATCH_NV(D, hipLaunchKernelGGL(plan_merge_kernel<NV>, grid, block, 0, s, x, L, D, info, frame_first,
                                       frame_count, frame_w, uniform_mean ? 1 : 0, merged, score));
  ET_LAUNCH_CHECK();
  return ET_OK;
}

int launch_select_policy(const float *score, int T, const int32_t *info, const int32_t *frame_dyn,
                         const int32_t *cu_tokens, int L, bool all_topk, int32_t *kept, hipStream_t s) {
  if (L > 15360) {
    set_error("tokens per frame %d above the supported 15360", L);
    return ET_ERR_UNSUPPORTED;
  }
  hipLaunchKernelGGL(select_policy_kernel, dim3(T), dim3(kSelThreads), (size_t)L * sizeof(uint32_t), s, score,
                     info, frame_dyn, cu_tokens, L, all_topk ? 1 : 0, kept);
  ET_LAUNCH_CHECK();
  return ET_OK;
}

int launch_compact_ragged(const uint16_t *merged, const int32_t *kept, int T, const int32_t *info,
                          const int32_t *cu_tokens, int L, int D, uint16_t *out, hipStream_t s) {
  dim3 grid((L + kRowsPerBlock - 1) / kRowsPerBlock, T);
  hipLaunchKernelGGL(compact_ragged_kernel, grid, dim3(kRowsPerBlock * kWave), 0, s, merged, kept, info,
                     cu_tokens, L, D, out);
  ET_LAUNCH_CHECK();
  return ET_OK;
}

}  // namespace et
