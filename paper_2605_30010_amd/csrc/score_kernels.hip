// Attention-received token scores (Sec. 3.3 / Alg. 2: the "per-token attention scores" A that the
// selection ranks).  The paper does not define how a per-token score is taken from the attention
// maps; this build's reading: score[f][j] = mean over heads h and queries i of
// softmax_h(Q K^T / sqrt(hd))[i][j] inside frame f, i.e. the attention token j RECEIVES.
//
// Three kernels over the q and k thirds of a [frames * L, 3 D] bf16 activation (every frame has L rows):
//   1. row statistics: for every (frame, head, query) the maximum m of the scaled logits (log2
//      domain) and 1 / sum_j exp2(s_j - m), by an online pass over 32-key tiles;
//   2. column sums: for every (frame, head, key) the sum over queries of exp2(s - m_i) / l_i,
//      accumulated in a fixed order inside one wavefront;
//   3. the sum over heads in ascending order, divided by heads * L (no atomics anywhere:
//      bit-reproducible).
// Both compute the logits with v_mfma_f32_32x32x16_bf16 on fragments loaded straight from global
// memory (the operand rows are 16-byte pieces of q / k rows); the head dimension is padded to a
// multiple of 16 with zero fragments.  This runs once per clip, so it is kept simple rather than
// staged through LDS.
#include "et_common.h"

namespace et {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kScoreWaves = 4;
constexpr int kMaxKSteps = 8;        // head_dim <= 128

__device__ __forceinline__ f32x16 mfma_bf16(u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                 0, 0, 0);
}

// 16-byte piece `chunk` (8 head dimensions) of a q / k row; zero past the head dimension.
__device__ __forceinline__ u32x4 load_piece(const uint16_t *row, int chunk, int head_dim) {
  if (chunk * 8 < head_dim) return *reinterpret_cast<const u32x4 *>(row + chunk * 8);
  return u32x4{0u, 0u, 0u, 0u};
}

// Pass 1.  grid (ceil(L / 128), heads, frames), 4 wavefronts, 32 queries per wavefront.
// S^T = K Q^T: keys on the accumulator's row axis, the query on its lane axis, so the running
// maximum and sum are per-lane scalars; the two lane halves see different keys and are combined
// at the end.  stats[(f * H + h) * L + i] = (m_i, 1 / l_i).
template <int KSTEPS>
__global__ __launch_bounds__(kScoreWaves * 64) void attn_rowstats_kernel(
    const uint16_t *__restrict__ qkv, int L, int D, int n_heads, int head_dim, float scale_log2,
    float2 *__restrict__ stats) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r32 = lane & 31, grp = lane >> 5;
  const int h = blockIdx.y, f = blockIdx.z;
  const int q0 = (blockIdx.x * kScoreWaves + wave) * 32;
  if (q0 >= L) return;                                         // wave-uniform
  const size_t row_stride = (size_t)3 * D;
  const uint16_t *frame = qkv + (size_t)f * L * row_stride + (size_t)h * head_dim;
  const int qi = q0 + r32 < L ? q0 + r32 : L - 1;              // clamped: rows past L are computed and dropped
  u32x4 qf[KSTEPS];
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks) qf[ks] = load_piece(frame + (size_t)qi * row_stride, 2 * ks + grp, head_dim);

  float m = -INFINITY, l = 0.f;
  for (int k0 = 0; k0 < L; k0 += 32) {
    const int kj = k0 + r32 < L ? k0 + r32 : L - 1;
    const uint16_t *krow = frame + (size_t)kj * row_stride + D;
    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) acc = mfma_bf16(load_piece(krow, 2 * ks + grp, head_dim), qf[ks], acc);
    float sv[16], tmax = -INFINITY;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int key = k0 + (i / 4) * 8 + 4 * grp + (i % 4);
      sv[i] = key < L ? acc[i] * scale_log2 : -INFINITY;
      tmax = fmaxf(tmax, sv[i]);
    }
    if (tmax > m) {                                            // (a tile of this half with no valid key leaves m alone)
      l *= __builtin_amdgcn_exp2f(m - tmax);                   // exp2(-inf) = 0 on the first tile
      m = tmax;
    }
    if (m > -INFINITY) {
#pragma unroll
      for (int i = 0; i < 16; ++i) l += __builtin_amdgcn_exp2f(sv[i] - m);
    }
  }
  const float m_o = __shfl_xor(m, 32), l_o = __shfl_xor(l, 32);
  const float mt = fmaxf(m, m_o);
  const float lt = (m > -INFINITY ? l * __builtin_amdgcn_exp2f(m - mt) : 0.f) +
                   (m_o > -INFINITY ? l_o * __builtin_amdgcn_exp2f(m_o - mt) : 0.f);
  if (grp == 0 && q0 + r32 < L) stats[((size_t)f * n_heads + h) * L + q0 + r32] = make_float2(mt, 1.0f / lt);
}

// Pass 2.  grid (ceil(L / 128), heads, frames), 4 wavefronts, 32 keys per wavefront; loops over
// 32-query tiles.  S = Q K^T: queries on the accumulator's row axis, the key on its lane axis.
// partial[(f * H + h) * L + j] = sum over queries i of softmax_h[i][j].
template <int KSTEPS>
__global__ __launch_bounds__(kScoreWaves * 64) void attn_colsum_kernel(
    const uint16_t *__restrict__ qkv, int L, int D, int n_heads, int head_dim, float scale_log2,
    const float2 *__restrict__ stats, float *__restrict__ partial) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r32 = lane & 31, grp = lane >> 5;
  const int h = blockIdx.y, f = blockIdx.z;
  const int k0 = (blockIdx.x * kScoreWaves + wave) * 32;       // (a wavefront past the last key computes on clamped rows and stores nothing)
  const size_t row_stride = (size_t)3 * D;
  const uint16_t *head = qkv + (size_t)f * L * row_stride + (size_t)h * head_dim;
  const float2 *st = stats + ((size_t)f * n_heads + h) * L;
  // the four wavefronts see the same 32 queries: their (m, 1/l) pairs go through LDS once per tile
  // instead of 16 scattered loads per lane; two buffers, so one barrier per tile is enough
  __shared__ float2 qstat[2][32];
  const int kj = k0 + r32 < L ? k0 + r32 : L - 1;
  u32x4 kf[KSTEPS];
#pragma unroll
  for (int ks = 0; ks < KSTEPS; ++ks) kf[ks] = load_piece(head + (size_t)kj * row_stride + D, 2 * ks + grp, head_dim);
  float col = 0.f;
  int buf = 0;
  for (int q0 = 0; q0 < L; q0 += 32, buf ^= 1) {
    if (threadIdx.x < 32) {
      const int q = q0 + (int)threadIdx.x;
      qstat[buf][threadIdx.x] = q < L ? st[q] : make_float2(INFINITY, 0.f);  // rows past L: exp2(-inf) * 0 = 0
    }
    const int qi = q0 + r32 < L ? q0 + r32 : L - 1;
    const uint16_t *qrow = head + (size_t)qi * row_stride;
    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KSTEPS; ++ks) acc = mfma_bf16(load_piece(qrow, 2 * ks + grp, head_dim), kf[ks], acc);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float2 ml = qstat[buf][(i / 4) * 8 + 4 * grp + (i % 4)];
      col += __builtin_amdgcn_exp2f(acc[i] * scale_log2 - ml.x) * ml.y;
    }
  }
  col += __shfl_xor(col, 32);
  if (grp == 0 && k0 + r32 < L) partial[((size_t)f * n_heads + h) * L + k0 + r32] = col;
}

// Pass 3: score[f][j] = (sum over heads, ascending, of partial) / (heads * L).
__global__ __launch_bounds__(256) void attn_score_reduce_kernel(const float *__restrict__ partial, int n_frames,
                                                                int L, int n_heads, float *__restrict__ score) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_frames * L) return;
  const int f = idx / L, j = idx - f * L;
  float t = 0.f;
  for (int h = 0; h < n_heads; ++h) t += partial[((size_t)f * n_heads + h) * L + j];
  score[idx] = t / ((float)n_heads * (float)L);
}

}  // namespace

// row statistics (float2) followed by the per-head column sums (float)
size_t attention_scores_workspace_bytes(int n_frames, int L, int n_heads) {
  return (size_t)n_frames * n_heads * L * (sizeof(float2) + sizeof(float));
}

int launch_attention_scores(const uint16_t *qkv, int n_frames, int L, int n_heads, int head_dim, void *stats_ws,
                            float *score, hipStream_t s) {
  if (n_frames <= 0 || L <= 0) return ET_OK;
  ET_REQUIRE(head_dim % 8 == 0 && head_dim >= 8 && head_dim <= kMaxKSteps * 16,
             "head_dim = %d must be a multiple of 8 in [8, %d]", head_dim, kMaxKSteps * 16);
  const int D = n_heads * head_dim;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)head_dim);
  float2 *stats = static_cast<float2 *>(stats_ws);
  float *partial = reinterpret_cast<float *>(stats + (size_t)n_frames * n_heads * L);
  const int blocks = (L + kScoreWaves * 32 - 1) / (kScoreWaves * 32);
  const dim3 g1(blocks, n_heads, n_frames), block(kScoreWaves * 64);
  switch ((head_dim + 15) / 16) {
#define ET_SCORE_CASE(KS)                                                                                           \
  case KS:                                                                                                          \
    hipLaunchKernelGGL(attn_rowstats_kernel<KS>, g1, block, 0, s, qkv, L, D, n_heads, head_dim, scale_log2, stats);  \
    hipLaunchKernelGGL(attn_colsum_kernel<KS>, g1, block, 0, s, qkv, L, D, n_heads, head_dim, scale_log2, stats,     \
                       partial);                                                                                    \
    break;
    ET_SCORE_CASE(1) ET_SCORE_CASE(2) ET_SCORE_CASE(3) ET_SCORE_CASE(4)
    ET_SCORE_CASE(5) ET_SCORE_CASE(6) ET_SCORE_CASE(7) ET_SCORE_CASE(8)
#undef ET_SCORE_CASE
    default: set_error("head_dim = %d unsupported", head_dim); return ET_ERR_INVALID_ARG;
  }
  hipLaunchKernelGGL(attn_score_reduce_kernel, dim3((n_frames * L + 255) / 256), dim3(256), 0, s, partial, n_frames,
                     L, n_heads, score);
  ET_LAUNCH_CHECK();
  return ET_OK;
}

}  // namespace et
