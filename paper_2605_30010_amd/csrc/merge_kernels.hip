// Bandwidth-bound compression kernels for gfx950: adjacent-frame similarity (Sec. 3.2),
// segment-boundary scan (Eq. 1, alpha = 1), per-position segment mean + token score,
// per-frame top-k (Eq. 4) by radix select, and the gather of kept tokens (Eq. 7).
//
// Layout: hidden states x are bf16 [T, L, D] row-major; one 64-lane wavefront owns one
// token row at a time and reads it as 16-byte vectors (8 bf16 per lane, lane-contiguous,
// so every load instruction covers a contiguous 1 KiB).  All reductions run in a fixed
// order (no floating-point atomics), so results are bit-reproducible run to run.
#include "select_common.h"

namespace et {

namespace {

// Wavefronts per workgroup in the row-streaming kernels.  Measured on [64, 729, 1152]: 2, 4 or 8
// per workgroup and 2048 to 8192 wavefronts per launch all give the same time within 2 % (the two
// passes over x run at about 5 TB/s whether x comes from HBM or from the last-level cache: the
// limit is the path between the compute dies and the memory side, not the kernels' shape).
constexpr int kRowsPerBlock = 4;
constexpr int kSimWaves = kRowsPerBlock;
constexpr int kMeanWaves = kRowsPerBlock;

// ---------------------------------------------------------------------------------------
// Similarity: cos[t-1, l] = <x[t,l], x[t-1,l]> / max(|x[t,l]| |x[t-1,l]|, 1e-8), t = 1..T-1.
// One wavefront = one position l and `chunk` consecutive pairs; the previous row stays in
// registers, so x is read (chunk + 1) / chunk times; two further rows are in flight while one
// is reduced.  The workgroup also leaves, per pair, the sum of its kSimWaves cosines in
// part[t-1, blockIdx.x] (added in wavefront order), so that the mean over positions needs
// L / kSimWaves values per pair instead of L (part may be NULL: not written).
// ---------------------------------------------------------------------------------------
constexpr int kSimMaxChunk = 16;

template <int NV>
__global__ __launch_bounds__(kSimWaves * kWave) void similarity_kernel(
    const uint16_t *__restrict__ x, int T, int L, int D, int chunk, float *__restrict__ cos_out,
    float *__restrict__ part) {
  __shared__ float csum[kSimWaves][kSimMaxChunk];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l = blockIdx.x * kSimWaves + wave;
  const int t_first = blockIdx.y * chunk + 1;                   // first pair's later frame
  const int t_last = min(t_first + chunk - 1, T - 1);           // (t_first <= T - 1 by the grid's size)
  if (lane < kSimMaxChunk) csum[wave][lane] = 0.f;              // positions past L add nothing
  if (l < L) {
    const size_t frame_stride = (size_t)L * D;
    const uint16_t *p = x + (size_t)(t_first - 1) * frame_stride + (size_t)l * D;
    uint4 raw[NV], raw1[NV], raw2[NV];
    Row<NV> prev, cur;
    load_row<NV>(p, D, lane, raw);
    load_row<NV>(p + frame_stride, D, lane, raw1);
    if (t_first < t_last) load_row<NV>(p + 2 * frame_stride, D, lane, raw2);
    unpack_row<NV>(raw, prev);
    float nn_prev = 0.f;
#pragma unroll
    for (int i = 0; i < NV * 8; ++i) nn_prev = fmaf(prev.v[i], prev.v[i], nn_prev);
    nn_prev = wave_sum(nn_prev);

    for (int t = t_first; t <= t_last; ++t) {
#pragma unroll
      for (int j = 0; j < NV; ++j) { raw[j] = raw1[j]; raw1[j] = raw2[j]; }
      if (t + 2 <= t_last) load_row<NV>(p + (size_t)(t - t_first + 3) * frame_stride, D, lane, raw2);
      unpack_row<NV>(raw, cur);
      float dot = 0.f, nn = 0.f;
#pragma unroll
      for (int i = 0; i < NV * 8; ++i) {
        dot = fmaf(cur.v[i], prev.v[i], dot);
        nn = fmaf(cur.v[i], cur.v[i], nn);
      }
      dot = wave_sum(dot);
      nn = wave_sum(nn);
      if (lane == 0) {
        const float den = fmaxf(sqrtf(nn) * sqrtf(nn_prev), 1e-8f);
        const float c = dot / den;
        cos_out[(size_t)(t - 1) * L + l] = c;
        csum[wave][t - t_first] = c;
      }
      nn_prev = nn;
#pragma unroll
      for (int i = 0; i < NV * 8; ++i) prev.v[i] = cur.v[i];
    }
  }
  __syncthreads();
  const int i = threadIdx.x;
  if (part && i <= t_last - t_first) {
    float a = csum[0][i];
#pragma unroll
    for (int w = 1; w < kSimWaves; ++w) a += csum[w][i];
    part[(size_t)(t_first - 1 + i) * gridDim.x + blockIdx.x] = a;
  }
}

// ---------------------------------------------------------------------------------------
// s_t = (sum of the n_src values of row t of `src`) / L: src is either the per-workgroup
// partial sums the similarity kernel left (n_src = its grid width) or the cosines themselves
// (n_src = L).  Fixed order: lane-strided partial sums, then a butterfly; one wavefront per
// pair.  Then the boundary scan of Eq. 1 with alpha = 1: frame t opens a segment iff
// !(s_t >= tau).  One workgroup; wavefront 0 does the scan with ballots.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void sim_mean_scan_kernel(
    const float *__restrict__ src, int n_src, int T, int L, float tau, float *__restrict__ sim,
    int32_t *__restrict__ seg_start, int32_t *__restrict__ n_seg, int do_mean, int do_scan) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
  if (do_mean) {
    // a wavefront sums four rows at a time, their loads issued together (the kernel is one round trip
    // to memory per 64 rows when a row has at most 256 values); each row's sum keeps its fixed order
    constexpr int U = 4;
    for (int t0 = wave; t0 < T - 1; t0 += U * n_waves) {
      float acc[U] = {0.f, 0.f, 0.f, 0.f};
      for (int i0 = lane; i0 < n_src; i0 += 4 * kWave) {
        float v[U][4];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int t = t0 + u * n_waves, i = i0 + j * kWave;
            v[u][j] = (t < T - 1 && i < n_src) ? src[(size_t)t * n_src + i] : 0.f;
          }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[u] += v[u][j];
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const float a = wave_sum(acc[u]);
        const int t = t0 + u * n_waves;
        if (lane == 0 && t < T - 1) sim[t] = a / (float)L;
      }
    }
  }
  if (!do_scan) return;
  __threadfence_block();
  __syncthreads();
  if (wave != 0) return;
  int count = 1;
  if (lane == 0) seg_start[0] = 0;
  for (int t0 = 1; t0 < T; t0 += kWave) {
    int t = t0 + lane;
    bool brk = false;
    if (t < T) brk = !(sim[t - 1] >= tau);
    unsigned long long m = __ballot(brk);
    int before = __popcll(m & ((1ull << lane) - 1ull));
    if (brk) seg_start[count + before] = t;
    count += __popcll(m);
  }
  if (lane == 0) {
    seg_start[count] = T;
    *n_seg = count;
  }
}

// ---------------------------------------------------------------------------------------
// Segment mean + score: merged[n, l, :] = (sum over the segment's frames, ascending t, fp32)
// / len, rounded once to bf16; score[n, l] = sum_d mean^2 from the unrounded fp32 mean.
// One wavefront per (n, l), four rows in flight; blockIdx.y runs over the maximum number of
// segments (T) and exits when n >= *n_seg, so no host round trip is needed between scan and merge.
// ---------------------------------------------------------------------------------------
template <int NV>
__global__ __launch_bounds__(kMeanWaves * kWave) void segment_mean_kernel(
    const uint16_t *__restrict__ x, int L, int D, const int32_t *__restrict__ seg_start,
    const int32_t *__restrict__ n_seg, uint16_t *__restrict__ merged, float *__restrict__ score) {
  const int n = blockIdx.y;
  if (n >= *n_seg) return;
  const int lane = threadIdx.x & 63;
  const int l = blockIdx.x * kMeanWaves + (threadIdx.x >> 6);
  if (l >= L) return;
  const int a = seg_start[n], b = seg_start[n + 1];
  const size_t frame_stride = (size_t)L * D;
  const uint16_t *p = x + (size_t)a * frame_stride + (size_t)l * D;

  Row<NV> acc, r;
#pragma unroll
  for (int i = 0; i < NV * 8; ++i) acc.v[i] = 0.f;
  uint4 raw[4][NV];
  int t = a;
  for (; t + 3 < b; t += 4) {           // four rows in flight per iteration, added in ascending t
#pragma unroll
    for (int u = 0; u < 4; ++u) load_row<NV>(p + (size_t)u * frame_stride, D, lane, raw[u]);
    p += 4 * frame_stride;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      unpack_row<NV>(raw[u], r);
#pragma unroll
      for (int i = 0; i < NV * 8; ++i) acc.v[i] += r.v[i];
    }
  }
  {                                     // the last b - t < 4 rows, loaded together
#pragma unroll
    for (int u = 0; u < 3; ++u)
      if (t + u < b) load_row<NV>(p + (size_t)u * frame_stride, D, lane, raw[u]);
#pragma unroll
    for (int u = 0; u < 3; ++u)
      if (t + u < b) {
        unpack_row<NV>(raw[u], r);
#pragma unroll
        for (int i = 0; i < NV * 8; ++i) acc.v[i] += r.v[i];
      }
  }
  const float len = (float)(b - a);
  float z = 0.f;
  uint16_t *q = merged + ((size_t)n * L + l) * D;
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    float m[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      m[e] = acc.v[j * 8 + e] / len;
      z = fmaf(m[e], m[e], z);
    }
    int c = (j * kWave + lane) * 8;
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
// Per-frame top-k: one 256-thread workgroup per frame, keys staged in LDS (select_common.h).
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSelThreads) void topk_kernel(
    const float *__restrict__ score, const int32_t *__restrict__ n_rows_dev, int L, int k,
    int32_t *__restrict__ kept, int32_t *__restrict__ cu_tokens) {
  extern __shared__ uint32_t keys[];     // [L]
  __shared__ SelectShared sh;
  const int n = blockIdx.x;
  const int n_rows = n_rows_dev ? *n_rows_dev : (int)gridDim.x;
  if (n >= n_rows) return;
  const int tid = threadIdx.x;
  if (cu_tokens && tid == 0) {
    cu_tokens[n] = n * k;
    if (n == 0) cu_tokens[n_rows] = n_rows * k;
  }
  const float *row = score + (size_t)n * L;
  for (int i = tid; i < L; i += kSelThreads) keys[i] = score_key(row[i]);
  radix_select_emit(keys, L, k, kept + (size_t)n * k, sh);
}

// ---------------------------------------------------------------------------------------
// Selection and gather in one launch (what the stage runs): gridDim.x workgroups per frame each
// repeat the frame's radix select (a few microseconds on L keys, all in LDS) into an LDS list and
// then copy their share of the kept rows, rows j = blockIdx.x * 4 + wavefront, + 4 gridDim.x, ...:
//   out[n*k + j, :] = merged[n, sel[j], :]   (Eq. 7).
// The repeated select costs nothing in time (the workgroups run side by side), and the gather no
// longer waits for a kernel boundary and a dependent index load.  Workgroup 0 of a frame also
// writes the kept positions and the token offsets.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kSelThreads) void topk_gather_kernel(
    const float *__restrict__ score, const uint16_t *__restrict__ merged, const int32_t *__restrict__ n_rows_dev,
    int L, int D, int k, int32_t *__restrict__ kept, int32_t *__restrict__ cu_tokens, uint16_t *__restrict__ out) {
  extern __shared__ uint32_t smem[];     // keys [L], then the kept positions [k]
  uint32_t *keys = smem;
  int32_t *sel = reinterpret_cast<int32_t *>(smem + L);
  __shared__ SelectShared sh;
  const int n = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // the frame's scores are fetched before the frame count is known (row n < gridDim.y lies inside the
  // score buffer whether or not the frame exists), so that the two loads overlap
  const float *row = score + (size_t)n * L;
  for (int i = tid; i < L; i += kSelThreads) keys[i] = score_key(row[i]);
  const int n_rows = *n_rows_dev;
  if (n >= n_rows) return;
  if (blockIdx.x == 0 && tid == 0) {
    cu_tokens[n] = n * k;
    if (n == 0) cu_tokens[n_rows] = n_rows * k;
  }
  radix_select_emit(keys, L, k, sel, sh);
  __syncthreads();
  if (blockIdx.x == 0)
    for (int j = tid; j < k; j += kSelThreads) kept[(size_t)n * k + j] = sel[j];
  // gather: a wavefront's rows (two with the launcher's grid) are all in flight at once
  const int chunks = D / 8;
  const int stride = 4 * gridDim.x;
  for (int j = blockIdx.x * 4 + wave; j < k; j += 2 * stride) {
    const int j2 = j + stride;
    const int l0 = sel[j], l1 = j2 < k ? sel[j2] : l0;
    const uint4 *s0 = reinterpret_cast<const uint4 *>(merged + ((size_t)n * L + l0) * D);
    const uint4 *s1 = reinterpret_cast<const uint4 *>(merged + ((size_t)n * L + l1) * D);
    uint4 *d0 = reinterpret_cast<uint4 *>(out + ((size_t)n * k + j) * D);
    uint4 *d1 = reinterpret_cast<uint4 *>(out + ((size_t)n * k + j2) * D);
    for (int c = lane; c < chunks; c += 4 * kWave) {
      uint4 v0[4], v1[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (c + u * kWave < chunks) { v0[u] = s0[c + u * kWave]; v1[u] = s1[c + u * kWave]; }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (c + u * kWave < chunks) {
          d0[c + u * kWave] = v0[u];
          if (j2 < k) d1[c + u * kWave] = v1[u];
        }
    }
  }
}

// ---------------------------------------------------------------------------------------
// Gather (Eq. 7): out[n*k + j, :] = merged[n, kept[n*k + j], :].  One wavefront per row.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kRowsPerBlock * kWave) void compact_kernel(
    const uint16_t *__restrict__ merged, const int32_t *__restrict__ kept,
    const int32_t *__restrict__ n_rows_dev, int L, int D, int k, uint16_t *__restrict__ out) {
  const int n = blockIdx.y;
  if (n_rows_dev && n >= *n_rows_dev) return;
  const int lane = threadIdx.x & 63;
  const int j = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (j >= k) return;
  const size_t orow = (size_t)n * k + j;
  const int l = kept[orow];
  if (l < 0 || l >= L) return;           // never follow a corrupt index out of bounds
  const uint4 *src = reinterpret_cast<const uint4 *>(merged + ((size_t)n * L + l) * D);
  uint4 *dst = reinterpret_cast<uint4 *>(out + orow * D);
  for (int c = lane; c < D / 8; c += kWave) dst[c] = src[c];
}

__global__ void identity_maps_kernel(int T, int L, int32_t *kept, int32_t *cu_tokens,
                                     int32_t *seg_start) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < T * L) kept[i] = i % L;
  if (i <= T) {
    cu_tokens[i] = i * L;
    seg_start[i] = i;
  }
}

__global__ void cu_uniform_kernel(int n, int step, int32_t *cu) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i <= n) cu[i] = i * step;
}

}  // namespace

int similarity_blocks(int L) { return (L + kSimWaves - 1) / kSimWaves; }

int launch_similarity(const uint16_t *x, int T, int L, int D, float *cos_out, float *part, hipStream_t s) {
  if (T < 2) return ET_OK;
  // pairs per wavefront: as many as keep about 4096 wavefronts in the grid (x is re-read 1 / chunk times)
  int chunk = (int)(((long long)(T - 1) * L + 4095) / 4096);
  chunk = chunk < 4 ? 4 : (chunk > kSimMaxChunk ? kSimMaxChunk : chunk);
  chunk = (T - 1 + (T - 1 + chunk - 1) / chunk - 1) / ((T - 1 + chunk - 1) / chunk);   // same number of wavefronts, even shares
  dim3 grid(similarity_blocks(L), (T - 1 + chunk - 1) / chunk);
  dim3 block(kSimWaves * kWave);
  ET_DISPATCH_NV(D, hipLaunchKernelGGL(similarity_kernel<NV>, grid, block, 0, s, x, T, L, D, chunk, cos_out, part));
  ET_LAUNCH_CHECK();
  return ET_OK;
}

int launch_sim_mean_scan(const float *src, int n_src, int T, int L, float tau, float *sim_out,
                         int32_t *seg_start, int32_t *n_seg, bool do_mean, bool do_scan,
                         hipStream_t s) {
  hipLaunchKernelGGL(sim_mean_scan_kernel, dim3(1), dim3(1024), 0, s, src, n_src, T, L, tau, sim_out,
                     seg_start, n_seg, do_mean ? 1 : 0, do_scan ? 1 : 0);
  ET_LAUNCH_CHECK();
  return ET_OK;
}

int launch_segment_mean(const uint16_t *x, int T, int L, int D, const int32_t *seg_start,
                        const int32_t *n_seg, uint16_t *merged, float *score, hipStream_t s) {
  dim3 grid((L + kMeanWaves - 1) / kMeanWaves, T);
  dim3 block(kMeanWaves * kWave);
  ET_DISPATCH_NV(D, hipLaunchKernelGGL(segment_mean_kernel<NV>, grid, block, 0, s, x, L, D, seg_start,
                                       n_seg, merged, score));
  ET_LAUNCH_CHECK();
  return ET_OK;
}

int launch_topk(const float *score, int n_rows_max, const int32_t *n_rows_dev, int L, int k,
                int32_t *kept, int32_t *cu_tokens, hipStream_t s) {
  if (L > 15360) {
    set_error("tokens per frame %d above the supported 15360", L);
    return ET_ERR_UNSUPPORTED;
  }
  hipLaunchKernelGGL(topk_kernel, dim3(n_rows_max), dim3(kSelThreads), (size_t)L * sizeof(uint32_t), s,
                     score, n_rows_dev, L, k, kept, cu_tokens);
  ET_LAUNCH_CHECK();
  return ET_OK;
}

int launch_topk_gather(const float *score, const uint16_t *merged, int n_rows_max, const int32_t *n_rows_dev, int L,
                       int D, int k, int32_t *kept, int32_t *cu_tokens, uint16_t *out, hipStream_t s) {
  if (L > 7680) {
    set_error("tokens per frame %d above the 7680 the fused selection supports", L);
    return ET_ERR_UNSUPPORTED;
  }
  int per_frame = (k + 7) / 8;             // workgroups per frame: two rows per wavefront, at most 32 workgroups
  per_frame = per_frame > 32 ? 32 : per_frame;
  hipLaunchKernelGGL(topk_gather_kernel, dim3(per_frame, n_rows_max), dim3(kSelThreads),
                     (size_t)(L + k) * sizeof(uint32_t), s, score, merged, n_rows_dev, L, D, k, kept, cu_tokens, out);
  ET_LAUNCH_CHECK();
  return ET_OK;
}

int launch_compact(const uint16_t *merged, const int32_t *kept, int n_rows_max,
                   const int32_t *n_rows_dev, int L, int D, int k, uint16_t *out, hipStream_t s) {
  dim3 grid((k + kRowsPerBlock - 1) / kRowsPerBlock, n_rows_max);
  hipLaunchKernelGGL(compact_kernel, grid, dim3(kRowsPerBlock * kWave), 0, s, merged, kept,
                     n_rows_dev, L, D, k, out);
  ET_LAUNCH_CHECK();
  return ET_OK;
}

int launch_identity_maps(int T, int L, int32_t *kept, int32_t *cu_tokens, int32_t *seg_start,
                         hipStream_t s) {
  int n = T * L > T + 1 ? T * L : T + 1;
  hipLaunchKernelGGL(identity_maps_kernel, dim3((n + 255) / 256), dim3(256), 0, s, T, L, kept,
                     cu_tokens, seg_start);
  ET_LAUNCH_CHECK();
  return ET_OK;
}

int launch_cu_uniform(int n, int step, int32_t *cu, hipStream_t s) {
  hipLaunchKernelGGL(cu_uniform_kernel, dim3((n + 256) / 256), dim3(256), 0, s, n, step, cu);
  ET_LAUNCH_CHECK();
  return ET_OK;
}

}  // namespace et
