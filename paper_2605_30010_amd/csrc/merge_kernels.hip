// Bandwidth-bound compression kernels for gfx950: adjacent-frame similarity (Sec. 3.2),
// segment-boundary scan (Eq. 1, alpha = 1), per-position segment mean + token score,
// per-frame top-k (Eq. 4) by radix select, and the gather of kept tokens (Eq. 7).
//
// Layout: hidden states x are bf16 [T, L, D] row-major; one 64-lane wavefront owns one
// token row at a time and reads it as 16-byte vectors (8 bf16 per lane, lane-contiguous,
// so every load instruction covers a contiguous 1 KiB).  All reductions run in a fixed
// order (no floating-point atomics), so results are bit-reproducible run to run.
#include "et_common.h"

namespace et {

namespace {

constexpr int kRowsPerBlock = 4;   // wavefronts per workgroup in the row-streaming kernels
constexpr int kSimChunk = 8;       // frame pairs handled by one wavefront before it re-reads a halo row

// ---------------------------------------------------------------------------------------
// Similarity: cos[t-1, l] = <x[t,l], x[t-1,l]> / max(|x[t,l]| |x[t-1,l]|, 1e-8), t = 1..T-1.
// One wavefront = one position l and kSimChunk consecutive pairs; the previous row stays in
// registers, so x is read (kSimChunk+1)/kSimChunk times.
// ---------------------------------------------------------------------------------------
template <int NV>
__global__ __launch_bounds__(kRowsPerBlock * kWave) void similarity_kernel(
    const uint16_t *__restrict__ x, int T, int L, int D, float *__restrict__ cos_out) {
  const int lane = threadIdx.x & 63;
  const int l = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (l >= L) return;
  const int t_first = blockIdx.y * kSimChunk + 1;               // first pair's later frame
  const int t_last = min(t_first + kSimChunk - 1, T - 1);
  if (t_first > t_last) return;
  const size_t frame_stride = (size_t)L * D;
  const uint16_t *p = x + (size_t)(t_first - 1) * frame_stride + (size_t)l * D;

  uint4 raw[NV], raw_next[NV];
  Row<NV> prev, cur;
  load_row<NV>(p, D, lane, raw);
  load_row<NV>(p + frame_stride, D, lane, raw_next);
  unpack_row<NV>(raw, prev);
  float nn_prev = 0.f;
#pragma unroll
  for (int i = 0; i < NV * 8; ++i) nn_prev = fmaf(prev.v[i], prev.v[i], nn_prev);
  nn_prev = wave_sum(nn_prev);

  for (int t = t_first; t <= t_last; ++t) {
#pragma unroll
    for (int j = 0; j < NV; ++j) raw[j] = raw_next[j];
    if (t < t_last) load_row<NV>(p + (size_t)(t - t_first + 2) * frame_stride, D, lane, raw_next);
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
      float den = fmaxf(sqrtf(nn) * sqrtf(nn_prev), 1e-8f);
      cos_out[(size_t)(t - 1) * L + l] = dot / den;
    }
    nn_prev = nn;
#pragma unroll
    for (int i = 0; i < NV * 8; ++i) prev.v[i] = cur.v[i];
  }
}

// ---------------------------------------------------------------------------------------
// s_t = mean_l cos[t-1, l] (fixed-order: lane-strided partial sums, then a butterfly), then
// the boundary scan of Eq. 1 with alpha = 1: frame t opens a segment iff !(s_t >= tau).
// One workgroup; wavefront 0 does the scan with ballots.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void sim_mean_scan_kernel(
    const float *__restrict__ cos_in, int T, int L, float tau, float *__restrict__ sim,
    int32_t *__restrict__ seg_start, int32_t *__restrict__ n_seg, int do_mean, int do_scan) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
  if (do_mean) {
    for (int t = wave; t < T - 1; t += n_waves) {
      const float *row = cos_in + (size_t)t * L;
      float acc = 0.f;
      for (int l = lane; l < L; l += kWave) acc += row[l];
      acc = wave_sum(acc);
      if (lane == 0) sim[t] = acc / (float)L;
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
// One wavefront per (n, l); blockIdx.y runs over the maximum number of segments (T) and
// exits when n >= *n_seg, so no host round trip is needed between scan and merge.
// ---------------------------------------------------------------------------------------
template <int NV>
__global__ __launch_bounds__(kRowsPerBlock * kWave) void segment_mean_kernel(
    const uint16_t *__restrict__ x, int L, int D, const int32_t *__restrict__ seg_start,
    const int32_t *__restrict__ n_seg, uint16_t *__restrict__ merged, float *__restrict__ score) {
  const int n = blockIdx.y;
  if (n >= *n_seg) return;
  const int lane = threadIdx.x & 63;
  const int l = blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
  if (l >= L) return;
  const int a = seg_start[n], b = seg_start[n + 1];
  const size_t frame_stride = (size_t)L * D;
  const uint16_t *p = x + (size_t)a * frame_stride + (size_t)l * D;

  Row<NV> acc, r;
#pragma unroll
  for (int i = 0; i < NV * 8; ++i) acc.v[i] = 0.f;
  uint4 raw0[NV], raw1[NV];
  int t = a;
  for (; t + 1 < b; t += 2) {           // two rows in flight per iteration, added in order
    load_row<NV>(p, D, lane, raw0);
    load_row<NV>(p + frame_stride, D, lane, raw1);
    p += 2 * frame_stride;
    unpack_row<NV>(raw0, r);
#pragma unroll
    for (int i = 0; i < NV * 8; ++i) acc.v[i] += r.v[i];
    unpack_row<NV>(raw1, r);
#pragma unroll
    for (int i = 0; i < NV * 8; ++i) acc.v[i] += r.v[i];
  }
  if (t < b) {
    load_row<NV>(p, D, lane, raw0);
    unpack_row<NV>(raw0, r);
#pragma unroll
    for (int i = 0; i < NV * 8; ++i) acc.v[i] += r.v[i];
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
// Per-frame top-k.  Scores are non-negative floats (or NaN), so key = bits + 1 (NaN -> 0)
// orders them as unsigned integers.  Four 8-bit radix passes find the k-th largest key v*
// and how many keys equal to v* still have to be taken; an ordered ballot compaction then
// emits, in ascending position, every key > v* plus the first `need_eq` keys == v*
// (lowest position wins ties).  One 256-thread workgroup per frame, keys staged in LDS.
// ---------------------------------------------------------------------------------------
constexpr int kSelThreads = 256;

__device__ __forceinline__ uint32_t score_key(float z) {
  uint32_t u = __float_as_uint(z);
  return (z != z) ? 0u : u + 1u;       // non-negative finite/inf floats: bits < 0x7F800001
}

// Exclusive prefix over the workgroup of a per-thread flag, in thread order; also the total.
__device__ __forceinline__ int block_prefix_flag(bool flag, int lane, int wave, int *wave_tot,
                                                 int &total) {
  unsigned long long m = __ballot(flag);
  int before = __popcll(m & ((1ull << lane) - 1ull));
  __syncthreads();                      // wave_tot may still be read from the previous use
  if (lane == 0) wave_tot[wave] = __popcll(m);
  __syncthreads();
  int base = 0;
  total = 0;
#pragma unroll
  for (int w = 0; w < kSelThreads / kWave; ++w) {
    int c = wave_tot[w];
    if (w < wave) base += c;
    total += c;
  }
  return base + before;
}

__global__ __launch_bounds__(kSelThreads) void topk_kernel(
    const float *__restrict__ score, const int32_t *__restrict__ n_rows_dev, int L, int k,
    int32_t *__restrict__ kept, int32_t *__restrict__ cu_tokens) {
  extern __shared__ uint32_t smem[];
  uint32_t *keys = smem;                 // [L]
  __shared__ int hist[256];
  __shared__ int scan[256];
  __shared__ int wave_tot[kSelThreads / kWave];
  __shared__ uint32_t sel_bin;
  __shared__ int sel_remaining;

  const int n = blockIdx.x;
  const int n_rows = n_rows_dev ? *n_rows_dev : (int)gridDim.x;
  if (n >= n_rows) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (cu_tokens && tid == 0) {
    cu_tokens[n] = n * k;
    if (n == 0) cu_tokens[n_rows] = n_rows * k;
  }
  const float *row = score + (size_t)n * L;
  for (int i = tid; i < L; i += kSelThreads) keys[i] = score_key(row[i]);

  uint32_t prefix = 0, mask = 0;
  int remaining = k;                     // how many of the keys matching `prefix` are wanted
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    hist[tid] = 0;
    __syncthreads();                     // also orders the key staging before the first pass
    for (int i = tid; i < L; i += kSelThreads) {
      uint32_t kk = keys[i];
      if ((kk & mask) == prefix) atomicAdd(&hist[(kk >> shift) & 255u], 1);
    }
    __syncthreads();
    // suffix[b] = number of candidates in bins > b  (inclusive scan of the reversed histogram)
    const int mine = hist[255 - tid];
    scan[tid] = mine;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
      int add = (tid >= off) ? scan[tid - off] : 0;
      __syncthreads();
      scan[tid] += add;
      __syncthreads();
    }
    const int incl = scan[tid];          // candidates in bins >= (255 - tid)
    const int above = incl - mine;       // candidates in bins >  (255 - tid)
    if (above < remaining && remaining <= incl) {
      sel_bin = 255u - (uint32_t)tid;
      sel_remaining = remaining - above;
    }
    __syncthreads();
    prefix |= sel_bin << shift;
    mask |= 0xFFu << shift;
    remaining = sel_remaining;
    __syncthreads();
  }
  const uint32_t vstar = prefix;
  const int need_eq = remaining;

  int eq_base = 0, out_base = 0;
  int32_t *dst = kept + (size_t)n * k;
  for (int i0 = 0; i0 < L; i0 += kSelThreads) {
    const int i = i0 + tid;
    const uint32_t kk = (i < L) ? keys[i] : 0u;
    const bool gt = (i < L) && kk > vstar;
    const bool eq = (i < L) && kk == vstar;
    int tot_eq, tot_keep;
    const int eq_rank = eq_base + block_prefix_flag(eq, lane, wave, wave_tot, tot_eq);
    const bool keep = gt || (eq && eq_rank < need_eq);
    const int pos = out_base + block_prefix_flag(keep, lane, wave, wave_tot, tot_keep);
    if (keep) dst[pos] = i;
    eq_base += tot_eq;
    out_base += tot_keep;
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

__global__ void fill_random_bf16_kernel(uint16_t *p, size_t n, uint32_t seed) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    uint32_t h = (uint32_t)i * 2654435761u ^ (seed * 0x9E3779B9u) ^ (uint32_t)(i >> 32);
    h ^= h >> 15; h *= 2246822519u; h ^= h >> 13; h *= 3266489917u; h ^= h >> 16;
    // sign 1 bit, exponent 0x70..0x7E (2^-15 .. 2^-1), mantissa 7 bits
    const uint32_t e = 0x70u + (h >> 8) % 15u;
    p[i] = (uint16_t)(((h & 1u) << 15) | (e << 7) | ((h >> 1) & 0x7Fu));
  }
}

}  // namespace

int launch_similarity(const uint16_t *x, int T, int L, int D, float *cos_out, hipStream_t s) {
  if (T < 2) return ET_OK;
  dim3 grid((L + kRowsPerBlock - 1) / kRowsPerBlock, (T - 1 + kSimChunk - 1) / kSimChunk);
  dim3 block(kRowsPerBlock * kWave);
  ET_DISPATCH_NV(D, hipLaunchKernelGGL(similarity_kernel<NV>, grid, block, 0, s, x, T, L, D, cos_out));
  ET_LAUNCH_CHECK();
  return ET_OK;
}

int launch_sim_mean_scan(const float *cos_in, int T, int L, float tau, float *sim_out,
                         int32_t *seg_start, int32_t *n_seg, bool do_mean, bool do_scan,
                         hipStream_t s) {
  hipLaunchKernelGGL(sim_mean_scan_kernel, dim3(1), dim3(1024), 0, s, cos_in, T, L, tau, sim_out,
                     seg_start, n_seg, do_mean ? 1 : 0, do_scan ? 1 : 0);
  ET_LAUNCH_CHECK();
  return ET_OK;
}

int launch_segment_mean(const uint16_t *x, int T, int L, int D, const int32_t *seg_start,
                        const int32_t *n_seg, uint16_t *merged, float *score, hipStream_t s) {
  dim3 grid((L + kRowsPerBlock - 1) / kRowsPerBlock, T);
  dim3 block(kRowsPerBlock * kWave);
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

int launch_fill_random_bf16(uint16_t *p, size_t n, uint32_t seed, hipStream_t s) {
  if (n == 0) return ET_OK;
  hipLaunchKernelGGL(fill_random_bf16_kernel, dim3(4096), dim3(256), 0, s, p, n, seed);
  ET_LAUNCH_CHECK();
  return ET_OK;
}

int launch_cu_uniform(int n, int step, int32_t *cu, hipStream_t s) {
  hipLaunchKernelGGL(cu_uniform_kernel, dim3((n + 256) / 256), dim3(256), 0, s, n, step, cu);
  ET_LAUNCH_CHECK();
  return ET_OK;
}

}  // namespace et
