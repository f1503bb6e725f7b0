// Per-frame top-k by radix select (Eq. 4), shared by the uniform selection (merge_kernels.hip) and
// the decoupled selection (policy_kernels.hip).  Device code only.
#pragma once
#include "et_common.h"

namespace et {

constexpr int kSelThreads = 256;                   // one workgroup of four wavefronts per frame
constexpr int kSelWaves = kSelThreads / kWave;

// Scores are non-negative floats (or NaN), so key = bits + 1 (NaN -> 0) orders them as unsigned
// integers: non-negative finite / infinite floats have bits < 0x7F800001.
__device__ __forceinline__ uint32_t score_key(float z) {
  const uint32_t u = __float_as_uint(z);
  return (z != z) ? 0u : u + 1u;
}

struct SelectShared {
  int hist[256];
  int wave_tot[kSelWaves];
  int eq_tot[2][kSelWaves], gt_tot[2][kSelWaves];   // double-buffered by chunk parity
  uint32_t sel_bin;
  int sel_remaining;
};

// Inclusive prefix sum over the lanes of a wavefront.
__device__ __forceinline__ int wave_inclusive_scan(int v, int lane) {
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int up = __shfl_up(v, o, kWave);
    if (lane >= o) v += up;
  }
  return v;
}

// keys[0..L) (LDS, already staged and visible to the whole workgroup) -> dst[0..k): the k positions
// that come first in the order (key descending, position ascending), written in ascending position.
// Four 8-bit radix passes find the k-th largest key v* and how many keys equal to v* are still
// wanted; per pass a 256-bin histogram (LDS atomics) is suffix-summed by the four wavefronts, 64 bins
// each (shuffle scan inside a wavefront, wavefront totals through LDS).  The emit pass ranks every
// position by two ballots: a kept key's slot is (#greater before it) + min(#equal before it, wanted).
// Must be called by all kSelThreads threads; 1 <= k <= L.
__device__ __forceinline__ void radix_select_emit(const uint32_t *keys, int L, int k, int32_t *dst,
                                                  SelectShared &sh) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint32_t prefix = 0, mask = 0;
  int remaining = k;                     // how many of the keys matching `prefix` are wanted
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    sh.hist[tid] = 0;
    __syncthreads();
    for (int i = tid; i < L; i += kSelThreads) {
      const uint32_t kk = keys[i];
      if ((kk & mask) == prefix) atomicAdd(&sh.hist[(kk >> shift) & 255u], 1);
    }
    __syncthreads();
    // thread t owns bin 255 - t: an inclusive scan in thread order counts the candidates in bins >= its own
    const int mine = sh.hist[255 - tid];
    const int incl_w = wave_inclusive_scan(mine, lane);
    if (lane == kWave - 1) sh.wave_tot[wave] = incl_w;
    __syncthreads();
    int base = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w)
      if (w < wave) base += sh.wave_tot[w];
    const int incl = base + incl_w;      // candidates in bins >= (255 - tid)
    const int above = incl - mine;       // candidates in bins >  (255 - tid)
    if (above < remaining && remaining <= incl) {      // exactly one thread
      sh.sel_bin = 255u - (uint32_t)tid;
      sh.sel_remaining = remaining - above;
    }
    __syncthreads();
    prefix |= sh.sel_bin << shift;
    mask |= 0xFFu << shift;
    remaining = sh.sel_remaining;
  }
  const uint32_t vstar = prefix;
  const int need_eq = remaining;

  int eq_base = 0, gt_base = 0, par = 0;
  for (int i0 = 0; i0 < L; i0 += kSelThreads, par ^= 1) {
    const int i = i0 + tid;
    const uint32_t kk = (i < L) ? keys[i] : 0u;
    const bool gt = (i < L) && kk > vstar;
    const bool eq = (i < L) && kk == vstar;
    const unsigned long long me = __ballot(eq), mg = __ballot(gt);
    const unsigned long long below = (1ull << lane) - 1ull;
    if (lane == 0) {
      sh.eq_tot[par][wave] = __popcll(me);
      sh.gt_tot[par][wave] = __popcll(mg);
    }
    __syncthreads();
    int eq_rank = eq_base + __popcll(me & below), gt_rank = gt_base + __popcll(mg & below);
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
      const int ce = sh.eq_tot[par][w], cg = sh.gt_tot[par][w];
      if (w < wave) { eq_rank += ce; gt_rank += cg; }
      eq_base += ce;
      gt_base += cg;
    }
    if (gt || (eq && eq_rank < need_eq)) dst[gt_rank + (eq_rank < need_eq ? eq_rank : need_eq)] = i;
  }
}

}  // namespace et
