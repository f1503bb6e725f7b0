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
  uint32_t wave_or[kSelWaves], wave_and[kSelWaves];
  uint32_t sel_bin;
  int sel_remaining;
};

// Cross-lane steps by data-parallel primitives (DPP: the operand of a vector instruction is taken
// from another lane of the same 16-lane row, or broadcast from the last lane of the previous row(s));
// a lane that has no source lane reads 0.  Much shorter latency than the LDS permute the generic
// shuffles go through.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_or_zero(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, false);
}

// Inclusive prefix sum over the lanes of a wavefront: shifts by 1, 2, 4, 8 inside each row of 16
// lanes, then lane 15 of rows 0 and 2 is added to rows 1 and 3, then lane 31 to rows 2 and 3.
__device__ __forceinline__ int wave_inclusive_scan(int v) {
  v += dpp_or_zero<0x111, 0xf>(v);     // row_shr:1
  v += dpp_or_zero<0x112, 0xf>(v);     // row_shr:2
  v += dpp_or_zero<0x114, 0xf>(v);     // row_shr:4
  v += dpp_or_zero<0x118, 0xf>(v);     // row_shr:8
  v += dpp_or_zero<0x142, 0xa>(v);     // row_bcast:15 into rows 1 and 3
  v += dpp_or_zero<0x143, 0xc>(v);     // row_bcast:31 into rows 2 and 3
  return v;
}

// OR over the lanes of a wavefront (same steps; the result is complete in lane 63).
__device__ __forceinline__ uint32_t wave_or_all(uint32_t u) {
  int v = (int)u;
  v |= dpp_or_zero<0x111, 0xf>(v);
  v |= dpp_or_zero<0x112, 0xf>(v);
  v |= dpp_or_zero<0x114, 0xf>(v);
  v |= dpp_or_zero<0x118, 0xf>(v);
  v |= dpp_or_zero<0x142, 0xa>(v);
  v |= dpp_or_zero<0x143, 0xc>(v);
  return (uint32_t)__builtin_amdgcn_readlane(v, 63);
}

// keys[0..L) (LDS, staged by this workgroup; the first barrier inside orders the staging) ->
// dst[0..k): the k positions that come first in the order (key descending, position ascending),
// written in ascending position.  Radix passes of up to 8 bits find the k-th largest key v* and how
// many keys equal to v* are still wanted.  The bits above the highest bit in which any two keys
// differ are skipped (scores of one frame share sign, exponent and often leading mantissa bits: a
// pass over those would send every key to one histogram bin, one LDS atomic after the other).  Per
// pass a histogram (LDS atomics) is suffix-summed by the four wavefronts, 64 bins each (shuffle
// scan inside a wavefront, wavefront totals through LDS).  The emit pass ranks every position by
// two ballots: a kept key's slot is (#greater before it) + min(#equal before it, wanted).
// Must be called by all kSelThreads threads; 1 <= k <= L.  dst may be LDS or global memory.
__device__ __forceinline__ void radix_select_emit(const uint32_t *keys, int L, int k, int32_t *dst,
                                                  SelectShared &sh) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  __syncthreads();
  uint32_t all_or = 0u, all_and = 0xFFFFFFFFu;
  for (int i = tid; i < L; i += kSelThreads) {
    const uint32_t kk = keys[i];
    all_or |= kk;
    all_and &= kk;
  }
  all_or = wave_or_all(all_or);
  all_and = ~wave_or_all(~all_and);                  // AND = NOT (OR of the complements)
  if (lane == 0) { sh.wave_or[wave] = all_or; sh.wave_and[wave] = all_and; }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) { all_or |= sh.wave_or[w]; all_and &= sh.wave_and[w]; }
  const uint32_t diff = all_or ^ all_and;
  const int top = diff ? 32 - __clz(diff) : 0;       // bits [0, top) are to be resolved
  uint32_t mask = top >= 32 ? 0u : ~((1u << top) - 1u);
  uint32_t prefix = all_and & mask;                  // the bits every key shares
  int remaining = k;                                 // how many of the keys matching `prefix` are wanted
  for (int hi = top; hi > 0;) {
    const int lo = hi > 8 ? hi - 8 : 0;
    const uint32_t bmask = (1u << (hi - lo)) - 1u;
    sh.hist[tid] = 0;
    __syncthreads();
    for (int i = tid; i < L; i += kSelThreads) {
      const uint32_t kk = keys[i];
      if ((kk & mask) == prefix) atomicAdd(&sh.hist[(kk >> lo) & bmask], 1);
    }
    __syncthreads();
    // thread t owns bin 255 - t: an inclusive scan in thread order counts the candidates in bins >= its own
    const int mine = sh.hist[255 - tid];
    const int incl_w = wave_inclusive_scan(mine);
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
    prefix |= sh.sel_bin << lo;
    mask |= bmask << lo;
    remaining = sh.sel_remaining;
    hi = lo;
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
