// Alg. 2 per query-block row in exact integers.
#ifndef SP_MASK_KERNEL_H
#define SP_MASK_KERNEL_H
#include "sp_common.h"

namespace {

// ---------------------------------------------------------------------------------------------
// mask kernel (Alg. 2 per row, exact integers)
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t wave_sum_u64(uint64_t x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}

__device__ __forceinline__ uint32_t quantise24(float s) {
  // bit tests, so the result does not depend on how the compiler treats NaN comparisons
  const uint32_t bits = __float_as_uint(s);
  if (bits & 0x80000000u) return 0u;         // negative (and -0, -NaN)
  if (bits > 0x7F800000u) return 0u;         // NaN
  if (bits >= 0x3F800000u) return 1u << 24;  // >= 1 (and +inf) clamps to 1
  return (uint32_t)rintf(s * 16777216.f);
}

// One wavefront per (map, row).  EPL > 0: the row lives in registers (nkb <= 64*EPL);
// EPL == 0: any nkb, the row is re-read from memory in every pass.
template <int EPL>
__global__ __launch_bounds__(256) void mask_kernel(const float *__restrict__ scores, int n_rows_total, int nqb,
                                                   int nkb, uint32_t gq, int32_t *__restrict__ kb_idx,
                                                   int32_t *__restrict__ kb_cnt, uint64_t *__restrict__ bitmask,
                                                   const int32_t *__restrict__ route) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= n_rows_total) return;
  const int i = row % nqb;
  // route (optional, [n_maps]): the map whose lists this map's rows become, negative = leave this map out
  int64_t orow = row;
  if (route) {
    const int dst = route[row / nqb];
    if (dst < 0) return;
    orow = (int64_t)dst * nqb + i;
  }
  const float *src = scores + (int64_t)row * nkb;
  const int nchunk = (i >> 6) + 1;  // 64-wide chunks that hold valid key blocks
  uint32_t u[EPL > 0 ? EPL : 1];
  auto get = [&](int e) -> uint32_t {
    if (EPL > 0) return u[e];
    const int j = e * 64 + lane;
    return (j <= i) ? quantise24(src[j]) : 0u;
  };
  if (EPL > 0) {
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      const int j = e * 64 + lane;
      u[e] = (j <= i) ? quantise24(src[j]) : 0u;
    }
  }
  auto sum_ge = [&](uint32_t v) -> uint64_t {
    uint64_t part = 0;
    if (EPL > 0) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) part += (u[e] >= v) ? u[e] : 0u;
    } else {
      for (int e = 0; e < nchunk; ++e) {
        const uint32_t x = get(e);
        part += (x >= v) ? x : 0u;
      }
    }
    return wave_sum_u64(part);
  };
  const uint64_t tot = sum_ge(1u);
  uint32_t vstar = 0xFFFFFFFFu;  // nothing reaches it: only forced blocks when tot == 0
  uint64_t need = 0;
  if (tot > 0) {
    uint64_t T = ((uint64_t)gq * tot + 16777215ull) >> 24;  // least integer prefix sum that reaches gamma
    if (T < 1) T = 1;
    uint32_t lo = 1u, hi = 16777217u;  // sum_ge(lo) >= T > sum_ge(hi)
    while (hi - lo > 1u) {
      const uint32_t mid = lo + ((hi - lo) >> 1);
      if (sum_ge(mid) >= T) lo = mid; else hi = mid;
    }
    vstar = lo;
    const uint64_t above = sum_ge(vstar + 1u);
    need = (T - above + vstar - 1) / vstar;  // ties taken, lowest key block first
  }
  int32_t *out = kb_idx + orow * nkb;
  const int nwords = (nkb + 63) >> 6;
  const uint64_t lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  uint32_t ties_before = 0, n_out = 0;
  const int nch_all = EPL > 0 ? EPL : nwords;
  for (int e = 0; e < nch_all; ++e) {
    if (e >= nwords) break;
    const int j = e * 64 + lane;
    uint32_t x = 0;
    if (EPL > 0) {
#pragma unroll
      for (int ee = 0; ee < EPL; ++ee)
        if (ee == e) x = u[ee];
    } else {
      x = (e < nchunk) ? get(e) : 0u;
    }
    const bool tie = (j <= i) && (x == vstar);
    const uint64_t tmask = __ballot(tie);
    const uint32_t trank = ties_before + __popcll(tmask & lt);
    ties_before += __popcll(tmask);
    const bool sel = (j <= i) && ((x > vstar && vstar != 0xFFFFFFFFu) || (tie && trank < need) || j == 0 || j == i);
    const uint64_t smask = __ballot(sel);
    if (sel) out[n_out + __popcll(smask & lt)] = j;
    n_out += __popcll(smask);
    if (bitmask && lane == 0) bitmask[orow * nwords + e] = smask;
  }
  for (int pos = n_out + lane; pos < nkb; pos += 64) out[pos] = -1;
  if (lane == 0) kb_cnt[orow] = (int32_t)n_out;
}

}  // namespace

#endif
