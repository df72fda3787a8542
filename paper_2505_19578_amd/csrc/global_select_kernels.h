// Alg. 2 over a flattened map (or over vectors) in exact integers: histogram passes, tie ranking, list emission.
#ifndef SP_GLOBAL_SELECT_KERNELS_H
#define SP_GLOBAL_SELECT_KERNELS_H
#include "sp_common.h"
#include "mask_kernel.h"

namespace {

// ---- Alg. 2 over the flattened map, exact integers -------------------------------------------
// With u = the 24-bit score, T = ceil(gamma_q * total / 2^24): the kept set is every entry above
// a threshold value v* plus the first `need` entries equal to v* in flat (row-major) order, where v*
// is the largest value with sum_{u >= v*} u >= T.  v* is found by two 12-bit histogram passes
// (sums of u per bin), the ties are ranked by a per-row count and a prefix sum over rows.
constexpr int GS_BINS = 4104;  // 4097 used by the first pass (u can equal 2^24), padded
struct GselState {
  uint64_t T, above, need;
  uint32_t bin_hi, vstar;
  uint32_t pad[8];
};
static_assert(sizeof(GselState) == 64, "GselState layout");

struct GselView {
  unsigned long long *hist1, *hist2;
  GselState *state;
  uint32_t *row_ties, *row_before;
};
// Shape of the maps a selection runs over.  A causal block map is n x n with only j <= row present; a plain
// vector of length n_rows * n_cols is a rectangular map whose row-major order is the vector's order.
struct GselGeom {
  int n_rows, n_cols;
  int tri;              // 1: entries j <= row only; 0: all n_cols entries of a row
  const int32_t *role;  // optional [n_maps / per_head]: a map is processed only if its owner's entry is -1
  int per_head;
};
__device__ __forceinline__ int gsel_width(const GselGeom &g, int row) { return g.tri ? row + 1 : g.n_cols; }
__device__ __forceinline__ bool gsel_skip(const GselGeom &g, int map) {
  return g.role != nullptr && g.role[map / g.per_head] != -1;
}
__host__ __device__ inline size_t gsel_map_bytes(int n_rows) {
  return (size_t)2 * GS_BINS * 8 + sizeof(GselState) + (((size_t)n_rows * 8 + 255) / 256) * 256;
}
__device__ __forceinline__ GselView gsel_view(char *scratch, int map, int nqb) {
  char *base = scratch + (size_t)map * gsel_map_bytes(nqb);
  GselView v;
  v.hist1 = reinterpret_cast<unsigned long long *>(base);
  v.hist2 = v.hist1 + GS_BINS;
  v.state = reinterpret_cast<GselState *>(v.hist2 + GS_BINS);
  v.row_ties = reinterpret_cast<uint32_t *>(v.state + 1);
  v.row_before = v.row_ties + nqb;
  return v;
}

__global__ __launch_bounds__(256) void gsel_zero_kernel(char *scratch, GselGeom g) {
  GselView v = gsel_view(scratch, blockIdx.x, g.n_rows);
  for (int x = threadIdx.x; x < 2 * GS_BINS; x += 256) v.hist1[x] = 0ull;
}

template <int PASS>
__global__ __launch_bounds__(256) void gsel_hist_kernel(const float *__restrict__ scores, GselGeom g, char *scratch) {
  __shared__ unsigned long long h[GS_BINS];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int map = blockIdx.y;
  if (gsel_skip(g, map)) return;
  GselView v = gsel_view(scratch, map, g.n_rows);
  for (int x = tid; x < GS_BINS; x += 256) h[x] = 0ull;
  __syncthreads();
  const uint32_t bin_hi = (PASS == 2) ? v.state->bin_hi : 0u;
  unsigned long long low = 0ull;  // first pass: bin 0 holds most of a softmaxed map; keep it out of the LDS atomics
  for (int row = blockIdx.x * 4 + w; row < g.n_rows; row += gridDim.x * 4) {
    const float *src = scores + ((int64_t)map * g.n_rows + row) * g.n_cols;
    const int width = gsel_width(g, row);
    for (int j = lane; j < width; j += 64) {
      const uint32_t u = quantise24(src[j]);
      if (PASS == 1) {
        const uint32_t bin = u >> 12;
        if (bin == 0)
          low += u;
        else
          atomicAdd(&h[bin], (unsigned long long)u);
      } else if (u != 0u && (u >> 12) == bin_hi) {
        atomicAdd(&h[u & 4095u], (unsigned long long)u);
      }
    }
  }
  if (PASS == 1) {
    low = wave_sum_u64(low);
    if (lane == 0 && low) atomicAdd(&h[0], low);
  }
  __syncthreads();
  unsigned long long *gh = (PASS == 1) ? v.hist1 : v.hist2;
  for (int x = tid; x < GS_BINS; x += 256)
    if (h[x]) atomicAdd(&gh[x], h[x]);
}

// One workgroup of 1024 threads per map.  Thread t owns bins [5t, 5t+5); a suffix sum over threads
// locates the bin in which the running sum from the top first reaches the target.
template <int PASS>
__global__ __launch_bounds__(1024) void gsel_scan_kernel(char *scratch, GselGeom g, uint32_t gq) {
  __shared__ unsigned long long wt[16];
  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  if (gsel_skip(g, blockIdx.x)) return;
  GselView v = gsel_view(scratch, blockIdx.x, g.n_rows);
  const unsigned long long *hist = (PASS == 1) ? v.hist1 : v.hist2;
  constexpr int NB = (PASS == 1) ? 4097 : 4096;
  unsigned long long mine[5], sum = 0ull;
#pragma unroll
  for (int x = 0; x < 5; ++x) {
    const int bin = 5 * t + x;
    mine[x] = (bin < NB) ? hist[bin] : 0ull;
    sum += mine[x];
  }
  unsigned long long incl = sum;  // sum over lanes >= this one
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const unsigned long long y = __shfl_down(incl, off, 64);
    if (lane + off < 64) incl += y;
  }
  if (lane == 0) wt[w] = incl;
  __syncthreads();
  unsigned long long above = incl - sum, tot = 0ull;
  for (int x = 0; x < 16; ++x) {
    tot += wt[x];
    if (x > w) above += wt[x];
  }
  unsigned long long T;
  if (PASS == 1) {
    const unsigned long long th = tot >> 24, tl = tot & 0xFFFFFFull;
    T = (unsigned long long)gq * th + (((unsigned long long)gq * tl + 0xFFFFFFull) >> 24);  // ceil(gq * tot / 2^24)
    if (T < 1) T = 1;
    if (tot == 0ull) {
      if (t == 0) {
        v.state->T = 0;
        v.state->above = 0;
        v.state->need = 0;
        v.state->bin_hi = 0xFFFFFFFFu;
        v.state->vstar = 0xFFFFFFFFu;  // nothing reaches it
      }
      return;
    }
  } else {
    if (v.state->vstar == 0xFFFFFFFFu && v.state->bin_hi == 0xFFFFFFFFu) return;  // empty map
    T = v.state->T - v.state->above;
  }
  if (above < T && T <= above + sum) {  // exactly one thread
    unsigned long long a = above;
    for (int x = 4; x >= 0; --x) {
      if (a + mine[x] >= T) {
        const uint32_t bin = (uint32_t)(5 * t + x);
        if (PASS == 1) {
          v.state->T = T;
          v.state->above = a;
          v.state->bin_hi = bin;
          v.state->vstar = 0u;
        } else {
          const uint32_t vs = (v.state->bin_hi << 12) | bin;
          const unsigned long long gt = v.state->above + a;  // sum of everything above v*
          v.state->vstar = vs;
          v.state->need = (v.state->T - gt + vs - 1) / vs;
        }
        break;
      }
      a += mine[x];
    }
  }
}

__global__ __launch_bounds__(256) void gsel_row_ties_kernel(const float *__restrict__ scores, GselGeom g, char *scratch) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), map = blockIdx.y;
  if (row >= g.n_rows || gsel_skip(g, map)) return;
  GselView v = gsel_view(scratch, map, g.n_rows);
  const uint32_t vstar = v.state->vstar;
  const float *src = scores + ((int64_t)map * g.n_rows + row) * g.n_cols;
  const int width = gsel_width(g, row);
  uint32_t n = 0;
  for (int j = lane; j < width; j += 64) n += (quantise24(src[j]) == vstar) ? 1u : 0u;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) n += __shfl_xor(n, off, 64);
  if (lane == 0) v.row_ties[row] = n;
}

// exclusive prefix sum of row_ties over the rows of one map (flat order = row-major)
__global__ __launch_bounds__(1024) void gsel_row_scan_kernel(GselGeom g, char *scratch) {
  __shared__ uint32_t wt[16];
  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  if (gsel_skip(g, blockIdx.x)) return;
  const int nqb = g.n_rows;
  GselView v = gsel_view(scratch, blockIdx.x, nqb);
  const int per = (nqb + 1023) / 1024;
  const int r0 = t * per, r1 = min(r0 + per, nqb);
  uint32_t sum = 0;
  for (int r = r0; r < r1; ++r) sum += v.row_ties[r];
  uint32_t incl = sum;  // sum over lanes <= this one
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t y = __shfl_up(incl, off, 64);
    if (lane >= off) incl += y;
  }
  if (lane == 63) wt[w] = incl;
  __syncthreads();
  uint32_t before = incl - sum;
  for (int x = 0; x < w; ++x) before += wt[x];
  for (int r = r0; r < r1; ++r) {
    v.row_before[r] = before;
    before += v.row_ties[r];
  }
}

// one wavefront per row: ascending list of the kept key blocks (+ sink and diagonal when forced)
__global__ __launch_bounds__(256) void gsel_emit_kernel(const float *__restrict__ scores, GselGeom g, char *scratch,
                                                        int forced, int32_t *__restrict__ kb_idx,
                                                        int32_t *__restrict__ kb_cnt,
                                                        const int32_t *__restrict__ route) {
  const int lane = threadIdx.x & 63;
  const int nqb = g.n_rows;
  const int i = blockIdx.x * 4 + (threadIdx.x >> 6), map = blockIdx.y;
  if (i >= nqb) return;
  int omap = map;
  if (route) {
    omap = route[map];
    if (omap < 0) return;
  }
  GselView v = gsel_view(scratch, map, nqb);
  const uint32_t vstar = v.state->vstar;
  const uint64_t need = v.state->need;
  const uint64_t before = v.row_before[i];
  const float *src = scores + ((int64_t)map * nqb + i) * nqb;
  int32_t *out = kb_idx + ((int64_t)omap * nqb + i) * nqb;
  const uint64_t lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  uint32_t ties_seen = 0, n_out = 0;
  for (int j0 = 0; j0 <= i; j0 += 64) {
    const int j = j0 + lane;
    const uint32_t x = (j <= i) ? quantise24(src[j]) : 0u;
    const bool tie = (j <= i) && (x == vstar);
    const uint64_t tmask = __ballot(tie);
    const uint64_t trank = before + ties_seen + __popcll(tmask & lt);
    ties_seen += __popcll(tmask);
    const bool sel = (j <= i) && ((x > vstar && vstar != 0xFFFFFFFFu) || (tie && trank < need) ||
                                  (forced && (j == 0 || j == i)));
    const uint64_t smask = __ballot(sel);
    if (sel) out[n_out + __popcll(smask & lt)] = j;
    n_out += __popcll(smask);
  }
  for (int pos = n_out + lane; pos < nqb; pos += 64) out[pos] = -1;
  if (lane == 0) kb_cnt[(int64_t)omap * nqb + i] = (int32_t)n_out;
}

// Selection over plain vectors (rectangular geometry): per (map, row) two flags instead of a list:
// bit 0 = some entry of the row is kept, bit 1 = some entry other than the row's first is kept.  bits (optional,
// n_cols a multiple of 64): the kept set itself, one bit per vector entry, [n_maps][n_rows * n_cols / 64] words.
__global__ __launch_bounds__(256) void gsel_emit_flags_kernel(const float *__restrict__ scores, GselGeom g, char *scratch,
                                                              int32_t *__restrict__ flags,
                                                              uint64_t *__restrict__ bits = nullptr) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), map = blockIdx.y;
  if (row >= g.n_rows || gsel_skip(g, map)) return;
  GselView v = gsel_view(scratch, map, g.n_rows);
  const uint32_t vstar = v.state->vstar;
  const uint64_t need = v.state->need;
  const uint64_t before = v.row_before[row];
  const float *src = scores + ((int64_t)map * g.n_rows + row) * g.n_cols;
  const int width = gsel_width(g, row);
  const uint64_t lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  uint32_t ties_seen = 0;
  int any = 0, any_after_first = 0;
  for (int j0 = 0; j0 < width; j0 += 64) {
    const int j = j0 + lane;
    const uint32_t x = (j < width) ? quantise24(src[j]) : 0u;
    const bool tie = (j < width) && (x == vstar);
    const uint64_t tmask = __ballot(tie);
    const uint64_t trank = before + ties_seen + __popcll(tmask & lt);
    ties_seen += __popcll(tmask);
    const bool sel = (j < width) && ((x > vstar && vstar != 0xFFFFFFFFu) || (tie && trank < need));
    const uint64_t smask = __ballot(sel);
    any |= smask != 0ull;
    any_after_first |= (j0 == 0 ? (smask & ~1ull) : smask) != 0ull;
    if (bits && lane == 0) bits[((int64_t)map * g.n_rows + row) * (g.n_cols / 64) + j0 / 64] = smask;
  }
  if (lane == 0) flags[(int64_t)map * g.n_rows + row] = any | (any_after_first << 1);
}

}  // namespace

#endif
