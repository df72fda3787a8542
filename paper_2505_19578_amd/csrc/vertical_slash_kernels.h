// Search Vertical Slash Pattern (Alg. 5) and its conversion to key-block lists.
#ifndef SP_VERTICAL_SLASH_KERNELS_H
#define SP_VERTICAL_SLASH_KERNELS_H
#include "sp_common.h"
#include "attn_kernel.h"
#include "mask_kernel.h"
#include "global_select_kernels.h"

namespace {

// ---- Search Vertical Slash Pattern (Alg. 5) ------------------------------------------------------
// Q_hat = the last `block` queries.  Their raw dot products with every key go to a workspace slab
// X[b][n][t][s] (fp32), three memory-bound passes turn it into the normalised vertical sums a_v[s] and
// slash sums a_s[t - s], the vector selection above keeps the shortest prefixes reaching gamma, and the kept
// keys / offsets become per-row key-block lists.
struct VsParams {
  const uint16_t *q, *k;
  int64_t q_sb, q_st, q_sh, k_sb, k_st, k_sh;
  int seq, group, n_heads, n_q_heads;
  float c;               // softmax scale * log2(e)
  float *x;              // [b][n][B][seq]
  float *stats;          // [b][n][B][2]  row max (log2 domain) and 1 / row sum
  float *sums;           // [b][n][2][seq] a_v then a_s
  const int32_t *role;   // optional [b][n_q_heads]: only heads whose entry is -1 are processed
  int32_t head_ids[SP_MAX_HEADS];
};
__device__ __forceinline__ bool vs_skip(const VsParams &p, int b, int n) {
  return p.role != nullptr && p.role[(int64_t)b * p.n_q_heads + p.head_ids[n]] != -1;
}

// X = Q_hat K^T with the queries as MFMA rows and the keys as columns, so that one accumulator register
// holds 32 consecutive keys of one query across the lanes and the stores coalesce.  A workgroup takes 128
// keys (32 per wavefront) against all B queries; operands come straight from the caller's Q and K.
template <int D, int B>
__global__ __launch_bounds__(256) void vs_logits_kernel(VsParams p) {
  constexpr int DS = D / 16;
  const int n = blockIdx.y, b = blockIdx.z;
  if (vs_skip(p, b, n)) return;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, h = lane >> 5, c = lane & 31;
  const int head = p.head_ids[n];
  const int s0 = blockIdx.x * 128 + 32 * w;
  if (s0 >= p.seq) return;  // seq is a multiple of 64, not necessarily of 128 (no barrier below)
  const uint16_t *kp = p.k + (int64_t)b * p.k_sb + (int64_t)(s0 + c) * p.k_st + (int64_t)(head / p.group) * p.k_sh + 8 * h;
  bf16x8 kf[DS];
#pragma unroll
  for (int ds = 0; ds < DS; ++ds) kf[ds] = *reinterpret_cast<const bf16x8 *>(kp + 16 * ds);
  float *xo = p.x + (((int64_t)b * p.n_heads + n) * B) * p.seq + s0 + c;
#pragma unroll
  for (int qt = 0; qt < B / 32; ++qt) {
    const uint16_t *qp = p.q + (int64_t)b * p.q_sb + (int64_t)(p.seq - B + 32 * qt + c) * p.q_st +
                         (int64_t)head * p.q_sh + 8 * h;
    f32x16 acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) {
      const bf16x8 qf = *reinterpret_cast<const bf16x8 *>(qp + 16 * ds);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, kf[ds], acc, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int t = 32 * qt + 8 * (r >> 2) + 4 * h + (r & 3);
      xo[(int64_t)t * p.seq] = acc[r];
    }
  }
}

// causal softmax statistics of each of the B query rows: one workgroup per row
template <int B>
__global__ __launch_bounds__(256) void vs_rowstats_kernel(VsParams p) {
  __shared__ float red[4];
  const int t = blockIdx.x, n = blockIdx.y, b = blockIdx.z;
  if (vs_skip(p, b, n)) return;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int last = p.seq - B + t;  // keys 0 .. last exist for this query
  const float *x = p.x + (((int64_t)b * p.n_heads + n) * B + t) * p.seq;
  float mx = -INFINITY;
  for (int s = tid; s <= last; s += 256) mx = fmaxf(mx, x[s]);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
  if (lane == 0) red[w] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3])) * p.c;
  __syncthreads();
  float sum = 0.f;
  for (int s = tid; s <= last; s += 256) sum += fast_exp2(__builtin_fmaf(x[s], p.c, -mx));
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
  if (lane == 0) red[w] = sum;
  __syncthreads();
  if (tid == 0) {
    float *st = p.stats + (((int64_t)b * p.n_heads + n) * B + t) * 2;
    st[0] = mx;
    st[1] = 1.f / (red[0] + red[1] + red[2] + red[3]);
  }
}

// thread i owns key i (vertical sum) and offset i (slash sum); the B queries are added in a fixed order
template <int B>
__global__ __launch_bounds__(256) void vs_sums_kernel(VsParams p) {
  __shared__ float st[B][2];
  const int n = blockIdx.y, b = blockIdx.z;
  if (vs_skip(p, b, n)) return;
  const int64_t hb = (int64_t)b * p.n_heads + n;
  for (int x = threadIdx.x; x < 2 * B; x += 256) st[x >> 1][x & 1] = p.stats[hb * B * 2 + x];
  __syncthreads();
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= p.seq) return;
  const float *x = p.x + hb * B * p.seq;
  const int t0 = p.seq - B;
  float av = 0.f, as = 0.f;
  for (int t = 0; t < B; ++t) {
    const int tabs = t0 + t;
    if (i <= tabs) {
      av += fast_exp2(__builtin_fmaf(x[(int64_t)t * p.seq + i], p.c, -st[t][0])) * st[t][1];
      as += fast_exp2(__builtin_fmaf(x[(int64_t)t * p.seq + (tabs - i)], p.c, -st[t][0])) * st[t][1];
    }
  }
  p.sums[(hb * 2) * p.seq + i] = av * (1.f / B);
  p.sums[(hb * 2 + 1) * p.seq + i] = as * (1.f / B);
}

// Kept keys / offsets -> key-block lists.  flags[b][n][2][nkb] come from the vector selection with rows of
// `block` entries: bit 0 = a kept entry in the row, bit 1 = a kept entry other than the row's first.  Block
// (i, j) holds a kept key iff row j of the vertical flags has bit 0; its token pairs realise the offsets
// (i-j)B - (B-1) .. (i-j)B + (B-1): all of slash row i-j, and slash row i-j-1 without its first entry.
__global__ __launch_bounds__(256) void vs_block_lists_kernel(VsParams p, const int32_t *__restrict__ flags, int nkb,
                                                             int forced, int by_head, int32_t *__restrict__ kb_idx,
                                                             int32_t *__restrict__ kb_cnt) {
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + (threadIdx.x >> 6), n = blockIdx.y, b = blockIdx.z;
  if (i >= nkb || vs_skip(p, b, n)) return;
  const int head = p.head_ids[n], n_heads = p.n_heads, n_q_heads = p.n_q_heads;
  const int32_t *fv = flags + (((int64_t)b * n_heads + n) * 2) * nkb, *fs = fv + nkb;
  // lists are stored per listed position, or per query head when they serve a whole layer
  const int64_t orow = (by_head ? ((int64_t)b * n_q_heads + head) : ((int64_t)b * n_heads + n)) * nkb + i;
  int32_t *out = kb_idx + orow * nkb;
  const uint64_t lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  uint32_t n_out = 0;
  for (int j0 = 0; j0 <= i; j0 += 64) {
    const int j = j0 + lane;
    bool sel = false;
    if (j <= i) {
      const int dlt = i - j;
      sel = (fv[j] & 1) || (fs[dlt] & 1) || (dlt >= 1 && (fs[dlt - 1] & 2)) || (forced && (j == 0 || j == i));
    }
    const uint64_t smask = __ballot(sel);
    if (sel) out[n_out + __popcll(smask & lt)] = j;
    n_out += __popcll(smask);
  }
  for (int pos = n_out + lane; pos < nkb; pos += 64) out[pos] = -1;
  if (lane == 0) kb_cnt[orow] = (int32_t)n_out;
}

}  // namespace

#endif
