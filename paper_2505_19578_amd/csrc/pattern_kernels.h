// Block-mean-logit score map (Sec. 5.2), last-row estimates, the Jensen-Shannon gate of Alg. 3 and pivot election (Alg. 1).
#ifndef SP_PATTERN_KERNELS_H
#define SP_PATTERN_KERNELS_H
#include "sp_common.h"
#include "attn_kernel.h"
#include "mask_kernel.h"

namespace {

// ---------------------------------------------------------------------------------------------
// pattern construction as printed in the paper (Sec. 5.2 "Sparse Attention Computation" and
// "Pivotal Pattern Construction"; Alg. 2): block-mean logits -> row softmax -> one selection over
// the flattened, globally normalised map
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_float(uint16_t x) { return __uint_as_float((uint32_t)x << 16); }

struct PoolParams {
  const uint16_t *q, *k;
  int64_t q_sb, q_st, q_sh, k_sb, k_st, k_sh;
  int nqb, group, n_heads, n_kv_heads;
  int row0, n_rows;  // query-block rows row0 .. row0 + n_rows - 1 are wanted
  float *qsum;       // [b][n][n_rows][D]   sum of the block's queries
  float *ksumT;      // [b][kvh][D][nqb]    sum of the block's keys, block index fastest
  float *diag;       // [b][n][n_rows]      sum over the diagonal block's causal entries of q_t . k_s
  float *out;        // [b][n][n_rows][nqb] row softmax of the block-mean logits
  float c_full, c_diag;
  const int32_t *head_dev;  // optional [b][n_heads]: head of listed position n chosen on the device, < 0 = empty
  int32_t head_ids[SP_MAX_HEADS];
};
__device__ __forceinline__ int pool_head(const PoolParams &p, int b, int n) {
  return p.head_dev ? p.head_dev[(int64_t)b * p.n_heads + n] : p.head_ids[n];
}

// The average of q_t . k_s over a full block is (sum_t q_t) . (sum_s k_s) / B^2, so the block-mean
// logits need only per-block sums of Q and K.  One thread per head dimension, one block per workgroup.
template <int D, int B>
__global__ __launch_bounds__(D) void key_pool_kernel(PoolParams p) {
  const int i = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z, e = threadIdx.x;
  const uint16_t *kp = p.k + (int64_t)b * p.k_sb + (int64_t)i * B * p.k_st + (int64_t)kvh * p.k_sh + e;
  float run = 0.f;
#pragma unroll 8
  for (int t = 0; t < B; ++t) run += bf16_bits_to_float(kp[(int64_t)t * p.k_st]);
  p.ksumT[(((int64_t)b * p.n_kv_heads + kvh) * D + e) * p.nqb + i] = run;
}

// Query sums of the wanted rows and, for the diagonal block (which keeps s <= t only), the sum
// sum_t q_t . (sum_{s<=t} k_s) from a running key sum walked once.
template <int D, int B>
__global__ __launch_bounds__(D) void query_pool_kernel(PoolParams p) {
  const int r = blockIdx.x, n = blockIdx.y, b = blockIdx.z, e = threadIdx.x;
  const int i = p.row0 + r;
  const int head = pool_head(p, b, n);
  if (head < 0) return;
  const uint16_t *qp = p.q + (int64_t)b * p.q_sb + (int64_t)i * B * p.q_st + (int64_t)head * p.q_sh + e;
  const uint16_t *kp = p.k + (int64_t)b * p.k_sb + (int64_t)i * B * p.k_st + (int64_t)(head / p.group) * p.k_sh + e;
  float run = 0.f, qs = 0.f, acc = 0.f;
#pragma unroll 8
  for (int t = 0; t < B; ++t) {
    const float kk = bf16_bits_to_float(kp[(int64_t)t * p.k_st]);
    const float qq = bf16_bits_to_float(qp[(int64_t)t * p.q_st]);
    run += kk;
    qs += qq;
    acc = fmaf(qq, run, acc);
  }
  const int64_t hr = ((int64_t)b * p.n_heads + n) * p.n_rows + r;
  p.qsum[hr * D + e] = qs;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
  if constexpr (D == 64) {
    if (e == 0) p.diag[hr] = acc;
  } else {
    __shared__ float part[D / 64];
    if ((e & 63) == 0) part[e >> 6] = acc;
    __syncthreads();
    if (e == 0) {
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < D / 64; ++w) s += part[w];
      p.diag[hr] = s;
    }
  }
}

// Four query-block rows per workgroup: thread j forms the four pooled dot products against key block j
// (block index fastest in ksumT, so the loads coalesce), then one wavefront per row applies the row
// softmax in place (Alg. 2, first step; Alg. 3's estimate when only the last row is asked for).
// Entries beyond the diagonal are written as 0.
template <int D>
__global__ __launch_bounds__(256) void mean_logit_softmax_kernel(PoolParams p) {
  constexpr int R = 4;
  __shared__ float qs[R][D];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int r0 = blockIdx.x * R;
  const int64_t hb = blockIdx.y;
  const int b = (int)(hb / p.n_heads), n = (int)(hb % p.n_heads);
  const int nqb = p.nqb;
  const int head = pool_head(p, b, n);
  if (head < 0) return;
  for (int x = tid; x < R * D; x += 256) {
    const int r = x / D, e = x % D;
    qs[r][e] = (r0 + r < p.n_rows) ? p.qsum[((hb * p.n_rows) + r0 + r) * D + e] : 0.f;
  }
  __syncthreads();
  const float *kT = p.ksumT + ((int64_t)b * p.n_kv_heads + head / p.group) * D * nqb;
  const int rmax = min(r0 + R - 1, p.n_rows - 1);
  const int imax = p.row0 + rmax;
  for (int j = tid; j <= imax; j += 256) {
    float acc[R] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
    for (int e = 0; e < D; ++e) {
      const float kv = kT[(int64_t)e * nqb + j];
#pragma unroll
      for (int r = 0; r < R; ++r) acc[r] = fmaf(qs[r][e], kv, acc[r]);
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int i = p.row0 + r0 + r;
      if (r0 + r < p.n_rows && j <= i)
        p.out[(hb * p.n_rows + r0 + r) * nqb + j] = (j < i) ? acc[r] * p.c_full : p.diag[hb * p.n_rows + r0 + r] * p.c_diag;
    }
  }
  __syncthreads();
  if (r0 + w >= p.n_rows) return;
  const int i = p.row0 + r0 + w;
  float *row = p.out + (hb * p.n_rows + r0 + w) * nqb;
  float mx = -INFINITY;
  for (int j = lane; j <= i; j += 64) mx = fmaxf(mx, row[j]);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
  float den = 0.f;
  for (int j = lane; j <= i; j += 64) den += expf(row[j] - mx);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) den += __shfl_xor(den, off, 64);
  for (int j = lane; j < nqb; j += 64) row[j] = (j <= i) ? expf(row[j] - mx) / den : 0.f;
}

// ---- Alg. 3 (Determine Sparse Pattern): Jensen-Shannon gate ------------------------------------
struct GateParams {
  const float *a_hat;     // [b][n][nkb] estimates of the listed heads
  float *dist;            // [b][n][2]   d_sparse, d_sim
  int32_t *head_pattern;  // [b][n_q_heads], entry of each listed head written
  int nkb, n_heads, n_q_heads;
  float delta, tau;
  int32_t head_ids[SP_MAX_HEADS];
  int32_t ref_pos[SP_MAX_HEADS];     // position of the head whose estimate is the representative, or -1
  int32_t shared_map[SP_MAX_HEADS];  // value written when the pattern is shared
};

// x ln(x/m) + y ln(y/m), m = (x+y)/2: one entry's contribution to 2*JSD, never negative
__device__ __forceinline__ double js_term(double x, double y) {
  const double m = 0.5 * (x + y);
  double t = 0.0;
  if (x > 0.0) t += x * log(x / m);
  if (y > 0.0) t += y * log(y / m);
  return t;
}
// sqrt(JSD(a || ref)) over n entries, natural logarithm, fp64; ref == nullptr: the uniform distribution.
// Called by a whole wavefront; every lane returns the result.
__device__ __forceinline__ double js_distance_wave(const float *a, const float *ref, int n, int lane) {
  const double u = 1.0 / (double)n;
  double sum = 0.0;
  for (int j = lane; j < n; j += 64) sum += js_term((double)a[j], ref ? (double)ref[j] : u);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off, 64);
  const double jsd = 0.5 * sum;
  return sqrt(jsd > 0.0 ? jsd : 0.0);
}

// Alg. 3's gate for the listed heads: one wavefront per (head, batch entry).
__global__ __launch_bounds__(64) void js_gate_kernel(GateParams p) {
  const int n = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
  const float *a = p.a_hat + ((int64_t)b * p.n_heads + n) * p.nkb;
  const int rp = p.ref_pos[n];
  const double d_sparse = js_distance_wave(a, nullptr, p.nkb, lane);
  const double d_sim = (rp >= 0) ? js_distance_wave(a, p.a_hat + ((int64_t)b * p.n_heads + rp) * p.nkb, p.nkb, lane) : 0.0;
  if (lane == 0) {
    const int64_t hb = (int64_t)b * p.n_heads + n;
    p.dist[hb * 2] = (float)d_sparse;
    p.dist[hb * 2 + 1] = (float)d_sim;
    const bool shared = d_sparse < (double)p.delta && d_sim < (double)p.tau;
    p.head_pattern[(int64_t)b * p.n_q_heads + p.head_ids[n]] = shared ? p.shared_map[n] : -1;
  }
}

// ---- dynamic pivotal pattern dictionary (Sec. 5.2; Alg. 1 with Alg. 3 and Alg. 4) ----------------
// Roles written per (batch entry, head): c >= 0 shares cluster c's dictionary pattern, -1 falls back
// (dense, no update), -2 is elected pivot of its cluster in this layer (dense + pattern construction).
struct ElectParams {
  const float *a_hat;   // [b][Hq][nkb] last-row estimates of every head
  float *dist;          // [b][Hq][2]
  int32_t *role;        // [b][Hq]
  int32_t *pivot_head;  // [b][n_slots] head elected for the slot's cluster in this layer, or -1
  int32_t *route;       // [b][n_slots] dictionary map (b * n_clusters + c) the slot's lists go to, or -1
  int32_t *act_n;       // [b] number of slots that elected a pivot
  int32_t *act_pos;     // [b][n_slots] those slots, ascending
  // the heads of the role-driven attention launch, split by weight class so that each class can be spread
  // evenly over the XCDs: positions (in that launch's slot table) of the heads that share a list, and of the
  // heads that fall back
  int32_t *shared_n, *shared_pos, *fallback_n, *fallback_pos;  // [b], [b][n_launch]
  int n_launch;
  int32_t launch_head[SP_MAX_HEADS];  // the launch's slot table: query head of each position
  int32_t *valid;       // dictionary [b][n_clusters]
  float *a_tilde;       // dictionary [b][n_clusters][nkb]
  int nkb, n_q_heads, n_slots, n_clusters;
  float delta, tau;
  int32_t head_cluster[SP_MAX_HEADS];  // global cluster id or -1
  int32_t head_slot[SP_MAX_HEADS];     // slot of the head's cluster, or -1
  int32_t slot_cluster[SP_MAX_HEADS];
};

// One workgroup per batch entry.  Heads are taken in ascending order as in Alg. 1: a cluster without a
// dictionary entry elects its first head that passes the sparsity test (there is no representative to
// compare with yet); every other head is tested against the entry's representative, or against the
// estimate of the pivot elected a moment ago.
__global__ __launch_bounds__(1024) void elect_kernel(ElectParams p) {
  __shared__ double ds[SP_MAX_HEADS];
  __shared__ int piv[SP_MAX_HEADS];
  __shared__ int had[SP_MAX_HEADS];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const float *ah = p.a_hat + (int64_t)b * p.n_q_heads * p.nkb;
  for (int h = w; h < p.n_q_heads; h += 16) {
    const double d = js_distance_wave(ah + (int64_t)h * p.nkb, nullptr, p.nkb, lane);
    if (lane == 0) ds[h] = d;
  }
  __syncthreads();
  if (tid < p.n_slots) {
    const int c = p.slot_cluster[tid];
    const int v = p.valid[(int64_t)b * p.n_clusters + c];
    int first = -1;
    if (!v && 0.0 < (double)p.tau)
      for (int h = p.n_q_heads - 1; h >= 0; --h)
        if (p.head_cluster[h] == c && ds[h] < (double)p.delta) first = h;
    piv[tid] = first;
    had[tid] = v;
    p.pivot_head[(int64_t)b * p.n_slots + tid] = first;
    p.route[(int64_t)b * p.n_slots + tid] = first >= 0 ? b * p.n_clusters + c : -1;
  }
  __syncthreads();
  if (tid == 0) {
    int na = 0;
    for (int s2 = 0; s2 < p.n_slots; ++s2)
      if (piv[s2] >= 0) p.act_pos[(int64_t)b * p.n_slots + na++] = s2;
    p.act_n[b] = na;
  }
  for (int h = w; h < p.n_q_heads; h += 16) {
    const int c = p.head_cluster[h], s = p.head_slot[h];
    int role = -1;
    double d_sim = 0.0;
    if (c >= 0) {
      if (piv[s] == h) {
        role = -2;
      } else {
        // heads met before the pivot of a new entry saw an empty dictionary: no representative for them
        const float *ref = had[s] ? p.a_tilde + ((int64_t)b * p.n_clusters + c) * p.nkb
                                  : (piv[s] >= 0 && piv[s] < h ? ah + (int64_t)piv[s] * p.nkb : nullptr);
        if (ref) {
          d_sim = js_distance_wave(ah + (int64_t)h * p.nkb, ref, p.nkb, lane);
          if (ds[h] < (double)p.delta && d_sim < (double)p.tau) role = c;
        }
      }
    }
    if (lane == 0) {
      p.role[(int64_t)b * p.n_q_heads + h] = role;
      p.dist[((int64_t)b * p.n_q_heads + h) * 2] = (float)ds[h];
      p.dist[((int64_t)b * p.n_q_heads + h) * 2 + 1] = (float)d_sim;
    }
  }
  __syncthreads();  // every read of the old representatives is done, every role is written
  if (tid == 0) {
    int ns = 0, nf = 0;
    for (int pos = 0; pos < p.n_launch; ++pos) {
      const int r = p.role[(int64_t)b * p.n_q_heads + p.launch_head[pos]];
      if (r >= 0) p.shared_pos[(int64_t)b * p.n_launch + ns++] = pos;
      if (r == -1) p.fallback_pos[(int64_t)b * p.n_launch + nf++] = pos;
    }
    p.shared_n[b] = ns;
    p.fallback_n[b] = nf;
  }
  for (int s = 0; s < p.n_slots; ++s) {
    if (piv[s] < 0) continue;
    const int c = p.slot_cluster[s];
    float *dst = p.a_tilde + ((int64_t)b * p.n_clusters + c) * p.nkb;
    const float *src = ah + (int64_t)piv[s] * p.nkb;
    for (int j = tid; j < p.nkb; j += 1024) dst[j] = src[j];
    if (tid == 0) p.valid[(int64_t)b * p.n_clusters + c] = 1;
  }
}

// Splits the heads of a role-driven attention launch into the two weight classes (sharing a list / falling
// back) so that each class can be spread evenly over the XCDs; positions refer to the launch's slot table.
struct ClassifyParams {
  const int32_t *role;  // [b][n_q_heads]
  int32_t *shared_n, *shared_pos, *fallback_n, *fallback_pos;  // [b], [b][n_launch]
  int n_q_heads, n_launch;
  int32_t launch_head[SP_MAX_HEADS];
};
__global__ __launch_bounds__(64) void classify_heads_kernel(ClassifyParams p) {
  const int b = blockIdx.x;
  if (threadIdx.x != 0) return;
  int ns = 0, nf = 0;
  for (int pos = 0; pos < p.n_launch; ++pos) {
    const int r = p.role[(int64_t)b * p.n_q_heads + p.launch_head[pos]];
    if (r >= 0) p.shared_pos[(int64_t)b * p.n_launch + ns++] = pos;
    if (r == -1) p.fallback_pos[(int64_t)b * p.n_launch + nf++] = pos;
  }
  p.shared_n[b] = ns;
  p.fallback_n[b] = nf;
}

}  // namespace

#endif
