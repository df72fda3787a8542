// SharePrefill prefill attention for one layer on gfx950 (MI355X): HIP kernels + C ABI.
//
// This file is the host side (argument checks, workspace layouts, launchers, the C ABI) and the only
// translation unit; the kernels live in the headers it includes.
//
// Kernels
//   pack_kv_kernel   K/V [token][kv head][d] -> per (kv head, 64-key sub-tile) images laid out
//                    in MFMA-operand order, so the attention kernels move a sub-tile from HBM
//                    to LDS as a straight copy (global_load_lds) and read every MFMA operand
//                    with one conflict-free ds_read_b128.
//   attn_kernel      flash-attention sweep (bf16 MFMA 32x32x16, fp32 online softmax in the
//                    log2 domain).  DENSE=true walks key blocks 0..i and records, per query
//                    and key block, the block-local log-sum-exp, from which the block-mass
//                    score map is reduced in the epilogue (Sec. 5.1 A(Q,K,V); Alg. 1 line 8).
//                    DENSE=false walks a per-row key-block index list (Sec. 5.1 A(Q,K,V,M)).
//   mask_kernel      Alg. 2 per query-block row in exact integer arithmetic, one wavefront
//                    per row: threshold search + ballot/popcount prefix sums.
//   key_pool_kernel, query_pool_kernel, mean_logit_softmax_kernel, gsel_*_kernel
//                    the pattern construction as the paper prints it: row softmax of the
//                    block-mean QK logits (Sec. 5.2) and Alg. 2 over the flattened map.
//
// MFMA operand mapping (v_mfma_f32_32x32x16_bf16, 64 lanes, lane = 32*h + c):
//   A (32 x 16): lane holds row c, k = 8h .. 8h+7        B (16 x 32): lane holds column c, same k
//   D (32 x 32): lane holds column c, rows 8*(r/4) + 4h + (r%4) for accumulator r = 0..15
// The kernel computes S^T = K Q^T (A = keys, B = queries) so that one lane owns one query:
// the row-wise softmax needs only a single cross-lane exchange (lane ^ 32).  The accumulator
// registers of S^T, rounded to bf16, are directly the B operand of O^T = V^T P^T provided the
// V^T operand uses the matching key order inside each 16-key step (slot (h,e) <-> key
// 4h+e for e<4, 8+4h+(e-4) for e>=4); pack_kv_kernel writes V in exactly that order.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "shareprefill.h"

#include "sp_common.h"
#include "pack_kernel.h"
#include "attn_kernel.h"
#include "mask_kernel.h"
#include "pattern_kernels.h"
#include "global_select_kernels.h"
#include "vertical_slash_kernels.h"
#include "vs_token_kernels.h"

namespace {

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

sp_status check_shape(const sp_shape *s) {
  if (!s) {
    set_err("shape is NULL");
    return SP_ERR_INVALID_ARG;
  }
  if (s->batch <= 0 || s->seq <= 0 || s->n_q_heads <= 0 || s->n_kv_heads <= 0) {
    set_err("batch/seq/head counts must be positive");
    return SP_ERR_INVALID_ARG;
  }
  if (s->n_q_heads % s->n_kv_heads) {
    set_err("n_q_heads (%d) is not a multiple of n_kv_heads (%d)", s->n_q_heads, s->n_kv_heads);
    return SP_ERR_INVALID_ARG;
  }
  if (s->head_dim != 64 && s->head_dim != 128) {
    set_err("head_dim %d unsupported (64 or 128)", s->head_dim);
    return SP_ERR_UNSUPPORTED;
  }
  if (s->block != 64 && s->block != 128) {
    set_err("block %d unsupported (64 or 128)", s->block);
    return SP_ERR_UNSUPPORTED;
  }
  if (s->seq % s->block) {
    set_err("seq %d is not a multiple of block %d", s->seq, s->block);
    return SP_ERR_UNSUPPORTED;
  }
  if (s->seq / s->block > 32768) {
    set_err("seq/block = %d exceeds 32768", s->seq / s->block);
    return SP_ERR_UNSUPPORTED;
  }
  if (s->n_q_heads > SP_MAX_HEADS) {
    set_err("n_q_heads %d exceeds %d", s->n_q_heads, SP_MAX_HEADS);
    return SP_ERR_UNSUPPORTED;
  }
  const int64_t st[] = {s->q_stride_b, s->q_stride_t, s->q_stride_h, s->kv_stride_b, s->kv_stride_t,
                        s->kv_stride_h, s->o_stride_b, s->o_stride_t, s->o_stride_h};
  for (int64_t x : st)
    if (x < 0 || (x % 8)) {
      set_err("strides must be non-negative multiples of 8 elements (got %lld)", (long long)x);
      return SP_ERR_INVALID_ARG;
    }
  if (s->q_stride_t < s->head_dim || s->kv_stride_t < s->head_dim || s->o_stride_t < s->head_dim ||
      (s->q_stride_h < s->head_dim && s->n_q_heads > 1) || (s->kv_stride_h < s->head_dim && s->n_kv_heads > 1) ||
      (s->o_stride_h < s->head_dim && s->n_q_heads > 1)) {
    set_err("token/head strides smaller than head_dim");
    return SP_ERR_INVALID_ARG;
  }
  if (!(s->softmax_scale >= 0.f) || std::isinf(s->softmax_scale)) {
    set_err("softmax_scale must be finite and >= 0 (0 selects 1/sqrt(head_dim))");
    return SP_ERR_INVALID_ARG;
  }
  return SP_OK;
}

size_t pack_bytes(const sp_shape *s) {
  return align_up((size_t)s->batch * s->n_kv_heads * s->seq * s->head_dim * 2 * 2, 256);
}
// block log-sum-exps of the scored heads: one float per (query, key block <= query block), i.e. the causal
// half [nqb(nqb+1)/2][block] per (batch entry, head)
size_t lws_bytes(const sp_shape *s, int n_dense) {
  const size_t nqb = s->seq / s->block;
  return align_up((size_t)s->batch * n_dense * (nqb * (nqb + 1) / 2) * s->block * sizeof(float), 256);
}
size_t scores_bytes(const sp_shape *s, int n_maps) {
  const size_t nqb = s->seq / s->block;
  return align_up((size_t)s->batch * n_maps * nqb * nqb * sizeof(float), 256);
}

// scratch of the pooled score path for n listed heads per batch entry and of the global selection
// for n maps per batch entry: [ksumT | qsum | diag | per-map selection scratch]
struct PatternLayout {
  size_t ksumT, qsum, diag, gsel, total;
};
PatternLayout pattern_layout(const sp_shape *s, int n) {
  const size_t nqb = s->seq / s->block, maps = (size_t)s->batch * n;
  PatternLayout L;
  L.ksumT = 0;
  L.qsum = L.ksumT + align_up((size_t)s->batch * s->n_kv_heads * nqb * s->head_dim * sizeof(float), 256);
  L.diag = L.qsum + align_up(maps * nqb * s->head_dim * sizeof(float), 256);
  L.gsel = L.diag + align_up(maps * nqb * sizeof(float), 256);
  L.total = L.gsel + align_up(maps * gsel_map_bytes((int)nqb), 256);
  return L;
}

sp_status check_ptr16(const void *p, const char *name) {
  if (!p) {
    set_err("%s is NULL", name);
    return SP_ERR_INVALID_ARG;
  }
  if ((uintptr_t)p % 16) {
    set_err("%s is not 16-byte aligned", name);
    return SP_ERR_INVALID_ARG;
  }
  return SP_OK;
}

sp_status check_heads(const sp_shape *s, const int32_t *ids, int n, const char *name) {
  if (!ids) {
    set_err("%s is NULL", name);
    return SP_ERR_INVALID_ARG;
  }
  if (n <= 0 || n > s->n_q_heads) {
    set_err("number of listed heads %d outside [1, %d]", n, s->n_q_heads);
    return SP_ERR_INVALID_ARG;
  }
  bool seen[SP_MAX_HEADS] = {false};
  for (int a = 0; a < n; ++a) {
    if (ids[a] < 0 || ids[a] >= s->n_q_heads) {
      set_err("%s[%d] = %d outside [0, %d)", name, a, ids[a], s->n_q_heads);
      return SP_ERR_INVALID_ARG;
    }
    if (seen[ids[a]]) {
      set_err("%s lists head %d twice", name, ids[a]);
      return SP_ERR_INVALID_ARG;
    }
    seen[ids[a]] = true;
  }
  return SP_OK;
}

sp_status hip_check(hipError_t e, const char *what) {
  if (e != hipSuccess) {
    set_err("%s: %s", what, hipGetErrorString(e));
    return SP_ERR_HIP;
  }
  return SP_OK;
}

sp_status launch_pack(const sp_shape *s, const void *k, const void *v, void *ws, hipStream_t st) {
  PackParams pp;
  pp.k = (const uint16_t *)k;
  pp.v = (const uint16_t *)v;
  pp.out = (char *)ws;
  pp.sb = s->kv_stride_b;
  pp.st = s->kv_stride_t;
  pp.sh = s->kv_stride_h;
  pp.n_kv_heads = s->n_kv_heads;
  pp.n_sub = s->seq / KT;
  dim3 grid(s->seq / KT, s->n_kv_heads, s->batch);
  ProfScope prof(KK_PACK, st);
  if (s->head_dim == 128)
    hipLaunchKernelGGL(pack_kv_kernel<128>, grid, dim3(256), 0, st, pp);
  else
    hipLaunchKernelGGL(pack_kv_kernel<64>, grid, dim3(256), 0, st, pp);
  return hip_check(hipGetLastError(), "pack_kv_kernel launch");
}

void fill_attn(AttnParams &ap, const sp_shape *s, const void *q, const void *kvp, void *o) {
  memset(&ap, 0, sizeof(ap));
  ap.q = (const uint16_t *)q;
  ap.kvp = (const char *)kvp;
  ap.o = (uint16_t *)o;
  ap.q_sb = s->q_stride_b;
  ap.q_st = s->q_stride_t;
  ap.q_sh = s->q_stride_h;
  ap.o_sb = s->o_stride_b;
  ap.o_st = s->o_stride_t;
  ap.o_sh = s->o_stride_h;
  ap.seq = s->seq;
  ap.nqb = s->seq / s->block;
  ap.n_kv_heads = s->n_kv_heads;
  ap.group = s->n_q_heads / s->n_kv_heads;
  const float scale = (s->softmax_scale > 0.f) ? s->softmax_scale : 1.0f / sqrtf((float)s->head_dim);
  ap.c = scale * 1.4426950408889634f;
}

// Host-side view of one attention launch: the listed heads in the caller's order.
struct HeadList {
  int n = 0;
  int32_t head[SP_MAX_HEADS];
  int32_t map[SP_MAX_HEADS];
};

// order of the slot table: heads that share a KV head, and among them those that walk the same list, adjacent
void sort_head_list(HeadList &hl, int group, bool dense) {
  struct Ent {
    int kvh, map, head;
  } ent[SP_MAX_HEADS];
  for (int a = 0; a < hl.n; ++a) ent[a] = {hl.head[a] / group, dense ? 0 : hl.map[a], hl.head[a]};
  std::stable_sort(ent, ent + hl.n, [](const Ent &x, const Ent &y) {
    if (x.kvh != y.kvh) return x.kvh < y.kvh;
    if (x.map != y.map) return x.map < y.map;
    return x.head < y.head;
  });
  for (int a = 0; a < hl.n; ++a) {
    hl.head[a] = ent[a].head;
    hl.map[a] = ent[a].map;
  }
}

// Builds the slot table and launches.  The listed heads are sorted by (kv head, list, head) and
// cut into 8 strands each and dealt to the 8 XCDs in contiguous runs, so heads that read the same K/V images
// (and, for the sparse kernel, walk the same list) run on one XCD together and meet in its L2.
template <bool DENSE>
sp_status launch_attn(const sp_shape *s, AttnParams ap, const HeadList &hl, hipStream_t st) {
  const int n = hl.n;
  struct Ent {
    int kvh, map, head, pos;
  } ent[SP_MAX_HEADS];
  for (int a = 0; a < n; ++a) ent[a] = {hl.head[a] / ap.group, DENSE ? 0 : hl.map[a], hl.head[a], a};
  std::stable_sort(ent, ent + n, [](const Ent &x, const Ent &y) {
    if (x.kvh != y.kvh) return x.kvh < y.kvh;
    if (x.map != y.map) return x.map < y.map;
    return x.head < y.head;
  });
  ap.n_heads = n;
  ap.rgroups = (ap.nqb + 7) / 8;
  for (int a = 0; a < n; ++a) {
    ap.head_ids[a] = ent[a].head;
    ap.head_map[a] = ent[a].map;
    ap.head_pos[a] = ent[a].pos;
  }
  const int64_t nwg = (int64_t)s->batch * 8 * n * ap.rgroups;
  if (nwg <= 0 || nwg > 0x7FFFFFFF) {
    set_err("grid too large");
    return SP_ERR_UNSUPPORTED;
  }
  dim3 grid((unsigned)nwg);
  const bool sc = DENSE && ap.scores != nullptr;
  ProfScope prof(DENSE ? KK_DENSE : KK_SPARSE, st);
#define SP_LAUNCH(D_, B_)                                                                           \
  do {                                                                                              \
    if (sc)                                                                                         \
      hipLaunchKernelGGL((attn_kernel<D_, B_, true, true>), grid, dim3(B_ * 2), 0, st, ap);        \
    else                                                                                            \
      hipLaunchKernelGGL((attn_kernel<D_, B_, DENSE, false>), grid, dim3(B_ * 2), 0, st, ap);      \
  } while (0)
  if (s->head_dim == 128 && s->block == 128)
    SP_LAUNCH(128, 128);
  else if (s->head_dim == 128 && s->block == 64)
    SP_LAUNCH(128, 64);
  else if (s->head_dim == 64 && s->block == 128)
    SP_LAUNCH(64, 128);
  else
    SP_LAUNCH(64, 64);
#undef SP_LAUNCH
  return hip_check(hipGetLastError(), DENSE ? "dense attn_kernel launch" : "sparse attn_kernel launch");
}

sp_status launch_mask(const float *scores, int n_maps, int nqb, int nkb, float gamma, int32_t *kb_idx,
                      int32_t *kb_cnt, uint64_t *bitmask, hipStream_t st, const int32_t *route = nullptr) {
  const uint32_t gq = (uint32_t)rintf(gamma * 16777216.f);
  const int64_t rows = (int64_t)n_maps * nqb;
  dim3 grid((unsigned)((rows + 3) / 4));
  ProfScope prof(KK_MASK, st);
  if (nkb <= 256)
    hipLaunchKernelGGL(mask_kernel<4>, grid, dim3(256), 0, st, scores, (int)rows, nqb, nkb, gq, kb_idx, kb_cnt, bitmask,
                       route);
  else if (nkb <= 1024)
    hipLaunchKernelGGL(mask_kernel<16>, grid, dim3(256), 0, st, scores, (int)rows, nqb, nkb, gq, kb_idx, kb_cnt, bitmask,
                       route);
  else
    hipLaunchKernelGGL(mask_kernel<0>, grid, dim3(256), 0, st, scores, (int)rows, nqb, nkb, gq, kb_idx, kb_cnt, bitmask,
                       route);
  return hip_check(hipGetLastError(), "mask_kernel launch");
}

// row softmax of the block-mean logits of the listed heads, query-block rows row0 .. row0+n_rows-1,
// into out[b][n][n_rows][nkb]
sp_status launch_mean_logit_scores(const sp_shape *s, const void *q, const void *k, const int32_t *heads, int n,
                                   int row0, int n_rows, float *out, char *pattern_ws, hipStream_t st,
                                   const int32_t *head_dev = nullptr) {
  if ((int64_t)s->batch * n > 65535) {
    set_err("batch * heads = %lld exceeds 65535", (long long)s->batch * n);
    return SP_ERR_UNSUPPORTED;
  }
  const PatternLayout L = pattern_layout(s, n);
  const int nqb = s->seq / s->block;
  PoolParams pp;
  memset(&pp, 0, sizeof(pp));
  pp.q = (const uint16_t *)q;
  pp.k = (const uint16_t *)k;
  pp.q_sb = s->q_stride_b;
  pp.q_st = s->q_stride_t;
  pp.q_sh = s->q_stride_h;
  pp.k_sb = s->kv_stride_b;
  pp.k_st = s->kv_stride_t;
  pp.k_sh = s->kv_stride_h;
  pp.nqb = nqb;
  pp.group = s->n_q_heads / s->n_kv_heads;
  pp.n_heads = n;
  pp.n_kv_heads = s->n_kv_heads;
  pp.row0 = row0;
  pp.n_rows = n_rows;
  pp.ksumT = (float *)(pattern_ws + L.ksumT);
  pp.qsum = (float *)(pattern_ws + L.qsum);
  pp.diag = (float *)(pattern_ws + L.diag);
  pp.out = out;
  pp.head_dev = head_dev;
  for (int a = 0; a < n; ++a) pp.head_ids[a] = heads ? heads[a] : 0;
  const float scale = (s->softmax_scale > 0.f) ? s->softmax_scale : 1.0f / sqrtf((float)s->head_dim);
  const float B = (float)s->block;
  pp.c_full = scale / (B * B);
  pp.c_diag = scale / (B * (B + 1.f) * 0.5f);
  ProfScope prof(KK_SCORE, st);
  dim3 gk(nqb, s->n_kv_heads, s->batch), gq(n_rows, n, s->batch), glog((n_rows + 3) / 4, s->batch * n);
#define SP_POOL(D_, B_)                                                              \
  do {                                                                               \
    hipLaunchKernelGGL((key_pool_kernel<D_, B_>), gk, dim3(D_), 0, st, pp);          \
    hipLaunchKernelGGL((query_pool_kernel<D_, B_>), gq, dim3(D_), 0, st, pp);        \
    hipLaunchKernelGGL((mean_logit_softmax_kernel<D_>), glog, dim3(256), 0, st, pp); \
  } while (0)
  if (s->head_dim == 128 && s->block == 128)
    SP_POOL(128, 128);
  else if (s->head_dim == 128 && s->block == 64)
    SP_POOL(128, 64);
  else if (s->head_dim == 64 && s->block == 128)
    SP_POOL(64, 128);
  else
    SP_POOL(64, 64);
#undef SP_POOL
  return hip_check(hipGetLastError(), "block-mean-logit score kernels launch");
}

// Alg. 3 for the listed heads: estimates (last query-block row of the score map) into a_hat, then the gate
sp_status launch_determine(const sp_shape *s, const void *q, const void *k, const int32_t *heads, int n,
                           const int32_t *ref_pos, const int32_t *shared_map, float delta, float tau, float *a_hat,
                           float *dist, int32_t *head_pattern, char *pattern_ws, hipStream_t st) {
  const int nqb = s->seq / s->block;
  sp_status rc = launch_mean_logit_scores(s, q, k, heads, n, nqb - 1, 1, a_hat, pattern_ws, st);
  if (rc) return rc;
  GateParams gp;
  memset(&gp, 0, sizeof(gp));
  gp.a_hat = a_hat;
  gp.dist = dist;
  gp.head_pattern = head_pattern;
  gp.nkb = nqb;
  gp.n_heads = n;
  gp.n_q_heads = s->n_q_heads;
  gp.delta = delta;
  gp.tau = tau;
  for (int a = 0; a < n; ++a) {
    gp.head_ids[a] = heads[a];
    gp.ref_pos[a] = ref_pos[a];
    gp.shared_map[a] = shared_map[a];
  }
  ProfScope prof(KK_SCORE, st);
  hipLaunchKernelGGL(js_gate_kernel, dim3(n, s->batch), dim3(64), 0, st, gp);
  return hip_check(hipGetLastError(), "js_gate_kernel launch");
}

void launch_gsel_threshold(const float *scores, int n_maps, const GselGeom &g, uint32_t gq, char *scratch,
                           hipStream_t st);

// workspace of the vertical-slash search for n listed heads per batch entry
struct VsLayout {
  size_t x, stats, sums, flags, gsel, total;
};
VsLayout vs_layout(const sp_shape *s, int n) {
  const size_t maps = (size_t)s->batch * n, nkb = s->seq / s->block;
  VsLayout L;
  L.x = 0;
  L.stats = L.x + align_up(maps * s->block * s->seq * sizeof(float), 256);
  L.sums = L.stats + align_up(maps * s->block * 2 * sizeof(float), 256);
  L.flags = L.sums + align_up(maps * 2 * s->seq * sizeof(float), 256);
  L.gsel = L.flags + align_up(maps * 2 * nkb * sizeof(int32_t), 256);
  L.total = L.gsel + align_up(maps * 2 * gsel_map_bytes((int)nkb), 256);
  return L;
}

// Alg. 5 for the listed heads: block lists into kb_idx / kb_cnt ([b][n] or, by_head, [b][n_q_heads]).
// role (device, [b][n_q_heads], needs the heads listed 0..n_q_heads-1) restricts the work to heads whose
// entry is -1.  sums_out (optional, [b][n][2][seq]) receives a_v and a_s.
sp_status launch_vertical_slash(const sp_shape *s, const void *q, const void *k, const int32_t *heads, int n,
                                float gamma, int forced, const int32_t *role, int by_head, float *sums_out,
                                int32_t *kb_idx, int32_t *kb_cnt, char *vs_ws, hipStream_t st,
                                uint64_t *keep_bits = nullptr) {
  if ((int64_t)s->batch * n * 2 > 65535) {
    set_err("batch * heads * 2 = %lld exceeds 65535", (long long)s->batch * n * 2);
    return SP_ERR_UNSUPPORTED;
  }
  const VsLayout L = vs_layout(s, n);
  const int nkb = s->seq / s->block;
  VsParams vp;
  memset(&vp, 0, sizeof(vp));
  vp.q = (const uint16_t *)q;
  vp.k = (const uint16_t *)k;
  vp.q_sb = s->q_stride_b;
  vp.q_st = s->q_stride_t;
  vp.q_sh = s->q_stride_h;
  vp.k_sb = s->kv_stride_b;
  vp.k_st = s->kv_stride_t;
  vp.k_sh = s->kv_stride_h;
  vp.seq = s->seq;
  vp.group = s->n_q_heads / s->n_kv_heads;
  vp.n_heads = n;
  vp.n_q_heads = s->n_q_heads;
  const float scale = (s->softmax_scale > 0.f) ? s->softmax_scale : 1.0f / sqrtf((float)s->head_dim);
  vp.c = scale * 1.4426950408889634f;
  vp.x = (float *)(vs_ws + L.x);
  vp.stats = (float *)(vs_ws + L.stats);
  vp.sums = sums_out ? sums_out : (float *)(vs_ws + L.sums);
  vp.role = role;
  for (int a = 0; a < n; ++a) vp.head_ids[a] = heads[a];
  int32_t *flags = (int32_t *)(vs_ws + L.flags);
  ProfScope prof(KK_VS, st);
  const dim3 glog((s->seq + 127) / 128, n, s->batch), gstat(s->block, n, s->batch), gsum((s->seq + 255) / 256, n, s->batch);
#define SP_VS(D_, B_)                                                                  \
  do {                                                                                 \
    hipLaunchKernelGGL((vs_logits_kernel<D_, B_>), glog, dim3(256), 0, st, vp);        \
    hipLaunchKernelGGL((vs_rowstats_kernel<B_>), gstat, dim3(256), 0, st, vp);         \
    hipLaunchKernelGGL((vs_sums_kernel<B_>), gsum, dim3(256), 0, st, vp);              \
  } while (0)
  if (s->head_dim == 128 && s->block == 128)
    SP_VS(128, 128);
  else if (s->head_dim == 128 && s->block == 64)
    SP_VS(128, 64);
  else if (s->head_dim == 64 && s->block == 128)
    SP_VS(64, 128);
  else
    SP_VS(64, 64);
#undef SP_VS
  sp_status rc = hip_check(hipGetLastError(), "vertical-slash sum kernels launch");
  if (rc) return rc;
  // the two selections of every head: vectors of seq entries seen as nkb rows of `block`
  GselGeom g;
  g.n_rows = nkb;
  g.n_cols = s->block;
  g.tri = 0;
  g.role = role;
  g.per_head = 2;
  const int n_maps = s->batch * n * 2;
  const uint32_t gq = (uint32_t)rintf(gamma * 16777216.f);
  launch_gsel_threshold(vp.sums, n_maps, g, gq, vs_ws + L.gsel, st);
  hipLaunchKernelGGL(gsel_emit_flags_kernel, dim3((nkb + 3) / 4, n_maps), dim3(256), 0, st, vp.sums, g,
                     vs_ws + L.gsel, flags, keep_bits);
  if (kb_idx)  // the pattern at block granularity (not needed by the token-level attention)
    hipLaunchKernelGGL(vs_block_lists_kernel, dim3((nkb + 3) / 4, n, s->batch), dim3(256), 0, st, vp, flags, nkb,
                       forced, by_head, kb_idx, kb_cnt);
  return hip_check(hipGetLastError(), "vertical-slash selection kernels launch");
}

// workspace of the token-level vertical-slash attention for n listed heads per batch entry, after the search's own
struct VsTokLayout {
  size_t search, bits, cumv, gpos, cumband, bandlist, act, gimg, total;
};
VsTokLayout vs_token_layout(const sp_shape *s, int n) {
  const size_t maps = (size_t)s->batch * n, nqb = s->seq / s->block;
  VsTokLayout L;
  L.search = 0;
  L.bits = L.search + vs_layout(s, n).total;
  L.cumv = L.bits + align_up(maps * 2 * (s->seq / 64) * sizeof(uint64_t), 256);
  L.gpos = L.cumv + align_up(maps * (nqb + 1) * sizeof(int32_t), 256);
  L.cumband = L.gpos + align_up(maps * s->seq * sizeof(int32_t), 256);
  L.bandlist = L.cumband + align_up(maps * nqb * sizeof(int32_t), 256);
  L.act = L.bandlist + align_up(maps * nqb * sizeof(int32_t), 256);
  L.gimg = L.act + align_up((maps + s->batch) * sizeof(int32_t), 256);
  L.total = L.gimg + align_up(maps * (size_t)s->seq * s->head_dim * 2 * 2, 256);
  return L;
}

// Alg. 5 for the listed heads and attention over its token-level pattern.  kvp: the packed K/V images of the call.
// role (device, [b][n_q_heads], heads listed 0..n_q_heads-1): only heads whose entry is -1 take part.
sp_status launch_vs_token_attn(const sp_shape *s, const void *q, const void *k, const void *v, const char *kvp,
                               const int32_t *heads, int n, float gamma, int forced, const int32_t *role, void *o,
                               uint64_t *keep_bits_out, int64_t *pairs, char *ws, hipStream_t st) {
  const VsTokLayout L = vs_token_layout(s, n);
  uint64_t *bits = keep_bits_out ? keep_bits_out : (uint64_t *)(ws + L.bits);
  sp_status rc = launch_vertical_slash(s, q, k, heads, n, gamma, forced, role, 0, nullptr, nullptr, nullptr,
                                       ws + L.search, st, bits);
  if (rc) return rc;
  VsTokParams tp;
  memset(&tp, 0, sizeof(tp));
  tp.q = (const uint16_t *)q;
  tp.k = (const uint16_t *)k;
  tp.v = (const uint16_t *)v;
  tp.kvp = kvp;
  tp.o = (uint16_t *)o;
  tp.q_sb = s->q_stride_b, tp.q_st = s->q_stride_t, tp.q_sh = s->q_stride_h;
  tp.kv_sb = s->kv_stride_b, tp.kv_st = s->kv_stride_t, tp.kv_sh = s->kv_stride_h;
  tp.o_sb = s->o_stride_b, tp.o_st = s->o_stride_t, tp.o_sh = s->o_stride_h;
  tp.seq = s->seq;
  tp.nqb = s->seq / s->block;
  tp.block = s->block;
  tp.n_kv_heads = s->n_kv_heads;
  tp.group = s->n_q_heads / s->n_kv_heads;
  tp.n_heads = n;
  tp.n_q_heads = s->n_q_heads;
  tp.forced = forced;
  const float scale = (s->softmax_scale > 0.f) ? s->softmax_scale : 1.0f / sqrtf((float)s->head_dim);
  tp.c = scale * 1.4426950408889634f;
  tp.bits = bits;
  tp.cumv = (int32_t *)(ws + L.cumv);
  tp.gpos = (int32_t *)(ws + L.gpos);
  tp.cumband = (int32_t *)(ws + L.cumband);
  tp.bandlist = (int32_t *)(ws + L.bandlist);
  tp.gimg = ws + L.gimg;
  tp.act_pos = (int32_t *)(ws + L.act);
  tp.act_n = tp.act_pos + (size_t)s->batch * n;
  tp.nch8 = ((tp.nqb + VST_TASK_ROWS - 1) / VST_TASK_ROWS + 7) / 8;
  tp.pairs = pairs;
  tp.role = role;
  for (int a = 0; a < n; ++a) tp.head_ids[a] = heads[a];
  ProfScope prof(KK_VS, st);
  hipLaunchKernelGGL(vs_token_prep_kernel, dim3(n, s->batch), dim3(1024), 0, st, tp);
  const dim3 ggather(s->seq / KT, n, s->batch), gattn((unsigned)((int64_t)s->batch * 8 * n * tp.nch8 * VST_TASK_ROWS));
  if (s->head_dim == 128)
    hipLaunchKernelGGL(vs_gather_kernel<128>, ggather, dim3(256), 0, st, tp);
  else
    hipLaunchKernelGGL(vs_gather_kernel<64>, ggather, dim3(256), 0, st, tp);
  if (s->head_dim == 128 && s->block == 128)
    hipLaunchKernelGGL((vs_token_attn_kernel<128, 128>), gattn, dim3(256), 0, st, tp);
  else if (s->head_dim == 128 && s->block == 64)
    hipLaunchKernelGGL((vs_token_attn_kernel<128, 64>), gattn, dim3(128), 0, st, tp);
  else if (s->head_dim == 64 && s->block == 128)
    hipLaunchKernelGGL((vs_token_attn_kernel<64, 128>), gattn, dim3(256), 0, st, tp);
  else
    hipLaunchKernelGGL((vs_token_attn_kernel<64, 64>), gattn, dim3(128), 0, st, tp);
  return hip_check(hipGetLastError(), "token-level vertical-slash kernels launch");
}

sp_status check_thresholds(float delta, float tau) {
  if (!(delta >= 0.f) || !(tau >= 0.f) || std::isinf(delta) || std::isinf(tau)) {
    set_err("delta %g / tau %g must be finite and >= 0", (double)delta, (double)tau);
    return SP_ERR_INVALID_ARG;
  }
  return SP_OK;
}

// the seven launches that leave, per map, the threshold value, the number of ties to take and every
// row's tie count prefix in the selection scratch
void launch_gsel_threshold(const float *scores, int n_maps, const GselGeom &g, uint32_t gq, char *scratch,
                           hipStream_t st) {
  const int row_groups = (g.n_rows + 3) / 4;
  const dim3 ghist(std::min(row_groups, 64), n_maps), grows(row_groups, n_maps);
  hipLaunchKernelGGL(gsel_zero_kernel, dim3(n_maps), dim3(256), 0, st, scratch, g);
  hipLaunchKernelGGL(gsel_hist_kernel<1>, ghist, dim3(256), 0, st, scores, g, scratch);
  hipLaunchKernelGGL(gsel_scan_kernel<1>, dim3(n_maps), dim3(1024), 0, st, scratch, g, gq);
  hipLaunchKernelGGL(gsel_hist_kernel<2>, ghist, dim3(256), 0, st, scores, g, scratch);
  hipLaunchKernelGGL(gsel_scan_kernel<2>, dim3(n_maps), dim3(1024), 0, st, scratch, g, gq);
  hipLaunchKernelGGL(gsel_row_ties_kernel, grows, dim3(256), 0, st, scores, g, scratch);
  hipLaunchKernelGGL(gsel_row_scan_kernel, dim3(n_maps), dim3(1024), 0, st, g, scratch);
}

// Alg. 2 over each flattened map; `scratch` holds n_maps * gsel_map_bytes(nqb) bytes
sp_status launch_mask_global(const float *scores, int n_maps, int nqb, float gamma, int forced, int32_t *kb_idx,
                             int32_t *kb_cnt, char *scratch, hipStream_t st, const int32_t *route = nullptr) {
  if (n_maps > 65535) {
    set_err("%d maps exceed 65535", n_maps);
    return SP_ERR_UNSUPPORTED;
  }
  const uint32_t gq = (uint32_t)rintf(gamma * 16777216.f);
  const int row_groups = (nqb + 3) / 4;
  const dim3 ghist(std::min(row_groups, 64), n_maps), grows(row_groups, n_maps);
  ProfScope prof(KK_MASK, st);
  GselGeom g;
  g.n_rows = nqb;
  g.n_cols = nqb;
  g.tri = 1;
  g.role = nullptr;
  g.per_head = 1;
  launch_gsel_threshold(scores, n_maps, g, gq, scratch, st);
  hipLaunchKernelGGL(gsel_emit_kernel, grows, dim3(256), 0, st, scores, g, scratch, forced, kb_idx, kb_cnt, route);
  return hip_check(hipGetLastError(), "global selection kernels launch");
}

sp_status check_ws(const void *ws, size_t have, size_t need) {
  if (need == 0) return SP_OK;
  if (!ws) {
    set_err("workspace is NULL (%zu bytes needed)", need);
    return SP_ERR_WORKSPACE;
  }
  if ((uintptr_t)ws % 256) {
    set_err("workspace is not 256-byte aligned");
    return SP_ERR_WORKSPACE;
  }
  if (have < need) {
    set_err("workspace too small: %zu bytes given, %zu needed", have, need);
    return SP_ERR_WORKSPACE;
  }
  return SP_OK;
}

}  // namespace

// Device memory of the one entry point that takes no workspace (sp_build_block_mask_global_static): a
// file-scope array, one copy per GPU the library runs on, held until the process ends.  The array's name
// is only a host-side handle; its device address is looked up once per device and every launch gets that
// pointer.
static __device__ __align__(256) char scratch[SP_STATIC_SCRATCH_BYTES];

namespace {

constexpr int SP_MAX_DEVICES = 64;
char *g_static_scratch[SP_MAX_DEVICES] = {nullptr};
std::mutex g_static_scratch_mutex;

// device address of `scratch` on the current device (no allocation: a symbol lookup, cached per device)
sp_status static_scratch_ptr(char **out) {
  int dev = -1;
  sp_status rc = hip_check(hipGetDevice(&dev), "hipGetDevice");
  if (rc) return rc;
  if (dev < 0 || dev >= SP_MAX_DEVICES) {
    set_err("device ordinal %d outside [0, %d)", dev, SP_MAX_DEVICES);
    return SP_ERR_UNSUPPORTED;
  }
  std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
  if (!g_static_scratch[dev]) {
    void *ptr = nullptr;
    if ((rc = hip_check(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)"))) return rc;
    if (!ptr || ((uintptr_t)ptr % 256)) {
      set_err("static scratch address %p is null or misaligned", ptr);
      return SP_ERR_HIP;
    }
    g_static_scratch[dev] = (char *)ptr;
  }
  *out = g_static_scratch[dev];
  return SP_OK;
}

}  // namespace

extern "C" {

const char *sp_status_string(sp_status s) {
  switch (s) {
    case SP_OK: return "SP_OK";
    case SP_ERR_INVALID_ARG: return "SP_ERR_INVALID_ARG";
    case SP_ERR_UNSUPPORTED: return "SP_ERR_UNSUPPORTED";
    case SP_ERR_WORKSPACE: return "SP_ERR_WORKSPACE";
    case SP_ERR_HIP: return "SP_ERR_HIP";
  }
  return "SP_ERR_UNKNOWN";
}

const char *sp_last_error(void) { return g_err; }


sp_status sp_profile_enable(int32_t on) {
  g_err[0] = 0;
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  if (on && !g_prof_events) {  // the events are created here, never while launches are being enqueued
    g_prof_events = new hipEvent_t[2 * SP_PROF_CAPACITY];
    for (int a = 0; a < 2 * SP_PROF_CAPACITY; ++a) {
      const hipError_t e = hipEventCreate(&g_prof_events[a]);
      if (e != hipSuccess) {
        for (int c = 0; c < a; ++c) (void)hipEventDestroy(g_prof_events[c]);
        delete[] g_prof_events;
        g_prof_events = nullptr;
        return hip_check(e, "hipEventCreate");
      }
    }
  }
  g_prof_count = 0;
  g_prof_dropped = 0;
  g_prof_on = on != 0;
  return SP_OK;
}

sp_status sp_profile_read(float *ms, int32_t *launches, int32_t reset) {
  g_err[0] = 0;
  if (!ms || !launches) {
    set_err("ms / launches must not be NULL");
    return SP_ERR_INVALID_ARG;
  }
  std::lock_guard<std::mutex> lock(g_prof_mutex);
  for (int a = 0; a < KK_COUNT; ++a) {
    ms[a] = 0.f;
    launches[a] = 0;
  }
  if (g_prof_dropped) {
    set_err("%d launches were not timed: more than %d launches between two reads", g_prof_dropped, SP_PROF_CAPACITY);
    return SP_ERR_UNSUPPORTED;
  }
  for (int r = 0; r < g_prof_count; ++r) {
    float t = 0.f;
    const hipError_t e = hipEventElapsedTime(&t, g_prof_events[2 * r], g_prof_events[2 * r + 1]);
    if (e != hipSuccess) return hip_check(e, "hipEventElapsedTime (synchronise the stream before sp_profile_read)");
    ms[g_prof_kind[r]] += t;
    launches[g_prof_kind[r]] += 1;
  }
  if (reset) g_prof_count = 0;
  return SP_OK;
}

sp_status sp_workspace_bytes(const sp_shape *shape, int32_t n_dense_heads, size_t *bytes) {
  g_err[0] = 0;
  sp_status rc = check_shape(shape);
  if (rc) return rc;
  if (!bytes) {
    set_err("bytes is NULL");
    return SP_ERR_INVALID_ARG;
  }
  if (n_dense_heads < 0 || n_dense_heads > shape->n_q_heads) {
    set_err("n_dense_heads %d outside [0, %d]", n_dense_heads, shape->n_q_heads);
    return SP_ERR_INVALID_ARG;
  }
  *bytes = pack_bytes(shape) + lws_bytes(shape, n_dense_heads) +
           std::max(pattern_layout(shape, n_dense_heads).total, pattern_layout(shape, shape->n_q_heads).total) +
           align_up((size_t)8 * shape->batch * shape->n_q_heads * sizeof(int32_t), 256) +
           scores_bytes(shape, n_dense_heads);  // the score maps, when the caller does not want them back
  return SP_OK;
}

sp_status sp_score_workspace_bytes(const sp_shape *shape, int32_t n_heads, size_t *bytes) {
  g_err[0] = 0;
  sp_status rc = check_shape(shape);
  if (rc) return rc;
  if (!bytes) {
    set_err("bytes is NULL");
    return SP_ERR_INVALID_ARG;
  }
  if (n_heads < 0 || n_heads > shape->n_q_heads) {
    set_err("n_heads %d outside [0, %d]", n_heads, shape->n_q_heads);
    return SP_ERR_INVALID_ARG;
  }
  *bytes = pattern_layout(shape, n_heads).gsel;  // the pooled sums only
  return SP_OK;
}

sp_status sp_mask_workspace_bytes(int32_t n_maps, int32_t nqb, size_t *bytes) {
  g_err[0] = 0;
  if (!bytes) {
    set_err("bytes is NULL");
    return SP_ERR_INVALID_ARG;
  }
  if (n_maps <= 0 || nqb <= 0 || nqb > 32768) {
    set_err("n_maps must be positive and nqb in [1, 32768]");
    return SP_ERR_INVALID_ARG;
  }
  *bytes = align_up((size_t)n_maps * gsel_map_bytes(nqb), 256);
  return SP_OK;
}

sp_status sp_dense_attn_with_block_scores(const sp_shape *shape, const void *q, const void *k, const void *v,
                                          const int32_t *head_ids, int32_t n_heads, void *o, float *block_scores,
                                          void *workspace, size_t workspace_bytes, void *hip_stream) {
  g_err[0] = 0;
  sp_status rc = check_shape(shape);
  if (rc) return rc;
  if ((rc = check_ptr16(q, "q")) || (rc = check_ptr16(k, "k")) || (rc = check_ptr16(v, "v")) ||
      (rc = check_ptr16(o, "o")))
    return rc;
  if ((rc = check_heads(shape, head_ids, n_heads, "head_ids"))) return rc;
  if (block_scores && ((uintptr_t)block_scores % 4)) {
    set_err("block_scores is misaligned");
    return SP_ERR_INVALID_ARG;
  }
  const size_t need = pack_bytes(shape) + (block_scores ? lws_bytes(shape, n_heads) : 0);
  if ((rc = check_ws(workspace, workspace_bytes, need))) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  if ((rc = launch_pack(shape, k, v, workspace, st))) return rc;
  AttnParams ap;
  fill_attn(ap, shape, q, workspace, o);
  HeadList hl;
  hl.n = n_heads;
  for (int a = 0; a < n_heads; ++a) hl.head[a] = head_ids[a];
  ap.lws = block_scores ? (float *)((char *)workspace + pack_bytes(shape)) : nullptr;
  ap.scores = block_scores;
  return launch_attn<true>(shape, ap, hl, st);
}

sp_status sp_build_block_mask(const float *block_scores, int32_t n_maps, int32_t nqb, int32_t nkb, float gamma,
                              int32_t *kb_idx, int32_t *kb_cnt, uint64_t *bitmask, void *hip_stream) {
  g_err[0] = 0;
  if (!block_scores || !kb_idx || !kb_cnt) {
    set_err("block_scores / kb_idx / kb_cnt must not be NULL");
    return SP_ERR_INVALID_ARG;
  }
  if (n_maps <= 0 || nqb <= 0 || nkb <= 0) {
    set_err("n_maps, nqb, nkb must be positive");
    return SP_ERR_INVALID_ARG;
  }
  if (nqb != nkb) {
    set_err("nqb (%d) != nkb (%d): causal prefill maps are square", nqb, nkb);
    return SP_ERR_INVALID_ARG;
  }
  if (nkb > 32768) {
    set_err("nkb %d exceeds 32768", nkb);
    return SP_ERR_UNSUPPORTED;
  }
  if (!(gamma > 0.f) || gamma > 1.f) {
    set_err("gamma %g outside (0, 1]", (double)gamma);
    return SP_ERR_INVALID_ARG;
  }
  if ((int64_t)n_maps * nqb > 0x7FFFFFF0ll) {
    set_err("too many rows");
    return SP_ERR_UNSUPPORTED;
  }
  return launch_mask(block_scores, n_maps, nqb, nkb, gamma, kb_idx, kb_cnt, bitmask, (hipStream_t)hip_stream);
}

static sp_status sparse_attn_impl(const sp_shape *shape, const void *q, const void *k, const void *v,
                                  const int32_t *head_ids, const int32_t *head_map, int32_t n_heads,
                                  const int32_t *kb_idx, const int32_t *kb_cnt, int32_t n_maps,
                                  const int32_t *head_pattern, void *o, void *workspace, size_t workspace_bytes,
                                  void *hip_stream) {
  g_err[0] = 0;
  sp_status rc = check_shape(shape);
  if (rc) return rc;
  if ((rc = check_ptr16(q, "q")) || (rc = check_ptr16(k, "k")) || (rc = check_ptr16(v, "v")) ||
      (rc = check_ptr16(o, "o")))
    return rc;
  if ((rc = check_heads(shape, head_ids, n_heads, "head_ids"))) return rc;
  if ((!head_map && !head_pattern) || !kb_idx || !kb_cnt) {
    set_err("head_map / head_pattern / kb_idx / kb_cnt must not be NULL");
    return SP_ERR_INVALID_ARG;
  }
  if (n_maps <= 0) {
    set_err("n_maps must be positive");
    return SP_ERR_INVALID_ARG;
  }
  for (int a = 0; head_map && a < n_heads; ++a)
    if (head_map[a] < 0 || head_map[a] >= n_maps) {
      set_err("head_map[%d] = %d outside [0, %d)", a, head_map[a], n_maps);
      return SP_ERR_INVALID_ARG;
    }
  if ((rc = check_ws(workspace, workspace_bytes, pack_bytes(shape)))) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  if ((rc = launch_pack(shape, k, v, workspace, st))) return rc;
  AttnParams ap;
  fill_attn(ap, shape, q, workspace, o);
  HeadList hl;
  hl.n = n_heads;
  ap.n_maps = n_maps;
  for (int a = 0; a < n_heads; ++a) {
    hl.head[a] = head_ids[a];
    hl.map[a] = head_map ? head_map[a] : 0;
  }
  ap.head_pattern = head_pattern;
  ap.n_q_heads = shape->n_q_heads;
  ap.kb_idx = kb_idx;
  ap.kb_cnt = kb_cnt;
  return launch_attn<false>(shape, ap, hl, st);
}

sp_status sp_block_sparse_attn(const sp_shape *shape, const void *q, const void *k, const void *v,
                               const int32_t *head_ids, const int32_t *head_map, int32_t n_heads,
                               const int32_t *kb_idx, const int32_t *kb_cnt, int32_t n_maps, void *o,
                               void *workspace, size_t workspace_bytes, void *hip_stream) {
  if (!head_map) {
    g_err[0] = 0;
    set_err("head_map must not be NULL");
    return SP_ERR_INVALID_ARG;
  }
  return sparse_attn_impl(shape, q, k, v, head_ids, head_map, n_heads, kb_idx, kb_cnt, n_maps, nullptr, o, workspace,
                          workspace_bytes, hip_stream);
}

sp_status sp_block_sparse_attn_gated(const sp_shape *shape, const void *q, const void *k, const void *v,
                                     const int32_t *head_ids, int32_t n_heads, const int32_t *kb_idx,
                                     const int32_t *kb_cnt, int32_t n_maps, const int32_t *head_pattern, void *o,
                                     void *workspace, size_t workspace_bytes, void *hip_stream) {
  if (!head_pattern) {
    g_err[0] = 0;
    set_err("head_pattern must not be NULL");
    return SP_ERR_INVALID_ARG;
  }
  return sparse_attn_impl(shape, q, k, v, head_ids, nullptr, n_heads, kb_idx, kb_cnt, n_maps, head_pattern, o,
                          workspace, workspace_bytes, hip_stream);
}

sp_status sp_determine_pattern(const sp_shape *shape, const void *q, const void *k, const int32_t *head_ids,
                               int32_t n_heads, const int32_t *ref_pos, const int32_t *shared_map, float delta,
                               float tau, float *a_hat, float *dist, int32_t *head_pattern, void *workspace,
                               size_t workspace_bytes, void *hip_stream) {
  g_err[0] = 0;
  sp_status rc = check_shape(shape);
  if (rc) return rc;
  if ((rc = check_ptr16(q, "q")) || (rc = check_ptr16(k, "k"))) return rc;
  if ((rc = check_heads(shape, head_ids, n_heads, "head_ids"))) return rc;
  if (!ref_pos || !shared_map || !a_hat || !dist || !head_pattern) {
    set_err("ref_pos / shared_map / a_hat / dist / head_pattern must not be NULL");
    return SP_ERR_INVALID_ARG;
  }
  for (int a = 0; a < n_heads; ++a)
    if (ref_pos[a] < -1 || ref_pos[a] >= n_heads) {
      set_err("ref_pos[%d] = %d outside [-1, %d)", a, ref_pos[a], n_heads);
      return SP_ERR_INVALID_ARG;
    }
  if ((rc = check_thresholds(delta, tau))) return rc;
  if ((rc = check_ws(workspace, workspace_bytes, pattern_layout(shape, n_heads).gsel))) return rc;
  return launch_determine(shape, q, k, head_ids, n_heads, ref_pos, shared_map, delta, tau, a_hat, dist, head_pattern,
                          (char *)workspace, (hipStream_t)hip_stream);
}

sp_status sp_block_mean_logit_scores(const sp_shape *shape, const void *q, const void *k, const int32_t *head_ids,
                                     int32_t n_heads, float *block_scores, void *workspace, size_t workspace_bytes,
                                     void *hip_stream) {
  g_err[0] = 0;
  sp_status rc = check_shape(shape);
  if (rc) return rc;
  if ((rc = check_ptr16(q, "q")) || (rc = check_ptr16(k, "k"))) return rc;
  if ((rc = check_heads(shape, head_ids, n_heads, "head_ids"))) return rc;
  if (!block_scores || ((uintptr_t)block_scores % 4)) {
    set_err("block_scores is NULL or misaligned");
    return SP_ERR_INVALID_ARG;
  }
  if ((rc = check_ws(workspace, workspace_bytes, pattern_layout(shape, n_heads).gsel))) return rc;
  return launch_mean_logit_scores(shape, q, k, head_ids, n_heads, 0, shape->seq / shape->block, block_scores,
                                  (char *)workspace,
                                  (hipStream_t)hip_stream);
}

static sp_status check_mask_global_args(const float *block_scores, int32_t n_maps, int32_t nqb, int32_t nkb, float gamma,
                                        const int32_t *kb_idx, const int32_t *kb_cnt) {
  if (!block_scores || !kb_idx || !kb_cnt) {
    set_err("block_scores / kb_idx / kb_cnt must not be NULL");
    return SP_ERR_INVALID_ARG;
  }
  if (n_maps <= 0 || nqb <= 0 || nkb <= 0) {
    set_err("n_maps, nqb, nkb must be positive");
    return SP_ERR_INVALID_ARG;
  }
  if (nqb != nkb) {
    set_err("nqb (%d) != nkb (%d): causal prefill maps are square", nqb, nkb);
    return SP_ERR_INVALID_ARG;
  }
  if (nkb > 32768 || n_maps > 65535) {
    set_err("nkb %d exceeds 32768 or n_maps %d exceeds 65535", nkb, n_maps);
    return SP_ERR_UNSUPPORTED;
  }
  if (!(gamma > 0.f) || gamma > 1.f) {
    set_err("gamma %g outside (0, 1]", (double)gamma);
    return SP_ERR_INVALID_ARG;
  }
  return SP_OK;
}

sp_status sp_build_block_mask_global(const float *block_scores, int32_t n_maps, int32_t nqb, int32_t nkb, float gamma,
                                     int32_t forced, int32_t *kb_idx, int32_t *kb_cnt, void *workspace,
                                     size_t workspace_bytes, void *hip_stream) {
  g_err[0] = 0;
  sp_status rc = check_mask_global_args(block_scores, n_maps, nqb, nkb, gamma, kb_idx, kb_cnt);
  if (rc) return rc;
  if ((rc = check_ws(workspace, workspace_bytes, align_up((size_t)n_maps * gsel_map_bytes(nqb), 256)))) return rc;
  return launch_mask_global(block_scores, n_maps, nqb, gamma, forced != 0, kb_idx, kb_cnt, (char *)workspace,
                            (hipStream_t)hip_stream);
}

sp_status sp_build_block_mask_global_static(const float *block_scores, int32_t n_maps, int32_t nqb, int32_t nkb,
                                            float gamma, int32_t forced, int32_t *kb_idx, int32_t *kb_cnt,
                                            void *hip_stream) {
  g_err[0] = 0;
  sp_status rc = check_mask_global_args(block_scores, n_maps, nqb, nkb, gamma, kb_idx, kb_cnt);
  if (rc) return rc;
  const size_t need = align_up((size_t)n_maps * gsel_map_bytes(nqb), 256);
  if (need > SP_STATIC_SCRATCH_BYTES) {
    set_err("selection scratch of %zu bytes (n_maps %d, nqb %d) exceeds the library's static %zu bytes; "
            "use sp_build_block_mask_global with a workspace", need, n_maps, nqb, (size_t)SP_STATIC_SCRATCH_BYTES);
    return SP_ERR_UNSUPPORTED;
  }
  char *scratch_dev = nullptr;
  if ((rc = static_scratch_ptr(&scratch_dev))) return rc;
  return launch_mask_global(block_scores, n_maps, nqb, gamma, forced != 0, kb_idx, kb_cnt, scratch_dev,
                            (hipStream_t)hip_stream);
}

// a_hat / dist / head_pattern all NULL: no gate (every clustered head shares its pivot's pattern)
static sp_status prefill_impl(const sp_shape *shape, const void *q, const void *k, const void *v,
                              const int32_t *head_to_cluster, const int32_t *pivot_heads, int32_t n_clusters,
                              float gamma, int32_t score_mode, int32_t select_mode, bool gated, float delta, float tau,
                              void *o, float *block_scores, int32_t *kb_idx, int32_t *kb_cnt, float *a_hat,
                              float *dist, int32_t *head_pattern, void *workspace, size_t workspace_bytes,
                              void *hip_stream) {
  g_err[0] = 0;
  sp_status rc = check_shape(shape);
  if (rc) return rc;
  if ((rc = check_ptr16(q, "q")) || (rc = check_ptr16(k, "k")) || (rc = check_ptr16(v, "v")) ||
      (rc = check_ptr16(o, "o")))
    return rc;
  if (!head_to_cluster || !pivot_heads || !kb_idx || !kb_cnt) {
    set_err("head_to_cluster / pivot_heads / kb_idx / kb_cnt must not be NULL");
    return SP_ERR_INVALID_ARG;
  }
  if (block_scores && ((uintptr_t)block_scores % 4)) {
    set_err("block_scores is misaligned");
    return SP_ERR_INVALID_ARG;
  }
  if ((score_mode != SP_SCORE_BLOCK_MASS && score_mode != SP_SCORE_MEAN_LOGIT) ||
      (select_mode != SP_SELECT_PER_ROW && select_mode != SP_SELECT_GLOBAL)) {
    set_err("unknown score_mode %d / select_mode %d", score_mode, select_mode);
    return SP_ERR_INVALID_ARG;
  }
  const int Hq = shape->n_q_heads;
  if (n_clusters <= 0 || n_clusters > Hq) {
    set_err("n_clusters %d outside [1, %d]", n_clusters, Hq);
    return SP_ERR_INVALID_ARG;
  }
  if (!(gamma > 0.f) || gamma > 1.f) {
    set_err("gamma %g outside (0, 1]", (double)gamma);
    return SP_ERR_INVALID_ARG;
  }
  bool is_pivot[SP_MAX_HEADS] = {false};
  for (int hq = 0; hq < Hq; ++hq)
    if (head_to_cluster[hq] < -1 || head_to_cluster[hq] >= n_clusters) {
      set_err("head_to_cluster[%d] = %d outside [-1, %d)", hq, head_to_cluster[hq], n_clusters);
      return SP_ERR_INVALID_ARG;
    }
  for (int c = 0; c < n_clusters; ++c) {
    const int ph = pivot_heads[c];
    if (ph < 0 || ph >= Hq) {
      set_err("pivot_heads[%d] = %d outside [0, %d)", c, ph, Hq);
      return SP_ERR_INVALID_ARG;
    }
    if (head_to_cluster[ph] != c) {
      set_err("pivot_heads[%d] = %d lies in cluster %d", c, ph, head_to_cluster[ph]);
      return SP_ERR_INVALID_ARG;
    }
    is_pivot[ph] = true;
  }
  if (gated) {
    if (!a_hat || !dist || !head_pattern) {
      set_err("a_hat / dist / head_pattern must not be NULL");
      return SP_ERR_INVALID_ARG;
    }
    if ((rc = check_thresholds(delta, tau))) return rc;
  }
  const bool mass = score_mode == SP_SCORE_BLOCK_MASS;
  const bool pattern_ws = !mass || select_mode == SP_SELECT_GLOBAL || gated;
  const size_t off_lws = pack_bytes(shape);
  const size_t off_pat = off_lws + (mass ? lws_bytes(shape, n_clusters) : 0);
  const PatternLayout PL = pattern_layout(shape, n_clusters);
  const PatternLayout PG = pattern_layout(shape, Hq);  // the gate pools every head
  const size_t off_tab = off_pat + (pattern_ws ? (gated ? PG.total : PL.total) : 0);
  const size_t off_sc = off_tab + (gated ? align_up((size_t)8 * shape->batch * Hq * sizeof(int32_t), 256) : 0);
  const size_t need = off_sc + (block_scores ? 0 : scores_bytes(shape, n_clusters));
  if ((rc = check_ws(workspace, workspace_bytes, need))) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  const int nqb = shape->seq / shape->block;
  char *ws = (char *)workspace;
  if (!block_scores) block_scores = (float *)(ws + off_sc);  // the caller does not want the maps back

  if ((rc = launch_pack(shape, k, v, workspace, st))) return rc;
  // 1. pivots: dense attention (Alg. 4: no pattern yet => all ones) and their block score map
  //    (Alg. 1 line 8): block mass from the same sweep, or the row softmax of the block-mean logits
  AttnParams ap;
  fill_attn(ap, shape, q, workspace, o);
  HeadList hl;
  hl.n = n_clusters;
  for (int c = 0; c < n_clusters; ++c) hl.head[c] = pivot_heads[c];
  if (mass) {
    ap.lws = (float *)(ws + off_lws);
    ap.scores = block_scores;
  }
  if ((rc = launch_attn<true>(shape, ap, hl, st))) return rc;
  if (!mass && (rc = launch_mean_logit_scores(shape, q, k, pivot_heads, n_clusters, 0, nqb, block_scores, ws + off_pat, st)))
    return rc;
  // 2. heads outside every cluster: dense, no scores
  fill_attn(ap, shape, q, workspace, o);
  hl.n = 0;
  for (int hq = 0; hq < Hq; ++hq)
    if (head_to_cluster[hq] < 0) hl.head[hl.n++] = hq;
  if (hl.n) {
    if ((rc = launch_attn<true>(shape, ap, hl, st))) return rc;
  }
  // 2b. Alg. 3: every head's last-row estimate, the pivot's serving as its cluster's representative;
  //     heads outside every cluster and pivots keep running dense whatever the gate says
  if (gated) {
    int32_t all[SP_MAX_HEADS], ref[SP_MAX_HEADS], smap[SP_MAX_HEADS];
    for (int hq = 0; hq < Hq; ++hq) {
      all[hq] = hq;
      ref[hq] = head_to_cluster[hq] >= 0 ? pivot_heads[head_to_cluster[hq]] : -1;
      smap[hq] = head_to_cluster[hq];  // -1 for unclustered heads: never shared
    }
    if ((rc = launch_determine(shape, q, k, all, Hq, ref, smap, delta, tau, a_hat, dist, head_pattern, ws + off_pat, st)))
      return rc;
  }
  // 3. one pattern per (batch, cluster) (Alg. 2: per query-block row, or over the flattened map)
  if (select_mode == SP_SELECT_PER_ROW)
    rc = launch_mask(block_scores, shape->batch * n_clusters, nqb, nqb, gamma, kb_idx, kb_cnt, nullptr, st);
  else
    rc = launch_mask_global(block_scores, shape->batch * n_clusters, nqb, gamma, 1, kb_idx, kb_cnt,
                            ws + off_pat + (gated ? PG.gsel : PL.gsel), st);
  if (rc) return rc;
  // 4. remaining heads share their cluster's pattern (Alg. 4) and run block-sparse (Sec. 5.1)
  fill_attn(ap, shape, q, workspace, o);
  hl.n = 0;
  for (int hq = 0; hq < Hq; ++hq)
    if (head_to_cluster[hq] >= 0 && !is_pivot[hq]) {
      hl.head[hl.n] = hq;
      hl.map[hl.n] = head_to_cluster[hq];
      ++hl.n;
    }
  if (hl.n && !gated) {
    ap.n_maps = n_clusters;
    ap.kb_idx = kb_idx;
    ap.kb_cnt = kb_cnt;
    ap.n_q_heads = Hq;
    if ((rc = launch_attn<false>(shape, ap, hl, st))) return rc;
  }
  if (hl.n && gated) {
    // the gate's decisions live on the device: split the heads there into those that share a list and those
    // that fall back to dense, and launch each class on its own, spread evenly over the XCDs
    sort_head_list(hl, Hq / shape->n_kv_heads, false);
    ClassifyParams cp;
    memset(&cp, 0, sizeof(cp));
    cp.role = head_pattern;
    cp.shared_pos = (int32_t *)(ws + off_tab);
    cp.fallback_pos = cp.shared_pos + (size_t)shape->batch * Hq;
    cp.shared_n = cp.fallback_pos + (size_t)shape->batch * Hq;
    cp.fallback_n = cp.shared_n + shape->batch;
    cp.n_q_heads = Hq;
    cp.n_launch = hl.n;
    for (int a = 0; a < hl.n; ++a) cp.launch_head[a] = hl.head[a];
    hipLaunchKernelGGL(classify_heads_kernel, dim3(shape->batch), dim3(64), 0, st, cp);
    if ((rc = hip_check(hipGetLastError(), "classify_heads_kernel launch"))) return rc;
    for (int cls = 0; cls < 2; ++cls) {
      fill_attn(ap, shape, q, workspace, o);
      ap.n_maps = n_clusters;
      ap.kb_idx = kb_idx;
      ap.kb_cnt = kb_cnt;
      ap.head_pattern = head_pattern;
      ap.n_q_heads = Hq;
      ap.act_n = cls == 0 ? cp.shared_n : cp.fallback_n;
      ap.act_pos = cls == 0 ? cp.shared_pos : cp.fallback_pos;
      if ((rc = launch_attn<false>(shape, ap, hl, st))) return rc;
    }
  }
  return SP_OK;
}

sp_status sp_prefill_layer_modes(const sp_shape *shape, const void *q, const void *k, const void *v,
                                 const int32_t *head_to_cluster, const int32_t *pivot_heads, int32_t n_clusters,
                                 float gamma, int32_t score_mode, int32_t select_mode, void *o, float *block_scores,
                                 int32_t *kb_idx, int32_t *kb_cnt, void *workspace, size_t workspace_bytes,
                                 void *hip_stream) {
  return prefill_impl(shape, q, k, v, head_to_cluster, pivot_heads, n_clusters, gamma, score_mode, select_mode, false,
                      0.f, 0.f, o, block_scores, kb_idx, kb_cnt, nullptr, nullptr, nullptr, workspace, workspace_bytes,
                      hip_stream);
}

sp_status sp_prefill_layer_gated(const sp_shape *shape, const void *q, const void *k, const void *v,
                                 const int32_t *head_to_cluster, const int32_t *pivot_heads, int32_t n_clusters,
                                 float gamma, float delta, float tau, int32_t score_mode, int32_t select_mode, void *o,
                                 float *block_scores, int32_t *kb_idx, int32_t *kb_cnt, float *a_hat, float *dist,
                                 int32_t *head_pattern, void *workspace, size_t workspace_bytes, void *hip_stream) {
  return prefill_impl(shape, q, k, v, head_to_cluster, pivot_heads, n_clusters, gamma, score_mode, select_mode, true,
                      delta, tau, o, block_scores, kb_idx, kb_cnt, a_hat, dist, head_pattern, workspace,
                      workspace_bytes, hip_stream);
}


sp_status sp_prefill_layer_dict(const sp_shape *shape, const void *q, const void *k, const void *v,
                                const int32_t *head_to_cluster, float gamma, float delta, float tau,
                                int32_t score_mode, int32_t select_mode, int32_t fallback_mode,
                                const sp_pattern_dict *dict, void *o, float *block_scores, int32_t *role, float *a_hat,
                                float *dist, int32_t *vs_idx, int32_t *vs_cnt, void *workspace, size_t workspace_bytes,
                                void *hip_stream) {
  g_err[0] = 0;
  sp_status rc = check_shape(shape);
  if (rc) return rc;
  if ((rc = check_ptr16(q, "q")) || (rc = check_ptr16(k, "k")) || (rc = check_ptr16(v, "v")) ||
      (rc = check_ptr16(o, "o")))
    return rc;
  if (!head_to_cluster || !dict || !block_scores || !role || !a_hat || !dist) {
    set_err("head_to_cluster / dict / block_scores / role / a_hat / dist must not be NULL");
    return SP_ERR_INVALID_ARG;
  }
  if (dict->n_clusters <= 0 || !dict->valid || !dict->a_tilde || !dict->kb_idx || !dict->kb_cnt) {
    set_err("dict: n_clusters must be positive and valid / a_tilde / kb_idx / kb_cnt non-NULL");
    return SP_ERR_INVALID_ARG;
  }
  if ((score_mode != SP_SCORE_BLOCK_MASS && score_mode != SP_SCORE_MEAN_LOGIT) ||
      (select_mode != SP_SELECT_PER_ROW && select_mode != SP_SELECT_GLOBAL)) {
    set_err("unknown score_mode %d / select_mode %d", score_mode, select_mode);
    return SP_ERR_INVALID_ARG;
  }
  if (!(gamma > 0.f) || gamma > 1.f) {
    set_err("gamma %g outside (0, 1]", (double)gamma);
    return SP_ERR_INVALID_ARG;
  }
  if ((rc = check_thresholds(delta, tau))) return rc;
  if (fallback_mode != SP_FALLBACK_DENSE && fallback_mode != SP_FALLBACK_VERTICAL_SLASH &&
      fallback_mode != SP_FALLBACK_VERTICAL_SLASH_TOKEN) {
    set_err("unknown fallback_mode %d", fallback_mode);
    return SP_ERR_INVALID_ARG;
  }
  const bool vs = fallback_mode == SP_FALLBACK_VERTICAL_SLASH;
  const bool vst = fallback_mode == SP_FALLBACK_VERTICAL_SLASH_TOKEN;
  if (vs && (!vs_idx || !vs_cnt)) {
    set_err("vs_idx / vs_cnt must not be NULL with the vertical-slash fallback");
    return SP_ERR_INVALID_ARG;
  }
  const int Hq = shape->n_q_heads, nqb = shape->seq / shape->block;
  if ((int64_t)shape->batch * dict->n_clusters > 65535) {
    set_err("batch * dict clusters exceeds 65535");
    return SP_ERR_UNSUPPORTED;
  }
  ElectParams ep;
  memset(&ep, 0, sizeof(ep));
  int n_slots = 0;
  for (int hq = 0; hq < Hq; ++hq) {
    const int c = head_to_cluster[hq];
    if (c < -1 || c >= dict->n_clusters) {
      set_err("head_to_cluster[%d] = %d outside [-1, %d)", hq, c, dict->n_clusters);
      return SP_ERR_INVALID_ARG;
    }
    ep.head_cluster[hq] = c;
    ep.head_slot[hq] = -1;
  }
  // slots = the distinct clusters of this layer, ascending: each may elect one pivot here
  for (int c = 0; c < dict->n_clusters; ++c) {
    bool used = false;
    for (int hq = 0; hq < Hq; ++hq)
      if (head_to_cluster[hq] == c) {
        used = true;
        ep.head_slot[hq] = n_slots;
      }
    if (used) ep.slot_cluster[n_slots++] = c;
  }
  const bool mass = score_mode == SP_SCORE_BLOCK_MASS;
  const PatternLayout PG = pattern_layout(shape, Hq);
  const size_t off_lws = pack_bytes(shape);
  const size_t off_pat = off_lws + (mass ? lws_bytes(shape, n_slots) : 0);
  const size_t off_tab = off_pat + PG.total;
  const size_t off_vs = off_tab + align_up((size_t)8 * shape->batch * Hq * sizeof(int32_t), 256);
  const size_t need = off_vs + (vs ? vs_layout(shape, Hq).total : 0) + (vst ? vs_token_layout(shape, Hq).total : 0);
  if ((rc = check_ws(workspace, workspace_bytes, need))) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  char *ws = (char *)workspace;
  int32_t *pivot_head = (int32_t *)(ws + off_tab);
  int32_t *route = pivot_head + (size_t)shape->batch * Hq;
  int32_t *act_pos = route + (size_t)shape->batch * Hq;
  int32_t *shared_pos = act_pos + (size_t)shape->batch * Hq;
  int32_t *fallback_pos = shared_pos + (size_t)shape->batch * Hq;
  int32_t *act_n = fallback_pos + (size_t)shape->batch * Hq;
  int32_t *shared_n = act_n + shape->batch, *fallback_n = shared_n + shape->batch;
  // the role-driven launch at the end lists every clustered head (every head with the vertical-slash fallback)
  HeadList rl;
  for (int hq = 0; hq < Hq; ++hq)
    if (head_to_cluster[hq] >= 0 || vs) {
      rl.head[rl.n] = hq;
      rl.map[rl.n] = head_to_cluster[hq] >= 0 ? head_to_cluster[hq] : dict->n_clusters + hq;
      ++rl.n;
    }
  sort_head_list(rl, shape->n_q_heads / shape->n_kv_heads, false);

  if ((rc = launch_pack(shape, k, v, workspace, st))) return rc;
  // 1. Alg. 3: every head's last-row estimate, then roles (election / sharing / fallback) on the device
  int32_t all[SP_MAX_HEADS];
  for (int hq = 0; hq < Hq; ++hq) all[hq] = hq;
  if ((rc = launch_mean_logit_scores(shape, q, k, all, Hq, nqb - 1, 1, a_hat, ws + off_pat, st))) return rc;
  ep.a_hat = a_hat;
  ep.dist = dist;
  ep.role = role;
  ep.pivot_head = pivot_head;
  ep.route = route;
  ep.act_n = act_n;
  ep.act_pos = act_pos;
  ep.shared_n = shared_n;
  ep.shared_pos = shared_pos;
  ep.fallback_n = fallback_n;
  ep.fallback_pos = fallback_pos;
  ep.n_launch = rl.n;
  for (int a = 0; a < rl.n; ++a) ep.launch_head[a] = rl.head[a];
  ep.valid = dict->valid;
  ep.a_tilde = dict->a_tilde;
  ep.nkb = nqb;
  ep.n_q_heads = Hq;
  ep.n_slots = n_slots;
  ep.n_clusters = dict->n_clusters;
  ep.delta = delta;
  ep.tau = tau;
  {
    ProfScope prof(KK_SCORE, st);
    hipLaunchKernelGGL(elect_kernel, dim3(shape->batch), dim3(1024), 0, st, ep);
    if ((rc = hip_check(hipGetLastError(), "elect_kernel launch"))) return rc;
  }
  AttnParams ap;
  HeadList hl;
  if (n_slots) {
    // 2. elected pivots: dense attention (Alg. 4: no pattern yet => all ones) + their block score map;
    //    one listed position per slot, its head read on the device, empty positions exit at once
    fill_attn(ap, shape, q, workspace, o);
    hl.n = n_slots;
    for (int s2 = 0; s2 < n_slots; ++s2) hl.head[s2] = 0;
    ap.head_dev = pivot_head;
    ap.act_n = act_n;
    ap.act_pos = act_pos;
    ap.n_q_heads = Hq;
    if (mass) {
      ap.lws = (float *)(ws + off_lws);
      ap.scores = block_scores;
    }
    if ((rc = launch_attn<true>(shape, ap, hl, st))) return rc;
    if (!mass && (rc = launch_mean_logit_scores(shape, q, k, nullptr, n_slots, 0, nqb, block_scores, ws + off_pat, st,
                                                pivot_head)))
      return rc;
    // 3. Alg. 2 for the elected slots, written straight into the dictionary
    if (select_mode == SP_SELECT_PER_ROW)
      rc = launch_mask(block_scores, shape->batch * n_slots, nqb, nqb, gamma, dict->kb_idx, dict->kb_cnt, nullptr, st,
                       route);
    else
      rc = launch_mask_global(block_scores, shape->batch * n_slots, nqb, gamma, 1, dict->kb_idx, dict->kb_cnt,
                              ws + off_pat + PG.gsel, st, route);
    if (rc) return rc;
  }
  if (vs) {
    // 4. Alg. 5 for every head whose role is -1 (fallback and heads outside every cluster), lists per head
    if ((rc = launch_vertical_slash(shape, q, k, all, Hq, gamma, 1, role, 1, nullptr, vs_idx, vs_cnt, ws + off_vs, st)))
      return rc;
  } else if (vst) {
    // 4. Alg. 5 and attention over its token-level pattern for every head whose role is -1
    if ((rc = launch_vs_token_attn(shape, q, k, v, (const char *)workspace, all, Hq, gamma, 1, role, o, nullptr,
                                   nullptr, ws + off_vs, st)))
      return rc;
  } else {
    // 4. heads outside every cluster: dense, no scores
    fill_attn(ap, shape, q, workspace, o);
    hl.n = 0;
    for (int hq = 0; hq < Hq; ++hq)
      if (head_to_cluster[hq] < 0) hl.head[hl.n++] = hq;
    if (hl.n) {
      if ((rc = launch_attn<true>(shape, ap, hl, st))) return rc;
    }
  }
  // 5. heads by role: shared -> the dictionary's lists, fallback -> dense or their vertical-slash lists,
  //    pivot -> done above.  Two launches over the same slot table, each restricted on the device to one
  //    weight class (a list-walking head costs a fraction of a falling-back one) and spread over all XCDs.
  if (rl.n) {
    for (int cls = 0; cls < (vst ? 1 : 2); ++cls) {  // token-level fallback heads are done already
      fill_attn(ap, shape, q, workspace, o);
      ap.n_maps = dict->n_clusters;
      ap.kb_idx = dict->kb_idx;
      ap.kb_cnt = dict->kb_cnt;
      ap.head_pattern = role;
      ap.n_q_heads = Hq;
      ap.act_n = cls == 0 ? shared_n : fallback_n;
      ap.act_pos = cls == 0 ? shared_pos : fallback_pos;
      if (vs) {
        ap.priv_idx = vs_idx;
        ap.priv_cnt = vs_cnt;
      }
      if ((rc = launch_attn<false>(shape, ap, rl, st))) return rc;
    }
  }
  return SP_OK;
}

sp_status sp_vs_workspace_bytes(const sp_shape *shape, int32_t n_heads, size_t *bytes) {
  g_err[0] = 0;
  sp_status rc = check_shape(shape);
  if (rc) return rc;
  if (!bytes) {
    set_err("bytes is NULL");
    return SP_ERR_INVALID_ARG;
  }
  if (n_heads < 0 || n_heads > shape->n_q_heads) {
    set_err("n_heads %d outside [0, %d]", n_heads, shape->n_q_heads);
    return SP_ERR_INVALID_ARG;
  }
  *bytes = vs_layout(shape, n_heads).total;
  return SP_OK;
}

sp_status sp_search_vertical_slash(const sp_shape *shape, const void *q, const void *k, const int32_t *head_ids,
                                   int32_t n_heads, float gamma, int32_t forced, float *sums, int32_t *kb_idx,
                                   int32_t *kb_cnt, void *workspace, size_t workspace_bytes, void *hip_stream) {
  g_err[0] = 0;
  sp_status rc = check_shape(shape);
  if (rc) return rc;
  if ((rc = check_ptr16(q, "q")) || (rc = check_ptr16(k, "k"))) return rc;
  if ((rc = check_heads(shape, head_ids, n_heads, "head_ids"))) return rc;
  if (!kb_idx || !kb_cnt) {
    set_err("kb_idx / kb_cnt must not be NULL");
    return SP_ERR_INVALID_ARG;
  }
  if (!(gamma > 0.f) || gamma > 1.f) {
    set_err("gamma %g outside (0, 1]", (double)gamma);
    return SP_ERR_INVALID_ARG;
  }
  if ((rc = check_ws(workspace, workspace_bytes, vs_layout(shape, n_heads).total))) return rc;
  return launch_vertical_slash(shape, q, k, head_ids, n_heads, gamma, forced != 0, nullptr, 0, sums, kb_idx, kb_cnt,
                               (char *)workspace, (hipStream_t)hip_stream);
}

sp_status sp_vs_token_workspace_bytes(const sp_shape *shape, int32_t n_heads, size_t *bytes) {
  g_err[0] = 0;
  sp_status rc = check_shape(shape);
  if (rc) return rc;
  if (!bytes) {
    set_err("bytes is NULL");
    return SP_ERR_INVALID_ARG;
  }
  if (n_heads < 0 || n_heads > shape->n_q_heads) {
    set_err("n_heads %d outside [0, %d]", n_heads, shape->n_q_heads);
    return SP_ERR_INVALID_ARG;
  }
  *bytes = pack_bytes(shape) + vs_token_layout(shape, n_heads).total;
  return SP_OK;
}

sp_status sp_vertical_slash_attn(const sp_shape *shape, const void *q, const void *k, const void *v,
                                 const int32_t *head_ids, int32_t n_heads, float gamma, int32_t forced, void *o,
                                 uint64_t *keep_bits, int64_t *pairs, void *workspace, size_t workspace_bytes,
                                 void *hip_stream) {
  g_err[0] = 0;
  sp_status rc = check_shape(shape);
  if (rc) return rc;
  if ((rc = check_ptr16(q, "q")) || (rc = check_ptr16(k, "k")) || (rc = check_ptr16(v, "v")) ||
      (rc = check_ptr16(o, "o")))
    return rc;
  if ((rc = check_heads(shape, head_ids, n_heads, "head_ids"))) return rc;
  if (!(gamma > 0.f) || gamma > 1.f) {
    set_err("gamma %g outside (0, 1]", (double)gamma);
    return SP_ERR_INVALID_ARG;
  }
  if ((keep_bits && ((uintptr_t)keep_bits % 8)) || (pairs && ((uintptr_t)pairs % 8))) {
    set_err("keep_bits / pairs must be 8-byte aligned");
    return SP_ERR_INVALID_ARG;
  }
  if ((int64_t)shape->batch * n_heads * 2 > 65535) {
    set_err("batch * heads * 2 = %lld exceeds 65535", (long long)shape->batch * n_heads * 2);
    return SP_ERR_UNSUPPORTED;
  }
  const size_t need = pack_bytes(shape) + vs_token_layout(shape, n_heads).total;
  if ((rc = check_ws(workspace, workspace_bytes, need))) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  if ((rc = launch_pack(shape, k, v, workspace, st))) return rc;
  return launch_vs_token_attn(shape, q, k, v, (const char *)workspace, head_ids, n_heads, gamma, forced != 0, nullptr,
                              o, keep_bits, pairs, (char *)workspace + pack_bytes(shape), st);
}

sp_status sp_prefill_layer(const sp_shape *shape, const void *q, const void *k, const void *v,
                           const int32_t *head_to_cluster, const int32_t *pivot_heads, int32_t n_clusters,
                           float gamma, void *o, float *block_scores, int32_t *kb_idx, int32_t *kb_cnt,
                           void *workspace, size_t workspace_bytes, void *hip_stream) {
  return sp_prefill_layer_modes(shape, q, k, v, head_to_cluster, pivot_heads, n_clusters, gamma, SP_SCORE_BLOCK_MASS,
                                SP_SELECT_PER_ROW, o, block_scores, kb_idx, kb_cnt, workspace, workspace_bytes,
                                hip_stream);
}

}  // extern "C"
