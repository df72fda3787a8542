// SharePrefill prefill attention for one layer on gfx950 (MI355X): HIP kernels + C ABI.
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
#include <vector>

#include "shareprefill.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int SP_MAX_HEADS = 128;
constexpr int KT = 64;  // keys per sub-tile

thread_local char g_err[512] = "";

// Optional per-kernel timing (sp_profile_enable / sp_profile_read): every launch is bracketed
// by two HIP events on the caller's stream.  Process-wide, not thread-safe; meant for benches.
enum KernelKind { KK_PACK = 0, KK_DENSE = 1, KK_MASK = 2, KK_SPARSE = 3, KK_SCORE = 4, KK_VS = 5, KK_COUNT = 6 };
struct ProfRec {
  int kind;
  hipEvent_t e0, e1;
};
bool g_prof_on = false;
std::vector<ProfRec> g_prof;

struct ProfScope {
  hipStream_t st;
  bool on;
  ProfRec rec;
  ProfScope(int kind, hipStream_t s) : st(s), on(g_prof_on) {
    if (!on) return;
    rec.kind = kind;
    if (hipEventCreate(&rec.e0) != hipSuccess || hipEventCreate(&rec.e1) != hipSuccess) {
      on = false;
      return;
    }
    (void)hipEventRecord(rec.e0, st);
  }
  ~ProfScope() {
    if (!on) return;
    (void)hipEventRecord(rec.e1, st);
    g_prof.push_back(rec);
  }
};

void set_err(const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

// ---------------------------------------------------------------------------------------------
// pack kernel
// ---------------------------------------------------------------------------------------------
struct PackParams {
  const uint16_t *k, *v;
  char *out;
  int64_t sb, st, sh;  // kv strides (elements)
  int n_kv_heads, n_sub;  // n_sub = seq / 64
};

// One workgroup packs one (batch, kv head, 64-key sub-tile): K image then V image.
template <int D>
__global__ __launch_bounds__(256) void pack_kv_kernel(PackParams p) {
  constexpr int IMG = KT * D * 2;       // bytes of one packed K (or V) image
  constexpr int NCH = IMG / 16;         // 16-byte chunks per image
  constexpr int DS = D / 16;
  constexpr int VROW = D + 8;           // padded LDS row (elements)
  __shared__ __attribute__((aligned(16))) uint16_t vs[KT * VROW];
  const int kt = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x;
  const int64_t base = (int64_t)b * p.sb + (int64_t)kt * KT * p.st + (int64_t)kvh * p.sh;
  char *out = p.out + (((int64_t)b * p.n_kv_heads + kvh) * p.n_sub + kt) * (int64_t)(2 * IMG);

  // stage V rows into LDS (row-major, padded)
  for (int c = tid; c < KT * (D / 8); c += 256) {
    const int key = c / (D / 8), part = c % (D / 8);
    const u32x4 val = *reinterpret_cast<const u32x4 *>(p.v + base + (int64_t)key * p.st + part * 8);
    *reinterpret_cast<u32x4 *>(&vs[key * VROW + part * 8]) = val;
  }
  // K image: fragment f = rb*DS + ds, lane holds key 32rb + c, d = 16ds + 8h ..+7
  for (int c = tid; c < NCH; c += 256) {
    const int f = c >> 6, lane = c & 63;
    const int rb = f / DS, ds = f % DS;
    const int key = 32 * rb + (lane & 31), dpos = 16 * ds + 8 * (lane >> 5);
    const u32x4 val = *reinterpret_cast<const u32x4 *>(p.k + base + (int64_t)key * p.st + dpos);
    *reinterpret_cast<u32x4 *>(out + (int64_t)c * 16) = val;
  }
  __syncthreads();
  // V image: fragment f = db*4 + ks, lane holds dd = 32db + c, keys 16ks + slot(h, e)
  for (int c = tid; c < NCH; c += 256) {
    const int f = c >> 6, lane = c & 63;
    const int db = f >> 2, ks = f & 3;
    const int dd = 32 * db + (lane & 31), h = lane >> 5;
    uint32_t w[4];
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      const int e = 2 * e2;
      const int key0 = 16 * ks + ((e < 4) ? (4 * h + e) : (8 + 4 * h + (e - 4)));
      const uint32_t lo = vs[key0 * VROW + dd], hi = vs[(key0 + 1) * VROW + dd];
      w[e2] = lo | (hi << 16);
    }
    u32x4 val = {w[0], w[1], w[2], w[3]};
    *reinterpret_cast<u32x4 *>(out + IMG + (int64_t)c * 16) = val;
  }
}

// ---------------------------------------------------------------------------------------------
// attention kernel
// ---------------------------------------------------------------------------------------------
constexpr int SP_MAX_SLOTS = SP_MAX_HEADS + 8;
struct AttnParams {
  const uint16_t *q;
  const char *kvp;  // packed K/V images
  uint16_t *o;
  int64_t q_sb, q_st, q_sh, o_sb, o_st, o_sh;
  int seq, nqb, n_kv_heads, group, n_heads, n_maps;
  int rgroups;  // ceil(nqb / 8): query-block rows per strand (see the workgroup mapping in attn_kernel)
  float c;    // softmax scale * log2(e)
  float *lws;     // dense: block-local log2-sum-exp [b][n][nqb][nkb][B], or null
  float *scores;  // dense: [b][n][nqb][nkb], or null
  const int32_t *kb_idx;  // sparse: [b][n_maps][nqb][nkb]
  const int32_t *kb_cnt;  // sparse: [b][n_maps][nqb]
  // sparse, optional: per (batch entry, query head) pattern chosen on the device (Alg. 3's gate):
  // a list index in [0, n_maps), or < 0 = no shared pattern, the head walks every key block 0..i
  const int32_t *head_pattern;  // [b][n_q_heads]; <= -2 = nothing to do for this head in this launch
  int n_q_heads;
  // optional: private lists per (batch entry, query head), used by a head whose head_pattern entry is -1
  // (its vertical-slash pattern) instead of the dense walk: [b][n_q_heads][nqb][nkb] / [b][n_q_heads][nqb]
  const int32_t *priv_idx, *priv_cnt;
  // optional: the query head of listed position n, chosen on the device (pivot election): [b][n_heads],
  // negative = this position is empty
  const int32_t *head_dev;
  // optional, with head_dev: how many listed positions are occupied per batch entry ([b]) and which ones
  // ([b][n_heads], ascending); the workgroup mapping then spreads just those over the XCDs
  const int32_t *act_n, *act_pos;
  int32_t head_ids[SP_MAX_SLOTS];  // query head of each slot, -1 = padding slot
  int32_t head_map[SP_MAX_SLOTS];  // sparse: which list the slot's head uses
  int32_t head_pos[SP_MAX_SLOTS];  // position of the head in the caller's list (scores / lws index)
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// max / sum of a value with its partner in lane ^ 32 (one v_permlane32_swap, no LDS round trip)
__device__ __forceinline__ float max_xor32(float x) {
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__builtin_bit_cast(float, (uint32_t)r[0]), __builtin_bit_cast(float, (uint32_t)r[1]));
}
__device__ __forceinline__ float sum_xor32(float x) {
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __builtin_bit_cast(float, (uint32_t)r[0]) + __builtin_bit_cast(float, (uint32_t)r[1]);
}

// Reference point of the online softmax.  The running reference m only has to stay within
// SP_MAX_SLACK (log2 units) of the true running max: P = 2^(x - m) is then at most 2^SP_MAX_SLACK,
// harmless in fp32 / bf16, and m, l, the block sums and O stay mutually consistent whatever m is.
// Moving m only when the max outgrows it by more than the slack makes O rescaling rare (a lane
// triggers it a handful of times per row instead of at every new maximum).
constexpr float SP_MAX_SLACK = 8.0f;
__device__ __forceinline__ float lazy_max(float m_ref, float tile_max) {
  return (tile_max > m_ref + SP_MAX_SLACK) ? tile_max : m_ref;
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 t = {a, b};
  bf16x2 r = __builtin_convertvector(t, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}

// One wavefront-wide 1 KiB copy HBM/L2 -> LDS without passing through registers: lane l moves the
// 16 bytes at g_uniform + lane_off to LDS byte address lds_base + 16 l (g_uniform and lds_base are
// wave-uniform).  Issued from inline assembly so that the compiler does not serialise it against
// the kernel's own LDS reads; the kernel counts these loads itself (wait_vm).
__device__ __forceinline__ void lds_dma16(const void *g_uniform, uint32_t lane_off, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(lane_off),
               "s"(g_uniform)
               : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Flash-attention sweep over 64-key sub-tiles t = 0 .. nsub-1, 32 queries per wavefront.
//
// Software pipeline (per wavefront), step t:
//     MFMA stream   S[t+1] = K[t+1] Q^T          then   O += V[t]^T P[t]^T
//     VALU stream   P[t] = 2^(S[t] c - m)        then   row max of S[t+1], running-max update
//   interleaved instruction by instruction (a hand-laid schedule), so the softmax runs in the
//   shadow of the matrix pipe.  Steps near the diagonal take a general path (causal mask / skip).
// K and V images ride in LDS rings (RK, RV slots) filled by LDS-direct loads issued DK resp. DV
// steps ahead, one chunk at a time from inside the MFMA groups; one workgroup barrier per step.
// One query block per workgroup (B/32 wavefronts); two workgroups per CU, so each SIMD holds two
// wavefronts of different workgroups and one's barrier / load-issue time is covered by the other.
template <int D, int B, bool DENSE, bool SCORES>
__global__ __launch_bounds__(B * 2, B / 64) void attn_kernel(AttnParams p) {
  constexpr int NW = B / 32;        // wavefronts per workgroup, 32 queries each
  constexpr int SPB = B / KT;       // sub-tiles per key block
  constexpr int IMG = KT * D * 2;   // bytes of a packed K (or V) image
  constexpr int STAGE = 2 * IMG;    // K image + V image in the packed buffer
  constexpr int DS = D / 16;        // k-steps of the QK^T product
  constexpr int DB = D / 32;        // 32-row blocks of O^T
  constexpr int DK = 2, DV = 2;                              // prefetch distances (steps)
  constexpr int RK = DK, RV = DV + 1;                        // ring slots
  constexpr int CH = IMG / 1024 / NW;                        // 1 KiB chunks per wavefront per image
  // Each step issues its CH chunks of K[t+DK] first, then its CH chunks of V[t+DV].  At the top of the next
  // step K[t+1] (issued a step ago) must have landed; the V chunks issued after it are for a later step and
  // may still be in flight (vmcnt counts in order).
  constexpr int VM_KEEP = CH;
  static_assert(IMG % (1024 * NW) == 0, "image must split evenly over the wavefronts");
  __shared__ __attribute__((aligned(1024))) char smem[(RK + RV) * IMG];
  const uint32_t lds_k = (uint32_t)(size_t)(__attribute__((address_space(3))) char *)smem;
  const uint32_t lds_v = lds_k + RK * IMG;

  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, c32 = lane & 31;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront index, kept scalar
  // workgroup -> (XCD, strand, query block, batch).  Workgroups are dealt round-robin to the 8 XCDs by the
  // hardware.  Every listed head is cut into 8 strands (the query blocks i with (nqb-1-i) % 8 == s, all of
  // about equal work and each spanning short and long rows); the 8n strands g = 8*slot + s, in slot-table
  // order, are dealt to the XCDs in contiguous runs of n, so whatever n is every XCD gets the same work and
  // works on at most ceil(n/8)+1 heads (heads that share a KV head sit next to each other and meet in its
  // L2).  Inside an XCD the dispatch order is rows from long to short, then strand number, then head: the
  // heads that walk the same list for the same row are neighbours in time.
  const int xcd = blockIdx.x & 7;
  int rest = blockIdx.x >> 3;
  const int b = rest / (p.n_heads * p.rgroups);
  rest %= p.n_heads * p.rgroups;
  // number of heads this launch really has for batch entry b (all listed ones unless the device says otherwise)
  const int n_act = p.act_n ? __builtin_amdgcn_readfirstlane(p.act_n[b]) : p.n_heads;
  if (n_act <= 0 || rest >= n_act * p.rgroups) return;
  int kk = rest % n_act;  // position inside the XCD's run, enumerated strand number first, head second
  rest /= n_act;
  const int g0 = xcd * n_act, g1 = g0 + n_act - 1;
  int strand = g0;
#pragma unroll
  for (int sn = 0; sn < 8; ++sn) {
    const int lo = (g0 >> 3) + (sn >= (g0 & 7) ? 0 : 1), hi = (g1 >> 3) - (sn <= (g1 & 7) ? 0 : 1);
    const int cnt = hi - lo + 1;  // heads of the run that own a strand number sn
    if (kk >= 0 && kk < cnt) strand = (lo + kk) * 8 + sn;
    kk -= (cnt > 0 ? cnt : 0);
  }
  int slot = strand >> 3;
  if (p.act_pos) slot = __builtin_amdgcn_readfirstlane(p.act_pos[(int64_t)b * p.n_heads + slot]);
  const int i = p.nqb - 1 - (rest * 8 + (strand & 7));
  if (i < 0) return;  // nqb is not a multiple of 8: this strand has one row fewer
  int head = p.head_ids[slot];
  const int nkb = p.nqb;
  const int hpos = p.head_pos[slot];
  if (p.head_dev) {
    head = __builtin_amdgcn_readfirstlane(p.head_dev[(int64_t)b * p.n_heads + hpos]);
    if (head < 0 || head >= p.n_q_heads) return;
  }
  const int kvh = head / p.group;

  const int tq = 32 * w + c32;  // this lane's query inside the block
  bf16x8 qf[DS];
  {
    const uint16_t *qp =
        p.q + (int64_t)b * p.q_sb + ((int64_t)i * B + tq) * p.q_st + (int64_t)head * p.q_sh + 8 * h;
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) qf[ds] = *reinterpret_cast<const bf16x8 *>(qp + 16 * ds);
  }

  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  float m = -INFINITY, l = 0.f, bs = 0.f;

  int nblk;
  const int32_t *list = nullptr;
  if (DENSE) {
    nblk = i + 1;
  } else {
    int map = p.head_map[slot];
    if (p.head_pattern) {
      map = __builtin_amdgcn_readfirstlane(p.head_pattern[(int64_t)b * p.n_q_heads + head]);
      map = map >= p.n_maps ? p.n_maps - 1 : map;
      if (map <= -2) return;
    }
    if (map < 0 && p.priv_idx) {
      const int64_t lrow_id = ((int64_t)b * p.n_q_heads + head) * p.nqb + i;
      nblk = p.priv_cnt[lrow_id];
      nblk = nblk < 0 ? 0 : (nblk > nkb ? nkb : nblk);
      list = p.priv_idx + lrow_id * nkb;
    } else if (map < 0) {
      nblk = i + 1;  // list stays null: dense walk
    } else {
      const int64_t lrow_id = ((int64_t)b * p.n_maps + map) * p.nqb + i;
      nblk = p.kb_cnt[lrow_id];
      nblk = nblk < 0 ? 0 : (nblk > nkb ? nkb : nblk);
      list = p.kb_idx + lrow_id * nkb;
    }
  }
  const int nsub = nblk * SPB;
  const char *kvbase = p.kvp + ((int64_t)b * p.n_kv_heads + kvh) * (int64_t)(p.seq / KT) * STAGE;
  float *lrow = nullptr;
  if (SCORES) lrow = p.lws + ((((int64_t)b * p.n_heads + hpos) * p.nqb + i) * nkb) * B + tq;

  // key block of sub-tile t (t clamped to the sequence; list entries clamped into [0, i]: memory-safe
  // whatever the list holds)
  auto block_of = [&](int t) -> int {
    int e = (t < nsub ? t : nsub - 1) / SPB;
    if (DENSE || list == nullptr) return e;
    const int j = list[e];
    return j < 0 ? 0 : (j > i ? i : j);
  };
  // what this wavefront has to do for sub-tile `sub` of key block j: 0 all of it, 1 causal mask, 2 nothing
  auto mode_of = [&](int j, int sub) -> int {
    if (j != i) return 0;
    const int klo = KT * sub, qlo = 32 * w;
    return (klo > qlo + 31) ? 2 : ((klo + KT - 1 <= qlo) ? 0 : 1);
  };
  // every wavefront moves CH chunks of the image of sub-tile t (clamped) into ring slot `slot_base`
  auto img_src = [&](int t, int j, bool is_v) -> const char * {
    const int tt = t < nsub ? t : nsub - 1;
    return kvbase + (int64_t)(j * SPB + tt % SPB) * STAGE + (is_v ? IMG : 0) + (w * CH) * 1024;
  };
  // chunk n (0 .. CH-1) of this wavefront's share of an image
  auto issue_chunk = [&](const char *src, uint32_t slot_base, int n) {
    lds_dma16(src + n * 1024, lane * 16, slot_base + (w * CH + n) * 1024);
  };
  auto issue_img = [&](int t, int j, bool is_v, uint32_t slot_base) {
    const char *src = img_src(t, j, is_v);
#pragma unroll
    for (int n = 0; n < CH; ++n) issue_chunk(src, slot_base, n);
  };

  auto qk = [&](const char *kbuf, f32x16(&s)[2]) {
    const char *kb = kbuf + lane * 16;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[rb][r] = 0.f;
#pragma unroll
    for (int ds = 0; ds < DS; ++ds)
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) {
        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(kb + (rb * DS + ds) * 1024);
        s[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ds], s[rb], 0, 0, 0);
      }
  };
  // Online softmax, split in two halves that sit in different pipeline steps.
  // tile_max: (optionally causal-masked) row max of a freshly computed S tile; moves the running max,
  // rescales the running sums, returns alpha = 2^(m_old - m_new) for the O accumulators.
  auto tile_max = [&](f32x16(&s)[2], int mode, int sub) -> float {
    if (mode == 1) {
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kk = KT * sub + 32 * rb + 8 * (r >> 2) + 4 * h + (r & 3);
          if (kk > tq) s[rb][r] = -INFINITY;
        }
    }
    float mx = fmaxf(s[0][0], s[0][1]);
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int r = (rb == 0 ? 2 : 0); r < 16; r += 2) mx = fmaxf(mx, fmaxf(s[rb][r], s[rb][r + 1]));
    mx = max_xor32(mx);
    const float m_new = lazy_max(m, mx * p.c);
    const float alpha = fast_exp2(m - m_new);
    m = m_new;
    l *= alpha;
    bs *= alpha;
    return alpha;
  };
  // tile_exp: P = 2^(S*c - m) for a tile whose max is already folded into m; adds the row sums,
  // leaves P rounded to bf16 in pb (the B operand of the PV product)
  auto tile_exp = [&](f32x16(&s)[2], bf16x8(&pb)[4]) {
    float rs0 = 0.f, rs1 = 0.f;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      u32x4 t;
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        const int r = 8 * (ks & 1) + 2 * e2;
        const float p0 = fast_exp2(__builtin_fmaf(s[ks >> 1][r], p.c, -m));
        const float p1 = fast_exp2(__builtin_fmaf(s[ks >> 1][r + 1], p.c, -m));
        rs0 += p0;
        rs1 += p1;
        t[e2] = pack_bf16(p0, p1);
      }
      pb[ks] = __builtin_bit_cast(bf16x8, t);
    }
    const float rs = sum_xor32(rs0 + rs1);
    l += rs;
    bs += rs;
  };
  auto rescale = [&](float alpha) {
    if (__any(alpha != 1.f)) {
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    }
  };
  auto pv = [&](const char *vbuf, const bf16x8(&pb)[4]) {
    const char *vb = vbuf + lane * 16;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(vb + (db * 4 + ks) * 1024);
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[ks], oacc[db], 0, 0, 0);
      }
  };

  // On entry to step t: s_cur = raw S[t] (masked where needed), m / l / bs / O already moved to the
  // running max that includes tile t.  jv = key block of the V image to fetch (tile t+DV), jk = of
  // the K image (tile t+DK).
  // sync_and_fill: wait until the images this step reads have landed for every wavefront, then
  // refill the ring slots the previous step freed.
  auto sync_and_fill = [&](int t, int jv, int jk) {
    wait_vm<VM_KEEP>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    issue_img(t + DK, jk, false, lds_k + ((t + DK) % RK) * IMG);
    issue_img(t + DV, jv, true, lds_v + ((t + DV) % RV) * IMG);
  };
  // fast step: tiles t and t+1 both off the diagonal.  One basic block up to the rescale test.
  auto fast_step = [&](int t, int j0, int jv, int jk, f32x16(&s_cur)[2], f32x16(&s_next)[2]) {
    // the ring refills (K for the step after next, then V for the same step) are dropped one chunk at a time
    // into the MFMA groups below instead of going out in a burst after the barrier
    wait_vm<VM_KEEP>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    const char *ksrc = img_src(t + DK, jk, false);
    const uint32_t kslot = lds_k + ((t + DK) % RK) * IMG;
    const char *vsrc = img_src(t + DV, jv, true);
    const uint32_t vslot = lds_v + ((t + DV) % RV) * IMG;
    const char *kb = smem + ((t + 1) % RK) * IMG + lane * 16;
    const char *vb = smem + (RK + t % RV) * IMG + lane * 16;
    // Hand-laid schedule: NM groups, each = one MFMA + one LDS read (PF fragments ahead) + a slice
    // of the VALU work; nothing may cross a group boundary (sched_barrier).
    //   groups 0 .. NQ-1   : S[t+1] += K frag * Q frag ; exp / row-sum / bf16 pack of S[t]
    //   groups NQ .. NM-1  : O += V frag * P frag       ; row max of S[t+1], running-max update
    constexpr int NQ = 2 * DS, NP = 4 * DB, NM = NQ + NP;
    constexpr int PF = 4;       // LDS fragments read ahead of the MFMA that uses them
    constexpr int MAXTAIL = 4;  // the running-max update sits this many groups before the end
    auto frag = [&](int n) -> bf16x8 {
      if (n < NQ) return *reinterpret_cast<const bf16x8 *>(kb + ((n % 2) * DS + n / 2) * 1024);
      const int np = n - NQ;
      return *reinterpret_cast<const bf16x8 *>(vb + ((np % DB) * 4 + np / DB) * 1024);
    };
    bf16x8 fr[PF + 1];
    bf16x8 pb[4];
    u32x4 pt;
    float rs0 = 0.f, rs1 = 0.f, mx = 0.f, lval = 0.f, alpha = 1.f;
    float xa[16], xb[16];
#pragma unroll
    for (int n = 0; n < PF; ++n) fr[n] = frag(n);
#pragma unroll
    for (int n = 0; n < NM; ++n) {
      if (n + PF < NM) fr[(n + PF) % (PF + 1)] = frag(n + PF);
      if (n < NQ) {
        if (n < 2) {
          f32x16 z;
#pragma unroll
          for (int r = 0; r < 16; ++r) z[r] = 0.f;
          s_next[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[n % (PF + 1)], qf[0], z, 0, 0, 0);
        } else {
          s_next[n % 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[n % (PF + 1)], qf[n / 2], s_next[n % 2], 0, 0, 0);
        }
      }
      // exp units u (2 scores each), three stages in consecutive groups so that no instruction waits
      // on the one just issued: scale+shift in group g(u), exp2 in g(u)+1, row sum + bf16 pack in g(u)+2
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int gu = u * NQ / 16;
        const int ks = u / 4, e2 = u % 4, r = 8 * (ks & 1) + 2 * e2;
        if (gu == n) {
          xa[u] = __builtin_fmaf(s_cur[ks >> 1][r], p.c, -m);
          xb[u] = __builtin_fmaf(s_cur[ks >> 1][r + 1], p.c, -m);
        }
        if (gu + 1 == n) {
          xa[u] = fast_exp2(xa[u]);
          xb[u] = fast_exp2(xb[u]);
        }
        if (gu + 2 == n) {
          rs0 += xa[u];
          rs1 += xb[u];
          pt[e2] = pack_bf16(xa[u], xb[u]);
          if (e2 == 3) pb[ks] = __builtin_bit_cast(bf16x8, pt);
        }
      }
      if (n == NQ + 2) {
        const float rs = sum_xor32(rs0 + rs1);
        l += rs;
        bs += rs;
        if (SCORES && t % SPB == SPB - 1) {  // end of key block j0: log2 of the block's exp-sum
          lval = m + fast_log2(bs);
          bs = 0.f;
        }
      }
      {
        constexpr int GAP = NM / (2 * CH);  // groups between two chunk loads
        if (n % GAP == 1 && n / GAP < CH) issue_chunk(ksrc, kslot, n / GAP);
        if (n % GAP == 1 && n / GAP >= CH && n / GAP < 2 * CH) issue_chunk(vsrc, vslot, n / GAP - CH);
      }
      if (n >= NQ) {
        const int np = n - NQ;
        oacc[np % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[n % (PF + 1)], pb[np / DB], oacc[np % DB], 0, 0, 0);
        // row max of S[t+1]: 16 max3 units spread over groups 2 .. NP-1-MAXTAIL, then the running-max
        // update MAXTAIL groups before the end (its dependent chain hides under the last MFMAs)
#pragma unroll
        for (int u = 0; u < 16; ++u) {
          if (2 + u * (NP - 2 - MAXTAIL) / 16 != np) continue;
          const float a0 = s_next[u / 8][2 * (u % 8)], a1 = s_next[u / 8][2 * (u % 8) + 1];
          mx = (u == 0) ? fmaxf(a0, a1) : fmaxf(mx, fmaxf(a0, a1));
        }
        if (np == NP - MAXTAIL) {
          mx = max_xor32(mx);
          const float m_new = lazy_max(m, mx * p.c);
          alpha = fast_exp2(m - m_new);
          m = m_new;
          l *= alpha;
          bs *= alpha;
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    rescale(alpha);
    if (SCORES && t % SPB == SPB - 1 && h == 0) lrow[(int64_t)j0 * B] = lval;
  };
  // general step: per-wavefront causal mask / skip near the diagonal, optional next tile
  auto slow_step = [&](int t, int j0, int j1, int jv, int jk, f32x16(&s_cur)[2], f32x16(&s_next)[2]) {
    sync_and_fill(t, jv, jk);
    const char *k_next = smem + ((t + 1) % RK) * IMG;
    const char *v_cur = smem + (RK + t % RV) * IMG;
    const int sub = t % SPB, sub1 = (t + 1) % SPB;
    const int mode0 = mode_of(j0, sub);
    const int mode1 = (t + 1 < nsub) ? mode_of(j1, sub1) : 2;
    if (mode1 != 2) qk(k_next, s_next);
    if (mode0 != 2) {
      bf16x8 pb[4];
      tile_exp(s_cur, pb);
      pv(v_cur, pb);
    }
    if (SCORES && sub == SPB - 1 && mode_of(j0, 0) != 2) {
      if (h == 0) lrow[(int64_t)j0 * B] = m + fast_log2(bs);
      bs = 0.f;
    }
    if (mode1 != 2) rescale(tile_max(s_next, mode1, sub1));
  };

  if (nsub > 0) {
    // leading run of sub-tiles that lie before the first diagonal entry of the list
    int nfast;
    if (DENSE || list == nullptr) {
      nfast = i * SPB;
    } else {
      int first = nblk;
      for (int e = lane; e < nblk; e += 64)
        if (list[e] >= i) first = first < e ? first : e;
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) {
        const int o2 = __shfl_xor(first, off, 64);
        first = first < o2 ? first : o2;
      }
      nfast = __builtin_amdgcn_readfirstlane(first) * SPB;
    }
    // fast steps need tile t+1 off the diagonal too; keep their count even (tail starts on even parity)
    nfast = nfast > 0 ? ((nfast - 1) & ~1) : 0;

    f32x16 s_a[2], s_b[2];
    // jw[n] = key block of sub-tile t + n
    int jw[6];
#pragma unroll
    for (int n = 0; n < 6; ++n) jw[n] = block_of(n);
    // prologue: K[0 .. DK-1], V[0 .. DV-1]
#pragma unroll
    for (int n = 0; n < DK; ++n) {
      if (n < DV && n < nsub) issue_img(n, jw[n], true, lds_v + (n % RV) * IMG);
      if (n < nsub) issue_img(n, jw[n], false, lds_k + (n % RK) * IMG);
    }
    wait_vm<0>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    {
      const int mode = mode_of(jw[0], 0);
      if (mode != 2) {
        qk(smem, s_a);
        tile_max(s_a, mode, 0);  // O is still zero: nothing to rescale
      }
    }
    int t = 0;
    for (; t < nfast; t += 2) {
      const int jn0 = block_of(t + 6), jn1 = block_of(t + 7);
      fast_step(t, jw[0], jw[DV], jw[DK], s_a, s_b);
      fast_step(t + 1, jw[1], jw[DV + 1], jw[DK + 1], s_b, s_a);
#pragma unroll
      for (int n = 0; n < 4; ++n) jw[n] = jw[n + 2];
      jw[4] = jn0;
      jw[5] = jn1;
    }
    for (; t < nsub; t += 2) {
      const int jn0 = block_of(t + 6), jn1 = block_of(t + 7);
      slow_step(t, jw[0], jw[1], jw[DV], jw[DK], s_a, s_b);
      if (t + 1 < nsub) slow_step(t + 1, jw[1], jw[2], jw[DV + 1], jw[DK + 1], s_b, s_a);
#pragma unroll
      for (int n = 0; n < 4; ++n) jw[n] = jw[n + 2];
      jw[4] = jn0;
      jw[5] = jn1;
    }
    wait_vm<0>();  // drain the ring's look-ahead loads before the LDS is reused or released
  }

  // ---- output: O = O^T accumulators / l, rounded to bf16 ----
  {
    const float inv = (l > 0.f) ? 1.f / l : 0.f;
    uint16_t *op = p.o + (int64_t)b * p.o_sb + ((int64_t)i * B + tq) * p.o_st + (int64_t)head * p.o_sh;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        u32x2 t;
        t[0] = pack_bf16(oacc[db][4 * gq] * inv, oacc[db][4 * gq + 1] * inv);
        t[1] = pack_bf16(oacc[db][4 * gq + 2] * inv, oacc[db][4 * gq + 3] * inv);
        *reinterpret_cast<u32x2 *>(op + 32 * db + 8 * gq + 4 * h) = t;
      }
  }

  // ---- block-mass scores: S[i][j] = (1/B) sum_t 2^(lws[j][t] - L_t) ----
  // Each wavefront takes 32 key blocks at a time.  Stage 1: lane <-> query, coalesced reads of the block
  // log-sum-exps, one partial per (key block, lane) into a wavefront-private LDS tile (rows padded to 65
  // floats).  Stage 2: lane <-> key block, the tile is read transposed and summed.  No cross-lane reduction
  // chain and several rows of loads in flight: the workspace rows were written long ago and come from HBM.
  if (SCORES) {
    constexpr int TPL = B / 64, PST = 65, JU = 8;
    constexpr int JB = (1024 + NW * 32 * PST * 4 <= (RK + RV) * IMG) ? 32 : 16;  // key blocks per tile
    constexpr int NPART = 64 / JB, PLEN = 64 / NPART;  // stage 2: NPART lanes share a key block, PLEN entries each
    static_assert(1024 + NW * JB * PST * 4 <= (RK + RV) * IMG, "score epilogue tiles must fit the idle rings");
    float *lse_sh = reinterpret_cast<float *>(smem);  // [B]; the rings are idle now
    float *part = reinterpret_cast<float *>(smem + 1024) + w * (JB * PST);
    __syncthreads();
    if (h == 0) lse_sh[tq] = m + fast_log2(l);
    __threadfence();
    __syncthreads();
    float lt[TPL];
#pragma unroll
    for (int tt = 0; tt < TPL; ++tt) lt[tt] = lse_sh[lane + 64 * tt];
    const float *lblk = p.lws + ((((int64_t)b * p.n_heads + hpos) * p.nqb + i) * nkb) * B;
    float *srow = p.scores + (((int64_t)b * p.n_heads + hpos) * p.nqb + i) * nkb;
    const int jr = lane % JB, jp = lane / JB;
    for (int j0 = w * JB; j0 <= i; j0 += NW * JB) {
#pragma unroll
      for (int u0 = 0; u0 < JB; u0 += JU) {
        float x[JU][TPL];
#pragma unroll
        for (int u = 0; u < JU; ++u) {
          const int j = (j0 + u0 + u <= i) ? j0 + u0 + u : i;
#pragma unroll
          for (int tt = 0; tt < TPL; ++tt) x[u][tt] = lblk[(int64_t)j * B + lane + 64 * tt];
        }
#pragma unroll
        for (int u = 0; u < JU; ++u) {
          float e = 0.f;
#pragma unroll
          for (int tt = 0; tt < TPL; ++tt) e += fast_exp2(x[u][tt] - lt[tt]);
          part[(u0 + u) * PST + lane] = e;
        }
      }
      // the tile is private to this wavefront: order its own LDS writes before its transposed reads
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      float acc = 0.f;
#pragma unroll
      for (int kq = 0; kq < PLEN; ++kq) acc += part[jr * PST + jp * PLEN + kq];
      acc = sum_xor32(acc);
      if (NPART == 4) acc += __shfl_xor(acc, 16, 64);
      if (jp == 0 && j0 + jr <= i) srow[j0 + jr] = acc * (1.f / B);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    for (int j = i + 1 + w * 64 + lane; j < nkb; j += NW * 64) srow[j] = 0.f;
  }
}

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
// bit 0 = some entry of the row is kept, bit 1 = some entry other than the row's first is kept.
__global__ __launch_bounds__(256) void gsel_emit_flags_kernel(const float *__restrict__ scores, GselGeom g, char *scratch,
                                                              int32_t *__restrict__ flags) {
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
  }
  if (lane == 0) flags[(int64_t)map * g.n_rows + row] = any | (any_after_first << 1);
}

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
  if (s->seq % 128) {
    set_err("seq %d is not a multiple of 128", s->seq);
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
size_t lws_bytes(const sp_shape *s, int n_dense) {
  const size_t nqb = s->seq / s->block;
  return align_up((size_t)s->batch * n_dense * nqb * nqb * s->block * sizeof(float), 256);
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
                                int32_t *kb_idx, int32_t *kb_cnt, char *vs_ws, hipStream_t st) {
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
  const dim3 glog(s->seq / 128, n, s->batch), gstat(s->block, n, s->batch), gsum((s->seq + 255) / 256, n, s->batch);
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
                     vs_ws + L.gsel, flags);
  hipLaunchKernelGGL(vs_block_lists_kernel, dim3((nkb + 3) / 4, n, s->batch), dim3(256), 0, st, vp, flags, nkb, forced,
                     by_head, kb_idx, kb_cnt);
  return hip_check(hipGetLastError(), "vertical-slash selection kernels launch");
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

// ---------------------------------------------------------------------------------------------
// step-mix probe (measurement aid): the instruction mix of one attention step, nothing around it
// ---------------------------------------------------------------------------------------------
namespace {

// Per step and wavefront: G MFMAs on four independent accumulators; a 1 KiB fragment read from LDS for
// every LP-th MFMA (4 groups ahead of its use, as in attn_kernel); C LDS-direct 1 KiB loads spread over
// the groups; V FMAs and E exp2 per MFMA; a barrier per step when there are loads.  LDS: a 32 KiB read
// window, above it the wavefronts' load windows.  Every workgroup streams its own 1 MiB of `src`.
template <int LP, int C, int V, int E, int G, int LDSB>
__global__ __launch_bounds__(256) void probe_kernel(const char *__restrict__ src, float *__restrict__ sink, int iters) {
  static_assert(32768 + 4 * C * 1024 <= LDSB, "load windows must fit");
  static_assert(G <= 64 && (C == 0 || G % C == 0), "group layout");
  __shared__ __attribute__((aligned(1024))) char smem[LDSB];
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const char *gsrc = src + (size_t)(blockIdx.x % 64) * (1 << 20);
  for (int i = tid; i < 32768 / 16; i += 256)
    reinterpret_cast<u32x4 *>(smem)[i] = reinterpret_cast<const u32x4 *>(gsrc)[i];
  __syncthreads();
  const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) char *)smem;
  const bf16x8 b = reinterpret_cast<const bf16x8 *>(gsrc + 65536)[tid];
  f32x16 acc[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[n][r] = 0.f;
  float x[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) x[i] = 0.5f + 0.01f * i + lane * 1e-4f;
  const char *rd = smem + lane * 16;
  constexpr int PF = 4;
  bf16x8 fr[PF + 1];
#pragma unroll
  for (int n = 0; n < PF + 1; ++n) fr[n] = b;
  for (int it = 0; it < iters; ++it) {
    if (C > 0) {
      wait_vm<C / 2>();
      __builtin_amdgcn_s_barrier();
    }
    const char *gs = gsrc + (size_t)(it & 7) * 65536 + (size_t)(w * C) * 1024 + 131072;
    const uint32_t wslot = lds0 + 32768 + (uint32_t)(w * C) * 1024;
#pragma unroll
    for (int n = 0; n < G; ++n) {
      if (LP > 0 && n % LP == 0)
        fr[(n + PF) % (PF + 1)] = *reinterpret_cast<const bf16x8 *>(rd + (n % 32) * 1024);
      acc[n % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[LP > 0 ? ((n / LP) * LP) % (PF + 1) : 0], b, acc[n % 4],
                                                           0, 0, 0);
#pragma unroll
      for (int v = 0; v < V; ++v) {
        const int i = (n * V + v) % 16;
        x[i] = __builtin_fmaf(x[i], 0.999f, 0.0007f);
      }
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const float y = fast_exp2(x[(n * E + e + 8) % 16]);
        asm volatile("" ::"v"(y));
      }
      if (C > 0 && n % (G / (C > 0 ? C : 1)) == 1) {
        constexpr int GAP = G / (C > 0 ? C : 1);
        lds_dma16(gs + (n / GAP) * 1024, lane * 16, wslot + (n / GAP) * 1024);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  wait_vm<0>();
  float s = 0.f;
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[n][r];
#pragma unroll
  for (int i = 0; i < 16; ++i) s += x[i];
  sink[(size_t)blockIdx.x * 256 + tid] = s;
}

template <int LP, int C, int V, int E, int G, int LDSB>
sp_status launch_probe(const void *operands, float *sink, int iters, int n_wg, hipStream_t st) {
  hipLaunchKernelGGL((probe_kernel<LP, C, V, E, G, LDSB>), dim3(n_wg), dim3(256), 0, st, (const char *)operands, sink,
                     iters);
  return hip_check(hipGetLastError(), "probe_kernel launch");
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
  g_prof_on = on != 0;
  return SP_OK;
}

sp_status sp_profile_read(float *ms, int32_t *launches, int32_t reset) {
  g_err[0] = 0;
  if (!ms || !launches) {
    set_err("ms / launches must not be NULL");
    return SP_ERR_INVALID_ARG;
  }
  for (int a = 0; a < KK_COUNT; ++a) {
    ms[a] = 0.f;
    launches[a] = 0;
  }
  sp_status rc = SP_OK;
  for (const ProfRec &r : g_prof) {
    float t = 0.f;
    const hipError_t e = hipEventElapsedTime(&t, r.e0, r.e1);
    if (e != hipSuccess) {
      rc = hip_check(e, "hipEventElapsedTime (synchronise the stream before sp_profile_read)");
      break;
    }
    ms[r.kind] += t;
    launches[r.kind] += 1;
  }
  if (reset && rc == SP_OK) {
    for (const ProfRec &r : g_prof) {
      (void)hipEventDestroy(r.e0);
      (void)hipEventDestroy(r.e1);
    }
    g_prof.clear();
  }
  return rc;
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
           align_up((size_t)8 * shape->batch * shape->n_q_heads * sizeof(int32_t), 256);
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

sp_status sp_build_block_mask_global(const float *block_scores, int32_t n_maps, int32_t nqb, int32_t nkb, float gamma,
                                     int32_t forced, int32_t *kb_idx, int32_t *kb_cnt, void *workspace,
                                     size_t workspace_bytes, void *hip_stream) {
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
  if (nkb > 32768 || n_maps > 65535) {
    set_err("nkb %d exceeds 32768 or n_maps %d exceeds 65535", nkb, n_maps);
    return SP_ERR_UNSUPPORTED;
  }
  if (!(gamma > 0.f) || gamma > 1.f) {
    set_err("gamma %g outside (0, 1]", (double)gamma);
    return SP_ERR_INVALID_ARG;
  }
  sp_status rc = check_ws(workspace, workspace_bytes, align_up((size_t)n_maps * gsel_map_bytes(nqb), 256));
  if (rc) return rc;
  return launch_mask_global(block_scores, n_maps, nqb, gamma, forced != 0, kb_idx, kb_cnt, (char *)workspace,
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
  if (!head_to_cluster || !pivot_heads || !block_scores || !kb_idx || !kb_cnt) {
    set_err("head_to_cluster / pivot_heads / block_scores / kb_idx / kb_cnt must not be NULL");
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
  const size_t need = off_tab + (gated ? align_up((size_t)8 * shape->batch * Hq * sizeof(int32_t), 256) : 0);
  if ((rc = check_ws(workspace, workspace_bytes, need))) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  const int nqb = shape->seq / shape->block;
  char *ws = (char *)workspace;

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
    // the gate's verdicts live on the device: split the heads there into those that share a list and those
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
  if (fallback_mode != SP_FALLBACK_DENSE && fallback_mode != SP_FALLBACK_VERTICAL_SLASH) {
    set_err("unknown fallback_mode %d", fallback_mode);
    return SP_ERR_INVALID_ARG;
  }
  const bool vs = fallback_mode == SP_FALLBACK_VERTICAL_SLASH;
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
  const size_t need = off_vs + (vs ? vs_layout(shape, Hq).total : 0);
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
    for (int cls = 0; cls < 2; ++cls) {
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

sp_status sp_prefill_layer(const sp_shape *shape, const void *q, const void *k, const void *v,
                           const int32_t *head_to_cluster, const int32_t *pivot_heads, int32_t n_clusters,
                           float gamma, void *o, float *block_scores, int32_t *kb_idx, int32_t *kb_cnt,
                           void *workspace, size_t workspace_bytes, void *hip_stream) {
  return sp_prefill_layer_modes(shape, q, k, v, head_to_cluster, pivot_heads, n_clusters, gamma, SP_SCORE_BLOCK_MASS,
                                SP_SELECT_PER_ROW, o, block_scores, kb_idx, kb_cnt, workspace, workspace_bytes,
                                hip_stream);
}

sp_status sp_probe_step_mix(int32_t mix, const void *operands, size_t operand_bytes, int32_t iters, float *sink,
                            size_t sink_bytes, double *mfma_flops, void *hip_stream) {
  g_err[0] = 0;
  if (!operands || !sink || !mfma_flops) {
    set_err("operands / sink / mfma_flops must not be NULL");
    return SP_ERR_INVALID_ARG;
  }
  if (((uintptr_t)operands & 15) || operand_bytes < SP_PROBE_OPERAND_BYTES || sink_bytes < SP_PROBE_SINK_BYTES) {
    set_err("operands must be 16-byte aligned and hold %zu bytes, sink %zu bytes", (size_t)SP_PROBE_OPERAND_BYTES,
            (size_t)SP_PROBE_SINK_BYTES);
    return SP_ERR_INVALID_ARG;
  }
  if (mix < SP_PROBE_MFMA || mix > SP_PROBE_STEP_64Q || iters < 1 || iters > 1000000) {
    set_err("mix %d outside [0, 4] or iters %d outside [1, 1000000]", mix, iters);
    return SP_ERR_INVALID_ARG;
  }
  int dev = 0, cus = 0;
  sp_status rc;
  if ((rc = hip_check(hipGetDevice(&dev), "hipGetDevice"))) return rc;
  if ((rc = hip_check(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev),
                      "hipDeviceGetAttribute")))
    return rc;
  // two workgroups of four wavefronts per CU (80 KiB of LDS each), one for the 64-query mix (160 KiB)
  const int wg_per_cu = mix == SP_PROBE_STEP_64Q ? 1 : 2;
  const int n_wg = cus * wg_per_cu;
  if (cus < 1 || (size_t)n_wg * 256 * sizeof(float) > SP_PROBE_SINK_BYTES) {
    set_err("device reports %d compute units", cus);
    return SP_ERR_UNSUPPORTED;
  }
  const int g = mix == SP_PROBE_STEP_64Q ? 64 : 32;
  *mfma_flops = (double)n_wg * 4 * (double)iters * g * (2.0 * 32 * 32 * 16);
  hipStream_t st = (hipStream_t)hip_stream;
  switch (mix) {
    case SP_PROBE_MFMA: return launch_probe<0, 0, 0, 0, 32, 80 * 1024>(operands, sink, iters, n_wg, st);
    case SP_PROBE_LDS_READ: return launch_probe<1, 0, 0, 0, 32, 80 * 1024>(operands, sink, iters, n_wg, st);
    case SP_PROBE_RING: return launch_probe<1, 8, 0, 0, 32, 80 * 1024>(operands, sink, iters, n_wg, st);
    case SP_PROBE_STEP: return launch_probe<1, 8, 4, 1, 32, 80 * 1024>(operands, sink, iters, n_wg, st);
    default: return launch_probe<2, 8, 4, 1, 64, 160 * 1024>(operands, sink, iters, n_wg, st);
  }
}

}  // extern "C"
