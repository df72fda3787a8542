// Dense / block-sparse flash-attention kernel (Sec. 5.1 A(Q,K,V) and A(Q,K,V,M)) with the block-mass score map.
#ifndef SP_ATTN_KERNEL_H
#define SP_ATTN_KERNEL_H
#include "sp_common.h"

namespace {

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
  float *lws;     // dense: block-local log2-sum-exp [b][n][nqb(nqb+1)/2][B] (row i, key block j <= i), or null
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
// P is rounded to bf16 for the PV product while the row sum l adds the unrounded values.  With m lagging the
// true max, a row's large weights 2^(x - m) are not exactly representable, so in a row that a few keys
// dominate numerator and normaliser would differ by those weights' rounding errors (up to 2^-9 of |O|).
// The kernel therefore keeps a second sum lc = sum of (bf16(p) - p) over every tile that can hold a weight
// above 1/SP_CARE of the row's running sum (the first tiles of a row, tiles with a sink or a heavy key, and
// all tiles near the diagonal), and normalises O by l + lc: every weight that matters enters the
// normaliser as PV saw it; the weights left out are each below 1/SP_CARE of the row, their rounding
// errors are independent and average out.  The block-mass scores keep using l, so their rows sum to 1.
constexpr float SP_MAX_SLACK = 8.0f;
constexpr float SP_CARE = 32.0f;
__device__ __forceinline__ float lazy_max(float m_ref, float tile_max) {
  return (tile_max > m_ref + SP_MAX_SLACK) ? tile_max : m_ref;
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 t = {a, b};
  bf16x2 r = __builtin_convertvector(t, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}

// sum of the eight bf16 values of a packed P fragment, as fp32
__device__ __forceinline__ float sum_bf16x8(bf16x8 v) {
  const u32x4 t = __builtin_bit_cast(u32x4, v);
  float a = 0.f, b = 0.f;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    a += __builtin_bit_cast(float, t[e] << 16);
    b += __builtin_bit_cast(float, t[e] & 0xffff0000u);
  }
  return a + b;
}
__device__ __forceinline__ float max3f(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
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
  float lc = 0.f;     // sum of bf16(p) - p over the tiles summed twice (see SP_CARE)
  bool care = true;   // the tile whose max was taken last may hold a weight that matters

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
  // block log-sum-exps: causal half, row i of a (batch entry, head) starts at i(i+1)/2 key-block slots
  const int64_t lws_row = ((int64_t)b * p.n_heads + hpos) * ((int64_t)p.nqb * (p.nqb + 1) / 2) + (int64_t)i * (i + 1) / 2;
  if (SCORES) lrow = p.lws + lws_row * B + tq;

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
  // move_reference: mx = raw row max of a fresh tile.  Moves the reference if the max outgrew the slack,
  // rescales the running sums, notes whether the tile's largest weight matters to the row (care), returns
  // alpha = 2^(m_old - m_new) for the O accumulators.
  auto move_reference = [&](float mx) -> float {
    const float m_new = lazy_max(m, mx * p.c);
    const float alpha = fast_exp2(m - m_new);
    m = m_new;
    l *= alpha;
    bs *= alpha;
    lc *= alpha;
    care = fast_exp2(__builtin_fmaf(mx, p.c, -m_new)) * SP_CARE > l;
    return alpha;
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
    return move_reference(mx);
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
    lc += sum_xor32(sum_bf16x8(pb[0]) + sum_bf16x8(pb[1]) + sum_bf16x8(pb[2]) + sum_bf16x8(pb[3])) - rs;
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
    float rs0 = 0.f, rs1 = 0.f, mx = 0.f, lval = 0.f, alpha = 1.f, rs_tile = 0.f;
    const bool care_t = care;  // set when this tile's max was taken
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
        rs_tile = rs;
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
          mx = (u == 0) ? fmaxf(a0, a1) : max3f(mx, a0, a1);
        }
        if (np == NP - MAXTAIL) alpha = move_reference(max_xor32(mx));
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (__any(care_t))  // rare: the tile summed again as PV saw it (alpha already holds the move after this tile)
      lc += (sum_xor32(sum_bf16x8(pb[0]) + sum_bf16x8(pb[1]) + sum_bf16x8(pb[2]) + sum_bf16x8(pb[3])) - rs_tile) * alpha;
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
    const float inv = (l > 0.f) ? 1.f / (l + lc) : 0.f;
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
    const float *lblk = p.lws + lws_row * B;
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

}  // namespace

#endif
