// Attention over the vertical-slash pattern of Alg. 5 at token granularity (Sec. 5.1 A(Q,K,V,M) with the mask M
// built from S = S_v U S_s): the kept keys of a head are gathered into packed images of their own, the kept
// offsets are walked as bands of key blocks with a bit mask inside every tile.
#ifndef SP_VS_TOKEN_KERNELS_H
#define SP_VS_TOKEN_KERNELS_H
#include <type_traits>
#include "sp_common.h"
#include "attn_kernel.h"
#include "vertical_slash_kernels.h"

namespace {

// Per listed head (hb = b * n_heads + n), all in the caller's workspace:
//   bits     [hb][2][seq/64] u64   kept keys (bit s) then kept offsets (bit o), written by the vector selection
//   cumv     [hb][nqb+1]           gathered keys with s < x*block (gathered = kept keys outside the forced sink block)
//   gpos     [hb][seq]             token index of gathered key g, ascending
//   cumband  [hb][nqb]             kept bands among 1 .. x (band d = the offsets (d-1)B+1 .. (d+1)B-1 a key block d
//                                  blocks below the diagonal can realise)
//   bandlist [hb][nqb]             the kept bands, ascending
//   gimg     [hb][seq/64][2][64*D] packed K and V images of the gathered keys, 64 keys each, zero padded
//   act_pos  [b][n_heads], act_n [b]  the listed positions that take part (role -1, or all without roles), ascending
constexpr int VST_TASK_ROWS = 16;  // consecutive query blocks of a head that one XCD runs side by side
struct VsTokParams {
  const uint16_t *q, *k, *v;
  const char *kvp;   // packed K/V images of the whole sequence (pack_kv_kernel)
  uint16_t *o;
  int64_t q_sb, q_st, q_sh, kv_sb, kv_st, kv_sh, o_sb, o_st, o_sh;
  int seq, nqb, block, n_kv_heads, group, n_heads, n_q_heads, forced;
  float c;  // softmax scale * log2(e)
  uint64_t *bits;
  int32_t *cumv, *gpos, *cumband, *bandlist, *act_pos, *act_n;
  char *gimg;
  int nch8;  // chunks of VST_TASK_ROWS query blocks per head and XCD: ceil(ceil(nqb / VST_TASK_ROWS) / 8)
  int64_t *pairs;        // optional [b][n]: number of (query, key) pairs of the pattern (statistics)
  const int32_t *role;   // optional [b][n_q_heads]: only heads whose entry is -1 are processed
  int32_t head_ids[SP_MAX_HEADS];
};
__device__ __forceinline__ bool vst_skip(const VsTokParams &p, int b, int n) {
  return p.role != nullptr && p.role[(int64_t)b * p.n_q_heads + p.head_ids[n]] != -1;
}

// exclusive prefix sum of one value per thread over a 1024-thread workgroup; returns the total in `total`
__device__ __forceinline__ int block_scan_1024(int x, int *sh, int &total) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  int inc = x;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int y = __shfl_up(inc, off, 64);
    if (lane >= off) inc += y;
  }
  if (lane == 63) sh[w] = inc;
  __syncthreads();
  int base = 0, tot = 0;
  for (int a = 0; a < 16; ++a) {
    const int s = sh[a];
    if (a < w) base += s;
    tot += s;
  }
  __syncthreads();
  total = tot;
  return base + inc - x;
}

// One workgroup of 1024 threads per listed head: the list of heads that take part, ranks of the kept keys, kept bands.
__global__ __launch_bounds__(1024) void vs_token_prep_kernel(VsTokParams p) {
  __shared__ int sh[16];
  const int n = blockIdx.x, b = blockIdx.y;
  {  // this head's rank among the heads that take part, and their number
    const int a = threadIdx.x;
    const bool on = a < p.n_heads && !vst_skip(p, b, a);
    const int total = __syncthreads_count(on), rank = __syncthreads_count(on && a < n);
    if (threadIdx.x == 0) {
      if (n == 0) p.act_n[b] = total;
      if (!vst_skip(p, b, n)) p.act_pos[(int64_t)b * p.n_heads + rank] = n;
    }
  }
  if (vst_skip(p, b, n)) return;
  const int64_t hb = (int64_t)b * p.n_heads + n;
  const int nw = p.seq / 64, B = p.block, wpb = B / 64;
  const uint64_t *bv = p.bits + hb * 2 * nw, *bs = bv + nw;
  int32_t *cumv = p.cumv + hb * (p.nqb + 1), *gpos = p.gpos + hb * (int64_t)p.seq;
  int32_t *cumband = p.cumband + hb * p.nqb, *bandlist = p.bandlist + hb * p.nqb;
  const int w_lo = p.forced ? wpb : 0;  // the forced sink block is walked as a block: its keys are not gathered
  int carry = 0;
  for (int w0 = 0; w0 < nw; w0 += 1024) {
    const int wd = w0 + threadIdx.x;
    uint64_t word = (wd < nw && wd >= w_lo) ? bv[wd] : 0ull;
    int total;
    int rank = carry + block_scan_1024(__popcll(word), sh, total);
    if (wd < nw && wd % wpb == 0) cumv[wd / wpb] = rank;
    while (word) {
      const int bit = __ffsll((unsigned long long)word) - 1;
      gpos[rank++] = wd * 64 + bit;
      word &= word - 1;
    }
    carry += total;
  }
  if (threadIdx.x == 0) {
    cumv[p.nqb] = carry;
    if (p.pairs) p.pairs[hb] = 0;
  }
  // band d >= 1 is kept iff an offset in [(d-1)B + 1, (d+1)B - 1] is kept
  carry = 0;
  for (int d0 = 0; d0 < p.nqb; d0 += 1024) {
    const int d = d0 + threadIdx.x;
    int on = 0;
    if (d >= 1 && d < p.nqb) {
      const int lo = (d - 1) * B + 1, hi = min((d + 1) * B - 1, p.seq - 1);
      for (int wd = lo / 64; wd <= hi / 64; ++wd) {
        uint64_t word = bs[wd];
        if (wd == lo / 64) word &= ~0ull << (lo % 64);
        if (wd == hi / 64 && hi % 64 != 63) word &= (2ull << (hi % 64)) - 1;
        on |= word != 0ull;
      }
    }
    int total;
    const int rank = carry + block_scan_1024(on, sh, total);
    if (d < p.nqb) cumband[d] = rank + on;
    if (on) bandlist[rank] = d;
    carry += total;
  }
}

// One workgroup per (gathered 64-key sub-tile, head): K image then V image in the operand order of pack_kv_kernel,
// rows taken at the gathered keys' positions (zero rows beyond the last gathered key).
template <int D>
__global__ __launch_bounds__(256) void vs_gather_kernel(VsTokParams p) {
  constexpr int IMG = KT * D * 2, NCH = IMG / 16, DS = D / 16, VROW = D + 8;
  __shared__ __attribute__((aligned(16))) uint16_t vs[KT * VROW];
  __shared__ int32_t pos[KT];
  const int mt = blockIdx.x, n = blockIdx.y, b = blockIdx.z;
  if (vst_skip(p, b, n)) return;
  const int64_t hb = (int64_t)b * p.n_heads + n;
  const int nv = p.cumv[hb * (p.nqb + 1) + p.nqb];
  if (mt * KT >= nv) return;
  const int tid = threadIdx.x, kvh = p.head_ids[n] / p.group;
  if (tid < KT) pos[tid] = (mt * KT + tid < nv) ? p.gpos[hb * (int64_t)p.seq + mt * KT + tid] : -1;
  __syncthreads();
  const int64_t base = (int64_t)b * p.kv_sb + (int64_t)kvh * p.kv_sh;
  char *out = p.gimg + (hb * (p.seq / KT) + mt) * (int64_t)(2 * IMG);
  const u32x4 zero = {0u, 0u, 0u, 0u};
  for (int c = tid; c < KT * (D / 8); c += 256) {
    const int key = c / (D / 8), part = c % (D / 8);
    const u32x4 val = pos[key] >= 0 ? *reinterpret_cast<const u32x4 *>(p.v + base + (int64_t)pos[key] * p.kv_st + part * 8) : zero;
    *reinterpret_cast<u32x4 *>(&vs[key * VROW + part * 8]) = val;
  }
  for (int c = tid; c < NCH; c += 256) {
    const int f = c >> 6, lane = c & 63;
    const int rb = f / DS, ds = f % DS;
    const int key = 32 * rb + (lane & 31), dpos = 16 * ds + 8 * (lane >> 5);
    const u32x4 val = pos[key] >= 0 ? *reinterpret_cast<const u32x4 *>(p.k + base + (int64_t)pos[key] * p.kv_st + dpos) : zero;
    *reinterpret_cast<u32x4 *>(out + (int64_t)c * 16) = val;
  }
  __syncthreads();
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

// f(integral_constant<int, G>) for G = FROM .. TO-1, expanded at compile time (the steps below index registers
// by G, so they must never be left as a run-time loop)
template <int FROM, int TO, class F>
__device__ __forceinline__ void static_for(F &&f) {
  if constexpr (FROM < TO) {
    f(std::integral_constant<int, FROM>{});
    static_for<FROM + 1, TO>(f);
  }
}

// One item of a row's work list: a packed K image followed by the V image of the same 64 keys.
// kind 0 sink block, 1 gathered keys, 2 band, 3 diagonal; j = key block (kinds 0, 2, 3), sub = 64-key sub-tile
struct VsItem {
  const char *src;
  int kind, j, sub;
};
// Wave-uniform part of an item's mask: three words of the kept-offset bitmap around the window the wavefront's 32
// queries see (word wi0 holds offset position start0 of the first query's window), the kept-key word of the item's
// 64 keys, and the geometry.
struct VsMaskPre {
  uint64_t w0, w1, w2, v;
  int start0, kind, nvalid, top0;
  bool restricted, live;
};

// One workgroup per (query block, listed head): B/32 wavefronts of 32 queries.  The row's work is a list of 64-key
// items, each a packed K/V image pair plus a 64-bit mask per query: the sink block (forced), the gathered kept keys
// below the query block, the kept bands (mask = kept offsets, minus the kept keys already gathered) and the
// diagonal block (causal; without forced blocks also restricted to kept keys / offsets).
// Same software pipeline as attn_kernel: K and V images ride in LDS rings filled two items ahead, one barrier per
// item; while the matrix pipe runs S[t+1] = K[t+1] Q^T and O += V[t]^T P[t]^T the VALU computes P[t], then masks
// S[t+1] and takes its row max (hand-laid groups).  The masks are built one item ahead from wave-uniform words of
// the bitmaps (scalar loads).  In the pipelined steps a wavefront computes every item (an item without an allowed key
// for its 32 queries contributes zeros); the general step of the last items skips such items.  Lazy softmax reference
// and the second normaliser sum as in attn_kernel.
template <int D, int B>
__global__ __launch_bounds__(B * 2, 2) void vs_token_attn_kernel(VsTokParams p) {
  constexpr int NW = B / 32, SPB = B / KT, IMG = KT * D * 2, STAGE = 2 * IMG, DS = D / 16, DB = D / 32;
  constexpr int RK = 2, RV = 3;             // ring slots: K and V are both fetched two items ahead
  constexpr int CH = IMG / 1024 / NW;       // 1 KiB chunks per wavefront per image
  constexpr int VM_KEEP = CH;               // at the top of an item only the V chunks issued last may be in flight
  static_assert(IMG % (1024 * NW) == 0, "image must split evenly over the wavefronts");
  __shared__ __attribute__((aligned(1024))) char smem[(RK + RV) * IMG];
  const uint32_t lds_k = (uint32_t)(size_t)(__attribute__((address_space(3))) char *)smem;
  const uint32_t lds_v = lds_k + RK * IMG;
  // workgroup -> (XCD, head, query block, batch).  Workgroups are dealt round-robin to the 8 XCDs by the hardware.
  // A task is VST_TASK_ROWS consecutive query blocks of one head; task (head a, chunk c) belongs to XCD
  // (a + c) % 8, so every XCD gets an eighth of every head (heads differ widely in how much they keep) and runs
  // its tasks from long rows to short.  The workgroups resident on an XCD at one time are then a few runs of
  // neighbouring rows, which walk nearly the same items at nearly the same time and find each other's images in
  // the XCD's L2.
  const int xcd = blockIdx.x & 7;
  int rest = blockIdx.x >> 3;
  const int per_batch = p.n_heads * p.nch8 * VST_TASK_ROWS;
  const int b = rest / per_batch;
  rest %= per_batch;
  const int n_act = __builtin_amdgcn_readfirstlane(p.act_n[b]);
  if (n_act <= 0 || rest >= n_act * p.nch8 * VST_TASK_ROWS) return;
  const int rr = rest % VST_TASK_ROWS, u = rest / VST_TASK_ROWS;
  const int a = u % n_act, c = 8 * (u / n_act) + ((xcd - a) & 7);
  const int n = __builtin_amdgcn_readfirstlane(p.act_pos[(int64_t)b * p.n_heads + a]);
  const int i = p.nqb - 1 - (c * VST_TASK_ROWS + rr);
  if (i < 0) return;  // the last chunks of a head may be short or empty
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, c32 = lane & 31;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int head = p.head_ids[n], kvh = head / p.group;
  const int64_t hb = (int64_t)b * p.n_heads + n;
  const int nwords = p.seq / 64;
  const uint64_t *__restrict__ bv = p.bits + hb * 2 * nwords, *__restrict__ bs = bv + nwords;
  const int tq = 32 * w + c32;
  bf16x8 qf[DS];
  {
    const uint16_t *qp = p.q + (int64_t)b * p.q_sb + ((int64_t)i * B + tq) * p.q_st + (int64_t)head * p.q_sh + 8 * h;
#pragma unroll
    for (int ds = 0; ds < DS; ++ds) qf[ds] = *reinterpret_cast<const bf16x8 *>(qp + 16 * ds);
  }
  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
  // m = running reference (-inf until a query has seen an allowed key), mref = m or 0 while m is -inf (so that no
  // inf - inf is ever formed), l = sum of weights, lc = sum of (bf16(p) - p) over the tiles that matter
  float m = -INFINITY, mref = 0.f, l = 0.f, lc = 0.f;
  bool care = true;

  // the row's items
  const int jmin = p.forced ? 1 : 0;
  const int n0 = (p.forced && i > 0) ? SPB : 0;
  const int G = p.cumv[hb * (p.nqb + 1) + i];
  // A row whose gathered items and kept bands together outnumber the key blocks below it walks all of those
  // blocks instead, each with the mask kept offsets | kept keys (a head that keeps nearly everything would
  // otherwise visit its kept keys twice: in the gathered images and, masked out, in the bands).
  const int ng_list = (G + KT - 1) / KT;
  const int nb_list = (i - jmin >= 1) ? p.cumband[hb * p.nqb + (i - jmin)] : 0;
  const int nbelow = (i - jmin > 0) ? i - jmin : 0;  // key blocks strictly between the forced sink block and the diagonal
  const bool walk_all = ng_list + nb_list * SPB > nbelow * SPB;
  const int ng = walk_all ? 0 : ng_list;
  const int nb = walk_all ? nbelow : nb_list;
  const int T = n0 + ng + nb * SPB + SPB;
  const char *kvbase = p.kvp + ((int64_t)b * p.n_kv_heads + kvh) * (int64_t)(p.seq / KT) * STAGE;
  const char *gbase = p.gimg + hb * (int64_t)(p.seq / KT) * STAGE;
  const int32_t *__restrict__ bandlist = p.bandlist + hb * p.nqb;
  auto item = [&](int t) -> VsItem {  // t beyond the list: the last item again (loaded, never used)
    t = t < T ? t : T - 1;
    if (t < n0) return VsItem{kvbase + (int64_t)t * STAGE, 0, 0, t};
    t -= n0;
    if (t < ng) return VsItem{gbase + (int64_t)t * STAGE, 1, 0, t};
    t -= ng;
    if (t < nb * SPB) {
      const int j = i - (walk_all ? 1 + t / SPB : bandlist[t / SPB]), sub = t % SPB;
      return VsItem{kvbase + (int64_t)(j * SPB + sub) * STAGE, 2, j, sub};
    }
    t -= nb * SPB;
    return VsItem{kvbase + (int64_t)(i * SPB + t) * STAGE, 3, i, t};
  };
  // word idx of a bitmap, 0 outside it (idx is wave-uniform)
  auto uword = [&](const uint64_t *__restrict__ bits, int idx) -> uint64_t {
    const int ic = idx < 0 ? 0 : (idx >= nwords ? nwords - 1 : idx);
    const uint64_t x = bits[ic];
    return ic == idx ? x : 0ull;
  };
  // The mask of item t for this lane's query: bit kk = key kk of the item is allowed.
  // Offsets of keys kk = 0 .. 63 of a band / diagonal item: o0 - kk with o0 = (i - j) B + tq - 64 sub, so the
  // window W[x] = kept(o0 - 63 + x), reversed, is the mask in key order; the window of the wavefront's first
  // query starts at bit start0, query c32's window c32 bits further.
  auto mask_pre = [&](const VsItem &it, int t) -> VsMaskPre {
    VsMaskPre pre;
    pre.live = t < T;
    pre.kind = it.kind;
    pre.nvalid = G - KT * it.sub;
    pre.restricted = it.kind == 2 || (it.kind == 3 && !p.forced);
    pre.start0 = (i - it.j) * B + 32 * w - KT * it.sub - 63;
    pre.top0 = 32 * w - KT * it.sub;
    const int wi0 = pre.start0 >> 6;  // floor, also for negative positions
    pre.w0 = uword(bs, wi0);
    pre.w1 = uword(bs, wi0 + 1);
    pre.w2 = uword(bs, wi0 + 2);
    pre.v = it.kind == 1 ? 0ull : bv[(it.j * B + KT * it.sub) >> 6];
    return pre;
  };
  auto mask_lane = [&](const VsMaskPre &pre) -> uint64_t {
    const int x = (pre.start0 & 63) + c32, sh = x & 63;
    const bool rel = x >= 64;
    const uint64_t lo = rel ? pre.w1 : pre.w0, hi = rel ? pre.w2 : pre.w1;
    const uint64_t win = (lo >> sh) | ((hi << 1) << (63 - sh));
    const uint64_t R = __builtin_bitreverse64(win);
    uint64_t M = pre.restricted ? ((pre.kind == 2 && !walk_all) ? (R & ~pre.v) : (R | pre.v)) : ~0ull;
    if (pre.kind == 1) M = pre.nvalid >= KT ? ~0ull : (pre.nvalid <= 0 ? 0ull : ((1ull << pre.nvalid) - 1));
    if (pre.kind == 3) {  // causal: key 64 sub + kk <= tq
      const int top = pre.top0 + c32;
      M &= top >= 63 ? ~0ull : (top < 0 ? 0ull : ((2ull << top) - 1));
    }
    return pre.live ? M : 0ull;
  };

  // every wavefront moves CH chunks of an image into a ring slot
  auto issue_chunk = [&](const char *src, uint32_t slot_base, int nchunk) {
    lds_dma16(src + nchunk * 1024, lane * 16, slot_base + (w * CH + nchunk) * 1024);
  };
  auto issue_img = [&](const VsItem &it, bool is_v, uint32_t slot_base) {
    const char *src = it.src + (is_v ? IMG : 0) + (w * CH) * 1024;
#pragma unroll
    for (int nchunk = 0; nchunk < CH; ++nchunk) issue_chunk(src, slot_base, nchunk);
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
  // score (rb, r) of this lane is key 32 rb + 8 (r / 4) + 4 h + r % 4 of the item: mw = the mask's word rb with the
  // 4 h already shifted out.  A score whose bit is clear becomes -inf (two instructions: bit -> 0 / -1, select).
  auto mask_score = [&](float s, uint32_t mw, int r) -> float {
    const int bit = 8 * (r >> 2) + (r & 3);
    const uint32_t keep = (uint32_t)((int32_t)(mw << (31 - bit)) >> 31);
    return __builtin_bit_cast(float, (__builtin_bit_cast(uint32_t, s) & keep) | (~keep & 0xff800000u));
  };
  auto apply_mask = [&](f32x16(&s)[2], uint64_t M) {
    const uint32_t mw0 = (uint32_t)M >> (4 * h), mw1 = (uint32_t)(M >> 32) >> (4 * h);
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[rb][r] = mask_score(s[rb][r], rb ? mw1 : mw0, r);
  };
  // mx = raw row max of a fresh (masked) tile, -inf if the query has no allowed key in it.  Moves the reference if
  // the max outgrew the slack, rescales the running sums, notes whether the tile's largest weight matters to the
  // row (care), returns alpha = 2^(m_old - m_new) for the O accumulators (1 while nothing has been accumulated).
  auto move_reference = [&](float mx) -> float {
    const float m_new = lazy_max(m, mx * p.c);
    const float mref_new = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = (m == -INFINITY) ? 1.f : fast_exp2(m - mref_new);
    m = m_new;
    mref = mref_new;
    l *= alpha;
    lc *= alpha;
    care = fast_exp2(__builtin_fmaf(mx, p.c, -mref_new)) * SP_CARE > l;
    return alpha;
  };
  auto tile_max = [&](f32x16(&s)[2]) -> float {
    float mx = fmaxf(s[0][0], s[0][1]);
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int r = (rb == 0 ? 2 : 0); r < 16; r += 2) mx = max3f(mx, s[rb][r], s[rb][r + 1]);
    return move_reference(max_xor32(mx));
  };
  auto tile_exp = [&](f32x16(&s)[2], bf16x8(&pb)[4]) {
    float rs0 = 0.f, rs1 = 0.f;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      u32x4 tt;
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        const int r = 8 * (ks & 1) + 2 * e2;
        const float p0 = fast_exp2(__builtin_fmaf(s[ks >> 1][r], p.c, -mref));
        const float p1 = fast_exp2(__builtin_fmaf(s[ks >> 1][r + 1], p.c, -mref));
        rs0 += p0;
        rs1 += p1;
        tt[e2] = pack_bf16(p0, p1);
      }
      pb[ks] = __builtin_bit_cast(bf16x8, tt);
    }
    const float rs = sum_xor32(rs0 + rs1);
    l += rs;
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

  // On entry to step t: s_cur = masked raw S[t] with its max folded into m / l / O (if this wavefront has anything
  // in item t), Mn = the mask of item t+1, it2 / pre2 = item t+2 and the uniform part of its mask.  Every step
  // returns the mask of item t+2.
  // fast step: this wavefront has work in items t and t+1.  One basic block up to the rescale test.
  auto fast_step = [&](int t, const VsItem &it2, const VsMaskPre &pre2, f32x16(&s_cur)[2], f32x16(&s_next)[2],
                       uint64_t Mn, auto masked_tag) __attribute__((always_inline)) -> uint64_t {
    constexpr bool MASKED = decltype(masked_tag)::value;
    wait_vm<VM_KEEP>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    const char *ksrc = it2.src + (w * CH) * 1024, *vsrc = ksrc + IMG;
    const uint32_t kslot = lds_k + ((t + 2) % RK) * IMG, vslot = lds_v + ((t + 2) % RV) * IMG;
    const char *kb = smem + ((t + 1) % RK) * IMG + lane * 16;
    const char *vb = smem + (RK + t % RV) * IMG + lane * 16;
    const uint32_t mw0 = (uint32_t)Mn >> (4 * h), mw1 = (uint32_t)(Mn >> 32) >> (4 * h);
    // NM groups, each = one MFMA + one LDS read (PF fragments ahead) + a slice of the VALU work:
    //   groups 0 .. NQ-1   : S[t+1] += K frag * Q frag ; exp / row-sum / bf16 pack of S[t]
    //   groups NQ .. NM-1  : O += V frag * P frag       ; mask and row max of S[t+1], reference update,
    //                                                     the mask of item t+2
    constexpr int NQ = 2 * DS, NP = 4 * DB, NM = NQ + NP;
    constexpr int PF = 3, MAXTAIL = 4;
    auto frag = [&](int g) -> bf16x8 {
      if (g < NQ) return *reinterpret_cast<const bf16x8 *>(kb + ((g % 2) * DS + g / 2) * 1024);
      const int np = g - NQ;
      return *reinterpret_cast<const bf16x8 *>(vb + ((np % DB) * 4 + np / DB) * 1024);
    };
    bf16x8 fr[PF + 1];
    bf16x8 pb[4];
    u32x4 pt;
    float rs0 = 0.f, rs1 = 0.f, mx = 0.f, alpha = 1.f, rs_tile = 0.f;
    const bool care_t = care;  // set when this tile's max was taken
    float xa[16], xb[16];
    uint64_t Mnn = 0ull;
#pragma unroll
    for (int g = 0; g < PF; ++g) fr[g] = frag(g);
    static_for<0, NM>([&](auto gc) __attribute__((always_inline)) {
      constexpr int g = decltype(gc)::value;
      if (g + PF < NM) fr[(g + PF) % (PF + 1)] = frag(g + PF);
      if (g < NQ) {
        if (g < 2) {
          f32x16 z;
#pragma unroll
          for (int r = 0; r < 16; ++r) z[r] = 0.f;
          s_next[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[g % (PF + 1)], qf[0], z, 0, 0, 0);
        } else {
          s_next[g % 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[g % (PF + 1)], qf[g / 2], s_next[g % 2], 0, 0, 0);
        }
      }
      // exp units u (2 scores each), three stages in consecutive groups
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int gu = u * NQ / 16;
        const int ks = u / 4, e2 = u % 4, r = 8 * (ks & 1) + 2 * e2;
        if (gu == g) {
          xa[u] = __builtin_fmaf(s_cur[ks >> 1][r], p.c, -mref);
          xb[u] = __builtin_fmaf(s_cur[ks >> 1][r + 1], p.c, -mref);
        }
        if (gu + 1 == g) {
          xa[u] = fast_exp2(xa[u]);
          xb[u] = fast_exp2(xb[u]);
        }
        if (gu + 2 == g) {
          rs0 += xa[u];
          rs1 += xb[u];
          pt[e2] = pack_bf16(xa[u], xb[u]);
          if (e2 == 3) pb[ks] = __builtin_bit_cast(bf16x8, pt);
        }
      }
      if (g == NQ + 2) {
        rs_tile = sum_xor32(rs0 + rs1);
        l += rs_tile;
      }
      {
        constexpr int GAP = NM / (2 * CH);  // groups between two chunk loads
        if (g % GAP == 1 && g / GAP < CH) issue_chunk(ksrc, kslot, g / GAP);
        if (g % GAP == 1 && g / GAP >= CH && g / GAP < 2 * CH) issue_chunk(vsrc, vslot, g / GAP - CH);
      }
      if (g >= NQ) {
        const int np = g - NQ;
        oacc[np % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[g % (PF + 1)], pb[np / DB], oacc[np % DB], 0, 0, 0);
        // S[t+1]: 16 units of two scores, masked one group before they enter the row max; the reference update
        // MAXTAIL groups before the end
#pragma unroll
        for (int u = 0; u < 16; ++u) {
          const int gm = 2 + u * (NP - 2 - MAXTAIL) / 16;
          const int rb = u / 8, r = 2 * (u % 8);
          if (MASKED && gm - 1 == np) {
            s_next[rb][r] = mask_score(s_next[rb][r], rb ? mw1 : mw0, r);
            s_next[rb][r + 1] = mask_score(s_next[rb][r + 1], rb ? mw1 : mw0, r + 1);
          }
          if (gm == np) {
            const float a0 = s_next[rb][r], a1 = s_next[rb][r + 1];
            mx = (u == 0) ? fmaxf(a0, a1) : max3f(mx, a0, a1);
          }
        }
        if (np == NP - MAXTAIL) alpha = move_reference(max_xor32(mx));
        if (MASKED && np == NP - 2) Mnn = mask_lane(pre2);
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    if (__any(care_t)) {  // rare: the tile summed again as PV saw it (alpha already holds the move after this tile)
      asm volatile("" ::: "memory");  // a real branch: not to be evaluated on every step
      lc += (sum_xor32(sum_bf16x8(pb[0]) + sum_bf16x8(pb[1]) + sum_bf16x8(pb[2]) + sum_bf16x8(pb[3])) - rs_tile) * alpha;
    }
    rescale(alpha);
    return Mnn;
  };
  // general step (the last items of a row): a wavefront whose 32 queries have no allowed key in an item skips its
  // matrix work; optional next item.  Returns whether s_next holds a tile.
  auto slow_step = [&](int t, const VsItem &it2, f32x16(&s_cur)[2], f32x16(&s_next)[2], uint64_t Mn,
                       bool act_cur) __attribute__((always_inline)) -> bool {
    wait_vm<VM_KEEP>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    issue_img(it2, false, lds_k + ((t + 2) % RK) * IMG);
    issue_img(it2, true, lds_v + ((t + 2) % RV) * IMG);
    const bool act_next = __any(Mn != 0ull);
    if (act_next) qk(smem + ((t + 1) % RK) * IMG, s_next);
    if (act_cur) {
      bf16x8 pb[4];
      tile_exp(s_cur, pb);
      pv(smem + (RK + t % RV) * IMG, pb);
    }
    if (act_next) {
      if (!__all(Mn == ~0ull)) apply_mask(s_next, Mn);
      rescale(tile_max(s_next));
    }
    return act_next;
  };

  // The leading items whose masks are all ones (the sink block, the full gathered items) go through the step
  // without the mask, the others through the step with it, both in pairs (the S tiles swap roles); the last one
  // or two items take the general step.  npairs counts the allowed (query, key) pairs of this lane's query.
  int npairs = 0;  // at most 64 per item
  {
    f32x16 s_a[2], s_b[2];
    const int U = n0 + (walk_all ? 0 : G / KT);     // items 0 .. U-1 have all-ones masks
    const int nfu = (U > 1) ? ((U - 1) & ~1) : 0;   // steps t < nfu: item t+1 is unmasked
    const int nfm = (T - 1 - nfu) & ~1;             // steps nfu <= t < nfu + nfm: the masked step (item t+1 exists)
    const VsItem it0 = item(0), it1 = item(1);
    const uint64_t M0 = mask_lane(mask_pre(it0, 0));
    npairs += __popcll(M0) + KT * nfu;  // items 1 .. nfu are full; the later ones are counted as their masks are built
    // prologue: K and V images of items 0 and 1
    issue_img(it0, true, lds_v);
    issue_img(it0, false, lds_k);
    issue_img(it1, true, lds_v + IMG);
    issue_img(it1, false, lds_k + IMG);
    wait_vm<0>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    qk(smem, s_a);
    if (!__all(M0 == ~0ull)) apply_mask(s_a, M0);
    tile_max(s_a);  // O is still zero: nothing to rescale
    int t = 0;
    {
      VsItem it2 = item(2), it3 = item(3);
      const VsMaskPre nopre{};
      for (; t < nfu; t += 2) {
        const VsItem it4 = item(t + 4), it5 = item(t + 5);
        fast_step(t, it2, nopre, s_a, s_b, 0ull, std::false_type{});
        fast_step(t + 1, it3, nopre, s_b, s_a, 0ull, std::false_type{});
        it2 = it4;
        it3 = it5;
      }
    }
    VsItem it2 = item(t + 2);
    uint64_t Mn = mask_lane(mask_pre(item(t + 1), t + 1));
    npairs += __popcll(Mn);
    {
      VsMaskPre pre2 = mask_pre(it2, t + 2);
      VsItem it3 = item(t + 3);
      for (const int tend = t + nfm; t < tend; t += 2) {
        const VsMaskPre pre3 = mask_pre(it3, t + 3);
        const VsItem it4 = item(t + 4);
        const uint64_t Mb = fast_step(t, it2, pre2, s_a, s_b, Mn, std::true_type{});
        const VsMaskPre pre4 = mask_pre(it4, t + 4);
        const VsItem it5 = item(t + 5);
        Mn = fast_step(t + 1, it3, pre3, s_b, s_a, Mb, std::true_type{});
        npairs += __popcll(Mb) + __popcll(Mn);
        it2 = it4;
        pre2 = pre4;
        it3 = it5;
      }
    }
    // one or two items are left (t + 2 >= T: no item t+2, its mask is empty)
    const bool act = slow_step(t, it2, s_a, s_b, Mn, true);
    if (t + 1 < T) slow_step(t + 1, it2, s_b, s_a, 0ull, act);
    wait_vm<0>();  // drain the rings' look-ahead loads before the LDS is released
  }
  {
    const float inv = (l > 0.f) ? 1.f / (l + lc) : 0.f;
    uint16_t *op = p.o + (int64_t)b * p.o_sb + ((int64_t)i * B + tq) * p.o_st + (int64_t)head * p.o_sh;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        u32x2 tt;
        tt[0] = pack_bf16(oacc[db][4 * gq] * inv, oacc[db][4 * gq + 1] * inv);
        tt[1] = pack_bf16(oacc[db][4 * gq + 2] * inv, oacc[db][4 * gq + 3] * inv);
        *reinterpret_cast<u32x2 *>(op + 32 * db + 8 * gq + 4 * h) = tt;
      }
  }
  if (p.pairs) {  // pairs of the pattern in this row: every query counted once (its two half-lanes hold the same mask)
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1) npairs += __shfl_xor(npairs, off, 64);
    if (lane == 0) atomicAdd(reinterpret_cast<unsigned long long *>(p.pairs + hb), (unsigned long long)(unsigned)npairs);
  }
}

}  // namespace

#endif
