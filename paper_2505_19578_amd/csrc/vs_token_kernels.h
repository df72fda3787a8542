// Attention over the vertical-slash pattern of Alg. 5 at token granularity (Sec. 5.1 A(Q,K,V,M) with the mask M
// built from S = S_v U S_s): the kept keys of a head are gathered into packed images of their own, the kept
// offsets are walked as bands of key blocks with a bit mask inside every tile.
#ifndef SP_VS_TOKEN_KERNELS_H
#define SP_VS_TOKEN_KERNELS_H
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
struct VsTokParams {
  const uint16_t *q, *k, *v;
  const char *kvp;   // packed K/V images of the whole sequence (pack_kv_kernel)
  uint16_t *o;
  int64_t q_sb, q_st, q_sh, kv_sb, kv_st, kv_sh, o_sb, o_st, o_sh;
  int seq, nqb, block, n_kv_heads, group, n_heads, n_q_heads, forced;
  float c;  // softmax scale * log2(e)
  uint64_t *bits;
  int32_t *cumv, *gpos, *cumband, *bandlist;
  char *gimg;
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

// One workgroup of 1024 threads per listed head: ranks of the kept keys, kept bands.
__global__ __launch_bounds__(1024) void vs_token_prep_kernel(VsTokParams p) {
  __shared__ int sh[16];
  const int n = blockIdx.x, b = blockIdx.y;
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

// 64 bits of a bit vector of nw words starting at bit position `start` (bits outside the vector read 0)
__device__ __forceinline__ uint64_t bit_window(const uint64_t *bits, int nw, int64_t start) {
  const int64_t wi = start >> 6;  // floor, also for negative positions
  const int sh = (int)(start & 63);
  const uint64_t a = (wi >= 0 && wi < nw) ? bits[wi] : 0ull;
  const uint64_t b2 = (wi + 1 >= 0 && wi + 1 < nw) ? bits[wi + 1] : 0ull;
  return sh ? ((a >> sh) | (b2 << (64 - sh))) : a;
}

// One workgroup per (query block, listed head): B/32 wavefronts of 32 queries.  The row's work is a list of 64-key
// items, each a packed K/V image pair plus a 64-bit mask per query: the sink block (forced), the gathered kept keys
// below the query block, the kept bands (mask = kept offsets, minus the kept keys already gathered) and the
// diagonal block (causal; without forced blocks also restricted to kept keys / offsets).  Items are double
// buffered in LDS (LDS-direct loads, one barrier per item); a wavefront whose 32 queries have no allowed key in an
// item skips its matrix work.  Lazy softmax reference as in attn_kernel; the row sum adds the bf16-rounded weights
// PV sees, every tile.
template <int D, int B>
__global__ __launch_bounds__(B * 2, 2) void vs_token_attn_kernel(VsTokParams p) {
  constexpr int NW = B / 32, SPB = B / KT, IMG = KT * D * 2, STAGE = 2 * IMG, DS = D / 16, DB = D / 32;
  constexpr int CH = STAGE / 1024 / NW;  // 1 KiB chunks per wavefront per item
  __shared__ __attribute__((aligned(1024))) char smem[2 * STAGE];
  const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) char *)smem;
  const int i = p.nqb - 1 - (int)blockIdx.x, n = blockIdx.y, b = blockIdx.z;
  if (vst_skip(p, b, n)) return;
  const int tid = threadIdx.x, lane = tid & 63, h = lane >> 5, c32 = lane & 31;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int head = p.head_ids[n], kvh = head / p.group;
  const int64_t hb = (int64_t)b * p.n_heads + n;
  const int nwords = p.seq / 64;
  const uint64_t *bv = p.bits + hb * 2 * nwords, *bs = bv + nwords;
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
  float m = -INFINITY, l = 0.f;

  // the row's items
  const int jmin = p.forced ? 1 : 0;
  const int n0 = (p.forced && i > 0) ? SPB : 0;
  const int G = p.cumv[hb * (p.nqb + 1) + i];
  const int ng = (G + KT - 1) / KT;
  const int nb = (i - jmin >= 1) ? p.cumband[hb * p.nqb + (i - jmin)] : 0;
  const int T = n0 + ng + nb * SPB + SPB;
  const char *kvbase = p.kvp + ((int64_t)b * p.n_kv_heads + kvh) * (int64_t)(p.seq / KT) * STAGE;
  const char *gbase = p.gimg + hb * (int64_t)(p.seq / KT) * STAGE;
  const int32_t *bandlist = p.bandlist + hb * p.nqb;
  // kind 0 sink block, 1 gathered keys, 2 band, 3 diagonal; j = key block (kinds 0, 2, 3), sub = 64-key half
  auto item = [&](int t, int &kind, int &j, int &sub) -> const char * {
    if (t < n0) {
      kind = 0, j = 0, sub = t;
      return kvbase + (int64_t)t * STAGE;
    }
    t -= n0;
    if (t < ng) {
      kind = 1, j = 0, sub = t;
      return gbase + (int64_t)t * STAGE;
    }
    t -= ng;
    if (t < nb * SPB) {
      kind = 2, j = i - bandlist[t / SPB], sub = t % SPB;
      return kvbase + (int64_t)(j * SPB + sub) * STAGE;
    }
    t -= nb * SPB;
    kind = 3, j = i, sub = t;
    return kvbase + (int64_t)(i * SPB + t) * STAGE;
  };
  auto issue = [&](int t) {
    int kind, j, sub;
    const char *src = item(t, kind, j, sub) + (w * CH) * 1024;
    const uint32_t dst = lds0 + (t & 1) * STAGE + (w * CH) * 1024;
#pragma unroll
    for (int c = 0; c < CH; ++c) lds_dma16(src + c * 1024, lane * 16, dst + c * 1024);
  };

  int64_t npairs = 0;
  issue(0);
  for (int t = 0; t < T; ++t) {
    wait_vm<0>();                    // this wavefront's share of item t has landed
    __builtin_amdgcn_s_barrier();    // ... everybody's has, and everybody is done with item t-1
    asm volatile("" ::: "memory");
    if (t + 1 < T) issue(t + 1);     // into the stage item t-1 occupied
    int kind, j, sub;
    item(t, kind, j, sub);
    // per-query mask over the item's 64 keys (bit kk = key kk of the item is allowed for this lane's query)
    uint64_t M = ~0ull;
    if (kind == 1) {
      const int nvalid = G - KT * sub;
      if (nvalid < KT) M = (1ull << nvalid) - 1;
    } else if (kind >= 2) {
      const bool restricted = kind == 2 || !p.forced;
      if (restricted) {
        // offsets of keys kk = 0 .. 63: o0 - kk with o0 = (i - j) B + tq - 64 sub; W[x] = kept(o0 - 63 + x)
        const int64_t o0 = (int64_t)(i - j) * B + tq - KT * sub;
        const uint64_t R = __builtin_bitreverse64(bit_window(bs, nwords, o0 - 63));
        const uint64_t V = bv[(j * B + KT * sub) / 64];
        M = kind == 2 ? (R & ~V) : (R | V);
      }
      if (kind == 3) {  // causal: key 64 sub + kk <= tq
        const int top = tq - KT * sub;
        M &= top >= 63 ? ~0ull : (top < 0 ? 0ull : ((2ull << top) - 1));
      }
    }
    npairs += __popcll(M);
    if (__all(M == 0ull)) continue;  // nothing for this wavefront (uniform per wavefront: no barrier inside)
    const char *kb = smem + (t & 1) * STAGE + lane * 16, *vb = kb + IMG;
    f32x16 s[2];
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
    if (!__all(M == ~0ull)) {
      const uint32_t m0 = (uint32_t)M >> (4 * h), m1 = (uint32_t)(M >> 32) >> (4 * h);
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int bit = 8 * (r >> 2) + (r & 3);  // key 32 rb + 8 (r/4) + 4 h + r%4, the 4 h already shifted out
          if (!(((rb ? m1 : m0) >> bit) & 1u)) s[rb][r] = -INFINITY;
        }
    }
    float mx = fmaxf(s[0][0], s[0][1]);
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int r = (rb == 0 ? 2 : 0); r < 16; r += 2) mx = max3f(mx, s[rb][r], s[rb][r + 1]);
    mx = max_xor32(mx);
    const float m_new = lazy_max(m, mx * p.c);  // the reference lags the max by at most SP_MAX_SLACK (see attn_kernel.h)
    const float mref = (m_new == -INFINITY) ? 0.f : m_new;  // no allowed key yet: every weight below is 0
    const float alpha = (m == -INFINITY) ? 0.f : fast_exp2(m - mref);
    m = m_new;
    if (__any(alpha != 1.f)) {
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
    }
    bf16x8 pb[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      u32x4 tt;
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        const int r = 8 * (ks & 1) + 2 * e2;
        tt[e2] = pack_bf16(fast_exp2(__builtin_fmaf(s[ks >> 1][r], p.c, -mref)),
                           fast_exp2(__builtin_fmaf(s[ks >> 1][r + 1], p.c, -mref)));
      }
      pb[ks] = __builtin_bit_cast(bf16x8, tt);
    }
    l = l * alpha + sum_xor32(sum_bf16x8(pb[0]) + sum_bf16x8(pb[1]) + sum_bf16x8(pb[2]) + sum_bf16x8(pb[3]));
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(vb + (db * 4 + ks) * 1024);
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[ks], oacc[db], 0, 0, 0);
      }
  }
  {
    const float inv = (l > 0.f) ? 1.f / l : 0.f;
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
    if (lane == 0) atomicAdd(reinterpret_cast<unsigned long long *>(p.pairs + hb), (unsigned long long)npairs);
  }
}

}  // namespace

#endif
