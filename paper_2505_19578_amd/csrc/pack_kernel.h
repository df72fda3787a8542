// K/V packing into MFMA-operand-ordered images (see the operand mapping in shareprefill.hip).
#ifndef SP_PACK_KERNEL_H
#define SP_PACK_KERNEL_H
#include "sp_common.h"

namespace {

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

}  // namespace

#endif
