// Step-mix probe (measurement aid): the instruction mix of one attention step, nothing around it.
#ifndef SP_PROBE_KERNEL_H
#define SP_PROBE_KERNEL_H
#include "sp_common.h"
#include "attn_kernel.h"

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
  constexpr int LPD = LP > 0 ? LP : 1;  // read period (unused when LP == 0)
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
      if (LP > 0 && n % LPD == 0)
        fr[(n + PF) % (PF + 1)] = *reinterpret_cast<const bf16x8 *>(rd + (n % 32) * 1024);
      acc[n % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[LP > 0 ? ((n / LPD) * LPD) % (PF + 1) : 0], b, acc[n % 4],
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

}  // namespace

#endif
