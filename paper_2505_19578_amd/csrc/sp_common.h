// Vector types, tile constants, error text and the optional per-kernel timing shared by every kernel file.
#ifndef SP_COMMON_H
#define SP_COMMON_H
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <mutex>

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

// Optional per-kernel timing for benchmarks (sp_profile_enable / sp_profile_read): while enabled, every
// launch is bracketed by two HIP events on the caller's stream, taken from a fixed pool that
// sp_profile_enable created beforehand (nothing is created or freed while work is being enqueued; launches
// beyond the pool are counted as dropped and reported by the next read).  Process-wide.
enum KernelKind { KK_PACK = 0, KK_DENSE = 1, KK_MASK = 2, KK_SPARSE = 3, KK_SCORE = 4, KK_VS = 5, KK_COUNT = 6 };
constexpr int SP_PROF_CAPACITY = 4096;
bool g_prof_on = false;
hipEvent_t *g_prof_events = nullptr;  // 2 * SP_PROF_CAPACITY, pairs (begin, end)
int g_prof_kind[SP_PROF_CAPACITY];
int g_prof_count = 0, g_prof_dropped = 0;
std::mutex g_prof_mutex;

struct ProfScope {
  hipStream_t st;
  int slot = -1;
  ProfScope(int kind, hipStream_t s) : st(s) {
    if (!g_prof_on) return;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (!g_prof_on || !g_prof_events) return;
    if (g_prof_count >= SP_PROF_CAPACITY) {
      ++g_prof_dropped;
      return;
    }
    slot = g_prof_count++;
    g_prof_kind[slot] = kind;
    (void)hipEventRecord(g_prof_events[2 * slot], st);
  }
  ~ProfScope() {
    if (slot >= 0) (void)hipEventRecord(g_prof_events[2 * slot + 1], st);
  }
};

void set_err(const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

}  // namespace

#endif
