// Vector types, tile constants, error text and the optional per-kernel timing shared by every kernel file.
#ifndef SP_COMMON_H
#define SP_COMMON_H
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
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

}  // namespace

#endif
