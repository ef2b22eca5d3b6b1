// Internal: optional per-kernel-class timing with HIP events recorded on the launch stream,
// so that a benchmark can report a kernel's average duration over the very region it times.
#pragma once
#include <hip/hip_runtime.h>

namespace ssdt {
namespace prof {

enum Cat { GEMM_MFMA_256 = 0, GEMM_MFMA_128, GEMM_GENERIC, TRANSPOSE, ATTN_FWD, ATTN_BWD, NORM_FWD, NORM_BWD, COLREDUCE, ADD, GEMM_MFMA_KM, NCAT };
extern bool g_on;
const char *name(int cat);
void begin(int cat, double flops, double bytes, hipStream_t s);
void end(hipStream_t s);
void set(bool on);
// folds finished measurements into the totals; returns false if some are still running
bool collect();
void totals(int cat, unsigned long long *launches, double *ms, double *flops, double *bytes);
void reset();

struct Scope {
  hipStream_t s;
  bool live;
  Scope(int cat, double flops, double bytes, hipStream_t st) : s(st), live(g_on) { if (live) begin(cat, flops, bytes, st); }
  ~Scope() { if (live) end(s); }
};

}  // namespace prof
}  // namespace ssdt
