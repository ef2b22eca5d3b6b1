#include "prof.h"

#include <vector>

namespace ssdt {
namespace prof {

bool g_on = false;
namespace {
struct Entry { int cat; hipEvent_t a, b; double flops, bytes; };
std::vector<Entry> pending;
std::vector<hipEvent_t> pool;
Entry cur{};
unsigned long long n_[NCAT];
double ms_[NCAT], fl_[NCAT], by_[NCAT];
hipEvent_t get() {
  if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
  hipEvent_t e;
  (void)hipEventCreate(&e);
  return e;
}
}  // namespace

const char *name(int cat) {
  static const char *n[NCAT] = {"gemm_nt256_k", "gemm_nt128_k", "gemm_generic_k", "transpose_k", "fa_fwd_k|attn_fwd_generic_k",
                                "fa_bwd_*|attn_bwd_*", "norm_fwd_k", "norm_bwd_dx_k", "colreduce*_k", "add_inplace_k", "gemm_km256_k"};
  return (cat >= 0 && cat < NCAT) ? n[cat] : "?";
}
void set(bool on) { g_on = on; }
void begin(int cat, double flops, double bytes, hipStream_t s) {
  cur = Entry{cat, get(), get(), flops, bytes};
  (void)hipEventRecord(cur.a, s);
}
void end(hipStream_t s) {
  (void)hipEventRecord(cur.b, s);
  pending.push_back(cur);
}
bool collect() {
  bool all = true;
  for (size_t i = 0; i < pending.size();) {
    Entry &e = pending[i];
    if (hipEventQuery(e.b) == hipSuccess) {
      float ms = 0;
      (void)hipEventElapsedTime(&ms, e.a, e.b);
      ++n_[e.cat]; ms_[e.cat] += ms; fl_[e.cat] += e.flops; by_[e.cat] += e.bytes;
      pool.push_back(e.a); pool.push_back(e.b);
      pending[i] = pending.back();
      pending.pop_back();
    } else {
      all = false;
      ++i;
    }
  }
  return all;
}
void totals(int cat, unsigned long long *launches, double *ms, double *flops, double *bytes) {
  *launches = n_[cat]; *ms = ms_[cat]; *flops = fl_[cat]; *bytes = by_[cat];
}
void reset() {
  collect();
  for (int c = 0; c < NCAT; ++c) { n_[c] = 0; ms_[c] = fl_[c] = by_[c] = 0; }
}

}  // namespace prof
}  // namespace ssdt
