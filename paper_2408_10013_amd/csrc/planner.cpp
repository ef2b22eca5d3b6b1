// Choice of the per-step offload amount from the model's per-layer activation sizes and times and the
// measured transfer rates (Sec. 3.1: the amount is set from the amount of computation, the activation
// size, the GPU throughput and the I/O bandwidth; Sec. 3.2: tensors are offloaded in forward order until
// that amount is reached).  Host arithmetic only.
#include <cmath>
#include <cstdint>
#include <vector>

#include "ssdt.h"

namespace {

struct Times {
  std::vector<double> fwd_end, bwd_start;  // per layer; backward runs the last layer first
  double t_fwd = 0;
};

Times timeline(const ssdt_plan_in &in) {
  Times t;
  const int n = in.num_layers;
  t.fwd_end.resize(n);
  t.bwd_start.resize(n);
  double run = 0;  // times accumulate left to right in double precision
  for (int l = 0; l < n; ++l) {
    run += in.fwd_s[l];
    t.fwd_end[l] = run;
  }
  t.t_fwd = run;
  double at = t.t_fwd;
  for (int l = n - 1; l >= 0; --l) {
    t.bwd_start[l] = at;
    at += in.bwd_s[l];
  }
  return t;
}

// Loads of the offloaded layers, topmost first, one queue; layer l's load is issued when the backward of
// layer l+d starts (end of forward if there is none) and has to be complete when layer l's backward starts.
bool loads_hidden(const std::vector<uint64_t> &amount, const Times &t, int n, double rate, int d) {
  double queue_free = 0;
  for (int l = (int)amount.size() - 1; l >= 0; --l) {
    const double issue = l + d < n ? t.bwd_start[l + d] : t.t_fwd;
    const double finish = std::fmax(queue_free, issue) + (double)amount[l] / rate;
    if (finish > t.bwd_start[l]) return false;
    queue_free = finish;
  }
  return true;
}

}  // namespace

extern "C" ssdt_status ssdt_plan(const ssdt_plan_in *in, ssdt_plan_out *out) {
  if (!in || !out || in->num_layers <= 0 || in->keep_last < 0 || !in->layer_bytes || !in->fwd_s || !in->bwd_s) return SSDT_E_INVAL;
  if (!(in->store_Bps > 0) || !(in->load_Bps > 0) || !(in->safety > 0) || !(in->safety <= 1)) return SSDT_E_INVAL;
  const int n = in->num_layers;
  for (int l = 0; l < n; ++l)
    if (!(in->fwd_s[l] >= 0) || !(in->bwd_s[l] >= 0)) return SSDT_E_INVAL;
  const Times t = timeline(*in);
  const double w = in->safety * in->store_Bps, r = in->safety * in->load_Bps;
  const int eligible = n - in->keep_last > 0 ? n - in->keep_last : 0;

  // stores: what has left the device when the forward pass ends
  std::vector<uint64_t> amount;
  double queue_free = 0;
  for (int l = 0; l < eligible; ++l) {
    const double start = std::fmax(queue_free, t.fwd_end[l]);
    const double finish = start + (double)in->layer_bytes[l] / w;
    if (finish <= t.t_fwd) {
      amount.push_back(in->layer_bytes[l]);
      queue_free = finish;
      continue;
    }
    if (t.t_fwd > start) {
      double part = std::floor((t.t_fwd - start) * w);
      if (part > (double)in->layer_bytes[l]) part = (double)in->layer_bytes[l];
      if (part >= 1) amount.push_back((uint64_t)part);
    }
    break;
  }

  ssdt_plan_out o{};
  while (!amount.empty()) {
    int dist = 0;
    for (int d = 1; d <= n && !dist; ++d)
      if (loads_hidden(amount, t, n, r, d)) dist = d;
    if (dist) {
      o.prefetch_distance = dist;
      double qf = 0;
      for (size_t l = 0; l < amount.size(); ++l) {
        o.budget_bytes += (int64_t)amount[l];
        if (amount[l] == in->layer_bytes[l]) ++o.layers;
        else o.partial_bytes = amount[l];
        qf = std::fmax(qf, t.fwd_end[l]) + (double)amount[l] / w;
      }
      o.store_done_s = qf;
      break;
    }
    amount.pop_back();  // no distance hides the loads: give up the partial layer, then the topmost layer
  }
  o.fwd_total_s = t.t_fwd;
  *out = o;
  return SSDT_OK;
}
