// Copy backend on the HIP runtime: one stream per direction (the paper's store and load
// pools, Sec. 3.3.2, both first-in-first-out), hipMemcpyAsync between device memory and a
// pinned host pool allocated once, and events for every ordering between streams.
#include <hip/hip_runtime.h>

#include "ctx.h"

namespace ssdt {
namespace {

class HipBackend : public Backend {
 public:
  hipStream_t q_[2] = {nullptr, nullptr};
  hipStream_t aux_ = nullptr;  // side stream for bandwidth-bound kernels that overlap the caller's GEMMs (default priority)
  void *pool_ = nullptr;
  std::vector<Ev *> free_[2];  // [timing]
  std::vector<Ev *> all_;

  bool check(hipError_t e, const char *what) {
    if (e == hipSuccess) return true;
    err = std::string(what) + ": " + hipGetErrorString(e);
    return false;
  }
  int dev_ = 0;
  void thread_init() override { (void)hipSetDevice(dev_); }
  bool init(size_t pool_bytes) {
    int n = 0;
    if (!check(hipGetDeviceCount(&n), "hipGetDeviceCount")) return false;
    if (n <= 0) {
      err = "no HIP device";
      return false;
    }
    if (!check(hipGetDevice(&dev_), "hipGetDevice")) return false;
    for (int d = 0; d < 2; ++d)
      if (!check(hipStreamCreateWithFlags(&q_[d], hipStreamNonBlocking), "hipStreamCreateWithFlags")) return false;
    if (!check(hipStreamCreateWithFlags(&aux_, hipStreamNonBlocking), "hipStreamCreateWithFlags")) return false;
    if (pool_bytes && !check(hipHostMalloc(&pool_, pool_bytes, hipHostMallocDefault), "hipHostMalloc(pool)")) return false;
    // a stock of events, so that the layer entry points create none in the steady state
    std::vector<Ev *> stock;
    for (int i = 0; i < 64; ++i) stock.push_back(get_ev(false));
    for (Ev *e : stock) recycle(e);
    return err.empty();
  }
  ~HipBackend() override {
    for (Ev *e : all_) {
      if (e->h) (void)hipEventDestroy((hipEvent_t)e->h);
      delete e;
    }
    for (int d = 0; d < 2; ++d)
      if (q_[d]) (void)hipStreamDestroy(q_[d]);
    if (aux_) (void)hipStreamDestroy(aux_);
    if (pool_) (void)hipHostFree(pool_);
  }
  bool is_sim() const override { return false; }
  uint64_t seq_ = 0;
  Ev *get_ev(bool timing) {
    auto &fl = free_[timing ? 1 : 0];
    if (!fl.empty()) {
      Ev *e = fl.back();
      fl.pop_back();
      e->refs = 0;
      e->seq = ++seq_;
      return e;
    }
    Ev *e = new Ev();
    e->timing = timing;
    hipEvent_t h;
    check(hipEventCreateWithFlags(&h, timing ? hipEventDefault : hipEventDisableTiming), "hipEventCreate");
    e->h = h;
    e->seq = ++seq_;
    all_.push_back(e);
    return e;
  }
  Ev *record(ssdt_stream s, bool timing) override {
    Ev *e = get_ev(timing);
    check(hipEventRecord((hipEvent_t)e->h, (hipStream_t)s), "hipEventRecord");
    return e;
  }
  void wait(ssdt_stream s, Ev *e) override {
    check(hipStreamWaitEvent((hipStream_t)s, (hipEvent_t)e->h, 0), "hipStreamWaitEvent");
  }
  bool done(Ev *e) override { return hipEventQuery((hipEvent_t)e->h) == hipSuccess; }
  Ev *copy(int dir, void *dst, const void *src, size_t n, Ev *after) override {
    if (after) wait(q_[dir], after);
    check(hipMemcpyAsync(dst, src, n, dir == 0 ? hipMemcpyDeviceToHost : hipMemcpyHostToDevice, q_[dir]),
          "hipMemcpyAsync");
    return record(q_[dir], false);
  }
  void wait_queue(int dir, Ev *e) override { wait(q_[dir], e); }
  ssdt_stream queue_stream(int dir) override { return q_[dir]; }
  ssdt_stream aux_stream() override { return aux_; }
  void recycle(Ev *e) override { free_[e->timing ? 1 : 0].push_back(e); }
  double elapsed_ms(Ev *a, Ev *b) override {
    float ms = 0;
    if (hipEventElapsedTime(&ms, (hipEvent_t)a->h, (hipEvent_t)b->h) != hipSuccess) return 0;
    return ms;
  }
  void sync_io() override {
    (void)hipStreamSynchronize(q_[0]);
    (void)hipStreamSynchronize(q_[1]);
  }
  void host_sync_event(Ev *e) override { (void)hipEventSynchronize((hipEvent_t)e->h); }
  void *pool() override { return pool_; }
};

}  // namespace

Backend *make_hip_backend(size_t pool_bytes, std::string *err) {
  auto *b = new HipBackend();
  if (!b->init(pool_bytes)) {
    *err = b->err;
    delete b;
    return nullptr;
  }
  return b;
}

}  // namespace ssdt
