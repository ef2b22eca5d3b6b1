// Simulated copy backend for host-side tests of the registry: "device" memory is host
// memory, a copy is a queued job that runs when the test completes it by hand, and an
// event on a compute stream is complete at once.  No GPU call is made.
#include <cstdlib>

#include "ctx.h"

namespace ssdt {
namespace {

struct Job {
  void *dst;
  const void *src;
  size_t n;
  Ev *ev;
};

class SimBackend : public Backend {
 public:
  std::deque<Job> q_[2];
  void *pool_ = nullptr;
  std::vector<Ev *> all_, free_;
  uint64_t seq_ = 0;
  int tag_[2] = {0, 0};  // addresses of these stand for the two queues

  ~SimBackend() override {
    for (Ev *e : all_) delete e;
    free(pool_);
  }
  bool is_sim() const override { return true; }
  Ev *get_ev() {
    Ev *e;
    if (!free_.empty()) {
      e = free_.back();
      free_.pop_back();
    } else {
      e = new Ev();
      all_.push_back(e);
    }
    e->refs = 0;
    e->done = true;
    e->seq = ++seq_;
    return e;
  }
  Ev *record(ssdt_stream, bool) override { return get_ev(); }
  void wait(ssdt_stream, Ev *e) override {
    // a stream that waits for a copy sees it finished: run the queues up to that copy
    for (int d = 0; d < 2 && !e->done; ++d) {
      bool mine = false;
      for (auto &j : q_[d]) mine |= (j.ev == e);
      while (mine && !e->done) sim_complete(d, 1);
    }
  }
  bool done(Ev *e) override { return e->done; }
  Ev *copy(int dir, void *dst, const void *src, size_t n, Ev *) override {
    Ev *e = get_ev();
    e->done = false;
    ++e->refs;  // the queue's own reference, dropped when the job runs
    q_[dir].push_back({dst, src, n, e});
    return e;
  }
  void wait_queue(int, Ev *) override {}
  ssdt_stream queue_stream(int dir) override { return &tag_[dir]; }
  void recycle(Ev *e) override { free_.push_back(e); }
  double elapsed_ms(Ev *, Ev *) override { return 0; }
  void sync_io() override {
    sim_complete(0, (int)q_[0].size());
    sim_complete(1, (int)q_[1].size());
  }
  void host_sync_event(Ev *) override {}
  int sim_complete(int dir, int n) override {
    if (dir < 0 || dir > 1) return 0;
    int k = 0;
    while (k < n && !q_[dir].empty()) {
      Job j = q_[dir].front();
      q_[dir].pop_front();
      memcpy(j.dst, j.src, j.n);
      j.ev->done = true;
      if (--j.ev->refs <= 0) recycle(j.ev);
      ++k;
    }
    return k;
  }
  void *pool() override { return pool_; }
};

}  // namespace

Backend *make_sim_backend(size_t pool_bytes, std::string *err) {
  auto *b = new SimBackend();
  if (pool_bytes) {
    // page aligned, as pinned memory is: the spill file may be open for direct I/O
    if (posix_memalign(&b->pool_, 4096, (pool_bytes + 4095) / 4096 * 4096) != 0) b->pool_ = nullptr;
    if (!b->pool_) {
      *err = "out of host memory for the simulated pool";
      delete b;
      return nullptr;
    }
  }
  return b;
}

}  // namespace ssdt
