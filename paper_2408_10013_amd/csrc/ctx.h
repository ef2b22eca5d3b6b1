// Internal declarations shared by the host-side sources of libssdt: the context (tensor
// cache registry, device arena, copy backend).  Not part of the public interface.
#pragma once
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <deque>
#include <mutex>
#include <thread>
#include <map>
#include <memory>
#include <string>
#include <unordered_map>
#include <vector>

#include "ssdt.h"

namespace ssdt {

constexpr size_t kAlignTensor = 256;
constexpr size_t kAlignPack = 4096;
inline size_t up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// An event of the copy backend.  For the HIP backend `h` is a hipEvent_t; for the
// simulated backend `done` is flipped by ssdt_sim_complete.
struct Ev {
  void *h = nullptr;
  bool done = true;
  bool timing = false;
  int refs = 0;  // holders: free blocks, records, pending wait measurements
  uint64_t seq = 0;  // order of creation: on one in-order stream a younger event implies every older one
};

// What the registry needs from the machine: events, cross-stream waits and the two
// in-order copy queues (store = device to host, load = host to device).
class Backend {
 public:
  virtual ~Backend() {}
  virtual bool is_sim() const = 0;
  virtual Ev *record(ssdt_stream s, bool timing) = 0;             // event after s's current work
  virtual void thread_init() {}                                   // called once by every helper thread that uses the backend
  virtual void wait(ssdt_stream s, Ev *e) = 0;                    // s waits for e
  virtual bool done(Ev *e) = 0;
  virtual Ev *copy(int dir, void *dst, const void *src, size_t n, Ev *after) = 0;
  virtual void wait_queue(int dir, Ev *e) = 0;                    // a copy queue waits for e
  virtual ssdt_stream queue_stream(int dir) = 0;                  // identity of a copy queue as a stream
  virtual ssdt_stream aux_stream() { return nullptr; }            // side stream for kernels that may overlap the caller's; null if none
  virtual void recycle(Ev *e) = 0;
  virtual double elapsed_ms(Ev *a, Ev *b) = 0;
  virtual void sync_io() = 0;
  virtual void host_sync_event(Ev *e) = 0;
  virtual int sim_complete(int dir, int n) { (void)dir; (void)n; return -1; }
  virtual void *pool() = 0;
  std::string err;  // last backend failure ("" = none)
};
Backend *make_hip_backend(size_t pool_bytes, std::string *err);
Backend *make_sim_backend(size_t pool_bytes, std::string *err);

struct Block {
  size_t size = 0;
  bool free = true;
  int refs = 0;
  Ev *ready = nullptr;            // free block: later users on another stream wait for this
  ssdt_stream ready_stream = nullptr;
};

struct Rec {
  ssdt_tid tid = 0;
  int64_t layer = 0;          // owning layer, as a key: (micro-batch << 20) | layer index
  int32_t cls = 0, state = 0;
  uint64_t bytes = 0;
  int64_t pack_offset = -1, pool_offset = -1;
  void *dev = nullptr;
  bool in_arena = false;
  bool holds_ref = false;     // the registry holds a reference on dev's arena block
  bool stored = false;        // a host copy exists or is being written
  bool forwarded = false;
  bool release_pending = false;  // released while its store was still in flight
  bool load_waited = false;
  bool spill_deferred = false; // spill mode: dropped from the device before its copy out was seen finished
  bool read_pending = false;  // spill mode: the file read of this record has been requested, its copy not yet issued
  std::vector<int64_t> scopes;  // scope keys: (micro-batch << 20) | scope
  Ev *store_ev = nullptr, *load_ev = nullptr;
};

// events are shared by reference count: hold() on taking one, drop() when done with it
static inline Ev *hold(Ev *e) {
  if (e) ++e->refs;
  return e;
}
static inline void drop(Backend *be, Ev *e) {
  if (e && --e->refs <= 0) be->recycle(e);
}

struct WaitPair { Ev *a, *b; int kind; uint64_t step; };

// Spill file: the tier behind the pinned pool (Sec. 3.1 names an SSD offloader beside the CPU
// offloader).  The pool is the staging buffer, the file holds the data at the same offsets.  The
// file is opened for direct I/O (no page cache behind the pool; every tensor starts on a 4 KiB
// boundary of pool and file when a spill file is configured) and served by a small pool of
// threads that take requests in order, a tensor being cut into chunks so that several requests are
// in flight at the device; each thread stages its chunk in a page-aligned buffer of its own, since
// pinned device-visible memory cannot be the buffer of a direct transfer.  A record is written once its device-to-host
// copy has completed (its pool bytes are then overwritten with a pattern, so a later load can
// only come from the file), and read back into the pool when a prefetch asks for it; a read asked
// for while the write is still going on is queued when the write ends.  The host-to-device copy
// of a record is issued by the next API call that finds its read complete.
struct Spill {
  int fd = -1;
  bool direct = false;           // O_DIRECT in effect (false where the file system refuses it)
  std::vector<std::thread> workers;
  std::mutex mu;
  std::condition_variable cv;
  struct Chunk { int kind; size_t key, at, len; };  // kind 0 write, 1 read; key = the tensor's pool offset
  std::deque<Chunk> chunks;
  struct Item { int st = 0, pending = 0; bool read_wanted = false; size_t bytes = 0; };
  std::map<size_t, Item> state;  // pool offset -> 1 write queued, 2 written, 3 read queued, 4 in pool again
  int busy = 0;
  bool stop = false;
  std::string error;             // first I/O error, sticky
  uint64_t bytes_written = 0, bytes_read = 0;
  // wall time during which at least one write / read chunk was at the device
  uint64_t write_ns = 0, read_ns = 0;
  int writes_in_flight = 0, reads_in_flight = 0;
  std::chrono::steady_clock::time_point w_since, r_since;
  char *pool = nullptr;
};
constexpr size_t kAlignSpill = 4096;       // tensor alignment in pool and file when a spill file is configured
constexpr size_t kSpillChunk = 8u << 20;   // bytes per file request

struct Ctx;
// first statement of every C ABI entry point that takes a context
struct ApiLock {
  std::unique_lock<std::recursive_mutex> l;
  explicit ApiLock(const Ctx *c);
};

struct Ctx {
  ssdt_config cfg{};
  std::unique_ptr<Backend> be;
  std::string last_error;
  // arena
  std::map<size_t, Block> blocks;  // offset -> block
  uint64_t in_use = 0, peak_in_use = 0, high_water = 0, n_allocs = 0;
  // registry
  int32_t num_layers = 0;
  std::vector<std::pair<const char *, size_t>> weights;
  std::vector<int64_t> stack;     // open forward scopes (keys)
  std::vector<int64_t> bwd_open;  // open backward scopes (keys)
  // Records are kept per micro-batch (Sec. 3.1): every scope id the caller passes is combined with the current
  // micro-batch into a key, so that several micro-batches can be between their forward and their backward.
  int32_t cur_mb = 0;
  std::map<int32_t, int32_t> mb_keep_last;  // per-micro-batch override of cfg.keep_last
  static constexpr int kScopeBits = 20;
  int64_t key(int32_t scope) const { return ((int64_t)cur_mb << kScopeBits) | (int64_t)scope; }
  static int32_t scope_of(int64_t k) { return (int32_t)(k & ((1 << kScopeBits) - 1)); }
  static int32_t mb_of(int64_t k) { return (int32_t)(k >> kScopeBits); }
  uint64_t next_stamp = 1;
  std::vector<Rec> recs;
  std::unordered_map<const void *, size_t> by_storage;
  std::unordered_map<ssdt_tid, size_t> by_tid;
  std::map<int64_t, size_t> pack_base, pack_cursor;  // by layer key
  size_t pool_cursor = 0;
  std::deque<size_t> storing;  // record indices with a store in flight, oldest first
  ssdt_stats st{};
  std::vector<WaitPair> waits;
  uint64_t step_no = 0;  // counts ssdt_step_begin calls: wait measurements belong to the step they were taken in
  std::unique_ptr<Spill> spill;
  // With a spill file a helper thread runs poll() a few thousand times a second, so that finished copies out of the
  // device are written to the file, and finished file reads are copied into the device, without waiting for the
  // caller's next call (a training loop runs a whole pass ahead of the GPU).  Every entry point of the C ABI then
  // holds this lock for its duration; without a spill file nobody takes it.
  mutable std::recursive_mutex api_mu;
  std::thread pump;
  std::atomic<bool> pump_stop{false};
  std::deque<size_t> spill_wait, reading;  // records waiting for their file write / file read

  ssdt_status fail(ssdt_status code, const char *fmt, ...);
  bool in_arena(const void *p) const {
    auto c = (const char *)p, b = (const char *)cfg.arena_base;
    return cfg.arena_base && c >= b && c < b + cfg.arena_bytes;
  }
  // arena
  ssdt_status alloc(size_t bytes, ssdt_stream s, void **out);
  void ref(void *p);
  void unref(void *p, Ev *ready, ssdt_stream ready_stream);
  bool try_alloc(size_t bytes, ssdt_stream s, void **out);
  // registry
  void poll();
  void reclaim(size_t idx);
  bool is_weight(const void *p) const;
  ssdt_status save(const void *base, size_t sbytes, size_t view_off, const int64_t *shape, int32_t ndim,
                   int32_t dtype, ssdt_tid *out);
  ssdt_status scope_begin(int32_t scope, int32_t phase);
  ssdt_status scope_end(int32_t scope, int32_t phase);
  ssdt_status offload(int32_t scope, ssdt_stream producer);
  ssdt_status prefetch(int32_t scope);
  ssdt_status get(ssdt_tid tid, ssdt_stream consumer, void **out);
  ssdt_status release(int32_t scope, ssdt_stream s);
  ssdt_status step_begin(int32_t n);
  ssdt_status micro_batch(int32_t mb, int32_t keep_last);
  void timed_wait(ssdt_stream s, Ev *e, int kind);
  ssdt_status spill_open(const char *path);
  void spill_close();
  ssdt_status spill_status(const char *who);
  void spill_request(int kind, size_t pool_off, size_t bytes);
  size_t tensor_align() const { return spill ? kAlignSpill : kAlignTensor; }
  bool spill_in_pool(size_t pool_off, bool block);
  void spill_drain();
  ssdt_status start_load(size_t idx, const char *who);
  ssdt_status issue_copy_in(size_t idx, const char *who);
  ssdt_status pump_reads();
};

}  // namespace ssdt

struct ssdt_ctx : ssdt::Ctx {};
