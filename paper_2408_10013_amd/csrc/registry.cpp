// The tensor cache: saved-tensor registry, device arena and offload/prefetch engine.
//
// Follows the paper's Sec. 3.1 (when offloads and prefetches start, kept last module),
// Sec. 3.2 (scope stack, pack/unpack hooks, release at scope exit), Sec. 3.3.1 (identity by
// storage stamp, weight exclusion), Sec. 3.3.2 (two in-order queues, data forwarding) and
// Algorithm 1 (order of the pack hook's tests).  Everything here is host code; the machine
// is reached only through `Backend`.
#include <algorithm>

#include "ctx.h"

#include <cerrno>
#include <fcntl.h>
#include <unistd.h>
#include "prof.h"

namespace ssdt {

ssdt_status Ctx::fail(ssdt_status code, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  last_error = buf;
  return code;
}


// ---------------------------------------------------------------------------------------
// arena: first-fit by address over a map of blocks; blocks are reference counted (the
// caller's reference from alloc, the registry's from save)
// ---------------------------------------------------------------------------------------

static void tidy(Ctx *c) {
  // forget ready-events that have completed, then merge neighbouring free blocks that carry none
  for (auto &kv : c->blocks) {
    Block &b = kv.second;
    if (b.free && b.ready && c->be->done(b.ready)) {
      drop(c->be.get(), b.ready);
      b.ready = nullptr;
    }
  }
  for (auto it = c->blocks.begin(); it != c->blocks.end();) {
    auto nx = std::next(it);
    if (nx == c->blocks.end()) break;
    Block &a = it->second, &b = nx->second;
    // neighbours merge when one event covers both: none at all, only one of them has one, or both
    // wait on the same in-order stream (then the younger event implies the older)
    bool ok = a.free && b.free && (!a.ready || !b.ready || a.ready_stream == b.ready_stream);
    if (ok) {
      if (b.ready && (!a.ready || b.ready->seq > a.ready->seq)) {
        drop(c->be.get(), a.ready);
        a.ready = b.ready;  // takes over b's reference
        a.ready_stream = b.ready_stream;
      } else {
        drop(c->be.get(), b.ready);
      }
      a.size += b.size;
      c->blocks.erase(nx);
    } else {
      it = nx;
    }
  }
}

// Large blocks are placed first-fit from the bottom of the arena, small ones (statistics, a few
// KiB each and long-lived) from the top, so that the small ones do not end up between large
// blocks and keep their neighbours from merging once those are freed.
bool Ctx::try_alloc(size_t bytes, ssdt_stream s, void **out) {
  const bool small = bytes < (1u << 20);
  std::map<size_t, Block>::iterator hit = blocks.end();
  if (!small) {
    for (auto it = blocks.begin(); it != blocks.end(); ++it)
      if (it->second.free && it->second.size >= bytes) { hit = it; break; }
  } else {
    for (auto it = blocks.end(); it != blocks.begin();) {
      --it;
      if (it->second.free && it->second.size >= bytes) { hit = it; break; }
    }
  }
  if (hit == blocks.end()) return false;
  if (hit->second.size > bytes) {
    Block rest = hit->second;
    rest.size = hit->second.size - bytes;
    hold(rest.ready);
    if (!small) {  // keep the low part
      blocks[hit->first + bytes] = rest;
      hit->second.size = bytes;
    } else {       // keep the high part
      Block mine = hit->second;
      mine.size = bytes;
      const size_t off = hit->first + rest.size;
      hit->second = rest;
      hit = blocks.emplace(off, mine).first;
    }
  }
  Block &b = hit->second;
  if (b.ready) {
    if (b.ready_stream != s) be->wait(s, b.ready);
    drop(be.get(), b.ready);
    b.ready = nullptr;
  }
  b.free = false;
  b.refs = 1;
  in_use += bytes;
  peak_in_use = std::max(peak_in_use, in_use);
  high_water = std::max<uint64_t>(high_water, hit->first + bytes);
  ++n_allocs;
  *out = (char *)cfg.arena_base + hit->first;
  return true;
}

ssdt_status Ctx::alloc(size_t bytes, ssdt_stream s, void **out) {
  if (!out || bytes == 0) return fail(SSDT_E_INVAL, "arena_alloc: null output or zero size");
  if (!cfg.arena_base) return fail(SSDT_E_NOMEM, "arena_alloc: the context has no arena");
  bytes = up(bytes, kAlignTensor);
  poll();
  tidy(this);
  if (try_alloc(bytes, s, out)) return SSDT_OK;
  // No room: tensors still being stored hold memory that returns once their copy is done
  // (Sec. 3.2).  Make the requesting stream wait for the oldest stores, in order.
  while (!storing.empty()) {
    size_t idx = storing.front();
    storing.pop_front();
    Rec &r = recs[idx];
    if (r.forwarded || r.state != SSDT_ST_STORING) continue;
    timed_wait(s, r.store_ev, 1);
    reclaim(idx);
    tidy(this);
    if (try_alloc(bytes, s, out)) return SSDT_OK;
  }
  return fail(SSDT_E_NOMEM, "arena_alloc: no room for %zu bytes (in use %llu of %zu)", bytes,
              (unsigned long long)in_use, cfg.arena_bytes);
}

void Ctx::ref(void *p) {
  auto it = blocks.find((char *)p - (char *)cfg.arena_base);
  if (it != blocks.end() && !it->second.free) ++it->second.refs;
}

void Ctx::unref(void *p, Ev *ready, ssdt_stream ready_stream) {
  auto it = blocks.find((char *)p - (char *)cfg.arena_base);
  if (it == blocks.end() || it->second.free) return;
  Block &b = it->second;
  if (--b.refs > 0) return;
  b.free = true;
  b.ready = hold(ready);
  b.ready_stream = ready_stream;
  in_use -= b.size;
  by_storage.erase(p);  // the address may now be reused by a different storage
}

// ---------------------------------------------------------------------------------------
// registry
// ---------------------------------------------------------------------------------------

bool Ctx::is_weight(const void *p) const {
  for (auto &w : weights)
    if ((const char *)p >= w.first && (const char *)p < w.first + w.second) return true;
  return false;
}

void Ctx::timed_wait(ssdt_stream s, Ev *e, int kind) {
  if (cfg.measure_waits && !be->is_sim()) {
    Ev *a = hold(be->record(s, true));
    be->wait(s, e);
    Ev *b = hold(be->record(s, true));
    waits.push_back({a, b, kind, step_no});
  } else {
    be->wait(s, e);
  }
}

// The store of record idx is complete (or `s` has been ordered after it): the registry gives up
// its reference on the device copy at that point (Sec. 3.2), which returns the block to the arena
// unless someone else still holds it.
void Ctx::reclaim(size_t idx) {
  Rec &r = recs[idx];
  bool finished = be->done(r.store_ev);
  if (r.holds_ref) {
    unref(r.dev, finished ? nullptr : r.store_ev, be->queue_stream(0));
    r.holds_ref = false;
  }
  r.dev = nullptr;
  r.state = r.release_pending ? SSDT_ST_RELEASED : SSDT_ST_OFFLOADED;
  if (spill && !r.release_pending) {
    if (finished) {
      spill_request(0, (size_t)r.pool_offset, r.bytes);
    } else {  // written once the copy is seen finished
      r.spill_deferred = true;
      spill_wait.push_back(idx);
    }
  }
}

// ---------------------------------------------------------------------------------------
// spill file
// ---------------------------------------------------------------------------------------

static bool rw_all(int fd, char *buf, size_t n, size_t off, bool write, std::string *err) {
  while (n) {
    ssize_t k = write ? pwrite(fd, buf, n, (off_t)off) : pread(fd, buf, n, (off_t)off);
    if (k < 0 && errno == EINTR) continue;
    if (k <= 0) {
      *err = std::string(write ? "spill write: " : "spill read: ") + (k == 0 ? "unexpected end of file" : strerror(errno));
      return false;
    }
    buf += k;
    off += (size_t)k;
    n -= (size_t)k;
  }
  return true;
}

// Queues the chunks of one tensor's write or read (caller holds the lock).  The range is padded to whole 4 KiB
// blocks: every tensor starts on such a boundary and owns the bytes up to the next one.
static void spill_push(Spill *sp, int kind, size_t key, size_t bytes) {
  Spill::Item &it = sp->state[key];
  it.st = kind == 0 ? 1 : 3;
  it.bytes = bytes;
  const size_t total = up(bytes, kAlignSpill);
  it.pending = 0;
  for (size_t o = 0; o < total; o += kSpillChunk) {
    sp->chunks.push_back({kind, key, key + o, std::min(kSpillChunk, total - o)});
    ++it.pending;
  }
}

static void spill_worker(Spill *sp) {
  // Direct I/O cannot take pinned device-visible memory as its buffer (the kernel refuses to pin those pages a
  // second time: EFAULT), so in direct mode every request goes through this thread's own page-aligned buffer.
  void *bounce = nullptr;
  if (sp->direct && posix_memalign(&bounce, kAlignSpill, kSpillChunk) != 0) bounce = nullptr;
  std::unique_lock<std::mutex> lk(sp->mu);
  for (;;) {
    sp->cv.wait(lk, [&] { return sp->stop || !sp->chunks.empty(); });
    if (sp->chunks.empty()) {  // stop requested and nothing left
      free(bounce);
      return;
    }
    Spill::Chunk c = sp->chunks.front();
    sp->chunks.pop_front();
    ++sp->busy;
    const auto now = std::chrono::steady_clock::now();
    if (c.kind == 0) { if (sp->writes_in_flight++ == 0) sp->w_since = now; }
    else { if (sp->reads_in_flight++ == 0) sp->r_since = now; }
    bool failed = !sp->error.empty();
    lk.unlock();
    std::string err;
    bool ok = true;
    if (!failed) {
      if (sp->direct && !bounce) {
        ok = false;
        err = "spill: no memory for the direct-I/O buffer";
      } else if (sp->direct) {
        if (c.kind == 0) memcpy(bounce, sp->pool + c.at, c.len);
        ok = rw_all(sp->fd, (char *)bounce, c.len, c.at, c.kind == 0, &err);
        if (ok && c.kind == 1) memcpy(sp->pool + c.at, bounce, c.len);
      } else {
        ok = rw_all(sp->fd, sp->pool + c.at, c.len, c.at, c.kind == 0, &err);
      }
      if (ok && c.kind == 0) memset(sp->pool + c.at, 0xEE, c.len);  // from here on only the file has it
    }
    lk.lock();
    const auto then = std::chrono::steady_clock::now();
    if (c.kind == 0) { if (--sp->writes_in_flight == 0) sp->write_ns += (uint64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(then - sp->w_since).count(); }
    else { if (--sp->reads_in_flight == 0) sp->read_ns += (uint64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(then - sp->r_since).count(); }
    if (!ok && sp->error.empty()) sp->error = err;
    Spill::Item &it = sp->state[c.key];
    if (--it.pending == 0) {  // the tensor's last chunk
      if (ok && !failed) (c.kind == 0 ? sp->bytes_written : sp->bytes_read) += it.bytes;
      it.st = c.kind == 0 ? 2 : 4;
      if (c.kind == 0 && it.read_wanted) {  // a prefetch came while the write was going on
        it.read_wanted = false;
        spill_push(sp, 1, c.key, it.bytes);
      }
    }
    --sp->busy;
    sp->cv.notify_all();
  }
}

ApiLock::ApiLock(const Ctx *c) {
  if (c && c->spill) l = std::unique_lock<std::recursive_mutex>(c->api_mu);
}

static void spill_pump(Ctx *c) {
  c->be->thread_init();
  while (!c->pump_stop.load()) {
    std::this_thread::sleep_for(std::chrono::microseconds(200));
    std::unique_lock<std::recursive_mutex> lk(c->api_mu, std::try_to_lock);
    if (lk.owns_lock()) c->poll();  // what the caller's next call would do first
  }
}

ssdt_status Ctx::spill_open(const char *path) {
  // direct I/O where the file system takes it: the pool is pinned memory, a second copy in the page cache would
  // only cost host bandwidth
  bool direct = true;
  int fd = open(path, O_RDWR | O_CREAT | O_TRUNC | O_DIRECT, 0600);
  if (fd < 0 && (errno == EINVAL || errno == EOPNOTSUPP || errno == ENOTSUP)) {
    direct = false;
    fd = open(path, O_RDWR | O_CREAT | O_TRUNC, 0600);
  }
  if (fd < 0) return fail(SSDT_E_IO, "cannot open the spill file %s: %s", path, strerror(errno));
  spill.reset(new Spill());
  spill->fd = fd;
  spill->direct = direct;
  spill->pool = (char *)be->pool();
  const int n = cfg.spill_threads > 0 ? std::min(cfg.spill_threads, 64) : 4;
  for (int i = 0; i < n; ++i) spill->workers.emplace_back(spill_worker, spill.get());
  pump_stop = false;
  pump = std::thread(spill_pump, this);
  return SSDT_OK;
}

void Ctx::spill_close() {
  if (!spill) return;
  pump_stop = true;
  if (pump.joinable()) pump.join();
  {
    std::lock_guard<std::mutex> g(spill->mu);
    spill->stop = true;
  }
  spill->cv.notify_all();
  for (auto &t : spill->workers) t.join();
  close(spill->fd);
  spill.reset();
}

void Ctx::spill_request(int kind, size_t off, size_t bytes) {
  {
    std::lock_guard<std::mutex> g(spill->mu);
    auto it = spill->state.find(off);
    if (kind == 1 && it != spill->state.end() && it->second.st == 1) {
      it->second.read_wanted = true;  // its write has not finished: the read is queued when it has
    } else {
      spill_push(spill.get(), kind, off, bytes);
    }
  }
  spill->cv.notify_all();
}

// True once the bytes at `off` have been read back into the pool; with `block`, waits for that.
bool Ctx::spill_in_pool(size_t off, bool block) {
  std::unique_lock<std::mutex> lk(spill->mu);
  if (block) spill->cv.wait(lk, [&] { return spill->state[off].st == 4; });
  return spill->state[off].st == 4;
}

void Ctx::spill_drain() {
  std::unique_lock<std::mutex> lk(spill->mu);
  spill->cv.wait(lk, [&] { return spill->chunks.empty() && spill->busy == 0; });
}

ssdt_status Ctx::spill_status(const char *who) {
  if (!spill) return SSDT_OK;
  std::lock_guard<std::mutex> g(spill->mu);
  if (spill->error.empty()) return SSDT_OK;
  return fail(SSDT_E_IO, "%s: %s", who, spill->error.c_str());
}

// Enqueues the host-to-device copy of record idx from the pool into its (already assigned) slot.
ssdt_status Ctx::issue_copy_in(size_t idx, const char *who) {
  Rec &r = recs[idx];
  r.read_pending = false;
  // a record dropped under memory pressure may still be on its way out: the copy in follows it
  Ev *after = (r.store_ev && !be->done(r.store_ev)) ? r.store_ev : nullptr;
  drop(be.get(), r.load_ev);
  r.load_ev = hold(be->copy(1, r.dev, (char *)be->pool() + r.pool_offset, r.bytes, after));
  if (!be->err.empty()) return fail(SSDT_E_HIP, "%s: %s", who, be->err.c_str());
  return SSDT_OK;
}

// Starts bringing an OFFLOADED record, whose new slot is already in r.dev, back to the device.
ssdt_status Ctx::start_load(size_t idx, const char *who) {
  Rec &r = recs[idx];
  r.state = SSDT_ST_LOADING;
  r.load_waited = false;
  ++st.loads;
  st.bytes_loaded += r.bytes;
  if (spill && !r.spill_deferred) {  // only the file has the bytes: read first, copy when that is done
    drop(be.get(), r.load_ev);
    r.load_ev = nullptr;
    r.read_pending = true;
    reading.push_back(idx);
    spill_request(1, (size_t)r.pool_offset, r.bytes);
    return SSDT_OK;
  }
  r.spill_deferred = false;  // taken straight from the pool; its write to the file is dropped
  return issue_copy_in(idx, who);
}

// Spill mode housekeeping: queue the writes of stores seen finished, issue the copies of finished reads.
ssdt_status Ctx::pump_reads() {
  if (!spill) return SSDT_OK;
  while (!spill_wait.empty()) {
    Rec &r = recs[spill_wait.front()];
    if (r.spill_deferred) {
      if (!be->done(r.store_ev)) break;  // stores finish in order
      r.spill_deferred = false;
      if (r.state == SSDT_ST_OFFLOADED) spill_request(0, (size_t)r.pool_offset, r.bytes);
    }
    spill_wait.pop_front();
  }
  while (!reading.empty()) {
    size_t idx = reading.front();
    Rec &r = recs[idx];
    if (r.read_pending) {
      if (!spill_in_pool((size_t)r.pool_offset, false)) break;  // reads finish in order
      ssdt_status e = spill_status("load");
      if (e != SSDT_OK) return e;
      e = issue_copy_in(idx, "load");
      if (e != SSDT_OK) return e;
    }
    reading.pop_front();
  }
  return SSDT_OK;
}

void Ctx::poll() {
  while (!storing.empty()) {
    size_t idx = storing.front();
    Rec &r = recs[idx];
    if (r.forwarded || r.state != SSDT_ST_STORING) {
      storing.pop_front();
      continue;
    }
    if (!be->done(r.store_ev)) break;
    storing.pop_front();
    reclaim(idx);
  }
  if (spill) (void)pump_reads();  // an I/O error stays recorded and is reported by spill_status()
}

ssdt_status Ctx::step_begin(int32_t n) {
  if (n <= 0) return fail(SSDT_E_INVAL, "step_begin: num_layers must be positive");
  if (!stack.empty()) return fail(SSDT_E_STATE, "step_begin: a forward scope is still open");
  for (auto &r : recs)
    if (!r.scopes.empty())
      return fail(SSDT_E_STATE, "step_begin: record %llu of the previous step has not been released",
                  (unsigned long long)r.tid);
  poll();
  if (!storing.empty()) {
    be->sync_io();
    poll();
  }
  if (spill) {
    spill_drain();
    spill->state.clear();
    spill_wait.clear();
    reading.clear();
    ssdt_status e = spill_status("step_begin");
    if (e != SSDT_OK) return e;
  }
  for (auto &r : recs) {
    drop(be.get(), r.store_ev);
    drop(be.get(), r.load_ev);
  }
  recs.clear();
  by_storage.clear();
  by_tid.clear();
  pack_base.clear();
  pack_cursor.clear();
  storing.clear();
  bwd_open.clear();
  cur_mb = 0;
  mb_keep_last.clear();
  pool_cursor = 0;
  num_layers = n;
  ++step_no;  // measurements of earlier steps still in `waits` are dropped when they are next looked at
  ssdt_stats z{};
  st = z;
  peak_in_use = in_use;
  high_water = 0;
  for (auto &kv : blocks)
    if (!kv.second.free) high_water = std::max<uint64_t>(high_water, kv.first + kv.second.size);
  return SSDT_OK;
}

ssdt_status Ctx::micro_batch(int32_t mb, int32_t keep_last) {
  if (mb < 0 || mb >= (1 << 20)) return fail(SSDT_E_INVAL, "micro_batch: id out of range");
  if (!stack.empty() || !bwd_open.empty()) return fail(SSDT_E_STATE, "micro_batch: a scope is still open");
  if (num_layers <= 0) return fail(SSDT_E_STATE, "micro_batch: no step in progress (call ssdt_step_begin)");
  cur_mb = mb;
  if (keep_last >= 0) mb_keep_last[mb] = keep_last;
  return SSDT_OK;
}

ssdt_status Ctx::scope_begin(int32_t scope_id, int32_t phase) {
  if (scope_id < 0 || scope_id >= (1 << kScopeBits)) return fail(SSDT_E_INVAL, "scope_begin: scope id out of range");
  const int64_t scope = key(scope_id);
  if (phase == SSDT_FWD) {
    if (num_layers <= 0) return fail(SSDT_E_STATE, "scope_begin: no step in progress (call ssdt_step_begin)");
    if (stack.empty() && !pack_base.count(scope)) {
      pool_cursor = up(pool_cursor, kAlignPack);
      pack_base[scope] = pool_cursor;
      pack_cursor[scope] = 0;
    }
    stack.push_back(scope);
    return SSDT_OK;
  }
  if (phase == SSDT_BWD) {
    bwd_open.push_back(scope);
    return SSDT_OK;
  }
  return fail(SSDT_E_INVAL, "scope_begin: unknown phase %d", phase);
}

ssdt_status Ctx::scope_end(int32_t scope_id, int32_t phase) {
  const int64_t scope = key(scope_id);
  if (phase == SSDT_FWD) {
    if (stack.empty() || stack.back() != scope)
      return fail(SSDT_E_STATE, "scope_end: scope %d is not on top of the forward scope stack", scope_id);
    stack.pop_back();
    if (stack.empty()) pool_cursor = up(pack_base[scope] + pack_cursor[scope], kAlignPack);
    return SSDT_OK;
  }
  if (phase == SSDT_BWD) {
    if (bwd_open.empty() || bwd_open.back() != scope)
      return fail(SSDT_E_STATE, "scope_end: backward scope %d is not open", scope_id);
    bwd_open.pop_back();
    return SSDT_OK;
  }
  return fail(SSDT_E_INVAL, "scope_end: unknown phase %d", phase);
}

ssdt_status Ctx::save(const void *base, size_t sbytes, size_t view_off, const int64_t *shape, int32_t ndim,
                      int32_t dtype, ssdt_tid *out) {
  if (!base || !out || !shape || ndim <= 0 || sbytes == 0) return fail(SSDT_E_INVAL, "save: null or empty argument");
  if (dtype != SSDT_F32 && dtype != SSDT_BF16) return fail(SSDT_E_INVAL, "save: unknown dtype %d", dtype);
  if (stack.empty()) return fail(SSDT_E_STATE, "save: no forward scope is open");
  uint64_t numel = 1;
  for (int i = 0; i < ndim; ++i) {
    if (shape[i] < 0) return fail(SSDT_E_INVAL, "save: negative extent");
    numel *= (uint64_t)shape[i];
  }
  size_t esize = dtype == SSDT_F32 ? 4 : 2;
  if (view_off + numel * esize > sbytes) return fail(SSDT_E_INVAL, "save: the view does not fit its storage");
  bool arena = in_arena(base);
  if (arena) {
    auto it = blocks.find((const char *)base - (const char *)cfg.arena_base);
    if (it == blocks.end() || it->second.free || it->second.size < sbytes)
      return fail(SSDT_E_INVAL, "save: storage is inside the arena but is not a live arena block");
  }
  ++st.save_calls;
  if (is_weight(base)) {  // Alg. 1, first test
    ++st.bypass_weight;
    *out = 0;
    return SSDT_OK;
  }
  const int64_t scope = stack.back(), layer = stack.front();
  auto hit = by_storage.find(base);
  if (hit != by_storage.end()) {  // a view of a storage already stamped (Sec. 3.3.1)
    Rec &r = recs[hit->second];
    ++st.dedup_hits;
    if (std::find(r.scopes.begin(), r.scopes.end(), scope) == r.scopes.end()) r.scopes.push_back(scope);
    *out = r.cls == SSDT_CLS_SMALL ? 0 : r.tid;
    return SSDT_OK;
  }
  Rec r;
  r.tid = next_stamp++;
  r.layer = layer;
  r.bytes = sbytes;
  r.dev = const_cast<void *>(base);
  r.in_arena = arena;
  r.state = SSDT_ST_RESIDENT;
  r.scopes.push_back(scope);
  ++st.unique;
  if (arena) {
    ref(r.dev);
    r.holds_ref = true;
  }
  if ((int64_t)numel < cfg.min_offload_elems) {  // Alg. 1: too small to be worth a transfer
    r.cls = SSDT_CLS_SMALL;
    ++st.bypass_small;
    st.bytes_small += sbytes;
    *out = 0;
  } else {
    auto kl = mb_keep_last.find(mb_of(layer));
    bool in_last = scope_of(layer) >= num_layers - (kl != mb_keep_last.end() ? kl->second : cfg.keep_last);
    bool over = cfg.budget_bytes >= 0 && st.bytes_offloaded + sbytes > (uint64_t)cfg.budget_bytes;
    size_t off = up(pack_cursor[layer], tensor_align());
    bool nomem = up(pack_base[layer] + off + sbytes, kAlignPack) > cfg.pool_bytes;
    const bool recomputing = !bwd_open.empty();  // a checkpointed module re-running its forward (Sec. 3.2)
    if (in_last || over || nomem || !arena || recomputing) {
      r.cls = SSDT_CLS_KEPT;
      ++st.kept;
      st.bytes_kept += sbytes;
    } else {
      r.cls = SSDT_CLS_OFFLOADED;
      r.pack_offset = (int64_t)off;
      r.pool_offset = (int64_t)(pack_base[layer] + off);
      pack_cursor[layer] = off + sbytes;
      ++st.offloaded;
      st.bytes_offloaded += sbytes;
      st.pool_bytes_used = up(pack_base[layer] + pack_cursor[layer], kAlignPack);
    }
    *out = r.tid;
  }
  by_storage[base] = recs.size();
  by_tid[r.tid] = recs.size();
  recs.push_back(r);
  return SSDT_OK;
}

ssdt_status Ctx::offload(int32_t scope_id, ssdt_stream producer) {
  const int64_t scope = key(scope_id);
  poll();
  if (ssdt_status e = spill_status("offload")) return e;
  Ev *after = nullptr;
  for (size_t i = 0; i < recs.size(); ++i) {
    Rec &r = recs[i];
    if (r.layer != scope || r.cls != SSDT_CLS_OFFLOADED || r.state != SSDT_ST_RESIDENT || r.stored || !r.dev)
      continue;
    if (!after) {
      after = hold(be->record(producer, false));
      be->wait_queue(0, after);  // the copy starts once the producing operators have finished
    }
    r.store_ev = hold(be->copy(0, (char *)be->pool() + r.pool_offset, r.dev, r.bytes, nullptr));
    if (!be->err.empty()) return fail(SSDT_E_HIP, "offload: %s", be->err.c_str());
    r.stored = true;
    r.state = SSDT_ST_STORING;
    storing.push_back(i);
  }
  drop(be.get(), after);
  return SSDT_OK;
}

ssdt_status Ctx::prefetch(int32_t scope_id) {
  const int64_t scope = key(scope_id);
  poll();
  if (ssdt_status e = spill_status("prefetch")) return e;
  std::vector<size_t> todo;
  for (size_t i = recs.size(); i-- > 0;) {  // reverse of the order recorded in forward (Sec. 3.1)
    Rec &r = recs[i];
    if (r.layer != scope || r.cls != SSDT_CLS_OFFLOADED || r.scopes.empty()) continue;
    if (r.state == SSDT_ST_STORING) {  // still being stored: forward the in-memory copy (Sec. 3.3.2)
      r.state = SSDT_ST_RESIDENT;
      r.forwarded = true;
      ++st.forwarded;
    } else if (r.state == SSDT_ST_OFFLOADED) {
      todo.push_back(i);
    }
  }
  ssdt_stream q = be->queue_stream(1);
  std::vector<void *> slots;
  for (size_t i : todo) {
    void *p = nullptr;
    if (alloc(recs[i].bytes, q, &p) != SSDT_OK) {
      for (void *s : slots) unref(s, nullptr, nullptr);
      return SSDT_E_NOMEM;  // message set by alloc; nothing was enqueued
    }
    slots.push_back(p);
  }
  for (size_t k = 0; k < todo.size(); ++k) {
    Rec &r = recs[todo[k]];
    r.dev = slots[k];
    r.holds_ref = true;  // the reference alloc() gave now belongs to the record
    by_storage[r.dev] = todo[k];
    ssdt_status e = start_load(todo[k], "prefetch");
    if (e != SSDT_OK) return e;
  }
  return SSDT_OK;
}

ssdt_status Ctx::get(ssdt_tid tid, ssdt_stream consumer, void **out) {
  if (!out) return fail(SSDT_E_INVAL, "get: null output");
  auto it = by_tid.find(tid);
  if (tid == 0 || it == by_tid.end()) return fail(SSDT_E_NOTFOUND, "get: unknown tensor id %llu", (unsigned long long)tid);
  poll();
  Rec &r = recs[it->second];
  if (r.state == SSDT_ST_RELEASED || r.scopes.empty())
    return fail(SSDT_E_STATE, "get: tensor %llu has been released", (unsigned long long)tid);
  if (r.state == SSDT_ST_STORING) {
    r.state = SSDT_ST_RESIDENT;
    r.forwarded = true;
    ++st.forwarded;
  } else if (r.state == SSDT_ST_OFFLOADED) {  // nobody prefetched it: load on demand
    void *p = nullptr;
    ssdt_stream q = be->queue_stream(1);
    if (alloc(r.bytes, q, &p) != SSDT_OK) return SSDT_E_NOMEM;
    r.dev = p;
    r.holds_ref = true;
    by_storage[p] = it->second;
    ++st.demand_loads;
    ssdt_status e = start_load(it->second, "get");
    if (e != SSDT_OK) return e;
  }
  if (r.read_pending) {  // spill mode: the host waits for the file, then the copy is enqueued
    spill_in_pool((size_t)r.pool_offset, true);
    ssdt_status e = spill_status("get");
    if (e == SSDT_OK) e = issue_copy_in(it->second, "get");
    if (e != SSDT_OK) return e;
  }
  if (r.load_ev) {
    if (!r.load_waited) {
      timed_wait(consumer, r.load_ev, 0);
      r.load_waited = true;
    } else {
      be->wait(consumer, r.load_ev);
    }
    if (r.state == SSDT_ST_LOADING) r.state = SSDT_ST_RESIDENT;
  }
  *out = r.dev;
  return SSDT_OK;
}

ssdt_status Ctx::release(int32_t scope_id, ssdt_stream s) {
  const int64_t scope = key(scope_id);
  poll();
  Ev *ev = nullptr;
  for (auto &r : recs) {
    auto f = std::find(r.scopes.begin(), r.scopes.end(), scope);
    if (f == r.scopes.end()) continue;
    r.scopes.erase(f);
    if (!r.scopes.empty()) continue;
    ++st.released;
    if (r.state == SSDT_ST_STORING && !r.forwarded) {
      r.release_pending = true;  // its memory returns when the store completes
      continue;
    }
    if (r.holds_ref && r.dev) {
      if (r.state == SSDT_ST_LOADING && r.read_pending) {
        r.read_pending = false;  // no copy was enqueued: nothing is in flight to the slot
        unref(r.dev, nullptr, nullptr);
      } else if (r.state == SSDT_ST_LOADING) {
        unref(r.dev, r.load_ev, be->queue_stream(1));
      } else {
        if (!ev) ev = hold(be->record(s, false));
        unref(r.dev, ev, s);
      }
      r.holds_ref = false;
    }
    r.dev = nullptr;
    r.state = SSDT_ST_RELEASED;
  }
  drop(be.get(), ev);
  return SSDT_OK;
}

}  // namespace ssdt

// ---------------------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------------------
using namespace ssdt;

extern "C" {

const char *ssdt_version(void) { return "ssdt 0.1 (gfx950)"; }

const char *ssdt_last_error(const ssdt_ctx *ctx) { return ctx ? ctx->last_error.c_str() : "null context"; }

ssdt_status ssdt_ctx_create(const ssdt_config *cfg, ssdt_ctx **out) {
  if (!cfg || !out) return SSDT_E_INVAL;
  *out = nullptr;
  if (cfg->arena_bytes && (!cfg->arena_base || ((uintptr_t)cfg->arena_base % kAlignTensor) != 0)) return SSDT_E_INVAL;
  if (cfg->keep_last < 0 || cfg->min_offload_elems < 0) return SSDT_E_INVAL;
  std::string err;
  Backend *be = nullptr;
  if (cfg->backend == SSDT_BACKEND_HIP) be = make_hip_backend(cfg->pool_bytes, &err);
  else if (cfg->backend == SSDT_BACKEND_SIM) be = make_sim_backend(cfg->pool_bytes, &err);
  else return SSDT_E_INVAL;
  if (!be) {
    fprintf(stderr, "ssdt_ctx_create: %s\n", err.c_str());
    return cfg->backend == SSDT_BACKEND_HIP ? SSDT_E_HIP : SSDT_E_NOMEM;
  }
  auto *c = new ssdt_ctx();
  c->cfg = *cfg;
  c->cfg.spill_path = nullptr;
  c->be.reset(be);
  if (cfg->arena_bytes) {
    Block b;
    b.size = cfg->arena_bytes / kAlignTensor * kAlignTensor;
    c->blocks[0] = b;
  }
  if (cfg->spill_path && cfg->spill_path[0]) {
    if (c->spill_open(cfg->spill_path) != SSDT_OK) {
      fprintf(stderr, "ssdt_ctx_create: %s\n", c->last_error.c_str());
      delete c;
      return SSDT_E_IO;
    }
  }
  *out = c;
  return SSDT_OK;
}

ssdt_status ssdt_ctx_destroy(ssdt_ctx *ctx) {
  if (!ctx) return SSDT_E_INVAL;
  ctx->be->sync_io();
  ctx->spill_close();
  delete ctx;
  return SSDT_OK;
}

ssdt_status ssdt_step_begin(ssdt_ctx *c, int32_t n) {
  if (!c) return SSDT_E_INVAL;
  ApiLock api_lock_(c);
  return c->step_begin(n);
}

ssdt_status ssdt_micro_batch(ssdt_ctx *c, int32_t mb, int32_t keep_last) {
  if (!c) return SSDT_E_INVAL;
  ApiLock api_lock_(c);
  return c->micro_batch(mb, keep_last);
}

ssdt_status ssdt_set_budget(ssdt_ctx *c, int64_t b) {
  ApiLock api_lock_(c);
  if (!c) return SSDT_E_INVAL;
  c->cfg.budget_bytes = b;
  return SSDT_OK;
}

ssdt_status ssdt_arena_alloc(ssdt_ctx *c, size_t bytes, ssdt_stream s, void **out) {
  ApiLock api_lock_(c);
  return c ? c->alloc(bytes, s, out) : SSDT_E_INVAL;
}

ssdt_status ssdt_arena_free(ssdt_ctx *c, void *p, ssdt_stream s) {
  ApiLock api_lock_(c);
  if (!c) return SSDT_E_INVAL;
  if (!p || !c->in_arena(p)) return c->fail(SSDT_E_INVAL, "arena_free: pointer is not inside the arena");
  auto it = c->blocks.find((char *)p - (char *)c->cfg.arena_base);
  if (it == c->blocks.end() || it->second.free) return c->fail(SSDT_E_STATE, "arena_free: not a live arena block");
  if (it->second.refs > 1) {
    c->unref(p, nullptr, nullptr);  // the registry still refers to it
    return SSDT_OK;
  }
  Ev *ev = c->be->record(s, false);
  ++ev->refs;
  c->unref(p, ev, s);
  if (--ev->refs <= 0) c->be->recycle(ev);
  return SSDT_OK;
}

ssdt_status ssdt_register_weight(ssdt_ctx *c, const void *base, size_t bytes) {
  ApiLock api_lock_(c);
  if (!c) return SSDT_E_INVAL;
  if (!base || !bytes) return c->fail(SSDT_E_INVAL, "register_weight: null or empty buffer");
  c->weights.emplace_back((const char *)base, bytes);
  return SSDT_OK;
}

ssdt_status ssdt_scope_begin(ssdt_ctx *c, int32_t scope, int32_t phase) {
  if (!c) return SSDT_E_INVAL;
  ApiLock api_lock_(c);
  return c->scope_begin(scope, phase);
}
ssdt_status ssdt_scope_end(ssdt_ctx *c, int32_t scope, int32_t phase) {
  if (!c) return SSDT_E_INVAL;
  ApiLock api_lock_(c);
  return c->scope_end(scope, phase);
}

ssdt_status ssdt_save(ssdt_ctx *c, const void *base, size_t sbytes, size_t off, const int64_t *shape, int32_t ndim,
                      int32_t dtype, ssdt_tid *out) {
  ApiLock api_lock_(c);
  return c ? c->save(base, sbytes, off, shape, ndim, dtype, out) : SSDT_E_INVAL;
}

ssdt_status ssdt_offload(ssdt_ctx *c, int32_t scope, ssdt_stream p) {
  if (!c) return SSDT_E_INVAL;
  ApiLock api_lock_(c);
  return c->offload(scope, p);
}
ssdt_status ssdt_prefetch(ssdt_ctx *c, int32_t scope) {
  if (!c) return SSDT_E_INVAL;
  ApiLock api_lock_(c);
  return c->prefetch(scope);
}
ssdt_status ssdt_get(ssdt_ctx *c, ssdt_tid t, ssdt_stream s, void **out) {
  if (!c) return SSDT_E_INVAL;
  ApiLock api_lock_(c);
  return c->get(t, s, out);
}
ssdt_status ssdt_release(ssdt_ctx *c, int32_t scope, ssdt_stream s) {
  if (!c) return SSDT_E_INVAL;
  ApiLock api_lock_(c);
  return c->release(scope, s);
}

ssdt_status ssdt_get_stats(ssdt_ctx *c, ssdt_stats *out) {
  ApiLock api_lock_(c);
  if (!c || !out) return SSDT_E_INVAL;
  // fold in the wait measurements whose closing event has completed
  for (size_t i = 0; i < c->waits.size();) {
    WaitPair w = c->waits[i];
    if (c->be->done(w.b)) {
      if (w.step == c->step_no) {  // the counters are per step, like every other one
        double ms = c->be->elapsed_ms(w.a, w.b);
        uint64_t ns = ms > 0 ? (uint64_t)(ms * 1e6) : 0;
        (w.kind == 0 ? c->st.exposed_load_wait_ns : c->st.exposed_store_wait_ns) += ns;
      }
      if (--w.a->refs <= 0) c->be->recycle(w.a);
      if (--w.b->refs <= 0) c->be->recycle(w.b);
      c->waits[i] = c->waits.back();
      c->waits.pop_back();
    } else {
      ++i;
    }
  }
  c->st.arena_in_use = c->in_use;
  c->st.arena_high_water = c->high_water;
  c->st.arena_peak_in_use = c->peak_in_use;
  c->st.arena_allocs = c->n_allocs;
  *out = c->st;
  return SSDT_OK;
}

ssdt_status ssdt_num_records(const ssdt_ctx *c, uint32_t *out) {
  ApiLock api_lock_(c);
  if (!c || !out) return SSDT_E_INVAL;
  *out = (uint32_t)c->recs.size();
  return SSDT_OK;
}

ssdt_status ssdt_get_record(const ssdt_ctx *c, uint32_t i, ssdt_record *out) {
  ApiLock api_lock_(c);
  if (!c || !out) return SSDT_E_INVAL;
  if (i >= c->recs.size()) return SSDT_E_NOTFOUND;
  const Rec &r = c->recs[i];
  out->tid = r.tid;
  out->layer = Ctx::scope_of(r.layer);
  out->micro_batch = Ctx::mb_of(r.layer);
  out->reserved = 0;
  out->cls = r.cls;
  out->state = r.state;
  out->n_scopes = (int32_t)r.scopes.size();
  out->bytes = r.bytes;
  out->pack_offset = r.pack_offset;
  out->pool_offset = r.pool_offset;
  out->device_ptr = r.dev;
  return SSDT_OK;
}

ssdt_status ssdt_pool_read(ssdt_ctx *c, size_t off, void *dst, size_t bytes) {
  ApiLock api_lock_(c);
  if (!c || !dst) return SSDT_E_INVAL;
  if (off + bytes > c->cfg.pool_bytes) return c->fail(SSDT_E_INVAL, "pool_read: range outside the pool");
  c->be->sync_io();
  if (c->spill) {  // the file is the store: finish the pending writes and read it
    c->poll();
    c->spill_drain();
    if (ssdt_status e = c->spill_status("pool_read")) return e;
    // the file may be open for direct I/O: read whole 4 KiB blocks into an aligned buffer
    const size_t lo = off / kAlignSpill * kAlignSpill, hi = up(off + bytes, kAlignSpill);
    void *tmp = nullptr;
    if (posix_memalign(&tmp, kAlignSpill, hi - lo) != 0) return c->fail(SSDT_E_NOMEM, "pool_read: no memory");
    std::string err;
    const bool ok = rw_all(c->spill->fd, (char *)tmp, hi - lo, lo, false, &err);
    if (ok) memcpy(dst, (char *)tmp + (off - lo), bytes);
    free(tmp);
    if (!ok) return c->fail(SSDT_E_IO, "pool_read: %s", err.c_str());
    return SSDT_OK;
  }
  memcpy(dst, (char *)c->be->pool() + off, bytes);
  return SSDT_OK;
}

ssdt_status ssdt_sim_complete(ssdt_ctx *c, int32_t dir, int32_t n, int32_t *done) {
  ApiLock api_lock_(c);
  if (!c) return SSDT_E_INVAL;
  int k = c->be->sim_complete(dir, n);
  if (k < 0) return c->fail(SSDT_E_UNSUPPORTED, "sim_complete: not the simulated backend");
  if (done) *done = k;
  return SSDT_OK;
}

ssdt_status ssdt_profile(ssdt_ctx *c, int32_t enable) {
  ApiLock api_lock_(c);
  if (!c) return SSDT_E_INVAL;
  if (c->be->is_sim()) return c->fail(SSDT_E_UNSUPPORTED, "profile: the simulated backend launches no kernels");
  if (enable) prof::reset();
  prof::set(enable != 0);
  return SSDT_OK;
}

ssdt_status ssdt_profile_read(ssdt_ctx *c, ssdt_kernel_time *out, uint32_t cap, uint32_t *n) {
  ApiLock api_lock_(c);
  if (!c || !out || !n) return SSDT_E_INVAL;
  if (c->be->is_sim()) return c->fail(SSDT_E_UNSUPPORTED, "profile: the simulated backend launches no kernels");
  prof::collect();
  uint32_t k = 0;
  for (int cat = 0; cat < prof::NCAT && k < cap; ++cat) {
    unsigned long long l;
    double ms, fl, by;
    prof::totals(cat, &l, &ms, &fl, &by);
    if (!l) continue;
    snprintf(out[k].name, sizeof out[k].name, "%s", prof::name(cat));
    out[k].launches = l; out[k].ms = ms; out[k].flops = fl; out[k].bytes = by;
    ++k;
  }
  *n = k;
  return SSDT_OK;
}

ssdt_status ssdt_sync_io(ssdt_ctx *c) {
  ApiLock api_lock_(c);
  if (!c) return SSDT_E_INVAL;
  c->be->sync_io();
  c->poll();
  if (c->spill) {
    c->spill_drain();
    c->poll();
    return c->spill_status("sync_io");
  }
  return SSDT_OK;
}

ssdt_status ssdt_spill_info(ssdt_ctx *c, ssdt_spill_info_t *out) {
  ApiLock api_lock_(c);
  if (!c || !out) return SSDT_E_INVAL;
  if (!c->spill) return c->fail(SSDT_E_STATE, "spill_info: the context has no spill file");
  std::lock_guard<std::mutex> g(c->spill->mu);
  out->direct_io = c->spill->direct ? 1 : 0;
  out->threads = (int32_t)c->spill->workers.size();
  out->bytes_written = c->spill->bytes_written;
  out->bytes_read = c->spill->bytes_read;
  out->write_busy_ns = c->spill->write_ns;
  out->read_busy_ns = c->spill->read_ns;
  return SSDT_OK;
}

ssdt_status ssdt_spill_stats(ssdt_ctx *c, uint64_t *bytes_written, uint64_t *bytes_read) {
  ApiLock api_lock_(c);
  if (!c) return SSDT_E_INVAL;
  if (!c->spill) return c->fail(SSDT_E_STATE, "spill_stats: the context has no spill file");
  std::lock_guard<std::mutex> g(c->spill->mu);
  if (bytes_written) *bytes_written = c->spill->bytes_written;
  if (bytes_read) *bytes_read = c->spill->bytes_read;
  return SSDT_OK;
}

}  // extern "C"
