// The third tier (Cross-tier Synergistic Storage): the backing file on SSD holds every page,
// host DRAM holds a bounded pool of whole extents, the GPU window sits in front of both.
//
// This file is host code only.  The file layout follows SSD-Aware Layout Planning (one segment
// per {layer, head} unit, cut into extents; inside a segment the pages of one cluster are
// neighbours); a step follows Parallel Sparse Synchronization (b) and (c): only the extents that
// hold a missed page are read, neighbouring extents as one read, several reads in flight, and
// they land directly in the pool — a fixed set of pinned buffers — so no staging copy in host
// memory is needed before the GPU takes the pages.
#include <errno.h>
#include <fcntl.h>
#include <stdlib.h>
#include <string.h>
#include <sys/stat.h>
#include <sys/types.h>
#include <sys/uio.h>
#include <unistd.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <mutex>
#include <thread>
#include <vector>

#include "kvd_internal.h"

namespace {

constexpr int kMaxQueueDepth = 64;
constexpr int kMaxRun = 64;

struct ReadOp {
  int64_t first;      // first extent in the file
  int32_t count;      // extents
  int32_t slot0;      // index into the slot list of the job
};

double now_ms() {
  using namespace std::chrono;
  return duration<double, std::milli>(steady_clock::now().time_since_epoch()).count();
}

}  // namespace

struct kvd_tier {
  kvd_tier_config cfg;
  int fd = -1;        // reads (O_DIRECT when taken)
  int wfd = -1;       // buffered writes of the set-up helper
  std::atomic<int> direct{0};   // 0 buffered reads; 1 O_DIRECT straight into the pool; 2 O_DIRECT into per-reader staging buffers
  std::vector<char*> staging;   // [readers] max_run_extents extents each, 4096-byte aligned (direct == 2)
  int last_errno = 0;
  int NE = 0;
  size_t extent_bytes = 0;
  int64_t total_extents = 0;
  char* pool = nullptr;

  std::vector<int32_t> position;    // [layers][U][NP]
  std::vector<int32_t> ext_slot;    // [total_extents] pool slot or -1
  std::vector<int64_t> slot_ext;    // [pool_extents] extent or -1
  std::vector<int32_t> slot_stamp;  // [pool_extents]
  std::vector<int32_t> free_slots;
  std::vector<uint32_t> mark;       // [total_extents] == epoch: needed by the running step
  uint32_t epoch = 0;
  int64_t n_pooled = 0;

  // the last step
  int64_t tr_counts[5] = {0, 0, 0, 0, 0};
  std::vector<int64_t> tr_runs, tr_evicted;

  // scratch of a step
  std::vector<int64_t> needed, reads;
  std::vector<std::pair<int32_t, int64_t>> cands;
  std::vector<ReadOp> ops;
  std::vector<int32_t> op_slots;    // pool slot of every extent of every op

  // readers
  std::vector<std::thread> workers;
  std::mutex mu;
  std::condition_variable cv_go, cv_done;
  uint64_t job_no = 0;
  int running = 0;
  bool quit = false;
  bool sequential = false;          // the job reads into per-reader scratch areas of the pool
  std::atomic<size_t> next_op{0};
  std::atomic<int> io_error{0};

  kvd_tier_stats stats = {};
};

namespace {

// Reads `count` extents starting at extent `first` into the given pool slots, as reader `me`;
// false on failure.
bool read_extents(kvd_tier* t, int me, int64_t first, int count, const int32_t* slots) {
  const off_t off = (off_t)first * (off_t)t->extent_bytes;
  const size_t want = (size_t)count * t->extent_bytes;
  if (t->direct.load(std::memory_order_relaxed) != 2) {
    struct iovec iov[kMaxRun];
    for (int i = 0; i < count; ++i) {
      iov[i].iov_base = t->pool + (size_t)slots[i] * t->extent_bytes;
      iov[i].iov_len = t->extent_bytes;
    }
    ssize_t got = preadv(t->fd, iov, count, off);
    if (got == (ssize_t)want) return true;
    if (got < 0 && errno == EFAULT && t->direct.load() != 0) {
      // The file system cannot pin the pool's memory for a direct transfer (memory page-locked by
      // a GPU driver may be mapped in a way that direct I/O does not take): from now on every
      // reader goes through its own aligned staging buffer.
      t->direct.store(2);
    } else {
      // short or failed: finish extent by extent
      for (int i = 0; i < count; ++i) {
        size_t done = 0;
        while (done < t->extent_bytes) {
          got = pread(t->fd, (char*)iov[i].iov_base + done, t->extent_bytes - done, off + (off_t)i * t->extent_bytes + done);
          if (got < 0 && errno == EINTR) continue;
          if (got <= 0) { t->io_error.store(got < 0 ? errno : EIO); return false; }
          done += (size_t)got;
        }
      }
      return true;
    }
  }
  char* buf = t->staging[me];
  size_t done = 0;
  while (done < want) {
    const ssize_t got = pread(t->fd, buf + done, want - done, off + (off_t)done);
    if (got < 0 && errno == EINTR) continue;
    if (got <= 0 || got % 4096 != 0) { t->io_error.store(got < 0 ? errno : EIO); return false; }
    done += (size_t)got;
  }
  for (int i = 0; i < count; ++i)
    memcpy(t->pool + (size_t)slots[i] * t->extent_bytes, buf + (size_t)i * t->extent_bytes, t->extent_bytes);
  return true;
}

void reader_main(kvd_tier* t, int me) {
  uint64_t seen = 0;
  for (;;) {
    {
      std::unique_lock<std::mutex> lk(t->mu);
      t->cv_go.wait(lk, [&] { return t->quit || t->job_no != seen; });
      if (t->quit) return;
      seen = t->job_no;
    }
    for (;;) {
      const size_t i = t->next_op.fetch_add(1);
      if (i >= t->ops.size()) break;
      const ReadOp& op = t->ops[i];
      if (t->sequential) {
        int32_t slots[kMaxRun];
        for (int j = 0; j < op.count; ++j) slots[j] = me * t->cfg.max_run_extents + j;
        read_extents(t, me, op.first, op.count, slots);
      } else {
        read_extents(t, me, op.first, op.count, t->op_slots.data() + op.slot0);
      }
    }
    {
      std::lock_guard<std::mutex> lk(t->mu);
      if (--t->running == 0) t->cv_done.notify_one();
    }
  }
}

// Runs t->ops on the readers and waits for them; returns the wall time in ms.
double run_reads(kvd_tier* t, bool sequential) {
  if (t->ops.empty()) return 0.0;
  const double t0 = now_ms();
  {
    std::lock_guard<std::mutex> lk(t->mu);
    t->sequential = sequential;
    t->next_op.store(0);
    t->io_error.store(0);
    t->running = (int)t->workers.size();
    ++t->job_no;
  }
  t->cv_go.notify_all();
  {
    std::unique_lock<std::mutex> lk(t->mu);
    t->cv_done.wait(lk, [&] { return t->running == 0; });
  }
  return now_ms() - t0;
}

void drop_pool(kvd_tier* t) {
  std::fill(t->ext_slot.begin(), t->ext_slot.end(), -1);
  std::fill(t->slot_ext.begin(), t->slot_ext.end(), (int64_t)-1);
  t->free_slots.clear();
  for (int64_t s = t->cfg.pool_extents - 1; s >= 0; --s) t->free_slots.push_back((int32_t)s);
  t->n_pooled = 0;
}

void release_extent(kvd_tier* t, int64_t x) {
  const int32_t s = t->ext_slot[x];
  if (s < 0) return;
  t->ext_slot[x] = -1;
  t->slot_ext[s] = -1;
  t->free_slots.push_back(s);
  --t->n_pooled;
}

}  // namespace

const kvd_tier_config* kvd_tier_config_of(const kvd_tier* t) { return &t->cfg; }
void* kvd_tier_pool_of(const kvd_tier* t) { return t->pool; }

extern "C" {

int kvd_tier_open(const kvd_tier_config* cfg, const char* path, void* pool_host, kvd_tier** out) {
  if (!cfg || !path || !pool_host || !out) return KVD_ERR_ARG;
  *out = nullptr;
  if (((uintptr_t)pool_host & 4095u) != 0) return KVD_ERR_ARG;
  if (cfg->n_layers < 1 || cfg->n_units < 1 || cfg->max_pages < 1 || cfg->extent_pages < 1 || cfg->page_bytes < 16 ||
      cfg->page_bytes % 16 != 0 || cfg->pool_extents < 1 || cfg->pool_extents > 0x7fffffff || cfg->queue_depth < 1 ||
      cfg->queue_depth > kMaxQueueDepth || cfg->max_run_extents < 1 || cfg->max_run_extents > kMaxRun)
    return KVD_ERR_SHAPE;
  kvd_tier* t = new kvd_tier();
  t->cfg = *cfg;
  t->NE = (cfg->max_pages + cfg->extent_pages - 1) / cfg->extent_pages;
  t->extent_bytes = (size_t)cfg->extent_pages * (size_t)cfg->page_bytes;
  t->total_extents = (int64_t)cfg->n_layers * cfg->n_units * t->NE;
  t->pool = static_cast<char*>(pool_host);
  const off_t file_bytes = (off_t)t->total_extents * (off_t)t->extent_bytes;
  t->wfd = open(path, O_RDWR | O_CREAT, 0644);
  if (t->wfd < 0) { t->last_errno = errno; delete t; return KVD_ERR_STATE; }
  struct stat st;
  if (fstat(t->wfd, &st) != 0 || (st.st_size < file_bytes && ftruncate(t->wfd, file_bytes) != 0)) {
    t->last_errno = errno; close(t->wfd); delete t; return KVD_ERR_STATE;
  }
  if (cfg->direct_io && t->extent_bytes % 4096 == 0) {
    // Direct I/O needs a file system that takes O_DIRECT.  Every reader also gets an ordinary
    // aligned staging buffer, for the case that the pool's memory turns out not to be usable for
    // direct transfers (see read_extents).
    t->fd = open(path, O_RDONLY | O_DIRECT);
    if (t->fd >= 0) {
      t->direct.store(1);
      for (int i = 0; i < cfg->queue_depth; ++i) {
        void* b = nullptr;
        if (posix_memalign(&b, 4096, (size_t)cfg->max_run_extents * t->extent_bytes) != 0) { t->direct.store(0); break; }
        t->staging.push_back(static_cast<char*>(b));
      }
      if (t->direct.load() == 0) {
        for (char* b : t->staging) free(b);
        t->staging.clear();
        close(t->fd);
        t->fd = -1;
      }
    }
  }
  if (t->fd < 0) t->fd = open(path, O_RDONLY);
  if (t->fd < 0) { t->last_errno = errno; close(t->wfd); delete t; return KVD_ERR_STATE; }
  const size_t un = (size_t)cfg->n_layers * cfg->n_units * cfg->max_pages;
  t->position.resize(un);
  for (size_t i = 0; i < un; ++i) t->position[i] = (int32_t)(i % (size_t)cfg->max_pages);
  t->ext_slot.assign((size_t)t->total_extents, -1);
  t->mark.assign((size_t)t->total_extents, 0u);
  t->slot_ext.assign((size_t)cfg->pool_extents, (int64_t)-1);
  t->slot_stamp.assign((size_t)cfg->pool_extents, 0);
  drop_pool(t);
  for (int i = 0; i < cfg->queue_depth; ++i) t->workers.emplace_back(reader_main, t, i);
  *out = t;
  return KVD_OK;
}

int kvd_tier_close(kvd_tier* t) {
  if (!t) return KVD_ERR_ARG;
  {
    std::lock_guard<std::mutex> lk(t->mu);
    t->quit = true;
  }
  t->cv_go.notify_all();
  for (auto& w : t->workers) w.join();
  if (t->fd >= 0) close(t->fd);
  if (t->wfd >= 0) close(t->wfd);
  for (char* b : t->staging) free(b);
  delete t;
  return KVD_OK;
}

int kvd_tier_last_errno(const kvd_tier* t) { return t ? t->last_errno : 0; }

int kvd_tier_set_layout(kvd_tier* t, int32_t layer, const int32_t* host_position) {
  if (!t || !host_position || layer < 0 || layer >= t->cfg.n_layers) return KVD_ERR_ARG;
  const int U = t->cfg.n_units, NP = t->cfg.max_pages;
  std::vector<uint8_t> seen((size_t)NP);
  for (int u = 0; u < U; ++u) {
    std::fill(seen.begin(), seen.end(), 0);
    for (int p = 0; p < NP; ++p) {
      const int32_t x = host_position[(size_t)u * NP + p];
      if (x < 0 || x >= NP || seen[x]) return KVD_ERR_ARG;
      seen[x] = 1;
    }
  }
  std::copy(host_position, host_position + (size_t)U * NP, t->position.begin() + (size_t)layer * U * NP);
  return KVD_OK;
}

int kvd_tier_write_layer(kvd_tier* t, int32_t layer, const void* host_pages) {
  if (!t || !host_pages || layer < 0 || layer >= t->cfg.n_layers) return KVD_ERR_ARG;
  const int U = t->cfg.n_units, NP = t->cfg.max_pages;
  const size_t pb = (size_t)t->cfg.page_bytes, seg = (size_t)t->NE * t->extent_bytes;
  std::vector<char> segment(seg);
  const char* src = static_cast<const char*>(host_pages);
  for (int u = 0; u < U; ++u) {
    std::fill(segment.begin(), segment.end(), 0);
    const int32_t* pos = t->position.data() + ((size_t)layer * U + u) * NP;
    for (int p = 0; p < NP; ++p) memcpy(segment.data() + (size_t)pos[p] * pb, src + ((size_t)u * NP + p) * pb, pb);
    const off_t off = (off_t)((size_t)layer * U + u) * (off_t)seg;
    size_t done = 0;
    while (done < seg) {
      const ssize_t w = pwrite(t->wfd, segment.data() + done, seg - done, off + (off_t)done);
      if (w < 0 && errno == EINTR) continue;
      if (w <= 0) { t->last_errno = w < 0 ? errno : EIO; return KVD_ERR_STATE; }
      done += (size_t)w;
    }
    for (int e = 0; e < t->NE; ++e) release_extent(t, ((int64_t)layer * U + u) * t->NE + e);
  }
  if (fsync(t->wfd) != 0) { t->last_errno = errno; return KVD_ERR_STATE; }
  return KVD_OK;
}

int kvd_tier_patch_page(kvd_tier* t, int32_t layer, int32_t unit, int32_t page, int64_t offset_in_page,
                        const void* host_src, int64_t nbytes) {
  if (!t || !host_src || layer < 0 || layer >= t->cfg.n_layers || unit < 0 || unit >= t->cfg.n_units || page < 0 ||
      page >= t->cfg.max_pages || offset_in_page < 0 || nbytes < 0 || offset_in_page + nbytes > t->cfg.page_bytes)
    return KVD_ERR_ARG;
  const int U = t->cfg.n_units, NP = t->cfg.max_pages, E = t->cfg.extent_pages;
  const int32_t place = t->position[((size_t)layer * U + unit) * NP + page];
  const int64_t x = ((int64_t)layer * U + unit) * t->NE + place / E;
  const int64_t in_extent = (int64_t)(place % E) * t->cfg.page_bytes + offset_in_page;
  const char* src = static_cast<const char*>(host_src);
  int64_t done = 0;
  while (done < nbytes) {
    const ssize_t w = pwrite(t->wfd, src + done, (size_t)(nbytes - done), (off_t)(x * (int64_t)t->extent_bytes + in_extent + done));
    if (w < 0 && errno == EINTR) continue;
    if (w <= 0) { t->last_errno = w < 0 ? errno : EIO; return KVD_ERR_STATE; }
    done += w;
  }
  const int32_t slot = t->ext_slot[x];
  if (slot >= 0) memcpy(t->pool + (size_t)slot * t->extent_bytes + in_extent, src, (size_t)nbytes);
  return KVD_OK;
}

int kvd_tier_fetch(kvd_tier* t, int32_t layer, int32_t step, const int32_t* miss_list, const int32_t* miss_count,
                   int32_t k, int64_t* src_offset) {
  if (!t || !miss_list || !miss_count || !src_offset || layer < 0 || layer >= t->cfg.n_layers || k < 1) return KVD_ERR_ARG;
  const double t_begin = now_ms();
  const int U = t->cfg.n_units, NP = t->cfg.max_pages, E = t->cfg.extent_pages, NE = t->NE;
  const int32_t* pos_l = t->position.data() + (size_t)layer * U * NP;
  // 1. the extents that hold a missed page
  if (++t->epoch == 0) { std::fill(t->mark.begin(), t->mark.end(), 0u); t->epoch = 1; }
  t->needed.clear();
  uint64_t n_pages = 0;
  for (int u = 0; u < U; ++u) {
    const int m = miss_count[u];
    if (m < 0 || m > k) return KVD_ERR_ARG;
    for (int j = 0; j < m; ++j) {
      const int32_t page = miss_list[((size_t)u * k + j) * 2];
      if (miss_list[((size_t)u * k + j) * 2 + 1] < 0) continue;
      if (page < 0 || page >= NP) return KVD_ERR_ARG;
      const int64_t x = ((int64_t)layer * U + u) * NE + pos_l[(size_t)u * NP + page] / E;
      ++n_pages;
      if (t->mark[x] != t->epoch) { t->mark[x] = t->epoch; t->needed.push_back(x); }
    }
  }
  std::sort(t->needed.begin(), t->needed.end());
  if ((int64_t)t->needed.size() > t->cfg.pool_extents) return KVD_ERR_CAPACITY;
  // 2. pooled extents are hits; the others are read
  t->reads.clear();
  int64_t n_hits = 0;
  for (int64_t x : t->needed) {
    const int32_t s = t->ext_slot[x];
    if (s >= 0) { t->slot_stamp[s] = step; ++n_hits; } else t->reads.push_back(x);
  }
  // 3. make room: pooled extents that this step does not need leave in (stamp, extent) order
  t->tr_evicted.clear();
  const int64_t n_evict = t->n_pooled + (int64_t)t->reads.size() - t->cfg.pool_extents;
  if (n_evict > 0) {
    t->cands.clear();
    for (int64_t s = 0; s < t->cfg.pool_extents; ++s) {
      const int64_t x = t->slot_ext[s];
      if (x >= 0 && t->mark[x] != t->epoch) t->cands.emplace_back(t->slot_stamp[s], x);
    }
    std::nth_element(t->cands.begin(), t->cands.begin() + (n_evict - 1), t->cands.end());
    for (int64_t i = 0; i < n_evict; ++i) t->tr_evicted.push_back(t->cands[i].second);
    std::sort(t->tr_evicted.begin(), t->tr_evicted.end());
    for (int64_t x : t->tr_evicted) release_extent(t, x);
  }
  // 4. slots for the new extents; neighbours in the file, inside one segment, are one read
  t->ops.clear();
  t->op_slots.clear();
  t->tr_runs.clear();
  for (int64_t x : t->reads) {
    const int32_t s = t->free_slots.back();
    t->free_slots.pop_back();
    t->ext_slot[x] = s;
    t->slot_ext[s] = x;
    t->slot_stamp[s] = step;
    ++t->n_pooled;
    if (!t->ops.empty()) {
      ReadOp& last = t->ops.back();
      if (x == last.first + last.count && x / NE == last.first / NE && last.count < t->cfg.max_run_extents) {
        ++last.count;
        t->op_slots.push_back(s);
        continue;
      }
    }
    t->ops.push_back(ReadOp{x, 1, (int32_t)t->op_slots.size()});
    t->op_slots.push_back(s);
  }
  for (const ReadOp& op : t->ops) { t->tr_runs.push_back(op.first); t->tr_runs.push_back(op.count); }
  t->tr_counts[0] = (int64_t)t->needed.size();
  t->tr_counts[1] = n_hits;
  t->tr_counts[2] = (int64_t)t->reads.size();
  t->tr_counts[3] = (int64_t)t->tr_evicted.size();
  t->tr_counts[4] = (int64_t)t->ops.size();
  const double t_planned = now_ms();
  // 5. the reads
  const double io_ms = run_reads(t, false);
  const int err = t->io_error.load();
  const double t_read = now_ms();
  t->stats.steps += 1;
  t->stats.pages_requested += n_pages;
  t->stats.extents_needed += t->needed.size();
  t->stats.extent_hits += (uint64_t)n_hits;
  t->stats.extent_reads += t->reads.size();
  t->stats.extent_evictions += t->tr_evicted.size();
  t->stats.reads_issued += t->ops.size();
  t->stats.bytes_read += (uint64_t)t->reads.size() * t->extent_bytes;
  t->stats.ms_io += io_ms;
  if (err != 0) {
    // what was to be read is not trusted: forget it
    for (int64_t x : t->reads) release_extent(t, x);
    t->last_errno = err;
    return KVD_ERR_STATE;
  }
  // 6. where the GPU finds every missed page
  const size_t pb = (size_t)t->cfg.page_bytes;
  for (int u = 0; u < U; ++u) {
    const int m = miss_count[u];
    for (int j = 0; j < m; ++j) {
      const int32_t page = miss_list[((size_t)u * k + j) * 2];
      if (miss_list[((size_t)u * k + j) * 2 + 1] < 0) { src_offset[(size_t)u * k + j] = -1; continue; }
      const int32_t place = pos_l[(size_t)u * NP + page];
      const int64_t x = ((int64_t)layer * U + u) * NE + place / E;
      src_offset[(size_t)u * k + j] = (int64_t)t->ext_slot[x] * (int64_t)t->extent_bytes + (int64_t)(place % E) * (int64_t)pb;
    }
  }
  t->stats.ms_plan += (t_planned - t_begin) + (now_ms() - t_read);
  return KVD_OK;
}

int kvd_tier_trace(const kvd_tier* t, int64_t* counts, int64_t* runs, int64_t cap_runs, int64_t* evicted,
                   int64_t cap_evicted) {
  if (!t || !counts) return KVD_ERR_ARG;
  for (int i = 0; i < 5; ++i) counts[i] = t->tr_counts[i];
  if (runs) {
    const int64_t n = std::min<int64_t>(cap_runs, (int64_t)t->tr_runs.size() / 2);
    std::copy(t->tr_runs.begin(), t->tr_runs.begin() + 2 * n, runs);
  }
  if (evicted) {
    const int64_t n = std::min<int64_t>(cap_evicted, (int64_t)t->tr_evicted.size());
    std::copy(t->tr_evicted.begin(), t->tr_evicted.begin() + n, evicted);
  }
  return KVD_OK;
}

int kvd_tier_pooled(const kvd_tier* t, int64_t* extents, int64_t cap, int64_t* n_pooled) {
  if (!t || !n_pooled) return KVD_ERR_ARG;
  *n_pooled = t->n_pooled;
  if (extents) {
    int64_t n = 0;
    for (int64_t x = 0; x < t->total_extents && n < cap; ++x)
      if (t->ext_slot[x] >= 0) extents[n++] = x;
  }
  return KVD_OK;
}

int kvd_tier_drop_pool(kvd_tier* t) {
  if (!t) return KVD_ERR_ARG;
  drop_pool(t);
  return KVD_OK;
}

int kvd_tier_get_stats(const kvd_tier* t, kvd_tier_stats* out) {
  if (!t || !out) return KVD_ERR_ARG;
  *out = t->stats;
  out->direct_io = t->direct.load();
  return KVD_OK;
}

int kvd_tier_reset_stats(kvd_tier* t) {
  if (!t) return KVD_ERR_ARG;
  t->stats = kvd_tier_stats{};
  return KVD_OK;
}

int kvd_tier_sequential_read_gbps(kvd_tier* t, double* gbps) {
  if (!t || !gbps) return KVD_ERR_ARG;
  const int R = t->cfg.max_run_extents;
  if ((int64_t)t->cfg.queue_depth * R > t->cfg.pool_extents) return KVD_ERR_CAPACITY;
  drop_pool(t);
  t->ops.clear();
  for (int64_t x = 0; x < t->total_extents; x += R)
    t->ops.push_back(ReadOp{x, (int32_t)std::min<int64_t>(R, t->total_extents - x), 0});
  const double ms = run_reads(t, true);
  t->ops.clear();
  if (t->io_error.load() != 0) { t->last_errno = t->io_error.load(); return KVD_ERR_STATE; }
  *gbps = ms > 0.0 ? (double)t->total_extents * (double)t->extent_bytes / (ms * 1e6) : 0.0;
  return KVD_OK;
}

}  // extern "C"
