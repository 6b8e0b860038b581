// Host-side types shared by the translation units that implement the C ABI: the graph object,
// the scratch of a BatchInsert call, and the functions that run one batch or one query launch.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <ctime>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "../../include/ann.h"
#include "ann_internal.hpp"

namespace annmi {

// records the message ann_last_error returns on this thread; returns `code`
int fail(int code, const char* fmt, ...);

#define HIP_TRY(expr)                                                                          \
  do {                                                                                         \
    hipError_t e_ = (expr);                                                                    \
    if (e_ != hipSuccess)                                                                      \
      return ::annmi::fail(e_ == hipErrorOutOfMemory ? ANN_ENOMEM : ANN_EHIP, "%s: %s", #expr, \
                           hipGetErrorString(e_));                                             \
  } while (0)

// Where device memory comes from: the caller's callbacks (ann_build_opts / ann_hnsw_opts), or
// hipMalloc / hipFree.  A call sets the allocator of its thread for its duration (AllocScope);
// every buffer remembers the allocator it came from and goes back to it.
struct Allocator {
  ann_alloc_fn alloc = nullptr;
  ann_free_fn free = nullptr;
  void* user = nullptr;
  void* stream = nullptr;  // handed to `alloc`: the stream the memory is first used on
  hipError_t get(void** p, size_t bytes) const {
    if (bytes == 0) bytes = 16;
    if (alloc == nullptr) return hipMalloc(p, bytes);
    *p = alloc(bytes, stream, user);
    return *p != nullptr ? hipSuccess : hipErrorOutOfMemory;
  }
  void put(void* p) const {
    if (p == nullptr) return;
    if (free != nullptr)
      free(p, user);
    else
      (void)hipFree(p);
  }
};
Allocator& current_allocator();  // of this thread
struct AllocScope {
  Allocator saved;
  explicit AllocScope(const Allocator& a) : saved(current_allocator()) { current_allocator() = a; }
  AllocScope(const AllocScope&) = delete;
  AllocScope& operator=(const AllocScope&) = delete;
  ~AllocScope() { current_allocator() = saved; }
};
// the allocator named by a pair of callbacks (both or neither); false if only one is given
bool allocator_from(ann_alloc_fn a, ann_free_fn f, void* user, void* stream, Allocator* out);

// what a C entry point returns for an exception that reached it (none may cross the boundary)
int on_exception();

// device buffer freed on scope exit
struct DevBuf {
  void* p = nullptr;
  Allocator al;
  DevBuf() = default;
  DevBuf(const DevBuf&) = delete;
  DevBuf& operator=(const DevBuf&) = delete;
  DevBuf(DevBuf&& o) noexcept : p(o.p), al(o.al) { o.p = nullptr; }
  DevBuf& operator=(DevBuf&& o) noexcept {
    if (this != &o) {
      release();
      p = o.p;
      al = o.al;
      o.p = nullptr;
    }
    return *this;
  }
  ~DevBuf() { release(); }
  void release() {
    al.put(p);
    p = nullptr;
  }
  hipError_t alloc(size_t bytes) {
    release();
    al = current_allocator();
    return al.get(&p, bytes);
  }
  template <typename T>
  T* as() const {
    return static_cast<T*>(p);
  }
};

// Page-locked host memory: small copies to and from it are queued without a staging copy, and the
// device reads it when the copy runs, so its contents must stay until then.
struct HostBuf {
  void* p = nullptr;
  HostBuf() = default;
  HostBuf(const HostBuf&) = delete;
  HostBuf& operator=(const HostBuf&) = delete;
  ~HostBuf() {
    if (p) (void)hipHostFree(p);
  }
  hipError_t alloc(size_t bytes) { return hipHostMalloc(&p, bytes, hipHostMallocDefault); }
  template <class T>
  T* as() const {
    return static_cast<T*>(p);
  }
};

u64 default_spill_keys(u64 batch);
u64 splitmix64(u64& state);
// Fisher-Yates from the front, SplitMix64(seed); *ready follows the number of final positions
void shuffle_in_place(u32* order, u64 m, u64 seed, std::atomic<u64>* ready = nullptr);

struct BatchScratch;

}  // namespace annmi

struct ann_graph {
  annmi::u64 n = 0;
  annmi::u64 cap = 0;  // rows and meta are allocated for this many points (>= n)
  annmi::u32 d = 0, R = 0;
  int dtype = 0, metric = 0;
  annmi::u32 start = 0;
  annmi::u64 rounds = 0;
  annmi::DistCfg cfg{};
  annmi::Allocator al;                   // where rows, meta, counters and the padded copies come from
  annmi::u32* rows = nullptr;            // device, n x R
  annmi::u32* meta = nullptr;            // device, n: degree | clean prefix length << 16
  float clean_alpha = 0.0f;       // the alpha the clean prefixes were pruned with
  annmi::DevCounters* counters = nullptr;  // device
  ann_stats stats{};
  annmi::u32 hash_bits = 0;
  annmi::u32 visited_cap = 0;
  annmi::u64 spill_keys = 0;  // 0 = default
  bool collect = false;
  annmi::u32 step1_parts = 0;  // 1: step 1 of a batch is never split into parts
  // u8/i8 rows whose size is not a multiple of 16 bytes: the kernels work on a copy with rows of
  // pad_stride bytes (zero tail, which changes no distance), made once per points array; queries
  // are copied the same way on every call.  cfg describes the padded rows.
  annmi::u64 pad_stride = 0;
  mutable void* pad_buf = nullptr;
  mutable const void* pad_src = nullptr;
  mutable annmi::u64 pad_cap = 0;   // rows pad_buf has room for
  mutable annmi::u64 pad_done = 0;  // leading rows of pad_src that pad_buf holds
  mutable void* qpad_buf = nullptr;
  mutable annmi::u64 qpad_rows = 0;
  // scratch of the insertions that follow the build (ann_insert_batch, ann_insert_points), kept
  // between calls: allocating and freeing it costs more than a batch of ten thousand points
  annmi::BatchScratch* scratch = nullptr;
};


namespace annmi {

// Scratch of one BatchInsert call, sized for `bmax` points.
struct BatchScratch {
  u64 bmax = 0;
  u32 vis_cap = 0;
  DevBuf qidx, vis, nvis, edges, edges_tmp, hist, lists, small, ovf_list, arena, spill, vis_where;
  u64 spill_cap = 0;    // keys
  u32 spill_chunk = 0;  // extra keys a spilled list gets on top of vis_cap
  u64 arena_cap = 0;
  // side streams (default priority): two of the three parts of a large batch's step 1 and three
  // of the four re-prune kernels of step 2 run on them; the events order them against the
  // caller's stream
  hipStream_t side[3] = {nullptr, nullptr, nullptr};
  hipEvent_t ev_plan = nullptr, ev_side[3] = {nullptr, nullptr, nullptr};
  u32* host_flag = nullptr;  // pinned: where the host reads the overflow count of a batch
  ~BatchScratch() {
    if (host_flag) (void)hipHostFree(host_flag);
    for (auto& s : side)
      if (s) (void)hipStreamDestroy(s);
    if (ev_plan) (void)hipEventDestroy(ev_plan);
    for (auto& e : ev_side)
      if (e) (void)hipEventDestroy(e);
  }
  // small: [0] overflow_count u32, [2] arena error flag, [3] "a visited list was lost" flag,
  // [4..5] arena_top u64, [6..7] spill_top u64, [8..10] work list counts
  // with_side = false: the re-prune kernels share the caller's stream (small batches)
  int alloc(u64 b, u32 R, u32 cap, u64 spill_keys, bool with_side = true) {
    bmax = b;
    vis_cap = cap;
    spill_chunk = 8192;
    spill_cap = spill_keys;
    const u64 E = b * R;
    // a spilled candidate list is longer than MERGE_SPILL_MIN and has at most R old entries
    arena_cap = E + (u64)R * (E / (MERGE_SPILL_MIN - R) + 1);
    HIP_TRY(qidx.alloc(b * 4));
    HIP_TRY(vis.alloc(b * cap * 8));
    HIP_TRY(nvis.alloc(b * 4));
    HIP_TRY(edges.alloc(E * 8));
    HIP_TRY(edges_tmp.alloc(E * 8));
    HIP_TRY(hist.alloc(radix_hist_entries(E) * 4));
    HIP_TRY(lists.alloc(3 * E * sizeof(MergeItem)));
    HIP_TRY(small.alloc(64));
    HIP_TRY(hipMemset(small.p, 0, 64));
    HIP_TRY(ovf_list.alloc(b * 4));
    HIP_TRY(arena.alloc(arena_cap * 8));
    HIP_TRY(spill.alloc(spill_cap * 8));
    HIP_TRY(vis_where.alloc(b * 8));
    HIP_TRY(hipHostMalloc(reinterpret_cast<void**>(&host_flag), 64, hipHostMallocDefault));
    if (with_side) {
      // the third stream is made when a batch first needs it (medium_stream): a process has few
      // hardware queues, and a stream nobody uses still takes its turn on one of them
      for (int i = 0; i < 2; ++i) HIP_TRY(hipStreamCreateWithFlags(&side[i], hipStreamNonBlocking));
      HIP_TRY(hipEventCreateWithFlags(&ev_plan, hipEventDisableTiming));
      for (int i = 0; i < 2; ++i) HIP_TRY(hipEventCreateWithFlags(&ev_side[i], hipEventDisableTiming));
    }
    return ANN_OK;
  }
  // The stream of the medium re-prune instance, made on first use.
  int medium_stream() {
    if (side[2] != nullptr) return ANN_OK;
    HIP_TRY(hipStreamCreateWithFlags(&side[2], hipStreamNonBlocking));
    HIP_TRY(hipEventCreateWithFlags(&ev_side[2], hipEventDisableTiming));
    return ANN_OK;
  }
};

// HIP events around the phases of every batch, read when the batches have finished.
struct PhaseTimer {
  // per batch: 0 start, 1 the caller's stream is through its searches, 2 every prune is over,
  // 3 sorted, 4 merged, 5 and 6 the side streams are through their searches (a batch whose
  // searches run in parts, see batch_insert; otherwise recorded with 1)
  static constexpr int PER_BATCH = 7;
  std::vector<hipEvent_t> ev;
  std::vector<int> parts;  // per batch: search launches (1 or 3)
  bool on = false;
  size_t cur = 0;  // batch being recorded
  int init(bool enable) {
    on = enable;
    return ANN_OK;
  }
  int begin_batch() {
    if (!on) return ANN_OK;
    cur = ev.size() / PER_BATCH;
    parts.push_back(1);
    for (int i = 0; i < PER_BATCH; ++i) {
      hipEvent_t e;
      HIP_TRY(hipEventCreate(&e));
      ev.push_back(e);
    }
    return ANN_OK;
  }
  void mark(int i, hipStream_t s) {
    if (on) (void)hipEventRecord(ev[cur * PER_BATCH + i], s);
  }
  void set_parts(int n) {
    if (on) parts[cur] = n;
  }
  void clear() {
    for (auto& e : ev) (void)hipEventDestroy(e);
    ev.clear();
    parts.clear();
  }
  ~PhaseTimer() { clear(); }
};


constexpr int ANN_LOST_LIST = 1;  // internal: a visited list fit nowhere in a batch issued without sync

// Start vertices of a batch's searches when every point has its own (layered index): position
// slot[i] (i itself when slot is null) of `cur` holds the start vertex of search i, and the same
// position of `next` receives the closest vertex the search visited, mapped through `down` when
// given (see SearchArgs).  slot_host is the host copy of slot.
struct StartsArgs {
  const u32* cur = nullptr;
  u32* next = nullptr;
  const u32* slot = nullptr;
  const u32* slot_host = nullptr;
  const u32* down = nullptr;
};

int new_graph(u64 n, u32 d, int dtype, int metric, u32 R, ann_graph** out);
int check_insert_params(const ann_graph* g, uint32_t L, float alpha);
// the graph gets the vertices n..n_total-1, with empty rows (its arrays grow when they have to)
int grow_graph(ann_graph* g, u64 n_total, hipStream_t st);
int resolve_points(const ann_graph* g, const void* points_dev, hipStream_t st, const void** out);
int resolve_queries(const ann_graph* g, const void* queries_dev, u64 nq, hipStream_t st, const void** out);
int graph_scratch(ann_graph* g, u64 b, u32 L, hipStream_t st, BatchScratch** out);
int batch_insert(ann_graph* g, const void* points, const u32* ids_host, const u32* ids_dev, u64 b, u32 L,
                 float alpha, BatchScratch& S, PhaseTimer& tm, hipStream_t st, bool sync,
                 const StartsArgs* starts = nullptr);
int finish_batches(ann_graph* g, BatchScratch& S, PhaseTimer& tm, hipStream_t st);
// One launch of the query search over `g` (points and queries already resolved to what the
// kernels read); `starts` as in batch_insert; out_ids / out_dists may be null.
int query_launch(const ann_graph* g, const void* pts, const void* queries, const u32* qidx, u64 nq, u32 k, u32 L,
                 float eps, const StartsArgs* starts, u32* out_ids, void* out_dists, hipStream_t st);

}  // namespace annmi
