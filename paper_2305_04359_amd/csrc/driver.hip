// Host side of the library: the C ABI of include/ann.h, the prefix-doubling schedule of Alg. 3
// (batchBuild) and the per-batch launch sequence of BatchInsert.
#include "driver_internal.hpp"

#include <algorithm>
#include <atomic>
#include <chrono>
#include <mutex>

using namespace annmi;

namespace annmi {

static thread_local std::string g_err;

int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

const char* last_error_text() { return g_err.c_str(); }

Allocator& current_allocator() {
  static thread_local Allocator a;
  return a;
}

bool allocator_from(ann_alloc_fn a, ann_free_fn f, void* user, void* stream, Allocator* out) {
  *out = Allocator{};
  if ((a == nullptr) != (f == nullptr)) return false;
  out->alloc = a;
  out->free = f;
  out->user = a != nullptr ? user : nullptr;
  out->stream = a != nullptr ? stream : nullptr;
  return true;
}

int on_exception() {
  try {
    throw;
  } catch (const std::bad_alloc&) {
    return fail(ANN_ENOMEM, "host allocation failed");
  } catch (const std::exception& e) {
    return fail(ANN_EINTERNAL, "exception: %s", e.what());
  } catch (...) {
    return fail(ANN_EINTERNAL, "unknown exception");
  }
}

bool make_cfg(uint32_t d, int dtype, int metric, DistCfg* cfg, std::string* why) {
  const u64 esz = dtype == ANN_F32 ? 4 : 1;
  const u64 rb = (u64)d * esz;
  if (dtype != ANN_U8 && dtype != ANN_I8 && dtype != ANN_F32) {
    *why = "unknown dtype";
    return false;
  }
  if (metric != ANN_L2SQ && metric != ANN_MIPS) {
    *why = "unknown metric";
    return false;
  }
  if (metric == ANN_MIPS && dtype != ANN_F32) {
    *why = "ANN_MIPS is supported for ANN_F32 only";
    return false;
  }
  if (d == 0) {
    *why = "d must be positive";
    return false;
  }
  if (rb % 16 != 0) {  // byte rows are padded by the caller of this function; f32 rows are not
    *why = "f32 needs d % 4 == 0";
    return false;
  }
  cfg->row_bytes = rb;
  cfg->kind = dtype == ANN_U8 ? 0 : dtype == ANN_I8 ? 1 : (metric == ANN_L2SQ ? 2 : 3);
  cfg->vec = 16;
  cfg->npieces = (u32)(rb / 16);
  const u32 per_lane = (cfg->npieces + 7) / 8;
  int nch = 1;
  while ((u32)nch < per_lane) nch *= 2;
  if (dtype == ANN_F32) {
    if (nch < 2) nch = 2;
    if (nch > 8) {
      *why = "f32 rows above 1024 bytes are not supported";
      return false;
    }
  } else if (nch > 4) {
    *why = "u8/i8 rows above 512 bytes are not supported";
    return false;
  }
  cfg->nch = nch;
  return true;
}

// keys of spill space for visited lists that outgrow their slot: room for 1 in 64 searches
u64 default_spill_keys(u64 batch) {
  const u64 k = (batch / 64 + 16) * (8192 + 1024);
  return k;
}

u32 bits_for(u64 n) {  // smallest b with 2^b - 1 >= n
  u32 b = 1;
  while (((1ull << b) - 1ull) < n) ++b;
  return b;
}

u64 splitmix64(u64& state) {
  u64 z = (state += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// Fisher-Yates from the front, driven by SplitMix64(seed): step i = 0 .. m-2 exchanges positions
// i and i + mulhi64(r, m - i), r the next output of the stream; position i is final once step i
// is done.  `ready`, when given, is raised to the number of final positions every few thousand
// steps, so that a build can hand the first batches to the GPU while the rest is still drawn
// (a hundred million steps take the host half a second).  A step's partner depends on the random
// stream alone, so it is known AHEAD steps early and its cache line is requested then: without
// that the walk waits for memory at every step.
void shuffle_in_place(u32* order, u64 m, u64 seed, std::atomic<u64>* ready) {
  constexpr u64 AHEAD = 32;
  u64 ring[AHEAD];
  u64 state = seed;
  const u64 steps = m > 1 ? m - 1 : 0;
  u64 drawn = 0;  // partners drawn so far
  for (; drawn < AHEAD && drawn < steps; ++drawn) {
    const u64 r = splitmix64(state);
    ring[drawn % AHEAD] = drawn + (u64)(((unsigned __int128)r * (unsigned __int128)(m - drawn)) >> 64);
    __builtin_prefetch(order + ring[drawn % AHEAD], 1);
  }
  for (u64 i = 0; i < steps; ++i) {
    const u64 j = ring[i % AHEAD];
    if (drawn < steps) {  // the slot of step i is free now: it takes the partner of step i + AHEAD
      const u64 r = splitmix64(state);
      ring[drawn % AHEAD] = drawn + (u64)(((unsigned __int128)r * (unsigned __int128)(m - drawn)) >> 64);
      __builtin_prefetch(order + ring[drawn % AHEAD], 1);
      ++drawn;
    }
    const u32 t = order[i];
    order[i] = order[j];
    order[j] = t;
    if (ready != nullptr && (i & 8191u) == 8191u) ready->store(i + 1, std::memory_order_release);
  }
  if (ready != nullptr) ready->store(m, std::memory_order_release);
}

}  // namespace annmi


namespace annmi {

// dst row r = src row r followed by zeros; one thread per 4-byte word of dst (rows of any byte
// length, so the source is read byte by byte at the ragged end)
__global__ __launch_bounds__(256) void pad_rows_kernel(const unsigned char* src, u64 nrows, u32 rb, u32* dst,
                                                       u32 stride) {
  const u64 w = (u64)blockIdx.x * blockDim.x + threadIdx.x;
  const u32 wpr = stride / 4u;
  if (w >= nrows * wpr) return;
  const u64 r = w / wpr;
  const u32 c = (u32)(w % wpr) * 4u;
  const unsigned char* p = src + r * rb;
  u32 v = 0;
#pragma unroll
  for (u32 k = 0; k < 4; ++k)
    if (c + k < rb) v |= (u32)p[c + k] << (8u * k);
  dst[w] = v;
}

// how many of the listed vertices have out-neighbours (degree in the low 16 bits of meta)
__global__ __launch_bounds__(256) void count_inserted_kernel(const u32* ids, u64 b, const u32* meta, u32* count) {
  const u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < b && (meta[ids[i]] & 0xFFFFu) != 0u) atomicAdd(count, 1u);
}

// positions among the ids other than s -> ids: every position from s on stands for the next id
__global__ __launch_bounds__(256) void skip_start_kernel(u32* ids, u64 count, u32 s) {
  const u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) ids[i] += ids[i] >= s ? 1u : 0u;
}

int pad_rows(const void* src, u64 nrows, u32 rb, void* dst, u64 stride, hipStream_t st) {
  const u64 words = nrows * (stride / 4);
  if (words == 0) return ANN_OK;
  hipLaunchKernelGGL(pad_rows_kernel, dim3((u32)((words + 255) / 256)), dim3(256), 0, st,
                     static_cast<const unsigned char*>(src), nrows, rb, static_cast<u32*>(dst), (u32)stride);
  HIP_TRY(hipGetLastError());
  return ANN_OK;
}

// The array the kernels read for `points_dev`: itself, or the graph's padded copy of it.  The
// copy follows the graph as it grows: rows already copied from the same array stay, only the new
// ones are added.
int resolve_points(const ann_graph* g, const void* points_dev, hipStream_t st, const void** out) {
  *out = points_dev;
  if (!g->pad_stride) return ANN_OK;
  if (g->pad_cap < g->n) {
    if (g->pad_buf) {
      HIP_TRY(hipDeviceSynchronize());  // earlier calls may still read the old copy
      g->al.put(g->pad_buf);
      g->pad_buf = nullptr;
    }
    g->pad_cap = 0;
    g->pad_src = nullptr;
    g->pad_done = 0;
    const u64 want = g->cap > g->n ? g->cap : g->n;
    HIP_TRY(g->al.get(&g->pad_buf, (size_t)want * g->pad_stride));
    g->pad_cap = want;
  }
  if (g->pad_src != points_dev) g->pad_done = 0;
  if (g->pad_done < g->n) {
    g->pad_src = nullptr;
    const u64 first = g->pad_done;
    int rc = pad_rows(static_cast<const char*>(points_dev) + first * g->d, g->n - first, g->d,
                      static_cast<char*>(g->pad_buf) + first * g->pad_stride, g->pad_stride, st);
    if (rc) return rc;
    g->pad_src = points_dev;
    g->pad_done = g->n;
  }
  *out = g->pad_buf;
  return ANN_OK;
}

int resolve_queries(const ann_graph* g, const void* queries_dev, u64 nq, hipStream_t st, const void** out) {
  *out = queries_dev;
  if (!g->pad_stride) return ANN_OK;
  if (g->qpad_rows < nq) {
    if (g->qpad_buf) {
      // an earlier call, on whatever stream it was issued, may still read the old buffer
      HIP_TRY(hipDeviceSynchronize());
      g->al.put(g->qpad_buf);
      g->qpad_buf = nullptr;
      g->qpad_rows = 0;
    }
    HIP_TRY(g->al.get(&g->qpad_buf, (size_t)nq * g->pad_stride));
    g->qpad_rows = nq;
  }
  int rc = pad_rows(queries_dev, nq, g->d, g->qpad_buf, g->pad_stride, st);
  if (rc) return rc;
  *out = g->qpad_buf;
  return ANN_OK;
}

// Adds up the phase times of all recorded batches (the caller has synchronised the stream).
void collect_phase_times(ann_graph* g, PhaseTimer& tm) {
  if (!tm.on) return;
  for (size_t k = 0; k + PhaseTimer::PER_BATCH <= tm.ev.size(); k += PhaseTimer::PER_BATCH) {
    // the search phase lasts until the last part's searches are over; prunes of parts that were
    // through earlier run inside it
    float ms = 0, srch = 0, both = 0;
    const int np = tm.parts[k / PhaseTimer::PER_BATCH];
    const int part_end[3] = {1, 5, 6};
    for (int c = 0; c < np; ++c) {
      (void)hipEventElapsedTime(&ms, tm.ev[k + 0], tm.ev[k + part_end[c]]);
      srch = ms > srch ? ms : srch;
      g->stats.ms_search_launches += ms;
    }
    g->stats.search_launches += (u64)np;
    (void)hipEventElapsedTime(&both, tm.ev[k + 0], tm.ev[k + 2]);
    g->stats.ms_search += srch;
    g->stats.ms_prune += both > srch ? both - srch : 0.0f;
    (void)hipEventElapsedTime(&ms, tm.ev[k + 2], tm.ev[k + 3]);
    g->stats.ms_sort += ms;
    (void)hipEventElapsedTime(&ms, tm.ev[k + 3], tm.ev[k + 4]);
    g->stats.ms_merge += ms;
    (void)hipEventElapsedTime(&ms, tm.ev[k + 0], tm.ev[k + 4]);
    g->stats.ms_total += ms;
  }
  tm.clear();
}

// batches of at least this many points run step 1 in three parts (see batch_insert)
constexpr u64 STEP1_PARTS_MIN = 8192;

// BatchInsert(P') of Alg. 3 for the b ids in ids_host (device copy made here).
// With `sync` the host waits after step 1 and redoes, with as much room as they need, the searches
// whose visited list fit neither its slot nor a spill chunk; without it nothing waits, such a
// search leaves its point unconnected and raises a flag that finish_batches reports.
int batch_insert(ann_graph* g, const void* points, const u32* ids_host, const u32* ids_dev, u64 b, u32 L,
                 float alpha, BatchScratch& S, PhaseTimer& tm, hipStream_t st, bool sync, const StartsArgs* starts) {
  if (b == 0) return ANN_OK;
  {
    int rc0 = tm.begin_batch();
    if (rc0) return rc0;
  }
  const u32 R = g->R;
  const u64 E = b * R;
  const long long a16 = llround((double)alpha * 65536.0);
  if (g->clean_alpha != alpha) {
    // prefixes pruned with another alpha say nothing about this one
    HIP_TRY(launch_meta_forget_clean(g->n, g->meta, st));
    g->clean_alpha = alpha;
  }
  u32* small = S.small.as<u32>();
  DevCounters* ctr = g->collect ? g->counters : nullptr;

  // per-batch counters: [0] overflow count, [4..5] arena top, [6..7] spill top, [8..10] work list
  // lengths; the flags [2] and [3] stay up once set.  The scratch starts zeroed; afterwards the
  // search kernel zeroes what the later steps count in, and the prune kernel the spill top.
  tm.mark(0, st);

  // step 1a: greedySearch(p, s, L, 1) over the frozen graph, visited lists to scratch
  SearchArgs sa{};
  sa.points = static_cast<const char*>(points);
  sa.graph = g->rows;
  sa.queries = static_cast<const char*>(points);
  sa.qidx = ids_dev;
  sa.qrow_bytes = g->cfg.row_bytes;
  sa.nq = (u32)b;
  sa.R = R;
  sa.start = g->start;
  if (starts) {
    sa.starts = starts->cur;
    sa.slot = starts->slot;
    sa.down = starts->down;
    sa.next_start = starts->next;
  }
  sa.L = L;
  sa.k = 1;
  sa.hash_buckets = search_hash_buckets(L, g->hash_bits);
  search_filter_mode(g->n, sa.hash_buckets, &sa.id_bits, &sa.tag_width);
  sa.batch_counters = small;
  sa.eps16 = -1;
  sa.epsf = 0.0f;
  sa.vis = S.vis.as<u64>();
  sa.nvis = S.nvis.as<u32>();
  sa.vis_cap = S.vis_cap;
  sa.spill = S.spill_cap ? S.spill.as<u64>() : nullptr;
  sa.spill_cap = S.spill_cap;
  sa.spill_top = reinterpret_cast<unsigned long long*>(small + 6);
  sa.spill_chunk = S.spill_chunk;
  sa.vis_where = S.vis_where.as<u64>();
  sa.counters = ctr;
  // A batch of many points runs step 1 in parts, each on a stream of its own (the caller's and
  // the side streams, idle until step 2): a part that is through its searches prunes while the
  // others still search, which fills the end of the search phase, when the chip runs empty
  // (C2 build 83.7 -> 81.5 ms, C5 19.85 -> 19.40 s with three parts; two parts gain less;
  // parts one after the other on one stream lose 12 ms at C2, each paying the tail).
  // Not for the synchronised attempt, whose host check reads one overflow list for the batch.
  const int nparts = (!sync && S.side[0] != nullptr && b >= STEP1_PARTS_MIN && g->step1_parts != 1) ? 3 : 1;
  u64 cut[4] = {0, b, b, b};
  if (nparts == 3) {  // a half for the caller's stream, then 30 % and 20 % (measured against other splits)
    cut[1] = b / 2;
    cut[2] = b * 4 / 5;
  }
  auto part_stream = [&](int c) { return c ? S.side[c - 1] : st; };
  if (nparts > 1) {
    HIP_TRY(hipEventRecord(S.ev_plan, st));
    for (int c = 1; c < nparts; ++c) HIP_TRY(hipStreamWaitEvent(S.side[c - 1], S.ev_plan, 0));
  }
  for (int c = 0; c < nparts; ++c) {
    SearchArgs sc = sa;
    sc.qidx = ids_dev + cut[c];
    sc.nq = (u32)(cut[c + 1] - cut[c]);
    sc.vis = sa.vis + cut[c] * S.vis_cap;
    sc.nvis = sa.nvis + cut[c];
    sc.vis_where = sa.vis_where + cut[c];
    if (c) sc.batch_counters = nullptr;  // the first part's first workgroup zeroes them
    if (starts) {  // the searches' own start vertices are indexed by slot, or by position
      if (starts->slot) {
        sc.slot = starts->slot + cut[c];
      } else {
        sc.starts = starts->cur + cut[c];
        if (starts->next) sc.next_start = starts->next + cut[c];
      }
    }
    HIP_TRY(launch_search(g->cfg, sc, part_stream(c)));
    tm.mark(c == 0 ? 1 : 4 + c, part_stream(c));
  }
  tm.set_parts(nparts);

  // step 1b: N_out(p) <- prune(p, V, R); reversed edges to the edge array
  PruneArgs pa{};
  pa.points = static_cast<const char*>(points);
  pa.graph = g->rows;
  pa.qidx = ids_dev;
  pa.slotmap = nullptr;
  pa.nq = (u32)b;
  pa.R = R;
  pa.vis = S.vis.as<u64>();
  pa.vis_rw = S.vis.as<u64>();
  pa.nvis = S.nvis.as<u32>();
  pa.vis_cap = S.vis_cap;
  pa.spill = S.spill.as<u64>();
  pa.spill_chunk = S.spill_chunk;
  pa.vis_where = S.vis_where.as<u64>();
  pa.spill_top_reset = reinterpret_cast<unsigned long long*>(small + 6);
  pa.lost_flag = small + 3;
  pa.meta = g->meta;
  pa.stage_bytes = prune_stage_bytes(R, g->cfg);
  pa.use_mfma = mfma_prune_ok(R, g->cfg) ? 1u : 0u;
  pa.edges = S.edges.as<u64>();
  pa.overflow_count = small + 0;
  pa.overflow_list = S.ovf_list.as<u32>();
  pa.a16 = a16;
  pa.af = alpha;
  pa.counters = ctr;
  if (nparts > 1) pa.spill_top_reset = nullptr;  // (a part's prune may start while another part still searches)
  for (int c = 0; c < nparts; ++c) {
    PruneArgs pc = pa;
    pc.qidx = ids_dev + cut[c];
    pc.nq = (u32)(cut[c + 1] - cut[c]);
    pc.vis = pa.vis + cut[c] * S.vis_cap;
    pc.vis_rw = pa.vis_rw + cut[c] * S.vis_cap;
    pc.nvis = pa.nvis + cut[c];
    pc.vis_where = pa.vis_where + cut[c];
    pc.edges = pa.edges + cut[c] * R;
    HIP_TRY(launch_prune(g->cfg, pc, part_stream(c)));
  }
  if (nparts > 1) {
    for (int c = 1; c < nparts; ++c) {
      HIP_TRY(hipEventRecord(S.ev_side[c - 1], S.side[c - 1]));
      HIP_TRY(hipStreamWaitEvent(st, S.ev_side[c - 1], 0));
    }
    HIP_TRY(hipMemsetAsync(small + 6, 0, 8, st));  // the spill top, for the next batch's searches
  }

  // searches whose visited list fit nowhere are redone with as much room as they need
  u32 novf = 0;
  if (sync) {
    HIP_TRY(hipMemcpyAsync(S.host_flag, small + 0, 4, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    novf = S.host_flag[0];
  }
  if (novf > 0) {
    std::vector<u32> slots(novf), nv(b);
    HIP_TRY(hipMemcpy(slots.data(), S.ovf_list.p, (size_t)novf * 4, hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(nv.data(), S.nvis.p, (size_t)b * 4, hipMemcpyDeviceToHost));
    u32 need = 0;
    std::vector<u32> ids2(novf);
    for (u32 i = 0; i < novf; ++i) {
      need = nv[slots[i]] > need ? nv[slots[i]] : need;
      ids2[i] = ids_host[slots[i]];
    }
    DevBuf ids2_d, slots_d, vis2, nvis2;
    HIP_TRY(ids2_d.alloc((size_t)novf * 4));
    HIP_TRY(slots_d.alloc((size_t)novf * 4));
    HIP_TRY(vis2.alloc((size_t)novf * need * 8));
    HIP_TRY(nvis2.alloc((size_t)novf * 4));
    HIP_TRY(hipMemcpy(ids2_d.p, ids2.data(), (size_t)novf * 4, hipMemcpyHostToDevice));
    HIP_TRY(hipMemcpy(slots_d.p, slots.data(), (size_t)novf * 4, hipMemcpyHostToDevice));
    HIP_TRY(hipMemsetAsync(small + 0, 0, 4, st));
    SearchArgs sb = sa;
    sb.qidx = ids2_d.as<u32>();
    sb.nq = novf;
    sb.vis = vis2.as<u64>();
    sb.nvis = nvis2.as<u32>();
    sb.vis_cap = need;
    sb.spill = nullptr;
    sb.batch_counters = nullptr;
    sb.vis_where = nullptr;
    sb.counters = nullptr;
    DevBuf pos2;
    if (starts) {
      // redone search i stands at the position of batch slot slots[i]
      std::vector<u32> p2(novf);
      for (u32 i = 0; i < novf; ++i) p2[i] = starts->slot_host ? starts->slot_host[slots[i]] : slots[i];
      HIP_TRY(pos2.alloc((size_t)novf * 4));
      HIP_TRY(hipMemcpy(pos2.p, p2.data(), (size_t)novf * 4, hipMemcpyHostToDevice));
      sb.slot = pos2.as<u32>();
    }
    HIP_TRY(launch_search(g->cfg, sb, st));
    PruneArgs pb = pa;
    pb.qidx = ids2_d.as<u32>();
    pb.slotmap = slots_d.as<u32>();
    pb.nq = novf;
    pb.vis = vis2.as<u64>();
    pb.vis_rw = vis2.as<u64>();
    pb.nvis = nvis2.as<u32>();
    pb.vis_cap = need;
    pb.vis_where = nullptr;
    pb.spill_top_reset = nullptr;
    HIP_TRY(launch_prune(g->cfg, pb, st));
    u32 again = 0;
    HIP_TRY(hipMemcpyAsync(&again, small + 0, 4, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (again != 0) return fail(ANN_EINTERNAL, "visited list overflowed again on retry");
    g->stats.redone += novf;
    HIP_TRY(hipMemsetAsync(small + 3, 0, 4, st));  // every lost list has been made up for
  }
  tm.mark(2, st);

  // step 2a: bring equal destinations together
  HIP_TRY(radix_sort_edges(S.edges.as<u64>(), S.edges_tmp.as<u64>(), S.hist.as<u32>(), radix_hist_entries(S.bmax * R), E,
                           bits_for(g->n), st));
  tm.mark(3, st);

  // step 2b: cut the keys into segments of equal destination; append where the row has room,
  // otherwise one wave per row prunes it again
  MergeArgs ma{};
  ma.points = static_cast<const char*>(points);
  ma.graph = g->rows;
  ma.meta = g->meta;
  ma.R = R;
  ma.keys = S.edges.as<u64>();
  ma.nkeys = E;
  ma.list_count = small + 8;
  for (int c = 0; c < 3; ++c) ma.list_items[c] = S.lists.as<MergeItem>() + (u64)c * E;
  ma.list_items[3] = ma.list_items[2] + (E - 1);  // grows down from the end of the large list's array
  ma.fast_amax = fast_path_amax(g->cfg);
  ma.gram_ok = gram_path_ok(g->cfg) ? 1u : 0u;
  ma.gram_tmax = gram_path_tmax();
  // rows between the matrix-core kernel's reach and 512 candidates are many where that kernel
  // does not apply (float rows, long rows) and in batches of millions of points: there they get
  // a kernel instance of their own; elsewhere one more launch per batch would cost more than
  // the few rows gain
  ma.medium_max = (!ma.gram_ok || E >= (1ull << 22)) ? MERGE_MEDIUM_MAX : 0u;
  ma.stage_bytes = prune_stage_bytes(R, g->cfg);
  ma.use_mfma = mfma_prune_ok(R, g->cfg) ? 1u : 0u;
  ma.arena = S.arena.as<u64>();
  ma.arena_cap = S.arena_cap;
  ma.arena_top = reinterpret_cast<unsigned long long*>(small + 4);
  ma.error_flag = small + 2;
  ma.a16 = a16;
  ma.af = alpha;
  ma.counters = ctr;
  HIP_TRY(launch_plan(ma, st));
  // grid-stride kernels over work lists whose lengths stay on the device: enough waves to fill
  // the chip, no more (idle workgroups are not free)
  const u64 want = E < 8192 ? E : 8192;
  // (a small batch's kernels are over before a wait between streams has been served)
  if (S.side[0] != nullptr && b >= 2048) {
    HIP_TRY(hipEventRecord(S.ev_plan, st));
    const int nside = ma.medium_max ? 3 : 2;
    if (nside == 3) {
      const int rc_side = S.medium_stream();
      if (rc_side) return rc_side;
    }
    for (int i = 0; i < nside; ++i) HIP_TRY(hipStreamWaitEvent(S.side[i], S.ev_plan, 0));
    HIP_TRY(launch_merge(g->cfg, ma, (u32)(want ? want : 1), st, S.side[0], S.side[1], S.side[2]));
    for (int i = 0; i < nside; ++i) {
      HIP_TRY(hipEventRecord(S.ev_side[i], S.side[i]));
      HIP_TRY(hipStreamWaitEvent(st, S.ev_side[i], 0));
    }
  } else {
    HIP_TRY(launch_merge(g->cfg, ma, (u32)(want ? want : 1), st, st, st, st));  // small batches: one stream
  }
  tm.mark(4, st);
  g->rounds += 1;
  g->stats.rounds += 1;
  return ANN_OK;
}

// Waits for the batches issued so far; reports a spill-arena failure (cannot happen with the
// arena sized as it is) or a lost visited list, and reads the phase times.
int finish_batches(ann_graph* g, BatchScratch& S, PhaseTimer& tm, hipStream_t st) {
  u32 flags[4] = {0, 0, 0, 0};
  HIP_TRY(hipMemcpyAsync(flags, S.small.p, 16, hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  collect_phase_times(g, tm);
  if (flags[2] != 0) return fail(ANN_EINTERNAL, "merge spill arena exhausted");
  if (flags[3] != 0) return ANN_LOST_LIST;
  return ANN_OK;
}

// The graph's own scratch with room for a batch of b points, made or enlarged when needed.
int graph_scratch(ann_graph* g, u64 b, u32 L, hipStream_t st, BatchScratch** out) {
  const u32 cap = g->visited_cap ? g->visited_cap : (4 * L > 256 ? 4 * L : 256);
  if (g->scratch && (g->scratch->bmax < b || g->scratch->vis_cap != cap)) {
    delete g->scratch;
    g->scratch = nullptr;
  }
  if (!g->scratch) {
    g->scratch = new (std::nothrow) BatchScratch();
    if (!g->scratch) return fail(ANN_ENOMEM, "host allocation failed");
    int rc = g->scratch->alloc(b, g->R, cap, g->spill_keys ? g->spill_keys : default_spill_keys(b));
    if (rc) {
      delete g->scratch;
      g->scratch = nullptr;
      return rc;
    }
  } else {
    HIP_TRY(hipMemsetAsync(g->scratch->small.p, 0, 64, st));  // flags of an earlier call that failed
  }
  *out = g->scratch;
  return ANN_OK;
}

int query_launch(const ann_graph* g, const void* pts, const void* queries, const u32* qidx, u64 nq, u32 k, u32 L,
                 float eps, const StartsArgs* starts, u32* out_ids, void* out_dists, hipStream_t st) {
  SearchArgs sa{};
  sa.points = static_cast<const char*>(pts);
  sa.graph = g->rows;
  sa.queries = static_cast<const char*>(queries);
  sa.qidx = qidx;
  sa.qrow_bytes = g->cfg.row_bytes;
  sa.nq = (u32)nq;
  sa.R = g->R;
  sa.start = g->start;
  if (starts) {
    sa.starts = starts->cur;
    sa.slot = starts->slot;
    sa.down = starts->down;
    sa.next_start = starts->next;
  }
  sa.L = L;
  sa.k = k;
  sa.hash_buckets = search_hash_buckets(L, g->hash_bits);
  search_filter_mode(g->n, sa.hash_buckets, &sa.id_bits, &sa.tag_width);
  sa.eps16 = eps >= 0.0f ? llround((double)eps * 65536.0) : -1;
  sa.epsf = eps >= 0.0f ? eps : 0.0f;
  sa.out_ids = out_ids;
  sa.out_dists = out_dists;
  sa.counters = g->collect ? g->counters : nullptr;
  HIP_TRY(launch_search(g->cfg, sa, st));
  return ANN_OK;
}

int check_insert_params(const ann_graph* g, uint32_t L, float alpha) {
  if (L < 1 || L > 512) return fail(ANN_EINVAL, "L must be in [1, 512]");
  if (!(alpha > 0.0f) || !std::isfinite(alpha) || alpha > 30000.0f) return fail(ANN_EINVAL, "alpha must be in (0, 30000]");
  // integer rows test alpha as round(alpha * 2^16) / 2^16: that must not be zero
  if (g->dtype != ANN_F32 && llround((double)alpha * 65536.0) < 1)
    return fail(ANN_EINVAL, "alpha is below 1/65536, the smallest value u8/i8 rows can be pruned with");
  if (g->metric == ANN_MIPS && alpha > 1.0f) return fail(ANN_EINVAL, "alpha must be <= 1 for ANN_MIPS");
  return ANN_OK;
}

int new_graph(u64 n, u32 d, int dtype, int metric, u32 R, ann_graph** out) {
  std::string why;
  DistCfg cfg{};
  u64 pad_stride = 0;
  if ((dtype == ANN_U8 || dtype == ANN_I8) && d % 16 != 0) {
    // multiple of 16 bytes; a power of two (whole cache lines) where that wastes at most a quarter
    const u64 s16 = ((u64)d + 15) / 16 * 16;
    u64 p2 = 16;
    while (p2 < s16) p2 *= 2;
    pad_stride = (p2 - s16) * 4 <= s16 ? p2 : s16;
  }
  if (!make_cfg(pad_stride ? (uint32_t)pad_stride : d, dtype, metric, &cfg, &why))
    return fail(ANN_EINVAL, "%s", why.c_str());
  if (n < 1 || n >= (1ull << 31)) return fail(ANN_EINVAL, "n must be in [1, 2^31)");
  if (R < 1 || R > 512) return fail(ANN_EINVAL, "R must be in [1, 512]");
  ann_graph* g = new (std::nothrow) ann_graph();
  if (!g) return fail(ANN_ENOMEM, "host allocation failed");
  g->n = n;
  g->cap = n;
  g->d = d;
  g->R = R;
  g->dtype = dtype;
  g->metric = metric;
  g->cfg = cfg;
  g->pad_stride = pad_stride;
  g->al = current_allocator();
  hipError_t e = g->al.get(reinterpret_cast<void**>(&g->rows), (size_t)n * R * sizeof(u32));
  if (e == hipSuccess) e = g->al.get(reinterpret_cast<void**>(&g->meta), (size_t)n * sizeof(u32));
  if (e == hipSuccess) e = hipMemset(g->meta, 0, (size_t)n * sizeof(u32));
  if (e == hipSuccess) e = g->al.get(reinterpret_cast<void**>(&g->counters), COUNTER_COPIES * sizeof(DevCounters));
  if (e == hipSuccess) e = hipMemset(g->counters, 0, COUNTER_COPIES * sizeof(DevCounters));
  if (e != hipSuccess) {
    ann_graph_free(g);
    return fail(e == hipErrorOutOfMemory ? ANN_ENOMEM : ANN_EHIP, "graph allocation: %s", hipGetErrorString(e));
  }
  *out = g;
  return ANN_OK;
}

// Room for `want` points: rows and meta move to larger arrays when the capacity is exceeded
// (everything that may still read the old ones is waited for first).
int reserve_rows(ann_graph* g, u64 want, hipStream_t st) {
  if (want <= g->cap) return ANN_OK;
  if (want >= (1ull << 31)) return fail(ANN_EINVAL, "n must stay below 2^31");
  u32* rows = nullptr;
  u32* meta = nullptr;
  hipError_t e = g->al.get(reinterpret_cast<void**>(&rows), (size_t)want * g->R * sizeof(u32));
  if (e == hipSuccess) e = g->al.get(reinterpret_cast<void**>(&meta), (size_t)want * sizeof(u32));
  if (e == hipSuccess)
    e = hipMemcpyAsync(rows, g->rows, (size_t)g->n * g->R * sizeof(u32), hipMemcpyDeviceToDevice, st);
  if (e == hipSuccess) e = hipMemcpyAsync(meta, g->meta, (size_t)g->n * sizeof(u32), hipMemcpyDeviceToDevice, st);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    g->al.put(rows);
    g->al.put(meta);
    return fail(e == hipErrorOutOfMemory ? ANN_ENOMEM : ANN_EHIP, "graph growth: %s", hipGetErrorString(e));
  }
  g->al.put(g->rows);
  g->al.put(g->meta);
  g->rows = rows;
  g->meta = meta;
  g->cap = want;
  return ANN_OK;
}

// The graph gets the vertices n..n_total-1, with empty rows.
int grow_graph(ann_graph* g, u64 n_total, hipStream_t st) {
  if (n_total > g->cap) {
    // at least half as much again, so that a stream of small additions copies the rows rarely
    u64 want = g->cap + g->cap / 2;
    if (want < n_total) want = n_total;
    if (want >= (1ull << 31)) want = n_total;
    int rc = reserve_rows(g, want, st);
    if (rc) return rc;
  }
  const u64 add = n_total - g->n;
  HIP_TRY(hipMemsetAsync(g->rows + g->n * g->R, 0xFF, (size_t)add * g->R * sizeof(u32), st));
  HIP_TRY(hipMemsetAsync(g->meta + g->n, 0, (size_t)add * sizeof(u32), st));
  g->n = n_total;
  return ANN_OK;
}

}  // namespace annmi

// ---------------------------------------------------------------------------------------------
// ann_search_noalloc: the query search for callers that cannot allocate.  The one buffer the
// search may need beyond its inputs and outputs, the zero-padded copy of the queries (byte rows
// that are not a multiple of 16 bytes), lives in a device array of this library instead of a
// hipMalloc'ed one.  Each device holds its own copy of the array, at its own address, until the
// process ends; the address is asked for once per device, with that device current.
// ---------------------------------------------------------------------------------------------
constexpr size_t NOALLOC_SCRATCH_BYTES = (size_t)ANN_NOALLOC_SCRATCH_MIB << 20;
static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES];  // per device: where `scratch` lives there (null: not asked yet)
std::mutex g_scratch_lock;

int noalloc_scratch(void** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return fail(ANN_EINVAL, "device %d is beyond the %d this call serves", dev, MAX_DEVICES);
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (p == nullptr) return fail(ANN_EINTERNAL, "the scratch array has no address on device %d", dev);
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return ANN_OK;
}
}  // namespace

extern "C" {

const char* ann_last_error(void) { return last_error_text(); }

void ann_graph_free(ann_graph* g) {
  if (!g) return;
  g->al.put(g->rows);
  g->al.put(g->meta);
  g->al.put(g->counters);
  g->al.put(g->pad_buf);
  g->al.put(g->qpad_buf);
  delete g->scratch;
  delete g;
}

int ann_graph_info(const ann_graph* g, ann_graph_info_t* info) try {
  if (!g || !info) return fail(ANN_EINVAL, "null argument");
  info->n = g->n;
  info->d = g->d;
  info->R = g->R;
  info->dtype = (uint32_t)g->dtype;
  info->metric = (uint32_t)g->metric;
  info->start = g->start;
  info->rounds = g->rounds;
  return ANN_OK;
} catch (...) {
  return annmi::on_exception();
}

int ann_get_stats(const ann_graph* g, ann_stats* stats) try {
  if (!g || !stats) return fail(ANN_EINVAL, "null argument");
  std::vector<DevCounters> copies(COUNTER_COPIES);
  HIP_TRY(hipMemcpy(copies.data(), g->counters, COUNTER_COPIES * sizeof(DevCounters), hipMemcpyDeviceToHost));
  DevCounters c{};
  for (const DevCounters& x : copies) {
    c.searches += x.searches;
    c.hops += x.hops;
    c.evals += x.evals;
    c.prunes += x.prunes;
    c.reprunes += x.reprunes;
    c.appends += x.appends;
    c.edges += x.edges;
    c.prune_evals += x.prune_evals;
    c.passes += x.passes;
    c.survivors += x.survivors;
    c.insert_hops += x.insert_hops;
  }
  *stats = g->stats;
  stats->searches = c.searches;
  stats->hops = c.hops;
  stats->evals = c.evals;
  stats->prunes = c.prunes;
  stats->reprunes = c.reprunes;
  stats->appends = c.appends;
  stats->edges = c.edges;
  stats->prune_evals = c.prune_evals;
  stats->passes = c.passes;
  stats->survivors = c.survivors;
  stats->insert_hops = c.insert_hops;
  return ANN_OK;
} catch (...) {
  return annmi::on_exception();
}

int ann_graph_set_stats(ann_graph* g, int on) {
  if (!g) return fail(ANN_EINVAL, "null argument");
  g->collect = on != 0;
  return ANN_OK;
}

int ann_graph_set_filter_bits(ann_graph* g, uint32_t hash_bits) {
  if (!g) return fail(ANN_EINVAL, "null argument");
  if (hash_bits && (hash_bits < 4 || hash_bits > 13)) return fail(ANN_EINVAL, "hash_bits must be in [4, 13]");
  g->hash_bits = hash_bits;
  return ANN_OK;
}

const uint32_t* ann_graph_device_rows(const ann_graph* g) { return g ? g->rows : nullptr; }

int ann_graph_copy_neighbors(const ann_graph* g, uint32_t* rows_host) try {
  if (!g || !rows_host) return fail(ANN_EINVAL, "null argument");
  HIP_TRY(hipMemcpy(rows_host, g->rows, (size_t)g->n * g->R * sizeof(u32), hipMemcpyDeviceToHost));
  return ANN_OK;
} catch (...) {
  return annmi::on_exception();
}

int ann_graph_from_host(const uint32_t* rows_host, uint64_t n, uint32_t d, ann_dtype dtype, ann_metric metric,
                        uint32_t R, uint32_t start, ann_graph** out) try {
  if (out) *out = nullptr;
  if (!rows_host || !out) return fail(ANN_EINVAL, "null argument");
  if (start >= n) return fail(ANN_EINVAL, "start vertex out of range");
  // every id must be a vertex or ANN_NONE: the kernels follow them without further checks
  for (u64 i = 0; i < n * R; ++i)
    if (rows_host[i] != ANN_NONE && rows_host[i] >= n) return fail(ANN_EINVAL, "neighbour id out of range");
  {
    // and no id twice in a row: a search takes the neighbours of a vertex as distinct candidates
    std::vector<u32> row(R);
    for (u64 v = 0; v < n; ++v) {
      u32 c = 0;
      for (u32 j = 0; j < R; ++j)
        if (rows_host[v * R + j] != ANN_NONE) row[c++] = rows_host[v * R + j];
      std::sort(row.begin(), row.begin() + c);
      for (u32 j = 1; j < c; ++j)
        if (row[j] == row[j - 1]) return fail(ANN_EINVAL, "vertex %llu lists neighbour %u twice", (unsigned long long)v, row[j]);
    }
  }
  ann_graph* g = nullptr;
  int rc = new_graph(n, d, dtype, metric, R, &g);
  if (rc) return rc;
  g->start = start;
  hipError_t e = hipMemcpy(g->rows, rows_host, (size_t)n * R * sizeof(u32), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = launch_meta_from_rows(g->rows, n, R, g->meta, nullptr);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    ann_graph_free(g);
    return fail(ANN_EHIP, "copy of rows: %s", hipGetErrorString(e));
  }
  *out = g;
  return ANN_OK;
} catch (...) {
  return annmi::on_exception();
}

int ann_start_vertex(const void* points_dev, uint64_t n, uint32_t d, ann_dtype dtype, void* stream,
                     uint32_t* start_out) try {
  if (!points_dev || !start_out || n < 1 || d < 1) return fail(ANN_EINVAL, "null argument or empty input");
  if (dtype != ANN_U8 && dtype != ANN_I8 && dtype != ANN_F32) return fail(ANN_EINVAL, "unknown dtype");
  u32 s = 0;
  HIP_TRY(start_vertex_device(points_dev, n, d, dtype, static_cast<hipStream_t>(stream), &s));
  *start_out = s;
  return ANN_OK;
} catch (...) {
  return annmi::on_exception();
}

int ann_sort_edges(uint64_t* keys_dev, uint64_t count, uint32_t key_bits, void* stream) try {
  if (!keys_dev && count) return fail(ANN_EINVAL, "null argument");
  if (key_bits < 1 || key_bits > 32) return fail(ANN_EINVAL, "key_bits must be in [1, 32]");
  if (count >= (1ull << 32)) return fail(ANN_EINVAL, "too many keys");
  hipStream_t st = static_cast<hipStream_t>(stream);
  DevBuf tmp, hist;
  HIP_TRY(tmp.alloc(count * 8));
  HIP_TRY(hist.alloc(radix_hist_entries(count) * 4));
  HIP_TRY(radix_sort_edges(keys_dev, tmp.as<u64>(), hist.as<u32>(), radix_hist_entries(count), count, key_bits, st));
  HIP_TRY(hipStreamSynchronize(st));
  return ANN_OK;
} catch (...) {
  return annmi::on_exception();
}


int ann_insert_batch(ann_graph* g, const void* points_dev, const uint32_t* ids_host, uint64_t b, uint32_t L,
                     float alpha, void* stream) try {
  if (!g || !points_dev || (!ids_host && b)) return fail(ANN_EINVAL, "null argument");
  int rc = check_insert_params(g, L, alpha);
  if (rc) return rc;
  if (b == 0) return ANN_OK;
  if (b * g->R >= (1ull << 32)) return fail(ANN_EINVAL, "batch too large");
  {
    // two searches of one point would write the same row
    std::vector<u64> seen((g->n + 63) / 64, 0ull);
    for (u64 i = 0; i < b; ++i) {
      const u32 id = ids_host[i];
      if (id >= g->n || id == g->start) return fail(ANN_EINVAL, "bad id in batch");
      if (seen[id >> 6] >> (id & 63) & 1ull) return fail(ANN_EINVAL, "id %u is listed twice in the batch", id);
      seen[id >> 6] |= 1ull << (id & 63);
    }
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  Allocator al = g->al;
  al.stream = stream;
  AllocScope scope(al);
  BatchScratch* Sp = nullptr;
  rc = graph_scratch(g, b, L, st, &Sp);
  if (rc) return rc;
  BatchScratch& S = *Sp;
  HIP_TRY(hipMemcpy(S.qidx.p, ids_host, (size_t)b * 4, hipMemcpyHostToDevice));
  {
    // a point that has out-neighbours is in the graph already: searching from s would reach it
    // and it would become its own candidate
    u32* flag = S.small.as<u32>() + 12;
    HIP_TRY(hipMemsetAsync(flag, 0, 4, st));
    hipLaunchKernelGGL(count_inserted_kernel, dim3((u32)((b + 255) / 256)), dim3(256), 0, st, S.qidx.as<u32>(), b,
                       g->meta, flag);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipMemcpyAsync(S.host_flag + 4, flag, 4, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (S.host_flag[4] != 0)
      return fail(ANN_EINVAL, "%u of the batch's points are in the graph already", S.host_flag[4]);
  }
  PhaseTimer tm;
  rc = tm.init(g->collect);
  if (rc) return rc;
  const void* pts = nullptr;
  rc = resolve_points(g, points_dev, st, &pts);
  if (rc) return rc;
  rc = batch_insert(g, pts, ids_host, S.qidx.as<u32>(), b, L, alpha, S, tm, st, /*sync=*/true);
  if (rc) return rc;
  rc = finish_batches(g, S, tm, st);
  return rc == ANN_LOST_LIST ? fail(ANN_EINTERNAL, "a visited list was lost in a synchronised batch") : rc;
} catch (...) {
  return annmi::on_exception();
}

int ann_graph_reserve(ann_graph* g, uint64_t n_cap, void* stream) try {
  if (!g) return fail(ANN_EINVAL, "null argument");
  return reserve_rows(g, n_cap, static_cast<hipStream_t>(stream));
} catch (...) {
  return annmi::on_exception();
}

int ann_insert_points(ann_graph* g, const void* points_dev, uint64_t n_total, uint32_t L, float alpha,
                      uint64_t seed, const ann_build_opts* opts, void* stream) try {
  if (!g || !points_dev) return fail(ANN_EINVAL, "null argument");
  int rc = check_insert_params(g, L, alpha);
  if (rc) return rc;
  if (n_total < g->n) return fail(ANN_EINVAL, "n_total is below the number of points in the graph");
  if (n_total >= (1ull << 31)) return fail(ANN_EINVAL, "n must stay below 2^31");
  ann_build_opts o{};
  if (opts) o = *opts;
  Allocator al = g->al;
  al.stream = stream;
  AllocScope scope(al);
  const u64 n_old = g->n, m = n_total - n_old;
  if (m == 0) return ANN_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool trace = getenv("ANN_TRACE_BUILD") != nullptr;  // wall-clock breakdown on stderr
  auto now_ms = [] {
    timespec ts;
    clock_gettime(CLOCK_MONOTONIC, &ts);
    return ts.tv_sec * 1e3 + ts.tv_nsec / 1e6;
  };
  const double t_begin = now_ms();

  // the new ids in the order they go in: as given, or shuffled like the ids of a build
  std::vector<u32> order(m);
  if (o.order) {
    std::vector<unsigned char> seen(m, 0);
    for (u64 i = 0; i < m; ++i) {
      const u32 id = o.order[i];
      if (id < n_old || id >= n_total || seen[id - n_old]) return fail(ANN_EINVAL, "order must list every new id once");
      seen[id - n_old] = 1;
      order[i] = id;
    }
  } else {
    for (u64 i = 0; i < m; ++i) order[i] = (u32)(n_old + i);
    shuffle_in_place(order.data(), m, seed);
  }

  // the schedule of the build carried on: a batch at most doubles what is there, theta caps it
  u64 theta = o.batch_cap ? o.batch_cap : (n_total / 50 > 1 ? n_total / 50 : 1);
  if (theta * g->R >= (1ull << 32)) theta = ((1ull << 32) - 1) / g->R;
  std::vector<u64> bounds{0};
  u64 bmax = 1;
  for (u64 taken = 0; taken < m;) {
    u64 size = (n_old - 1) + taken + 2;
    if (size > theta) size = theta;
    if (size > m - taken) size = m - taken;
    taken += size;
    bounds.push_back(taken);
    bmax = size > bmax ? size : bmax;
  }

  const double t_order = now_ms();
  rc = grow_graph(g, n_total, st);
  if (rc) return rc;
  const double t_grow = now_ms();
  BatchScratch* Sp = nullptr;
  rc = graph_scratch(g, bmax, L, st, &Sp);
  if (rc) return rc;
  BatchScratch& S = *Sp;
  PhaseTimer tm;
  rc = tm.init(g->collect);
  if (rc) return rc;
  const void* pts = nullptr;
  rc = resolve_points(g, points_dev, st, &pts);
  if (rc) return rc;
  const double t_alloc = now_ms();
  // Every batch waits on the host after step 1 (the check for visited lists that fit nowhere):
  // unlike a build, an insertion cannot start over from the empty graph.
  for (size_t r = 0; r + 1 < bounds.size(); ++r) {
    if (o.max_rounds && r >= o.max_rounds) break;
    const u64 lo = bounds[r], b = bounds[r + 1] - bounds[r];
    HIP_TRY(hipMemcpyAsync(S.qidx.p, order.data() + lo, b * 4, hipMemcpyHostToDevice, st));
    rc = batch_insert(g, pts, order.data() + lo, S.qidx.as<u32>(), b, L, alpha, S, tm, st, /*sync=*/true);
    if (rc) return rc;
  }
  rc = finish_batches(g, S, tm, st);
  if (trace)
    fprintf(stderr, "ann_insert_points: order %.2f ms, growth %.2f ms, scratch %.2f ms, %zu batches %.2f ms\n",
            t_order - t_begin, t_grow - t_order, t_alloc - t_grow, bounds.size() - 1, now_ms() - t_alloc);
  return rc == ANN_LOST_LIST ? fail(ANN_EINTERNAL, "a visited list was lost in a synchronised batch") : rc;
} catch (...) {
  return annmi::on_exception();
}

int ann_build(const void* points_dev, uint64_t n, uint32_t d, ann_dtype dtype, ann_metric metric, uint32_t R,
              uint32_t L, float alpha, uint64_t seed, const ann_build_opts* opts, void* stream, ann_graph** out) try {
  if (out) *out = nullptr;
  if (!points_dev || !out) return fail(ANN_EINVAL, "null argument");
  ann_build_opts o{};
  o.start = ANN_NONE;
  if (opts) o = *opts;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Allocator al;
  if (!allocator_from(o.alloc, o.free, o.alloc_user, stream, &al))
    return fail(ANN_EINVAL, "alloc and free must be given together");
  AllocScope scope(al);

  const bool trace = getenv("ANN_TRACE_BUILD") != nullptr;  // wall-clock breakdown on stderr
  auto now_ms = [] {
    timespec ts;
    clock_gettime(CLOCK_MONOTONIC, &ts);
    return ts.tv_sec * 1e3 + ts.tv_nsec / 1e6;
  };
  const double t_begin = now_ms();
  // Insertion order: the ids other than s, shuffled (Fisher-Yates from the front, driven by
  // SplitMix64).  The shuffle moves positions, whatever they hold, so it runs on the positions
  // 0..m-1 on a host thread (position j stands for the j-th id other than s) while the graph is
  // allocated and the GPU finds s, and goes on while the first batches run: its first `ready`
  // positions are final, and a batch waits only for its own.
  const u64 m = n ? n - 1 : 0;
  std::vector<u32> order(m && n < (1ull << 31) ? m : 1);
  // Large inputs (the shuffle of 10^8 positions takes the host half a second): page-locked
  // positions, handed to the device batch by batch while the shuffle goes on (from ordinary
  // memory every such copy would wait for the batch before it).  Small inputs: the shuffle is
  // over before the GPU has found s, page-locking would cost more than it saves, and the whole
  // order goes to the device in one copy.
  const bool stream_order = m >= (1ull << 23);
  HostBuf pos_buf;
  std::vector<u32> pos_vec;
  std::atomic<u64> ready{0};
  std::thread shuffler;
  u32* pos = nullptr;
  if (!o.order && n >= 1 && n < (1ull << 31)) {
    if (stream_order) {
      HIP_TRY(pos_buf.alloc(m * sizeof(u32)));
      pos = pos_buf.as<u32>();
    } else {
      pos_vec.resize(m ? m : 1);
      pos = pos_vec.data();
    }
    shuffler = std::thread([pos, &ready, m, seed] {
      for (u64 i = 0; i < m; ++i) pos[i] = (u32)i;
      shuffle_in_place(pos, m, seed, &ready);
    });
  }
  struct Joiner {
    std::thread& t;
    ~Joiner() {
      if (t.joinable()) t.join();
    }
  } joiner{shuffler};

  ann_graph* g = nullptr;
  int rc = new_graph(n, d, dtype, metric, R, &g);
  if (rc) return rc;
  struct Guard {
    ann_graph* g;
    ~Guard() {
      if (g) ann_graph_free(g);
    }
  } guard{g};
  rc = check_insert_params(g, L, alpha);
  if (rc) return rc;
  g->collect = o.collect_stats != 0;
  g->step1_parts = o.step1_parts;
  g->hash_bits = o.hash_bits;
  if (g->hash_bits && (g->hash_bits < 4 || g->hash_bits > 13)) return fail(ANN_EINVAL, "hash_bits must be in [4, 13]");
  g->visited_cap = o.visited_cap;
  g->spill_keys = o.spill_cap;
  HIP_TRY(hipMemsetAsync(g->rows, 0xFF, (size_t)n * R * sizeof(u32), st));

  // (scratch is allocated here, while the shuffle runs)
  // batches of 2, 4, 8, ... points, never more than theta
  u64 theta = o.batch_cap ? o.batch_cap : (n / 50 > 1 ? n / 50 : 1);
  if (theta * R >= (1ull << 32)) theta = ((1ull << 32) - 1) / R;
  std::vector<u64> bounds{0};
  for (u64 done = 0; done < m;) {
    u64 size = done + 2;
    if (size > theta) size = theta;
    if (size > m - done) size = m - done;
    done += size;
    bounds.push_back(done);
  }
  u64 bmax = 1;
  for (size_t r = 0; r + 1 < bounds.size(); ++r) bmax = bounds[r + 1] - bounds[r] > bmax ? bounds[r + 1] - bounds[r] : bmax;

  DevBuf order_dev;
  HIP_TRY(order_dev.alloc(m * 4));
  BatchScratch S;
  const u32 cap = g->visited_cap ? g->visited_cap : (4 * L > 256 ? 4 * L : 256);
  rc = S.alloc(bmax, R, cap, g->spill_keys ? g->spill_keys : default_spill_keys(bmax));
  if (rc) return rc;
  PhaseTimer tm;
  rc = tm.init(g->collect);
  if (rc) return rc;

  // start vertex s: present from the beginning with an empty row, never inserted again
  if (o.use_start) {
    if (o.start >= n) return fail(ANN_EINVAL, "start vertex out of range");
    g->start = o.start;
  } else {
    u32 s = 0;
    HIP_TRY(start_vertex_device(points_dev, n, d, dtype, st, &s));
    g->start = s;
  }

  const double t_start = now_ms();
  if (o.order) {
    std::vector<unsigned char> seen(n, 0);
    for (u64 i = 0; i < m; ++i) {
      const u32 id = o.order[i];
      if (id >= n || id == g->start || seen[id]) return fail(ANN_EINVAL, "order must list every id but the start once");
      seen[id] = 1;
      order[i] = id;
    }
  }
  // ids of the positions [lo, hi) of the order, on the host and on the device (waits for the
  // shuffle where it has not come that far yet)
  u64 filled = o.order ? m : 0;
  auto fill_order = [&](u64 hi) -> int {
    if (hi <= filled) return ANN_OK;
    while (ready.load(std::memory_order_acquire) < hi) std::this_thread::sleep_for(std::chrono::microseconds(20));
    const u32 s = g->start;
    for (u64 i = filled; i < hi; ++i) order[i] = pos[i] + (pos[i] >= s ? 1u : 0u);  // (the host's copy)
    const u64 cnt = hi - filled;
    HIP_TRY(hipMemcpyAsync(order_dev.as<u32>() + filled, pos + filled, cnt * 4, hipMemcpyHostToDevice, st));
    hipLaunchKernelGGL(skip_start_kernel, dim3((u32)((cnt + 255) / 256)), dim3(256), 0, st, order_dev.as<u32>() + filled,
                       cnt, s);
    HIP_TRY(hipGetLastError());
    filled = hi;
    return ANN_OK;
  };

  if (!o.order && !stream_order) {
    shuffler.join();
    const u32 s = g->start;
    for (u64 i = 0; i < m; ++i) order[i] = pos[i] + (pos[i] >= s ? 1u : 0u);
    filled = m;
  }
  const double t_order = now_ms();
  if (filled == m && m) HIP_TRY(hipMemcpyAsync(order_dev.p, order.data(), m * 4, hipMemcpyHostToDevice, st));
  const void* pts = nullptr;
  rc = resolve_points(g, points_dev, st, &pts);
  if (rc) return rc;

  const double t_alloc = now_ms();
  // First try: every batch is issued without waiting for the previous one.  A search whose
  // visited list fits neither its slot nor a spill chunk spoils that attempt (it is detected at
  // the end); the build is then repeated from the empty graph with a host check after step 1 of
  // every batch, which redoes such searches with as much room as they need.
  for (int attempt = 0; attempt < 2; ++attempt) {
    const bool sync = attempt == 1;
    for (size_t r = 0; r + 1 < bounds.size(); ++r) {
      if (o.max_rounds && r >= o.max_rounds) break;
      const u64 lo = bounds[r], b = bounds[r + 1] - bounds[r];
      rc = fill_order(bounds[r + 1]);
      if (rc) return rc;
      rc = batch_insert(g, pts, order.data() + lo, order_dev.as<u32>() + lo, b, L, alpha, S, tm, st, sync);
      if (rc) return rc;
    }
    rc = finish_batches(g, S, tm, st);
    if (rc != ANN_LOST_LIST) break;
    if (sync) return fail(ANN_EINTERNAL, "a visited list was lost in a synchronised batch");
    // start over
    HIP_TRY(hipMemsetAsync(g->rows, 0xFF, (size_t)n * R * sizeof(u32), st));
    HIP_TRY(hipMemsetAsync(g->meta, 0, (size_t)n * sizeof(u32), st));
    HIP_TRY(hipMemsetAsync(g->counters, 0, COUNTER_COPIES * sizeof(DevCounters), st));
    HIP_TRY(hipMemsetAsync(S.small.p, 0, 64, st));
    const u64 redone = g->stats.redone;
    g->stats = ann_stats{};
    g->stats.redone = redone;
    g->stats.restarts = 1;
    g->rounds = 0;
  }
  if (rc) return rc;
  if (trace)
    fprintf(stderr, "ann_build: graph alloc + start vertex %.2f ms, order %.2f ms, scratch %.2f ms, batches %.2f ms\n",
            t_start - t_begin, t_order - t_start, t_alloc - t_order, now_ms() - t_alloc);
  guard.g = nullptr;
  *out = g;
  return ANN_OK;
} catch (...) {
  return annmi::on_exception();
}

int ann_search(const ann_graph* g, const void* points_dev, const void* queries_dev, uint64_t nq, uint32_t k,
               uint32_t L, uint32_t* ids_dev, void* dists_dev, void* stream) {
  return ann_search_eps(g, points_dev, queries_dev, nq, k, L, -1.0f, ids_dev, dists_dev, stream);
}

int ann_search_eps(const ann_graph* g, const void* points_dev, const void* queries_dev, uint64_t nq, uint32_t k,
                   uint32_t L, float eps, uint32_t* ids_dev, void* dists_dev, void* stream) try {
  if (!g || !points_dev) return fail(ANN_EINVAL, "null argument");
  if (!(eps < 16384.0f)) return fail(ANN_EINVAL, "eps must be below 16384 (negative: no pruning)");
  if (nq == 0) return ANN_OK;
  if (!queries_dev || !ids_dev || !dists_dev) return fail(ANN_EINVAL, "null argument");
  if (k < 1 || k > L) return fail(ANN_EINVAL, "need 1 <= k <= L");
  if (L > 2048) return fail(ANN_EINVAL, "L must be at most 2048");
  if (nq >= (1ull << 31)) return fail(ANN_EINVAL, "too many queries");
  hipStream_t st_ = static_cast<hipStream_t>(stream);
  const void* pts = nullptr;
  const void* qsp = nullptr;
  int rc_ = resolve_points(g, points_dev, st_, &pts);
  if (rc_) return rc_;
  rc_ = resolve_queries(g, queries_dev, nq, st_, &qsp);
  if (rc_) return rc_;
  rc_ = query_launch(g, pts, qsp, nullptr, nq, k, L, eps, nullptr, ids_dev, dists_dev, st_);
  if (rc_) return rc_;
  return ANN_OK;
} catch (...) {
  return annmi::on_exception();
}

int ann_search_noalloc(const ann_graph* g, const void* points_dev, const void* queries_dev, uint64_t nq, uint32_t k,
                       uint32_t L, float eps, uint32_t* ids_dev, void* dists_dev, void* stream) try {
  if (!g || !points_dev) return fail(ANN_EINVAL, "null argument");
  if (!(eps < 16384.0f)) return fail(ANN_EINVAL, "eps must be below 16384 (negative: no pruning)");
  if (nq == 0) return ANN_OK;
  if (!queries_dev || !ids_dev || !dists_dev) return fail(ANN_EINVAL, "null argument");
  if (k < 1 || k > L) return fail(ANN_EINVAL, "need 1 <= k <= L");
  if (L > 2048) return fail(ANN_EINVAL, "L must be at most 2048");
  if (nq >= (1ull << 31)) return fail(ANN_EINVAL, "too many queries");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const void* pts = points_dev;
  const void* qsp = queries_dev;
  if (g->pad_stride) {
    // the padded copy of the points is the graph's, made by the build or by an earlier search
    if (g->pad_buf == nullptr || g->pad_src != points_dev || g->pad_done < g->n || g->pad_cap < g->n)
      return fail(ANN_EINVAL, "the graph holds no padded copy of this points array yet: ann_build makes it, and so "
                              "does one call of ann_search");
    if (nq * g->pad_stride > NOALLOC_SCRATCH_BYTES)
      return fail(ANN_EINVAL, "%llu queries of %llu padded bytes exceed the %d MiB this call can stage (at most %llu queries)",
                  (unsigned long long)nq, (unsigned long long)g->pad_stride, ANN_NOALLOC_SCRATCH_MIB,
                  (unsigned long long)(NOALLOC_SCRATCH_BYTES / g->pad_stride));
    void* sp = nullptr;
    int rc = noalloc_scratch(&sp);
    if (rc) return rc;
    // every word of the rows used is written (zero tails included): nothing of an earlier call shows
    rc = pad_rows(queries_dev, nq, g->d, sp, g->pad_stride, st);
    if (rc) return rc;
    pts = g->pad_buf;
    qsp = sp;
  }
  return query_launch(g, pts, qsp, nullptr, nq, k, L, eps, nullptr, ids_dev, dists_dev, st);
} catch (...) {
  return annmi::on_exception();
}

}  // extern "C"
