// The layered index of Sec. 4.2 (ParlayHNSW) on top of the kernels of the flat graph: every layer
// is a graph of its own that BatchInsert of Alg. 3 fills batch by batch, searched with beam 1 on
// the way down and with the full beam on the bottom layer.
//
// Layer 0 is a graph over the caller's points (degree bound 2m).  Layer l >= 1 holds the points of
// level >= l only (a fraction m^-l of them), so it is a graph over a compact copy of those points
// with ids of its own, 0..n_l-1 in ascending order of the global ids (so ties between distances
// break the same way in both numberings); every kernel of the flat graph runs on it unchanged.
// down[l][c] is the id that vertex c of layer l has one layer below.
//
// One batch: all its points search layer l with beam 1 from their current start vertices (the
// entry point at the top) and note the vertex they reach, mapped one layer down; the points that
// belong to layer l then search it again with beam efc and are inserted, and their note is
// replaced by the closest vertex that search visited.  Layer 0 is BatchInsert with those notes as
// start vertices.
#include <algorithm>

#include "driver_internal.hpp"

using namespace annmi;

struct ann_hnsw {
  u64 n = 0;
  u32 d = 0, m = 0;
  int dtype = 0, metric = 0;
  u32 top = 0;
  u32 entry = 0;  // global id
  u64 rounds = 0;
  u64 level_seed = 0;  // levels are a function of this seed and the point's id
  Allocator al;        // where the index's device memory comes from
  std::vector<u32> level;             // host, n
  std::vector<ann_graph*> layer;      // 0..top
  std::vector<std::vector<u32>> ids;  // ids[l], l >= 1: global ids of the layer's vertices, ascending
  std::vector<DevBuf> pts;            // pts[l], l >= 1: the layer's vectors, n_l x d
  std::vector<DevBuf> down;           // down[l], l >= 1: n_l ids one layer below
  std::vector<u32> entry_c;           // the entry point's id on every layer
  DevBuf walk;  // the upper layers, from the top, as the descent kernel reads them (DescendLayer)
  // where each query of a call enters the bottom layer
  mutable DevBuf qcur;
  mutable u64 qcur_cap = 0;
};

namespace {

u64 level_draw(u64 seed, u64 id) {  // the (id+1)-th output of SplitMix64(seed)
  u64 z = seed + (id + 1) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// largest l with r <= floor((2^64 - 1) / m^l): P(level >= l) = m^-l
u32 level_of(u64 r, u32 m) {
  u32 l = 0;
  for (u64 t = ~0ull / m; t != 0 && r <= t; t /= m) ++l;
  return l;
}

__global__ __launch_bounds__(256) void gather_rows_kernel(const unsigned char* src, const u32* ids, u64 nrows,
                                                          u32 row_bytes, unsigned char* dst) {
  const u64 t = (u64)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= nrows * row_bytes) return;
  const u64 r = t / row_bytes;
  const u32 c = (u32)(t % row_bytes);
  dst[t] = src[(u64)ids[r] * row_bytes + c];
}

__global__ __launch_bounds__(256) void fill_u32_kernel(u32* p, u64 count, u32 v) {
  const u64 t = (u64)blockIdx.x * blockDim.x + threadIdx.x;
  if (t < count) p[t] = v;
}

int fill_u32(u32* p, u64 count, u32 v, hipStream_t st) {
  if (count == 0) return ANN_OK;
  hipLaunchKernelGGL(fill_u32_kernel, dim3((u32)((count + 255) / 256)), dim3(256), 0, st, p, count, v);
  HIP_TRY(hipGetLastError());
  return ANN_OK;
}

void free_hnsw(ann_hnsw* h) {
  if (!h) return;
  for (ann_graph* g : h->layer)
    if (g) ann_graph_free(g);
  delete h;
}

int reset_layers(ann_hnsw* h, hipStream_t st) {
  for (ann_graph* g : h->layer) {
    HIP_TRY(hipMemsetAsync(g->rows, 0xFF, (size_t)g->n * g->R * sizeof(u32), st));
    HIP_TRY(hipMemsetAsync(g->meta, 0, (size_t)g->n * sizeof(u32), st));
    HIP_TRY(hipMemsetAsync(g->counters, 0, COUNTER_COPIES * sizeof(DevCounters), st));
    const u64 redone = g->stats.redone;
    g->stats = ann_stats{};
    g->stats.redone = redone;
    g->rounds = 0;
  }
  return ANN_OK;
}

// The layers of an index whose levels and entry point are set: vertices, compact vectors, maps
// one layer down, empty rows.
int make_layers(ann_hnsw* h, const void* points_dev, hipStream_t st) {
  const u32 top = h->top, m = h->m, d = h->d;
  const u64 n = h->n;
  h->layer.assign(top + 1, nullptr);
  h->ids.resize(top + 1);
  h->pts.resize(top + 1);
  h->down.resize(top + 1);
  h->entry_c.assign(top + 1, 0);
  const u64 esz = h->dtype == ANN_F32 ? 4 : 1;
  int rc = new_graph(n, d, h->dtype, h->metric, 2 * m, &h->layer[0]);
  if (rc) return rc;
  for (u32 l = 1; l <= top; ++l)
    for (u64 i = 0; i < n; ++i)
      if (h->level[i] >= l) h->ids[l].push_back((u32)i);
  for (u32 l = 1; l <= top; ++l) {
    const std::vector<u32>& mine = h->ids[l];
    const u64 nl = mine.size();
    rc = new_graph(nl, d, h->dtype, h->metric, m, &h->layer[l]);
    if (rc) return rc;
    std::vector<u32> dn(nl);
    if (l == 1) {
      dn = mine;
    } else {
      const std::vector<u32>& below = h->ids[l - 1];
      u64 j = 0;
      for (u64 c = 0; c < nl; ++c) {
        while (below[j] != mine[c]) ++j;  // both ascending, mine is a subset
        dn[c] = (u32)j;
      }
    }
    DevBuf idsd;
    HIP_TRY(idsd.alloc(nl * 4));
    HIP_TRY(hipMemcpyAsync(idsd.p, mine.data(), nl * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(h->down[l].alloc(nl * 4));
    HIP_TRY(hipMemcpyAsync(h->down[l].p, dn.data(), nl * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(h->pts[l].alloc(nl * d * esz));
    const u64 bytes = nl * d * esz;
    hipLaunchKernelGGL(gather_rows_kernel, dim3((u32)((bytes + 255) / 256)), dim3(256), 0, st,
                       static_cast<const unsigned char*>(points_dev), idsd.as<u32>(), nl, (u32)(d * esz),
                       h->pts[l].as<unsigned char>());
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(st));  // idsd and the host vectors go out of scope
    h->entry_c[l] = (u32)(std::lower_bound(mine.begin(), mine.end(), h->entry) - mine.begin());
  }
  h->entry_c[0] = h->entry;
  for (u32 l = 0; l <= top; ++l) {
    ann_graph* g = h->layer[l];
    g->start = h->entry_c[l];
    HIP_TRY(hipMemsetAsync(g->rows, 0xFF, (size_t)g->n * g->R * sizeof(u32), st));
  }
  return ANN_OK;
}

// The table the descent kernel reads: the upper layers from the top.
int make_walk(ann_hnsw* h, hipStream_t st) {
  if (h->top == 0) return ANN_OK;
  std::vector<DescendLayer> walk;
  for (u32 l = h->top; l >= 1; --l) {
    const void* pl = nullptr;
    int rc = resolve_points(h->layer[l], h->pts[l].p, st, &pl);
    if (rc) return rc;
    DescendLayer y{};
    y.points = static_cast<const char*>(pl);
    y.graph = h->layer[l]->rows;
    y.down = h->down[l].as<u32>();
    y.R = h->m;
    walk.push_back(y);
  }
  HIP_TRY(h->walk.alloc(walk.size() * sizeof(DescendLayer)));
  HIP_TRY(hipMemcpy(h->walk.p, walk.data(), walk.size() * sizeof(DescendLayer), hipMemcpyHostToDevice));
  return ANN_OK;
}

// The batches bounds[r]..bounds[r+1] of `order` go into the index.  With may_restart the first
// attempt runs without host waits and, if a search lost its visited list, every layer is emptied
// and the run repeated with a host check in every batch (a build); without it the one run has
// those checks (insertion into an index that cannot be started over).
int run_batches(ann_hnsw* h, const void* points_dev, const std::vector<u32>& order, const std::vector<u64>& bounds,
                u32 efc, float alpha, u64 max_rounds, bool collect, bool may_restart, hipStream_t st) {
  const u32 top = h->top, m = h->m;
  const size_t nrounds = bounds.size() - 1;
  const u64 cnt = bounds.back();
  u64 bmax = 1;
  for (size_t r = 0; r < nrounds; ++r) bmax = std::max(bmax, bounds[r + 1] - bounds[r]);
  int rc = ANN_OK;
  // per layer l >= 1: the batch points that belong to it, batch after batch: their ids on that
  // layer and their positions in their batch
  std::vector<std::vector<u32>> ins_c(top + 1), ins_slot(top + 1);
  std::vector<std::vector<u64>> ins_off(top + 1, std::vector<u64>(nrounds + 1, 0));
  for (size_t r = 0; r < nrounds; ++r) {
    for (u64 i = bounds[r]; i < bounds[r + 1]; ++i) {
      const u32 p = order[i];
      for (u32 l = 1; l <= h->level[p]; ++l) {
        const std::vector<u32>& mine = h->ids[l];
        ins_c[l].push_back((u32)(std::lower_bound(mine.begin(), mine.end(), p) - mine.begin()));
        ins_slot[l].push_back((u32)(i - bounds[r]));
      }
    }
    for (u32 l = 1; l <= top; ++l) ins_off[l][r + 1] = ins_c[l].size();
  }
  DevBuf order_dev;
  std::vector<DevBuf> ins_c_dev(top + 1), ins_slot_dev(top + 1);
  HIP_TRY(order_dev.alloc(cnt * 4));
  if (cnt) HIP_TRY(hipMemcpyAsync(order_dev.p, order.data(), cnt * 4, hipMemcpyHostToDevice, st));
  for (u32 l = 1; l <= top; ++l) {
    const u64 k = ins_c[l].size();
    HIP_TRY(ins_c_dev[l].alloc(k * 4));
    HIP_TRY(ins_slot_dev[l].alloc(k * 4));
    if (k) {
      HIP_TRY(hipMemcpyAsync(ins_c_dev[l].p, ins_c[l].data(), k * 4, hipMemcpyHostToDevice, st));
      HIP_TRY(hipMemcpyAsync(ins_slot_dev[l].p, ins_slot[l].data(), k * 4, hipMemcpyHostToDevice, st));
    }
  }

  // Two scratch areas and two streams: the upper layers of a batch do not depend on layer 0, so
  // they run on a stream of their own, up to two batches ahead of the bottom layer's stream, and
  // their small kernels fill the gaps the large ones leave.
  constexpr int RING = 2;
  BatchScratch S0, Su;
  const u32 vcap = 4 * efc > 256 ? 4 * efc : 256;
  rc = S0.alloc(bmax, 2 * m, vcap, default_spill_keys(bmax));
  if (rc) return rc;
  u64 bup = 1;
  for (u32 l = 1; l <= top; ++l)
    for (size_t r = 0; r < nrounds; ++r) bup = std::max(bup, ins_off[l][r + 1] - ins_off[l][r]);
  if (top > 0) {
    rc = Su.alloc(bup, m, vcap, default_spill_keys(bup), /*with_side=*/false);
    if (rc) return rc;
  }
  struct UpStream {
    hipStream_t s = nullptr;
    hipEvent_t cur_ready[RING] = {}, cur_free[RING] = {}, setup = nullptr;
    ~UpStream() {
      if (s) (void)hipStreamDestroy(s);
      for (auto& e : cur_ready)
        if (e) (void)hipEventDestroy(e);
      for (auto& e : cur_free)
        if (e) (void)hipEventDestroy(e);
      if (setup) (void)hipEventDestroy(setup);
    }
  } us;
  DevBuf cur_a[RING], cur_b[RING];
  if (top > 0) {
    HIP_TRY(hipStreamCreateWithFlags(&us.s, hipStreamNonBlocking));
    HIP_TRY(hipEventCreateWithFlags(&us.setup, hipEventDisableTiming));
    for (int k = 0; k < RING; ++k) {
      HIP_TRY(hipEventCreateWithFlags(&us.cur_ready[k], hipEventDisableTiming));
      HIP_TRY(hipEventCreateWithFlags(&us.cur_free[k], hipEventDisableTiming));
      HIP_TRY(cur_a[k].alloc(bmax * 4));
      HIP_TRY(cur_b[k].alloc(bmax * 4));
    }
  }
  PhaseTimer tm, tm_off;
  rc = tm.init(collect);
  if (rc) return rc;
  (void)tm_off.init(false);

  // what the kernels read: the layers' vectors (padded copies where the row size asks for it)
  std::vector<const void*> lp(top + 1, nullptr);
  rc = resolve_points(h->layer[0], points_dev, st, &lp[0]);
  if (rc) return rc;
  for (u32 l = 1; l <= top; ++l) {
    rc = resolve_points(h->layer[l], h->pts[l].p, st, &lp[l]);
    if (rc) return rc;
  }

  for (int attempt = may_restart ? 0 : 1; attempt < 2; ++attempt) {
    const bool sync = attempt == 1;
    // the second attempt waits on the host in every batch: one stream serves it
    hipStream_t up = sync ? st : us.s;
    if (top > 0) {
      HIP_TRY(hipEventRecord(us.setup, st));
      HIP_TRY(hipStreamWaitEvent(up, us.setup, 0));
    }
    for (size_t r = 0; r < nrounds; ++r) {
      if (max_rounds && r >= max_rounds) break;
      const u64 lo = bounds[r], b = bounds[r + 1] - bounds[r];
      const int k = (int)(r % RING);
      u32* cur = cur_a[k].as<u32>();
      u32* nxt = cur_b[k].as<u32>();
      if (top > 0) {
        // this pair of arrays was last read by the bottom layer's search RING batches ago
        if (r >= (size_t)RING) HIP_TRY(hipStreamWaitEvent(up, us.cur_free[k], 0));
        rc = fill_u32(cur, b, h->entry_c[top], up);
        if (rc) return rc;
      }
      for (u32 l = top; l >= 1; --l) {
        ann_graph* g = h->layer[l];
        // everyone: beam 1 from the current start vertex, over the layer as it stands
        StartsArgs sd;
        sd.cur = cur;
        sd.next = nxt;
        sd.down = h->down[l].as<u32>();
        rc = query_launch(g, lp[l], lp[0], order_dev.as<u32>() + lo, b, 1, 1, -1.0f, &sd, nullptr, nullptr, up);
        if (rc) return rc;
        // the layer's own points: BatchInsert from the same start vertices
        const u64 i0 = ins_off[l][r], bl = ins_off[l][r + 1] - i0;
        if (bl) {
          StartsArgs si = sd;
          si.slot = ins_slot_dev[l].as<u32>() + i0;
          si.slot_host = ins_slot[l].data() + i0;
          rc = batch_insert(g, lp[l], ins_c[l].data() + i0, ins_c_dev[l].as<u32>() + i0, bl, efc, alpha, Su, tm_off, up,
                            sync, &si);
          if (rc) return rc;
        }
        std::swap(cur, nxt);
      }
      if (top > 0) {
        HIP_TRY(hipEventRecord(us.cur_ready[k], up));
        HIP_TRY(hipStreamWaitEvent(st, us.cur_ready[k], 0));
      }
      StartsArgs s0;
      s0.cur = cur;
      rc = batch_insert(h->layer[0], lp[0], order.data() + lo, order_dev.as<u32>() + lo, b, efc, alpha, S0, tm, st, sync,
                        top > 0 ? &s0 : nullptr);
      if (rc) return rc;
      if (top > 0) HIP_TRY(hipEventRecord(us.cur_free[k], st));
      h->rounds += 1;
    }
    // the bottom layer's stream has waited for everything the other one was given
    rc = finish_batches(h->layer[0], S0, tm, st);
    if (top > 0 && (rc == ANN_OK || rc == ANN_LOST_LIST)) {
      const int rc_up = finish_batches(h->layer[1], Su, tm_off, st);
      if (rc_up != ANN_OK) rc = rc_up;
    }
    if (rc != ANN_LOST_LIST) break;
    if (sync) return fail(ANN_EINTERNAL, "a visited list was lost in a synchronised batch");
    rc = reset_layers(h, st);  // start over, waiting after step 1 of every batch
    if (rc) return rc;
    HIP_TRY(hipMemsetAsync(S0.small.p, 0, 64, st));
    if (top > 0) HIP_TRY(hipMemsetAsync(Su.small.p, 0, 64, st));
    h->layer[0]->stats.restarts = 1;
    h->rounds = 0;
  }
  if (rc) return rc;
  return rc;
}

}  // namespace

extern "C" {

void ann_hnsw_free(ann_hnsw* h) { free_hnsw(h); }

int ann_hnsw_build(const void* points_dev, uint64_t n, uint32_t d, ann_dtype dtype, ann_metric metric, uint32_t m,
                   uint32_t efc, float alpha, uint64_t seed, const ann_hnsw_opts* opts, void* stream,
                   ann_hnsw** out) try {
  if (out) *out = nullptr;
  if (!points_dev || !out) return fail(ANN_EINVAL, "null argument");
  if (m < 2 || m > 256) return fail(ANN_EINVAL, "m must be in [2, 256]");
  if (n < 1 || n >= (1ull << 31)) return fail(ANN_EINVAL, "n must be in [1, 2^31)");
  ann_hnsw_opts o{};
  if (opts) o = *opts;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Allocator al;
  if (!allocator_from(o.alloc, o.free, o.alloc_user, stream, &al))
    return fail(ANN_EINVAL, "alloc and free must be given together");
  AllocScope scope(al);

  ann_hnsw* h = new (std::nothrow) ann_hnsw();
  if (!h) return fail(ANN_ENOMEM, "host allocation failed");
  struct Guard {
    ann_hnsw* h;
    ~Guard() { free_hnsw(h); }
  } guard{h};
  h->al = al;
  h->n = n;
  h->d = d;
  h->m = m;
  h->dtype = dtype;
  h->metric = metric;
  h->level_seed = seed;

  // levels (several host threads: a hundred million draws take a third of a second on one)
  h->level.resize(n);
  if (o.level) {
    for (u64 i = 0; i < n; ++i) {
      if (o.level[i] > 63) return fail(ANN_EINVAL, "levels must be at most 63");
      h->level[i] = o.level[i];
    }
  } else {
    const unsigned nt = n < 200000 ? 1u : 8u;
    std::vector<std::thread> workers;
    u32* lv = h->level.data();
    for (unsigned t = 0; t < nt; ++t)
      workers.emplace_back([=] {
        for (u64 i = n * t / nt; i < n * (t + 1) / nt; ++i) lv[i] = level_of(level_draw(seed, i), m);
      });
    for (auto& w : workers) w.join();
  }
  // entry point: highest level, smallest id
  h->entry = 0;
  for (u64 i = 1; i < n; ++i)
    if (h->level[i] > h->level[h->entry]) h->entry = (u32)i;
  h->top = h->level[h->entry];

  // insertion order: the ids other than the entry point, shuffled as in ann_build
  const u64 cnt = n - 1;
  std::vector<u32> order(cnt ? cnt : 1);
  if (o.order) {
    std::vector<unsigned char> seen(n, 0);
    for (u64 i = 0; i < cnt; ++i) {
      const u32 id = o.order[i];
      if (id >= n || id == h->entry || seen[id])
        return fail(ANN_EINVAL, "order must list every id but the entry point once");
      seen[id] = 1;
      order[i] = id;
    }
  } else {
    for (u64 i = 0; i < cnt; ++i) order[i] = (u32)i;
    shuffle_in_place(order.data(), cnt, seed);
    for (u64 i = 0; i < cnt; ++i) order[i] += order[i] >= h->entry ? 1u : 0u;
  }

  int rc = make_layers(h, points_dev, st);
  if (rc) return rc;
  rc = check_insert_params(h->layer[0], efc, alpha);
  if (rc) return rc;
  for (ann_graph* g : h->layer) g->collect = o.collect_stats != 0;

  // schedule of Alg. 3
  u64 theta = o.batch_cap ? o.batch_cap : (n / 50 > 1 ? n / 50 : 1);
  if (theta * 2 * m >= (1ull << 32)) theta = ((1ull << 32) - 1) / (2 * m);
  std::vector<u64> bounds{0};
  for (u64 done = 0; done < cnt;) {
    u64 size = done + 2;
    if (size > theta) size = theta;
    if (size > cnt - done) size = cnt - done;
    done += size;
    bounds.push_back(done);
  }
  rc = run_batches(h, points_dev, order, bounds, efc, alpha, o.max_rounds, o.collect_stats != 0, /*may_restart=*/true, st);
  if (rc) return rc;
  rc = make_walk(h, st);
  if (rc) return rc;
  guard.h = nullptr;
  *out = h;
  return ANN_OK;
} catch (...) {
  return annmi::on_exception();
}

int ann_hnsw_insert_points(ann_hnsw* h, const void* points_dev, uint64_t n_total, uint32_t efc, float alpha,
                           uint64_t seed, const ann_hnsw_opts* opts, void* stream) try {
  if (!h || !points_dev) return fail(ANN_EINVAL, "null argument");
  int rc = check_insert_params(h->layer[0], efc, alpha);
  if (rc) return rc;
  if (n_total < h->n) return fail(ANN_EINVAL, "n_total is below the number of points in the index");
  if (n_total >= (1ull << 31)) return fail(ANN_EINVAL, "n must stay below 2^31");
  ann_hnsw_opts o{};
  if (opts) o = *opts;
  const u64 n_old = h->n, mnew = n_total - n_old;
  if (mnew == 0) return ANN_OK;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Allocator al = h->al;
  al.stream = stream;
  AllocScope scope(al);
  const u32 top = h->top, m = h->m, d = h->d;
  const u64 esz = h->dtype == ANN_F32 ? 4 : 1;

  // levels of the new points, by the index's own rule, none above the index's highest layer
  std::vector<u32> lv(mnew);
  for (u64 i = 0; i < mnew; ++i) {
    u32 x = o.level ? o.level[i] : level_of(level_draw(h->level_seed, n_old + i), m);
    lv[i] = x > top ? top : x;
  }
  // their order: as given, or shuffled like the ids of a build
  std::vector<u32> order(mnew);
  if (o.order) {
    std::vector<unsigned char> seen(mnew, 0);
    for (u64 i = 0; i < mnew; ++i) {
      const u32 id = o.order[i];
      if (id < n_old || id >= n_total || seen[id - n_old]) return fail(ANN_EINVAL, "order must list every new id once");
      seen[id - n_old] = 1;
      order[i] = id;
    }
  } else {
    for (u64 i = 0; i < mnew; ++i) order[i] = (u32)(n_old + i);
    shuffle_in_place(order.data(), mnew, seed);
  }
  // the build's schedule carried on
  u64 theta = o.batch_cap ? o.batch_cap : (n_total / 50 > 1 ? n_total / 50 : 1);
  if (theta * 2 * m >= (1ull << 32)) theta = ((1ull << 32) - 1) / (2 * m);
  std::vector<u64> bounds{0};
  for (u64 taken = 0; taken < mnew;) {
    u64 size = (n_old - 1) + taken + 2;
    if (size > theta) size = theta;
    if (size > mnew - taken) size = mnew - taken;
    taken += size;
    bounds.push_back(taken);
  }

  // the layers grow: new members go behind the old ones (their ids are larger), so every vertex
  // keeps its number on every layer
  h->level.insert(h->level.end(), lv.begin(), lv.end());
  rc = grow_graph(h->layer[0], n_total, st);
  if (rc) return rc;
  for (u32 l = 1; l <= top; ++l) {
    std::vector<u32> fresh;
    for (u64 i = 0; i < mnew; ++i)
      if (lv[i] >= l) fresh.push_back((u32)(n_old + i));
    if (fresh.empty()) continue;
    std::vector<u32>& mine = h->ids[l];
    const u64 nl0 = mine.size(), nl1 = nl0 + fresh.size();
    std::vector<u32> dn(fresh.size());
    for (size_t c = 0; c < fresh.size(); ++c) {
      if (l == 1) {
        dn[c] = fresh[c];
      } else {
        const std::vector<u32>& below = h->ids[l - 1];  // already grown
        dn[c] = (u32)(std::lower_bound(below.begin(), below.end(), fresh[c]) - below.begin());
      }
    }
    mine.insert(mine.end(), fresh.begin(), fresh.end());
    rc = grow_graph(h->layer[l], nl1, st);
    if (rc) return rc;
    DevBuf npts, ndown, idsd;
    HIP_TRY(npts.alloc(nl1 * d * esz));
    HIP_TRY(ndown.alloc(nl1 * 4));
    HIP_TRY(idsd.alloc(fresh.size() * 4));
    HIP_TRY(hipMemcpyAsync(npts.p, h->pts[l].p, nl0 * d * esz, hipMemcpyDeviceToDevice, st));
    HIP_TRY(hipMemcpyAsync(ndown.p, h->down[l].p, nl0 * 4, hipMemcpyDeviceToDevice, st));
    HIP_TRY(hipMemcpyAsync(ndown.as<u32>() + nl0, dn.data(), dn.size() * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(hipMemcpyAsync(idsd.p, fresh.data(), fresh.size() * 4, hipMemcpyHostToDevice, st));
    const u64 bytes = fresh.size() * d * esz;
    hipLaunchKernelGGL(gather_rows_kernel, dim3((u32)((bytes + 255) / 256)), dim3(256), 0, st,
                       static_cast<const unsigned char*>(points_dev), idsd.as<u32>(), (u64)fresh.size(), (u32)(d * esz),
                       npts.as<unsigned char>() + nl0 * d * esz);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipDeviceSynchronize());  // the old arrays may still be read; the host vectors go out of scope
    h->pts[l] = std::move(npts);
    h->down[l] = std::move(ndown);
  }
  h->n = n_total;
  rc = make_walk(h, st);
  if (rc) return rc;
  return run_batches(h, points_dev, order, bounds, efc, alpha, o.max_rounds, h->layer[0]->collect, /*may_restart=*/false,
                     st);
} catch (...) {
  return annmi::on_exception();
}

int ann_hnsw_from_host(const void* points_dev, uint64_t n, uint32_t d, ann_dtype dtype, ann_metric metric, uint32_t m,
                       const uint32_t* level_host, uint32_t entry, const uint32_t* const* rows_host, void* stream,
                       ann_hnsw** out) try {
  if (out) *out = nullptr;
  if (!points_dev || !out || !level_host || !rows_host) return fail(ANN_EINVAL, "null argument");
  if (m < 2 || m > 256) return fail(ANN_EINVAL, "m must be in [2, 256]");
  if (n < 1 || n >= (1ull << 31)) return fail(ANN_EINVAL, "n must be in [1, 2^31)");
  if (entry >= n) return fail(ANN_EINVAL, "entry point out of range");
  hipStream_t st = static_cast<hipStream_t>(stream);
  ann_hnsw* h = new (std::nothrow) ann_hnsw();
  if (!h) return fail(ANN_ENOMEM, "host allocation failed");
  struct Guard {
    ann_hnsw* h;
    ~Guard() { free_hnsw(h); }
  } guard{h};
  h->n = n;
  h->d = d;
  h->m = m;
  h->dtype = dtype;
  h->metric = metric;
  h->entry = entry;
  h->level.assign(level_host, level_host + n);
  u32 top = 0;
  for (u64 i = 0; i < n; ++i) {
    if (h->level[i] > 63) return fail(ANN_EINVAL, "levels must be at most 63");
    top = h->level[i] > top ? h->level[i] : top;
  }
  if (h->level[entry] != top) return fail(ANN_EINVAL, "the entry point must be on the highest layer");
  h->top = top;
  for (u32 l = 0; l <= top; ++l)
    if (!rows_host[l]) return fail(ANN_EINVAL, "null layer");
  int rc = make_layers(h, points_dev, st);
  if (rc) return rc;
  // rows: ids of members of the layer only, translated to the layer's own numbering
  for (u32 l = 0; l <= top; ++l) {
    ann_graph* g = h->layer[l];
    const u32 R = g->R;
    const std::vector<u32>& mine = h->ids[l];
    std::vector<u32> rows((size_t)g->n * R, ANN_NONE);
    for (u64 c = 0; c < g->n; ++c) {
      const u64 p = l ? mine[c] : c;
      const u32* src = rows_host[l] + p * R;
      u32 deg = 0;
      for (u32 j = 0; j < R && src[j] != ANN_NONE; ++j) {
        const u32 q = src[j];
        if (q >= n || h->level[q] < l) return fail(ANN_EINVAL, "neighbour id out of range or not on the layer");
        rows[c * R + deg++] = l ? (u32)(std::lower_bound(mine.begin(), mine.end(), q) - mine.begin()) : q;
      }
    }
    HIP_TRY(hipMemcpyAsync(g->rows, rows.data(), rows.size() * sizeof(u32), hipMemcpyHostToDevice, st));
    HIP_TRY(launch_meta_from_rows(g->rows, g->n, R, g->meta, st));
    HIP_TRY(hipStreamSynchronize(st));
  }
  rc = make_walk(h, st);
  if (rc) return rc;
  guard.h = nullptr;
  *out = h;
  return ANN_OK;
} catch (...) {
  return annmi::on_exception();
}

int ann_hnsw_search(const ann_hnsw* h, const void* points_dev, const void* queries_dev, uint64_t nq, uint32_t k,
                    uint32_t L, float eps, uint32_t* ids_dev, void* dists_dev, void* stream) try {
  if (!h || !points_dev) return fail(ANN_EINVAL, "null argument");
  if (!(eps < 16384.0f)) return fail(ANN_EINVAL, "eps must be below 16384 (negative: no pruning)");
  if (nq == 0) return ANN_OK;
  if (!queries_dev || !ids_dev || !dists_dev) return fail(ANN_EINVAL, "null argument");
  if (k < 1 || k > L) return fail(ANN_EINVAL, "need 1 <= k <= L");
  if (L > 2048) return fail(ANN_EINVAL, "L must be at most 2048");
  if (nq >= (1ull << 31)) return fail(ANN_EINVAL, "too many queries");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const ann_graph* g0 = h->layer[0];
  const void* p0 = nullptr;
  const void* qs = nullptr;
  int rc = resolve_points(g0, points_dev, st, &p0);
  if (rc) return rc;
  rc = resolve_queries(g0, queries_dev, nq, st, &qs);
  if (rc) return rc;
  if (h->top == 0) return query_launch(g0, p0, qs, nullptr, nq, k, L, eps, nullptr, ids_dev, dists_dev, st);
  if (h->qcur_cap < nq) {
    HIP_TRY(hipDeviceSynchronize());  // an earlier call, on whatever stream, may still use the old array
    Allocator al = h->al;
    al.stream = stream;
    AllocScope scope(al);
    HIP_TRY(h->qcur.alloc(nq * 4));
    h->qcur_cap = nq;
  }
  // the upper layers in one launch, then the bottom layer from where each query arrived
  DescendArgs da{};
  da.queries = static_cast<const char*>(qs);
  da.qrow_bytes = g0->cfg.row_bytes;
  da.nq = (u32)nq;
  da.nlayers = h->top;
  da.entry = h->entry_c[h->top];
  da.layers = h->walk.as<DescendLayer>();
  da.out = h->qcur.as<u32>();
  HIP_TRY(launch_descend(g0->cfg, da, st));
  StartsArgs s0;
  s0.cur = h->qcur.as<u32>();
  return query_launch(g0, p0, qs, nullptr, nq, k, L, eps, &s0, ids_dev, dists_dev, st);
} catch (...) {
  return annmi::on_exception();
}

int ann_hnsw_info(const ann_hnsw* h, ann_hnsw_info_t* info) try {
  if (!h || !info) return fail(ANN_EINVAL, "null argument");
  info->n = h->n;
  info->d = h->d;
  info->m = h->m;
  info->dtype = (uint32_t)h->dtype;
  info->metric = (uint32_t)h->metric;
  info->top = h->top;
  info->entry = h->entry;
  info->rounds = h->rounds;
  return ANN_OK;
} catch (...) {
  return annmi::on_exception();
}

int ann_hnsw_copy_levels(const ann_hnsw* h, uint32_t* level_host) try {
  if (!h || !level_host) return fail(ANN_EINVAL, "null argument");
  memcpy(level_host, h->level.data(), h->n * sizeof(u32));
  return ANN_OK;
} catch (...) {
  return annmi::on_exception();
}

int ann_hnsw_layer_size(const ann_hnsw* h, uint32_t layer, uint64_t* count) try {
  if (!h || !count) return fail(ANN_EINVAL, "null argument");
  if (layer > h->top) return fail(ANN_EINVAL, "no such layer");
  *count = h->layer[layer]->n;
  return ANN_OK;
} catch (...) {
  return annmi::on_exception();
}

int ann_hnsw_copy_layer(const ann_hnsw* h, uint32_t layer, uint32_t* ids_host, uint32_t* rows_host) try {
  if (!h || !ids_host || !rows_host) return fail(ANN_EINVAL, "null argument");
  if (layer > h->top) return fail(ANN_EINVAL, "no such layer");
  const ann_graph* g = h->layer[layer];
  HIP_TRY(hipMemcpy(rows_host, g->rows, (size_t)g->n * g->R * sizeof(u32), hipMemcpyDeviceToHost));
  if (layer == 0) {
    for (u64 i = 0; i < g->n; ++i) ids_host[i] = (u32)i;
    return ANN_OK;
  }
  const std::vector<u32>& mine = h->ids[layer];
  memcpy(ids_host, mine.data(), mine.size() * sizeof(u32));
  for (u64 i = 0; i < g->n * g->R; ++i)
    if (rows_host[i] != ANN_NONE) rows_host[i] = mine[rows_host[i]];
  return ANN_OK;
} catch (...) {
  return annmi::on_exception();
}

int ann_hnsw_get_stats(const ann_hnsw* h, uint32_t layer, ann_stats* stats) try {
  if (!h || !stats) return fail(ANN_EINVAL, "null argument");
  if (layer > h->top) return fail(ANN_EINVAL, "no such layer");
  return ann_get_stats(h->layer[layer], stats);
} catch (...) {
  return annmi::on_exception();
}

}  // extern "C"
