// Wavefront-parallel alpha-prune (Sec. 4.1 of the paper) and the two places BatchInsert (Alg. 3)
// uses it: step 1, prune(p, V, R) for every batch point, and step 2, the merge of reversed edges
// into existing rows with a re-prune of the rows that overflow R.
//
// prune(p, C, R) is stated as a scan over C sorted by distance to p.  The same result is
// obtained without sorting: the next selected point is always the (distance, id)-minimum of the
// candidates that are still alive, because every candidate ahead of it in sorted order has been
// selected or removed.  One wave keeps the alive candidates as a compact array of keys, takes the
// minimum with a wave reduction, and tests the others against it eight at a time.
#include "ann_device.hpp"
#include "ann_internal.hpp"
#include "ann_dispatch.hpp"

namespace annmi {

// Select at most R of cand[0..m) (keys with the distance to p; ids distinct, p absent).
// Selected ids go to out[0..return) in selection order.  cand is overwritten.
template <int KIND, int VEC, int NCH>
__device__ __forceinline__ u32 robust_prune(const VecTable& T, u64* cand, u32 m, u32 R, const AlphaParam& al,
                                            u32* out, int lane, u32& pair_evals) {
  u32 nout = 0;
  while (m > 0) {
    u64 best = KEY_INF;
    for (u32 i = lane; i < m; i += 64) {
      const u64 k = cand[i];
      best = k < best ? k : best;
    }
    best = wave_min_u64(best);
    const u32 bid = key_id(best);
    if (lane == 0) out[nout] = bid;
    ++nout;
    if (nout == R) break;

    const QueryRegs<KIND, VEC, NCH> S =
        load_query<KIND, VEC, NCH>(T.base + (u64)bid * T.row_bytes, T.npieces, lane);
    u32 w = 0;
    for (u32 base = 0; base < m; base += 64) {
      const u32 cnt = m - base < 64u ? m - base : 64u;
      const u32 c = cand_of_lane(lane);
      const u64 mykey = c < cnt ? cand[base + c] : KEY_INF;
      const u64* cb = cand + base;
      const u32 dk = eval_up_to_64<KIND, VEC, NCH>(T, S, [cb](u32 i) { return key_id(cb[i]); }, cnt, lane);
      const bool keep = mykey != KEY_INF && mykey != best && !alpha_dominates<KIND>(al, dk, key_dkey(mykey));
      const u64 km = ballot(keep);
      __syncthreads();  // all reads of this block of 64 are done
      if (keep) cand[w + (u32)__builtin_popcountll(km & lanemask_lt(lane))] = mykey;
      w += (u32)__builtin_popcountll(km);
      pair_evals += cnt;
    }
    __syncthreads();
    m = w;
  }
  __syncthreads();
  return nout;
}

// ---------------------------------------------------------------------------------------------
// step 1: N_out(p) <- prune(p, V, R) for every batch point; emit the reversed edges
// ---------------------------------------------------------------------------------------------
template <int KIND, int VEC, int NCH>
__global__ __launch_bounds__(64) void prune_kernel(PruneArgs a, VecTable T) {
  __shared__ u64 cand_lds[PRUNE_LDS_CAP];
  extern __shared__ __align__(16) unsigned char smem[];
  u32* out = reinterpret_cast<u32*>(smem);  // R entries

  const int lane = threadIdx.x;
  const u32 qi = blockIdx.x;
  const u32 p = a.qidx[qi];
  const u32 slot = a.slotmap ? a.slotmap[qi] : qi;
  const u32 nv = a.nvis[qi];
  u64* edges = a.edges + (u64)slot * a.R;

  if (nv > a.vis_cap) {
    // the visited list did not fit: leave this point to the host's retry
    if (lane == 0) {
      const u32 o = atomicAdd(a.overflow_count, 1u);
      a.overflow_list[o] = qi;
    }
    for (u32 j = lane; j < a.R; j += 64) edges[j] = KEY_INF;
    return;
  }

  const AlphaParam al{a.a16, a.af};
  u64* cand;
  u64* vis = a.vis_rw + (u64)qi * a.vis_cap;
  if (nv <= PRUNE_LDS_CAP) {
    for (u32 i = lane; i < nv; i += 64) cand_lds[i] = vis[i] & ~1ull;
    cand = cand_lds;
  } else {
    for (u32 i = lane; i < nv; i += 64) vis[i] &= ~1ull;
    cand = vis;
  }
  __syncthreads();
  u32 pair_evals = 0;
  const u32 cnt = robust_prune<KIND, VEC, NCH>(T, cand, nv, a.R, al, out, lane, pair_evals);

  u32* row = a.graph + (u64)p * a.R;
  for (u32 j = lane; j < a.R; j += 64) {
    const bool ok = j < cnt;
    const u32 b = ok ? out[j] : NONE_ID;
    row[j] = b;
    edges[j] = ok ? (((u64)b << 32) | p) : KEY_INF;
  }
  if (a.counters != nullptr && lane == 0) {
    atomicAdd(&a.counters->prunes, 1ull);
    atomicAdd(&a.counters->prune_evals, (unsigned long long)pair_evals);
  }
}

template <int KIND, int VEC, int NCH>
static hipError_t launch_prune_t(const PruneArgs& a, const VecTable& T, hipStream_t s) {
  hipLaunchKernelGGL((prune_kernel<KIND, VEC, NCH>), dim3(a.nq), dim3(64), a.R * sizeof(u32), s, a, T);
  return hipGetLastError();
}

hipError_t launch_prune(const DistCfg& cfg, const PruneArgs& a, hipStream_t s) {
  if (a.nq == 0) return hipSuccess;
  VecTable T{a.points, cfg.row_bytes, cfg.npieces};
  ANN_DISPATCH_CFG(launch_prune_t, a, T, s);
}

// ---------------------------------------------------------------------------------------------
// step 2: segments of equal destination in the sorted edge keys
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void segments_kernel(const u64* keys, u64 nkeys, u32* seg_count, u32* seg_start) {
  const u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
  bool head = false;
  if (i < nkeys) {
    const u32 b = (u32)(keys[i] >> 32);
    head = b != NONE_ID && (i == 0 || (u32)(keys[i - 1] >> 32) != b);
  }
  // one atomic per wave; which slot a segment lands in does not influence any result, each
  // segment is processed on its own
  const u64 hm = ballot(head);
  if (hm) {
    const int lane = threadIdx.x & 63;
    const int leader = __builtin_ctzll(hm);
    u32 base = 0;
    if (lane == leader) base = atomicAdd(seg_count, (u32)__builtin_popcountll(hm));
    base = readlane_u32(base, leader);
    if (head) seg_start[base + (u32)__builtin_popcountll(hm & lanemask_lt(lane))] = (u32)i;
  }
}

hipError_t launch_segments(const u64* keys, u64 nkeys, u32* seg_count, u32* seg_start, hipStream_t s) {
  if (nkeys == 0) return hipSuccess;
  const u32 grid = (u32)((nkeys + 255) / 256);
  hipLaunchKernelGGL(segments_kernel, dim3(grid), dim3(256), 0, s, keys, nkeys, seg_count, seg_start);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// step 2: N_out(b) <- N_out(b) U N; prune(b, N_out(b), R) if it grew beyond R
// ---------------------------------------------------------------------------------------------
template <int KIND, int VEC, int NCH>
__global__ __launch_bounds__(64) void merge_kernel(MergeArgs a, VecTable T) {
  __shared__ u64 cand_lds[PRUNE_LDS_CAP];
  extern __shared__ __align__(16) unsigned char smem[];
  u32* out = reinterpret_cast<u32*>(smem);  // R entries

  const int lane = threadIdx.x;
  const u32 nseg = *a.seg_count;
  const AlphaParam al{a.a16, a.af};
  unsigned long long n_app = 0, n_rep = 0, n_edges = 0, n_pair = 0;

  for (u32 sidx = blockIdx.x; sidx < nseg; sidx += gridDim.x) {
    const u64 i0 = a.seg_start[sidx];
    const u32 b = (u32)(a.keys[i0] >> 32);

    // length of the segment
    u32 cnt = 0;
    for (;;) {
      const u64 i = i0 + cnt + lane;
      const bool same = i < a.nkeys && (u32)(a.keys[i] >> 32) == b;
      const u64 sm = ballot(same);
      if (sm == ~0ull) {
        cnt += 64;
        continue;
      }
      cnt += (u32)__builtin_ctzll(~sm);
      break;
    }
    n_edges += cnt;

    // current degree of b (rows are compact)
    u32* row = a.graph + (u64)b * a.R;
    u32 deg = 0;
    for (u32 base = 0; base < a.R; base += 64) {
      const u32 j = base + lane;
      const u64 vm = ballot(j < a.R && row[j] != NONE_ID);
      deg += (u32)__builtin_popcountll(vm);
      if (vm != ~0ull) break;
    }

    const u32 total = deg + cnt;
    if (total <= a.R) {
      for (u32 j = lane; j < cnt; j += 64) row[deg + j] = (u32)(a.keys[i0 + j] & 0xFFFFFFFFull);
      ++n_app;
      continue;
    }

    // candidate list U = N_out(b) followed by the new sources
    u64* cand;
    if (total <= PRUNE_LDS_CAP) {
      cand = cand_lds;
    } else {
      unsigned long long off = 0;
      if (lane == 0) off = atomicAdd(a.arena_top, (unsigned long long)total);
      off = readlane_u64(off, 0);
      if (off + total > a.arena_cap) {  // cannot happen with the arena sized by the host
        if (lane == 0) *a.error_flag = 1u;
        continue;
      }
      cand = a.arena + off;
    }
    for (u32 j = lane; j < total; j += 64) {
      const u32 id = j < deg ? row[j] : (u32)(a.keys[i0 + (j - deg)] & 0xFFFFFFFFull);
      cand[j] = make_key(0u, id);
    }
    __syncthreads();

    // distances d(b, x) for every x in U
    const QueryRegs<KIND, VEC, NCH> Q =
        load_query<KIND, VEC, NCH>(T.base + (u64)b * T.row_bytes, T.npieces, lane);
    for (u32 base = 0; base < total; base += 64) {
      const u32 c64 = total - base < 64u ? total - base : 64u;
      const u64* cb = cand + base;
      const u32 dk = eval_up_to_64<KIND, VEC, NCH>(T, Q, [cb](u32 i) { return key_id(cb[i]); }, c64, lane);
      const u32 c = cand_of_lane(lane);
      const u32 id = c < c64 ? key_id(cb[c]) : 0u;
      __syncthreads();
      if (c < c64) cand[base + c] = make_key(dk, id);
    }
    __syncthreads();

    u32 pair_evals = total;
    const u32 kept = robust_prune<KIND, VEC, NCH>(T, cand, total, a.R, al, out, lane, pair_evals);
    for (u32 j = lane; j < a.R; j += 64) row[j] = j < kept ? out[j] : NONE_ID;
    __syncthreads();
    ++n_rep;
    n_pair += pair_evals;
  }

  if (a.counters != nullptr && lane == 0) {
    if (n_app) atomicAdd(&a.counters->appends, n_app);
    if (n_rep) atomicAdd(&a.counters->reprunes, n_rep);
    if (n_edges) atomicAdd(&a.counters->edges, n_edges);
    if (n_pair) atomicAdd(&a.counters->prune_evals, n_pair);
  }
}

template <int KIND, int VEC, int NCH>
static hipError_t launch_merge_t(const MergeArgs& a, const VecTable& T, u32 grid, hipStream_t s) {
  hipLaunchKernelGGL((merge_kernel<KIND, VEC, NCH>), dim3(grid), dim3(64), a.R * sizeof(u32), s, a, T);
  return hipGetLastError();
}

hipError_t launch_merge(const DistCfg& cfg, const MergeArgs& a, u32 grid, hipStream_t s) {
  if (grid == 0) return hipSuccess;
  VecTable T{a.points, cfg.row_bytes, cfg.npieces};
  ANN_DISPATCH_CFG(launch_merge_t, a, T, grid, s);
}

}  // namespace annmi
