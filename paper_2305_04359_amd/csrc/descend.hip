// The way of a query down the upper layers of the layered index (Sec. 4.2): on every layer a
// greedy search with beam 1 (Alg. 1 with L = 1), one wavefront per query, all layers in one
// launch.
//
// With a beam of one the search of Alg. 1 is a walk: the vertex in the beam is expanded, and the
// closest of its neighbours replaces it if it is closer under (distance, id); otherwise the search
// ends there.  A neighbour whose distance was taken at an earlier step lost to a vertex of the
// walk then, and the walk has only come closer since, so taking its distance again changes
// nothing: no visited set is kept.
#include "ann_device.hpp"
#include "ann_dispatch.hpp"
#include "ann_internal.hpp"

namespace annmi {

__device__ __forceinline__ u64 wave_min_key(u64 v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const u64 o = __shfl_xor(v, off, 64);
    v = o < v ? o : v;
  }
  return v;
}

template <int KIND, int VEC, int NCH>
__global__ __launch_bounds__(64) void descend_kernel(DescendArgs a, u32 row_bytes, u32 npieces) {
  __shared__ u32 ids[64];  // the 64 neighbour ids under evaluation
  const int lane = threadIdx.x;
  const u32 qi = blockIdx.x;
  const QueryRegs<KIND, VEC, NCH> Q = load_query<KIND, VEC, NCH>(a.queries + (u64)qi * a.qrow_bytes, npieces, lane);
  u32 cur = a.entry;
  for (u32 li = 0; li < a.nlayers; ++li) {
    const DescendLayer Y = a.layers[li];
    const VecTable T{Y.points, row_bytes, npieces};
    u32 dk = eval_up_to_64<KIND, VEC, NCH>(T, Q, [cur](u32) { return cur; }, 1u, lane);
    u64 curkey = make_key(readlane_u32(dk, 0), cur);
    for (;;) {
      u64 best = curkey;
      const u32* row = Y.graph + (u64)cur * Y.R;
      for (u32 c0 = 0; c0 < Y.R; c0 += 64) {
        const u32 mine = c0 + (u32)lane < Y.R ? row[c0 + lane] : NONE_ID;
        const u32 cnt = (u32)__builtin_popcountll(ballot(mine != NONE_ID));  // rows are compact
        if (cnt == 0) break;
        __syncthreads();
        ids[lane] = mine;
        __syncthreads();
        const u32 d = eval_up_to_64<KIND, VEC, NCH>(T, Q, [&](u32 c) { return ids[c]; }, cnt, lane);
        const u32 c = cand_of_lane(lane);
        const u64 key = c < cnt ? make_key(d, ids[c]) : KEY_INF;
        const u64 m = wave_min_key(key);
        best = m < best ? m : best;
        if (cnt < 64) break;
      }
      if (best == curkey) break;
      curkey = best;
      cur = key_id(best);
    }
    cur = Y.down[cur];
  }
  if (lane == 0) a.out[qi] = cur;
}

template <int KIND, int VEC, int NCH>
static hipError_t launch_descend_t(const DescendArgs& a, u32 row_bytes, u32 npieces, hipStream_t s) {
  hipLaunchKernelGGL((descend_kernel<KIND, VEC, NCH>), dim3(a.nq), dim3(64), 0, s, a, row_bytes, npieces);
  return hipGetLastError();
}

hipError_t launch_descend(const DistCfg& cfg, const DescendArgs& a, hipStream_t s) {
  if (a.nq == 0) return hipSuccess;
  ANN_DISPATCH_CFG(launch_descend_t, a, (u32)cfg.row_bytes, cfg.npieces, s);
}

}  // namespace annmi
