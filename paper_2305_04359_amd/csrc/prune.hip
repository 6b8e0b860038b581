// Step 1 of BatchInsert (Alg. 3 of the paper): N_out(p) <- prune(p, V, R) for every batch point,
// one wavefront per point, and emission of the reversed edges for step 2.
#include "ann_device.hpp"
#include "ann_internal.hpp"
#include "ann_dispatch.hpp"
#include "prune_device.hpp"

namespace annmi {

// ---------------------------------------------------------------------------------------------
// step 1: N_out(p) <- prune(p, V, R) for every batch point; emit the reversed edges
// ---------------------------------------------------------------------------------------------
template <int KIND, int VEC, int NCH>
__global__ __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(4, 4))) void prune_kernel(PruneArgs a, VecTable T) {
  __shared__ u64 cand_lds[PRUNE_LDS_CAP];
  extern __shared__ __align__(16) unsigned char smem[];
  u32* out = reinterpret_cast<u32*>(smem);  // R entries
  u32* selxx = out + a.R;                   // R entries
  SelStage st;
  st.stride = stage_stride(T.row_bytes);
  st.xx = selxx;
  unsigned char* blk = smem + ((a.R * 8u + 15u) & ~15u);  // 8 rows + 8 norms
  st.vec = a.stage_bytes ? blk + 8u * st.stride + 32u : nullptr;
  constexpr bool kMfma = MfmaPruneOk<KIND, VEC, NCH>::value;
  const MfmaLds M = mfma_lds_carve(smem + ((a.R * 4u + 15u) & ~15u), a.R, T.row_bytes);  // used when a.use_mfma

  const int lane = threadIdx.x;
  const u32 qi = blockIdx.x;
  const u32 p = a.qidx[qi];
  const u32 slot = a.slotmap ? a.slotmap[qi] : qi;
  const u32 nv = a.nvis[qi];
  u64* edges = a.edges + (u64)slot * a.R;
  if (a.spill_top_reset != nullptr && qi == 0 && lane == 0) *a.spill_top_reset = 0ull;  // every search of this batch is over

  const u64 where = a.vis_where != nullptr ? a.vis_where[qi] : ~0ull;
  const u32 room = where == ~0ull ? a.vis_cap : a.vis_cap + a.spill_chunk;
  if (nv > room) {
    // the visited list did not fit anywhere: leave this point to the host
    if (lane == 0) {
      const u32 o = atomicAdd(a.overflow_count, 1u);
      a.overflow_list[o] = qi;
      *a.lost_flag = 1u;
    }
    for (u32 j = lane; j < a.R; j += 64) edges[j] = KEY_INF;
    return;
  }

  const AlphaParam al{a.a16, a.af};
  u64* vis = where == ~0ull ? a.vis_rw + (u64)qi * a.vis_cap : a.spill + where;
  u32 pair_evals = 0;
  u32 cnt;
  if (nv <= PRUNE_LDS_CAP) {
    u32 n2 = 64;
    while (n2 < nv) n2 <<= 1;
    for (u32 i = lane; i < n2; i += 64) cand_lds[i] = i < nv ? (vis[i] & ~1ull) : KEY_INF;
    __syncthreads();
    bitonic_sort_keys(cand_lds, n2, lane);
    bool done = false;
    cnt = 0;
    if constexpr (kMfma) {
      if (a.use_mfma) {
        cnt = prune_sorted_mfma<KIND, VEC, NCH>(T, M, cand_lds, nv, a.R, a.a16, out, lane, pair_evals);
        done = true;
      }
    }
    if (!done) cnt = prune_sorted<KIND, VEC, NCH>(T, st, blk, cand_lds, nv, a.R, al, out, lane, pair_evals);
  } else {
    for (u32 i = lane; i < nv; i += 64) vis[i] &= ~1ull;
    __syncthreads();
    SelStage st2 = st;
    if (a.use_mfma) st2.vec = nullptr;  // the LDS areas are laid out for the matrix-core walk
    cnt = prune_unsorted<KIND, VEC, NCH>(T, st2, vis, nv, a.R, al, out, lane, pair_evals);
  }
  __syncthreads();

  u32* row = a.graph + (u64)p * a.R;
  for (u32 j = lane; j < a.R; j += 64) {
    const bool ok = j < cnt;
    const u32 b = ok ? out[j] : NONE_ID;
    row[j] = b;
    edges[j] = ok ? (((u64)b << 32) | p) : KEY_INF;
  }
  if (lane == 0) a.meta[p] = cnt | (cnt << 16);  // the whole row is the output of a prune
  if (a.counters != nullptr && lane == 0) {
    atomicAdd(&block_counters(a.counters)->prunes, 1ull);
    atomicAdd(&block_counters(a.counters)->prune_evals, (unsigned long long)pair_evals);
  }
}

template <int KIND, int VEC, int NCH>
static hipError_t launch_prune_t(const PruneArgs& a, const VecTable& T, hipStream_t s) {
  const u32 lds = a.use_mfma ? ((a.R * 4u + 15u) & ~15u) + mfma_lds_bytes(a.R, T.row_bytes)
                            : ((a.R * 8u + 15u) & ~15u) + 8u * stage_stride(T.row_bytes) + 32u + a.stage_bytes;
  hipLaunchKernelGGL((prune_kernel<KIND, VEC, NCH>), dim3(a.nq), dim3(64), lds, s, a, T);
  return hipGetLastError();
}

hipError_t launch_prune(const DistCfg& cfg, const PruneArgs& a, hipStream_t s) {
  if (a.nq == 0) return hipSuccess;
  VecTable T{a.points, (u32)cfg.row_bytes, cfg.npieces};
  ANN_DISPATCH_CFG(launch_prune_t, a, T, s);
}

}  // namespace annmi
