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

#include <utility>

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
// prune of a short candidate list of u8/i8 vectors with the matrix cores
//
// An overflowing row has R old entries plus a few new ones.  For such a list every pair
// distance the scan of prune() can ask for is an entry of the Gram matrix of the candidate
// vectors, a small dense contraction.  The wave stages the vectors in LDS (u8 shifted by -128 so
// that they are int8; distances are translation invariant), sorts the candidates by
// (d(b,.), id), forms the Gram matrix of the sorted list with v_mfma_i32_32x32x32_i8 (exact in
// int32), reduces each entry at once to the bit "i removes j" (alpha * D(i,j) <= d(b,j), as the
// equivalent D(i,j) <= floor(d(b,j) * 2^16 / a16)), and then replays the scan of prune() on bit
// masks with scalar instructions.
// ---------------------------------------------------------------------------------------------
constexpr u32 SM_TMAX = 96;     // candidates handled by this path
constexpr u32 SM_STRIDE = 144;  // bytes between staged vectors (128 + 16: spreads LDS banks)
constexpr u32 MERGE_BUF_BYTES = SM_TMAX * SM_STRIDE;
constexpr u32 MERGE_LDS_CAP = MERGE_BUF_BYTES / 8;  // keys the generic path can hold instead
static_assert(MERGE_LDS_CAP == MERGE_SPILL_MIN, "the host sizes the spill arena from MERGE_SPILL_MIN");

struct SmallLds {
  u64 key[SM_TMAX];   // by arrival index
  u32 uid[SM_TMAX];   // ids by arrival index
  u32 nrm[SM_TMAX];   // squared norms of the shifted vectors, by arrival index
  u32 sid[SM_TMAX];   // ids, sorted by (distance to b, id)
  u32 snrm[SM_TMAX];  // norms, sorted
  i32 sthr[SM_TMAX];  // largest D(i,j) that still removes j, sorted
  u32 inv[SM_TMAX];   // sorted position -> arrival index
};

typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef int v16i_t __attribute__((ext_vector_type(16)));

template <int VEC, int NCH>
struct SmallPathOk {
  static constexpr bool value = (8 * NCH * VEC <= 128);
};

// floor(d * 2^16 / a16) for 0 <= d < 2^31, 0 < a16 < 2^31, clamped to INT32_MAX
__device__ __forceinline__ i32 alpha_threshold(i32 d, i64 a16) {
  const u64 x = (u64)(u32)d << 16;
  u64 t = (u64)__builtin_floor((double)x / (double)a16);
  if (t * (u64)a16 > x)
    --t;
  else if ((t + 1) * (u64)a16 <= x)
    ++t;
  return t > 0x7FFFFFFFull ? 0x7FFFFFFF : (i32)t;
}

// One 32x32 tile of the Gram matrix of the sorted candidates: rows 32*RB.., columns 32*CB...
// Accumulator register r of lane l is entry (row 8*(r/4) + 4*(l/32) + r%4, column l%32), so one
// ballot per register yields the 32 "removes" bits of two rows, which go to the lanes that own
// those rows.
template <int RB, int CB, int R_>
__device__ __forceinline__ void gram_tile_reg(const v16i_t& acc, const SmallLds& S, bool colok, i32 ncol, i32 tcol,
                                              u32 half, u32& Klo, u32& Khi) {
  constexpr int mlo = 32 * RB + 8 * (R_ / 4) + (R_ % 4);
  const i32 nrow = (i32)S.snrm[mlo + 4 * half];
  const i32 D = nrow + ncol - 2 * acc[R_];
  const u64 bm = ballot(colok && D <= tcol);
  const u32 lo = (u32)bm, hi = (u32)(bm >> 32);
  if constexpr (mlo < 64) {
    Klo = writelane_u32<mlo>(Klo, lo);
    Klo = writelane_u32<mlo + 4>(Klo, hi);
  } else if constexpr (CB == 2) {
    Khi = writelane_u32<mlo - 64>(Khi, lo);
    Khi = writelane_u32<mlo + 4 - 64>(Khi, hi);
  }
}

template <int RB, int CB, int... Rs>
__device__ __forceinline__ void gram_tile_regs(const v16i_t& acc, const SmallLds& S, bool colok, i32 ncol, i32 tcol,
                                               u32 half, u32& Klo, u32& Khi, std::integer_sequence<int, Rs...>) {
  (gram_tile_reg<RB, CB, Rs>(acc, S, colok, ncol, tcol, half, Klo, Khi), ...);
}

template <int RB, int CB>
__device__ __forceinline__ void gram_tile(const unsigned char* Xs, const SmallLds& S, u32 total, u32 ksteps, int lane,
                                          u32& Klo, u32& Khi) {
  const u32 half = (u32)lane >> 5;
  const u32 ia = 32u * RB + (lane & 31), ib = 32u * CB + (lane & 31);
  const u32 ra = ia < total ? S.inv[ia] : 0u;
  const u32 rb = ib < total ? S.inv[ib] : 0u;
  const unsigned char* pa = Xs + ra * SM_STRIDE + 16u * half;
  const unsigned char* pb = Xs + rb * SM_STRIDE + 16u * half;
  v16i_t acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
  for (u32 ks = 0; ks < ksteps; ++ks) {
    const v4i_t av = *reinterpret_cast<const v4i_t*>(pa + 32u * ks);
    const v4i_t bv = *reinterpret_cast<const v4i_t*>(pb + 32u * ks);
    acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(av, bv, acc, 0, 0, 0);
  }
  const bool colok = ib < total;
  const i32 ncol = colok ? (i32)S.snrm[ib] : 0;
  const i32 tcol = colok ? S.sthr[ib] : -1;
  gram_tile_regs<RB, CB>(acc, S, colok, ncol, tcol, half, Klo, Khi, std::make_integer_sequence<int, 16>{});
}

// S.uid[0..total) holds the candidate ids (old row entries first).  Writes the pruned row.
template <int KIND, int VEC, int NCH>
__device__ __forceinline__ void reprune_small_int(const VecTable& T, const QueryRegs<KIND, VEC, NCH>& Q,
                                                  unsigned char* Xs, SmallLds& S, u32 total, u32 R, i64 a16,
                                                  u32* row, int lane) {
  constexpr int PB = PassBatch<VEC, NCH>::value;
  const int sub = lane & (LPC - 1);
  const u32 grp = (u32)lane >> 3;
  const u32 npass = (total + 7u) >> 3;
  const u32 flip = KIND == K_U8 ? 0x80808080u : 0u;

  // stage the vectors, take d(b, x) and the norms
  for (u32 t0 = 0; t0 < npass; t0 += PB) {
    Piece<VEC> x[PB][NCH];
    u32 ids[PB];
#pragma unroll
    for (int tt = 0; tt < PB; ++tt) {
      const u32 c = 8u * (t0 + tt) + grp;
      const bool ok = c < total;
      ids[tt] = ok ? S.uid[c] : 0u;
      const char* src = T.base + (u64)ids[tt] * T.row_bytes;
#pragma unroll
      for (int u = 0; u < NCH; ++u) {
        const u32 pc = sub + LPC * u;
        x[tt][u] = (ok && pc < T.npieces) ? load_piece<VEC>(src + (u64)pc * VEC) : zero_piece<VEC>();
      }
    }
#pragma unroll
    for (int tt = 0; tt < PB; ++tt) {
      const u32 c = 8u * (t0 + tt) + grp;
      const u32 dk = distance_key<KIND, VEC, NCH>(Q, x[tt]);
      i32 nn = 0;
#pragma unroll
      for (int u = 0; u < NCH; ++u) {
        const u32 pc = sub + LPC * u;
#pragma unroll
        for (int i = 0; i < VEC / 4; ++i) {
          const u32 wv = pc < T.npieces ? (x[tt][u].w[i] ^ flip) : 0u;
          nn = __builtin_amdgcn_sdot4((i32)wv, (i32)wv, nn, false);
          if (c < total) *reinterpret_cast<u32*>(Xs + c * SM_STRIDE + pc * VEC + 4 * i) = wv;
        }
      }
      nn = group_sum(nn);
      if (sub == 0 && c < total) {
        S.key[c] = make_key(dk, ids[tt]);
        S.nrm[c] = (u32)nn;
      }
    }
  }
  __syncthreads();

  // rank of every candidate under (distance, id); keys are distinct
  {
    const u32 j0 = lane, j1 = lane + 64;
    const u64 k0 = j0 < total ? S.key[j0] : KEY_INF;
    const u64 k1 = j1 < total ? S.key[j1] : KEY_INF;
    u32 r0 = 0, r1 = 0;
    for (u32 i = 0; i < total; ++i) {
      const u64 ki = S.key[i];
      r0 += ki < k0 ? 1u : 0u;
      r1 += ki < k1 ? 1u : 0u;
    }
    if (j0 < total) {
      S.sid[r0] = key_id(k0);
      S.snrm[r0] = S.nrm[j0];
      S.sthr[r0] = alpha_threshold(int_from_dkey(key_dkey(k0)), a16);
      S.inv[r0] = j0;
    }
    if (j1 < total) {
      S.sid[r1] = key_id(k1);
      S.snrm[r1] = S.nrm[j1];
      S.sthr[r1] = alpha_threshold(int_from_dkey(key_dkey(k1)), a16);
      S.inv[r1] = j1;
    }
  }
  __syncthreads();

  // Gram matrix tile by tile; K0[c] of lane i = bits "sorted candidate i removes candidate 32c+j",
  // K1 the same for candidates 64..95 (only column block 2 matters there)
  const u32 nb = (total + 31u) >> 5;
  const u32 ksteps = (u32)((T.row_bytes + 31) / 32);
  u32 K0[3] = {0u, 0u, 0u};
  u32 K1 = 0u;
  gram_tile<0, 0>(Xs, S, total, ksteps, lane, K0[0], K1);
  if (nb > 1) {
    gram_tile<0, 1>(Xs, S, total, ksteps, lane, K0[1], K1);
    gram_tile<1, 1>(Xs, S, total, ksteps, lane, K0[1], K1);
  }
  if (nb > 2) {
    gram_tile<0, 2>(Xs, S, total, ksteps, lane, K0[2], K1);
    gram_tile<1, 2>(Xs, S, total, ksteps, lane, K0[2], K1);
    gram_tile<2, 2>(Xs, S, total, ksteps, lane, K0[2], K1);
  }

  // the scan of prune(): walk the sorted list, select what is still alive, remove what it removes
  const u32 nlo = total < 64u ? total : 64u;
  u64 rem_lo = nlo == 64u ? ~0ull : ((1ull << nlo) - 1ull);
  u32 rem_hi = total > 64u ? ((total - 64u) >= 32u ? ~0u : ((1u << (total - 64u)) - 1u)) : 0u;
  u64 sel_lo = 0;
  u32 sel_hi = 0, nout = 0;
  while (rem_lo != 0 && nout < R) {
    const int i = __builtin_ctzll(rem_lo);
    sel_lo |= 1ull << i;
    ++nout;
    const u64 klo = (u64)readlane_u32(K0[0], i) | ((u64)readlane_u32(K0[1], i) << 32);
    rem_lo &= ~klo;
    rem_lo &= ~(1ull << i);
    rem_hi &= ~readlane_u32(K0[2], i);
  }
  while (rem_hi != 0 && nout < R) {
    const int i = __builtin_ctz(rem_hi);
    sel_hi |= 1u << i;
    ++nout;
    rem_hi &= ~readlane_u32(K1, i);
    rem_hi &= ~(1u << i);
  }

  // write the row: selected ids in sorted order, then padding
  if ((sel_lo >> lane) & 1ull) row[__builtin_popcountll(sel_lo & lanemask_lt(lane))] = S.sid[lane];
  if (lane < 32 && ((sel_hi >> lane) & 1u))
    row[__builtin_popcountll(sel_lo) + __builtin_popcount(sel_hi & ((1u << lane) - 1u))] = S.sid[64 + lane];
  for (u32 j = nout + lane; j < R; j += 64) row[j] = NONE_ID;
  __syncthreads();
}

// ---------------------------------------------------------------------------------------------
// step 2: N_out(b) <- N_out(b) U N; prune(b, N_out(b), R) if it grew beyond R
// ---------------------------------------------------------------------------------------------
template <int KIND, int VEC, int NCH>
__global__ __launch_bounds__(64) void merge_kernel(MergeArgs a, VecTable T) {
  __shared__ __align__(16) unsigned char buf[MERGE_BUF_BYTES];  // staged vectors, or candidate keys
  __shared__ SmallLds small;
  u64* cand_lds = reinterpret_cast<u64*>(buf);
  extern __shared__ __align__(16) unsigned char smem[];
  u32* out = reinterpret_cast<u32*>(smem);  // R entries
  constexpr bool kSmall = KindTraits<KIND>::is_int && SmallPathOk<VEC, NCH>::value;

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

    if constexpr (kSmall) {
      if (total <= SM_TMAX) {
        for (u32 j = lane; j < total; j += 64)
          small.uid[j] = j < deg ? row[j] : (u32)(a.keys[i0 + (j - deg)] & 0xFFFFFFFFull);
        __syncthreads();
        const QueryRegs<KIND, VEC, NCH> Qb =
            load_query<KIND, VEC, NCH>(T.base + (u64)b * T.row_bytes, T.npieces, lane);
        reprune_small_int<KIND, VEC, NCH>(T, Qb, buf, small, total, a.R, al.a16, row, lane);
        ++n_rep;
        n_pair += (unsigned long long)total * (total + 1) / 2;
        continue;
      }
    }

    // candidate list U = N_out(b) followed by the new sources
    u64* cand;
    if (total <= MERGE_LDS_CAP) {
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
