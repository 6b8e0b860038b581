// Step 2 of BatchInsert (Alg. 3 of the paper): for every existing point b that was chosen by
// batch points, N_out(b) <- N_out(b) U N, and prune(b, N_out(b), R) if that exceeds R.
//
// The sorted edge keys are cut into segments of equal destination by a planning kernel, which
// appends directly where the row has room and otherwise files the segment under one of three
// kinds of re-prune, each served by its own kernel (one wavefront per row):
//
//   fast     the row still starts with the output of its last prune (its "clean prefix": sorted
//            by distance to b and free of pairs where one removes the other, which is what prune
//            guarantees of what it keeps) and only a few entries are new.  Only pairs with a new
//            entry can change anything, so the wave measures every candidate against b and
//            against the new entries in one sweep and replays the scan on bit masks.
//   gram     u8/i8 rows of at most 96 candidates: all pair distances from the int8 Gram matrix
//            on the matrix cores (exact), then the scan on bit masks.
//   generic  everything else: the wave-wide scan of prune_device.hpp, candidates in LDS or, for
//            very long lists, in a spill arena in device memory.
//
// Every path computes exactly prune(b, U, R) with U = old row followed by the new sources in
// batch order; they differ only in which distances they have to take.
#include <utility>

#include "ann_device.hpp"
#include "ann_internal.hpp"
#include "ann_dispatch.hpp"
#include "prune_device.hpp"

namespace annmi {

__device__ __forceinline__ u32 meta_deg(u32 m) { return m & 0xFFFFu; }
__device__ __forceinline__ u32 meta_clean(u32 m) { return m >> 16; }
__device__ __forceinline__ u32 make_meta(u32 deg, u32 clean) { return deg | (clean << 16); }

// ---------------------------------------------------------------------------------------------
// planning: one thread per edge key; the first key of each segment does the work
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void plan_kernel(MergeArgs a) {
  __shared__ u32 cnt_lds[4];
  __shared__ u32 base_lds[4];
  __shared__ u32 stat_lds[2];  // appends, appended edges
  if (threadIdx.x < 4) cnt_lds[threadIdx.x] = 0;
  if (threadIdx.x < 2) stat_lds[threadIdx.x] = 0;
  __syncthreads();

  const u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
  int kind = -1;  // 0 fast, 1 gram, 2 generic with a long candidate list, 3 generic with a list of up to 512
  u32 slot = 0, cnt = 0, b = 0, m = 0;
  if (i < a.nkeys) {
    b = (u32)(a.keys[i] >> 32);
    const bool head = b != NONE_ID && (i == 0 || (u32)(a.keys[i - 1] >> 32) != b);
    if (head) {
      // length of the segment: gallop, then bisect (keys are sorted by destination)
      u64 lo = i, step = 1;
      while (i + step < a.nkeys && (u32)(a.keys[i + step] >> 32) == b) {
        lo = i + step;
        step <<= 1;
      }
      u64 hi = i + step < a.nkeys ? i + step : a.nkeys;
      while (hi - lo > 1) {
        const u64 mid = (lo + hi) >> 1;
        if ((u32)(a.keys[mid] >> 32) == b)
          lo = mid;
        else
          hi = mid;
      }
      cnt = (u32)(hi - i);
      m = a.meta[b];
      const u32 deg = meta_deg(m), clean = meta_clean(m);
      if (!a.force_prune && deg + cnt <= a.R) {
        u32* row = a.graph + (u64)b * a.R;
        for (u32 j = 0; j < cnt; ++j) row[deg + j] = (u32)(a.keys[i + j] & 0xFFFFFFFFull);
        a.meta[b] = make_meta(deg + cnt, clean);
        if (a.counters != nullptr) {
          atomicAdd(&stat_lds[0], 1u);
          atomicAdd(&stat_lds[1], cnt);
        }
      } else {
        const u32 fresh = deg - clean + cnt;
        if (a.force_prune)
          kind = (a.gram_ok && deg + cnt <= a.gram_tmax) ? 1 : 2;  // (the fast path presumes a clean prefix)
        else if (clean <= 64 && fresh <= a.fast_amax)
          kind = 0;
        else if (a.gram_ok && deg + cnt <= a.gram_tmax)
          kind = 1;
        else
          kind = 2;
        if (kind == 2 && deg + cnt <= a.medium_max) kind = 3;
        slot = atomicAdd(&cnt_lds[kind], 1u);
      }
    }
  }
  __syncthreads();
  // one global atomic per work list and workgroup; the order of a list has no influence on any
  // result, every segment is processed on its own
  if (threadIdx.x < 4 && cnt_lds[threadIdx.x] != 0)
    base_lds[threadIdx.x] = atomicAdd(&a.list_count[threadIdx.x], cnt_lds[threadIdx.x]);
  if (a.counters != nullptr && threadIdx.x == 0 && stat_lds[0] != 0) {
    atomicAdd(&block_counters(a.counters)->appends, (unsigned long long)stat_lds[0]);
    atomicAdd(&block_counters(a.counters)->edges, (unsigned long long)stat_lds[1]);
  }
  __syncthreads();
  if (kind >= 0) {
    const long long at = (long long)(base_lds[kind] + slot);
    a.list_items[kind][kind == 3 ? -at : at] = MergeItem{(u32)i, cnt, b, m};
  }
}

hipError_t launch_plan(const MergeArgs& a, hipStream_t s) {
  if (a.nkeys == 0) return hipSuccess;
  const u32 grid = (u32)((a.nkeys + 255) / 256);
  hipLaunchKernelGGL(plan_kernel, dim3(grid), dim3(256), 0, s, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// fast path: clean prefix plus at most FastAMax new entries
// ---------------------------------------------------------------------------------------------
template <int NCH>
struct FastAMax {
  static constexpr int value = NCH <= 2 ? 4 : (NCH <= 4 ? 2 : 1);
};

// lane-local part of the distance between a query and the row pieces x; `xx` is the shared
// <x,x> part for the integer kinds
template <int KIND, int VEC, int NCH>
__device__ __forceinline__ i32 xx_part(const Piece<VEC> (&x)[NCH]) {
  i32 xx = 0;
  if constexpr (KIND == K_U8) {
#pragma unroll
    for (int u = 0; u < NCH; ++u)
#pragma unroll
      for (int i = 0; i < VEC / 4; ++i) xx = (i32)__builtin_amdgcn_udot4(x[u].w[i], x[u].w[i], (u32)xx, false);
  } else if constexpr (KIND == K_I8) {
#pragma unroll
    for (int u = 0; u < NCH; ++u)
#pragma unroll
      for (int i = 0; i < VEC / 4; ++i) xx = __builtin_amdgcn_sdot4((i32)x[u].w[i], (i32)x[u].w[i], xx, false);
  }
  return xx;
}

template <int KIND, int VEC, int NCH>
__device__ __forceinline__ u32 distance_key_xx(const QueryRegs<KIND, VEC, NCH>& Q, const Piece<VEC> (&x)[NCH], i32 xx) {
  if constexpr (KIND == K_U8) {
    u32 qx = 0;
#pragma unroll
    for (int u = 0; u < NCH; ++u)
#pragma unroll
      for (int i = 0; i < VEC / 4; ++i) qx = __builtin_amdgcn_udot4(Q.q[u].w[i], x[u].w[i], qx, false);
    return dkey_from_int(group_sum(xx - 2 * (i32)qx) + Q.qq);
  } else if constexpr (KIND == K_I8) {
    i32 qx = 0;
#pragma unroll
    for (int u = 0; u < NCH; ++u)
#pragma unroll
      for (int i = 0; i < VEC / 4; ++i) qx = __builtin_amdgcn_sdot4((i32)Q.q[u].w[i], (i32)x[u].w[i], qx, false);
    return dkey_from_int(group_sum(xx - 2 * qx) + Q.qq);
  } else {
    return distance_key<KIND, VEC, NCH>(Q, x);
  }
}

// One row of the fast path with exactly NA new entries (a compile-time count keeps every loop
// over the new entries fully unrolled and free of guards).
template <int KIND, int VEC, int NCH, int NA>
__device__ __forceinline__ u32 fast_item(const MergeArgs& a, const VecTable& T, const AlphaParam& al, u32* ids_lds,
                                         u32 (*dk_lds)[64], u32 b, u32 i0, u32 clean, u32 stale, u32* row, u32 R,
                                         int lane) {
  // all nine passes (eight over the clean prefix, one over the new entries) requested at once when
  // the pieces fit the register file: one trip to memory instead of three
  constexpr int PBF = VEC * NCH <= 16 ? 9 : (VEC * NCH <= 32 ? 5 : (PassBatch<VEC, NCH>::value > 4 ? 4 : PassBatch<VEC, NCH>::value));
  constexpr u32 na = NA;
  const int sub = lane & (LPC - 1);
  const u32 grp = (u32)lane >> 3;
    const u32 myid = (u32)lane < clean ? row[lane] : NONE_ID;
    u32 mynew = NONE_ID;
    if ((u32)lane < na) mynew = (u32)lane < stale ? row[clean + lane] : (u32)(a.keys[i0 + (lane - stale)] & 0xFFFFFFFFull);
    ids_lds[lane] = myid;
    if ((u32)lane < na) ids_lds[64 + lane] = mynew;

    const QueryRegs<KIND, VEC, NCH> Qb = load_query<KIND, VEC, NCH>(T.base + (u64)b * T.row_bytes, T.npieces, lane);
    QueryRegs<KIND, VEC, NCH> Qn[NA];
    u32 nid[NA];
#pragma unroll
    for (int k = 0; k < NA; ++k) {
      nid[k] = readlane_u32(mynew, k);
      if ((u32)k < na)
        Qn[k] = load_query<KIND, VEC, NCH>(T.base + (u64)nid[k] * T.row_bytes, T.npieces, lane);
      else
        Qn[k] = Qb;
    }
    __syncthreads();

    // one sweep over the clean prefix and the new entries: candidate index c < clean is row
    // position c, index 64 + k is new entry k; each is measured against b and every new entry
    u32 res[1 + NA];
#pragma unroll
    for (int q = 0; q <= NA; ++q) res[q] = 0;
    u32 newres[1 + NA];  // the same for the pass over the new entries (valid in lanes 8k)
#pragma unroll
    for (int q = 0; q <= NA; ++q) newres[q] = 0;
    const u32 npass_clean = (clean + 7u) >> 3;
    for (u32 t0 = 0; t0 < npass_clean + 1; t0 += PBF) {
      Piece<VEC> x[PBF][NCH];
#pragma unroll
      for (int tt = 0; tt < PBF; ++tt) {
        const u32 t = t0 + tt;
        // passes 0..npass_clean-1 cover the clean prefix, pass npass_clean the new entries
        const bool newpass = t == npass_clean;
        const u32 c = newpass ? grp : 8u * t + grp;
        const bool ok = newpass ? (grp < na) : (t < npass_clean && c < clean);
        const u32 id = ok ? ids_lds[newpass ? 64 + grp : c] : 0u;
        const char* src = T.base + (u64)id * T.row_bytes;
#pragma unroll
        for (int u = 0; u < NCH; ++u) {
          const u32 pc = sub + LPC * u;
          x[tt][u] = (ok && pc < T.npieces) ? load_piece<VEC>(src + (u64)pc * VEC) : zero_piece<VEC>();
        }
      }
#pragma unroll
      for (int tt = 0; tt < PBF; ++tt) {
        const u32 t = t0 + tt;
        if (t <= npass_clean) {  // uniform
          const i32 xx = xx_part<KIND, VEC, NCH>(x[tt]);
          const bool newpass = t == npass_clean;
          const u32 d0 = distance_key_xx<KIND, VEC, NCH>(Qb, x[tt], xx);
          if (newpass)
            newres[0] = d0;
          else if ((u32)sub == t)
            res[0] = d0;
#pragma unroll
          for (int k = 0; k < NA; ++k) {
            if ((u32)k < na) {  // uniform
              const u32 dkk = distance_key_xx<KIND, VEC, NCH>(Qn[k], x[tt], xx);
              if (newpass)
                newres[1 + k] = dkk;
              else if ((u32)sub == t)
                res[1 + k] = dkk;
            }
          }
        }
      }
    }
    // lane l holds the results of row position cand_of_lane(l); bring them to lane = position
    {
      const u32 c = cand_of_lane(lane);
#pragma unroll
      for (int q = 0; q <= NA; ++q) dk_lds[q][c] = res[q];
    }
    __syncthreads();
    const bool isc = (u32)lane < clean;
    const u32 dB = dk_lds[0][lane];
    const u64 keyc = isc ? make_key(dB, myid) : KEY_INF;

    // per new entry k: its key, its place among the clean entries, what it removes, what removes it
    u64 keyn[NA];
    u32 rank[NA];
    u64 removes[NA], removed_by[NA];
    u32 dBn[NA];
#pragma unroll
    for (int k = 0; k < NA; ++k) {
      dBn[k] = readlane_u32(newres[0], 8 * k);
      keyn[k] = make_key(dBn[k], nid[k]);
      const u32 dkj = dk_lds[1 + k][lane];  // distance new entry k <-> clean entry `lane`
      rank[k] = (u32)__builtin_popcountll(ballot(isc && keyc < keyn[k]));
      removes[k] = ballot(isc && alpha_dominates<KIND>(al, dkj, dB));
      removed_by[k] = ballot(isc && alpha_dominates<KIND>(al, dkj, dBn[k]));
    }
    // replay the scan: clean entries never remove each other, so only the new entries matter
    u64 alive = clean >= 64 ? ~0ull : ((1ull << clean) - 1ull);
    u32 selnew = 0;
#pragma unroll
    for (int r = 0; r < NA; ++r) {
      // the new entry that is r-th among the new entries in (distance, id) order
#pragma unroll
      for (int k = 0; k < NA; ++k) {
        if ((u32)k < na) {
          u32 ord = 0;
#pragma unroll
          for (int l = 0; l < NA; ++l)
            if ((u32)l < na && keyn[l] < keyn[k]) ++ord;
          if (ord == (u32)r) {
            const u64 before = rank[k] >= 64 ? ~0ull : ((1ull << rank[k]) - 1ull);
            bool killed = (removed_by[k] & alive & before) != 0;
#pragma unroll
            for (int l = 0; l < NA; ++l) {
              if ((u32)l < na && l != k && ((selnew >> l) & 1u) && keyn[l] < keyn[k]) {
                // distance new l <-> new k: query l against candidate k of the new pass
                const u32 dlk = readlane_u32(newres[1 + l], 8 * k);
                killed = killed || alpha_dominates<KIND>(al, dlk, dBn[k]);
              }
            }
            if (!killed) {
              selnew |= 1u << k;
              alive &= ~(removes[k] & ~before);
            }
          }
        }
      }
    }
    // positions in the merged order, cut at R
    u32 pos = (u32)__builtin_popcountll(alive & lanemask_lt(lane));
    u32 newpos = 0;
#pragma unroll
    for (int k = 0; k < NA; ++k) {
      if ((u32)k < na && ((selnew >> k) & 1u)) {
        if (rank[k] <= (u32)lane) ++pos;  // new entry k precedes clean entry `lane`
        const u64 before = rank[k] >= 64 ? ~0ull : ((1ull << rank[k]) - 1ull);
        u32 pk = (u32)__builtin_popcountll(alive & before);
#pragma unroll
        for (int l = 0; l < NA; ++l)
          if ((u32)l < na && ((selnew >> l) & 1u) && keyn[l] < keyn[k]) ++pk;
        if (lane == k) newpos = pk;
      }
    }
    const u32 nsel = (u32)__builtin_popcountll(alive) + (u32)__builtin_popcount(selnew);
    const u32 kept = nsel < R ? nsel : R;
    __syncthreads();
    if (isc && ((alive >> lane) & 1ull) && pos < R) row[pos] = myid;
    if ((u32)lane < na && ((selnew >> lane) & 1u) && newpos < R) row[newpos] = mynew;
    for (u32 j = kept + lane; j < R; j += 64) row[j] = NONE_ID;
    if (lane == 0) a.meta[b] = make_meta(kept, kept);
    return kept;
}

template <int KIND, int VEC, int NCH>
__global__ __launch_bounds__(64) void merge_fast_kernel(MergeArgs a, VecTable T) {
  constexpr int AMAX = FastAMax<NCH>::value;
  __shared__ u32 ids_lds[64 + AMAX];    // clean ids by row position, then the new ids
  __shared__ u32 dk_lds[1 + AMAX][64];  // distance keys by row position: to b, to each new entry

  const int lane = threadIdx.x;
  const u32 nitems = a.list_count[0];
  const AlphaParam al{a.a16, a.af};
  unsigned long long n_rep = 0, n_edges = 0, n_pair = 0;

  for (u32 it = blockIdx.x; it < nitems; it += gridDim.x) {
    const MergeItem item = a.list_items[0][it];
    const u32 i0 = item.i0, cnt = item.cnt, b = item.b, m = item.meta;
    const u32 deg = meta_deg(m), clean = meta_clean(m);
    const u32 stale = deg - clean;  // appended since the last prune
    const u32 na = stale + cnt;     // 1 <= na <= AMAX
    u32* row = a.graph + (u64)b * a.R;
    u32 kept = 0;
    // uniform dispatch on the number of new entries
#define ANN_FAST_CASE(N)                                                                                     \
  case N:                                                                                                    \
    if constexpr (AMAX >= N)                                                                                 \
      kept = fast_item<KIND, VEC, NCH, N>(a, T, al, ids_lds, dk_lds, b, i0, clean, stale, row, a.R, lane);   \
    break;
    switch (na) {
      ANN_FAST_CASE(1)
      ANN_FAST_CASE(2)
      ANN_FAST_CASE(3)
      ANN_FAST_CASE(4)
      ANN_FAST_CASE(5)
      ANN_FAST_CASE(6)
      ANN_FAST_CASE(7)
      ANN_FAST_CASE(8)
      default: break;
    }
#undef ANN_FAST_CASE
    (void)kept;
    ++n_rep;
    n_edges += cnt;
    n_pair += (unsigned long long)(clean + na) * (na + 1);
  }
  if (a.counters != nullptr && lane == 0 && n_rep) {
    atomicAdd(&block_counters(a.counters)->reprunes, n_rep);
    atomicAdd(&block_counters(a.counters)->edges, n_edges);
    atomicAdd(&block_counters(a.counters)->prune_evals, n_pair);
  }
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

struct SmallLds {
  u64 key[SM_TMAX];   // by arrival index
  u32 uid[SM_TMAX];   // ids by arrival index
  u32 nrm[SM_TMAX];   // squared norms of the shifted vectors, by arrival index
  u32 sid[SM_TMAX];   // ids, sorted by (distance to b, id)
  u32 snrm[SM_TMAX];  // norms, sorted
  i32 sthr[SM_TMAX];  // largest D(i,j) that still removes j, sorted
  u32 inv[SM_TMAX];   // sorted position -> arrival index
  // the entries behind the clean prefix ("new"), by their index among the new entries
  u32 nnrm[32];  // norms
  i32 nthr[32];  // largest D that still removes the new entry
  u32 npos[32];  // sorted positions
};

template <int VEC, int NCH>
struct SmallPathOk {
  static constexpr bool value = (8 * NCH * VEC <= 128);
};

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
  if constexpr (mlo < 64) {
    Klo = writelane_pair<mlo, mlo + 4>(Klo, bm);
  } else if constexpr (CB == 2) {
    Khi = writelane_pair<mlo - 64, mlo + 4 - 64>(Khi, bm);
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
  // all four k-steps unconditionally: operands beyond the row's last step are zeroed
  v4i_t av[4], bv[4];
#pragma unroll
  for (u32 ks = 0; ks < 4; ++ks) {
    const u32 kk = ks < ksteps ? ks : ksteps - 1u;
    const v4i_t x = *reinterpret_cast<const v4i_t*>(pa + 32u * kk);
    const v4i_t y = *reinterpret_cast<const v4i_t*>(pb + 32u * kk);
    av[ks] = ks < ksteps ? x : v4i_t{0, 0, 0, 0};
    bv[ks] = y;
  }
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(av[ks], bv[ks], acc, 0, 0, 0);
  const bool colok = ib < total;
  const i32 ncol = colok ? (i32)S.snrm[ib] : 0;
  const i32 tcol = colok ? S.sthr[ib] : -1;
  gram_tile_regs<RB, CB>(acc, S, colok, ncol, tcol, half, Klo, Khi, std::make_integer_sequence<int, 16>{});
}

// The same tile with the NEW entries as rows (new entry t in row t, at most 32 of them) and the
// sorted candidates 32*CB.. as columns.  Each accumulator register that holds rows below `na`
// yields two ballots: "new t removes sorted candidate j" (alpha * D <= d(b, j)) and "sorted
// candidate j removes new t" (alpha * D <= d(b, t)); lane t collects word CB of both masks.
template <int CB, int R_>
__device__ __forceinline__ void newrow_tile_reg(const v16i_t& acc, const i32 (&rown)[16], const i32 (&rowt)[16], u32 na,
                                                bool colok, i32 ncol, i32 tcol, u32 half, u32& rem, u32& rby) {
  constexpr int mlo = 8 * (R_ / 4) + (R_ % 4);
  if (na > (u32)(8 * (R_ / 4))) {  // uniform: rows 8*(R_/4).. exist
    const u32 t = (u32)mlo + 4u * half;
    const bool ok = colok && t < na;
    const i32 D = rown[R_] + ncol - 2 * acc[R_];
    const u64 b1 = ballot(ok && D <= tcol);
    const u64 b2 = ballot(ok && D <= rowt[R_]);
    rem = writelane_pair<mlo, mlo + 4>(rem, b1);
    rby = writelane_pair<mlo, mlo + 4>(rby, b2);
  }
}
template <int CB, int... Rs>
__device__ __forceinline__ void newrow_tile_regs(const v16i_t& acc, const i32 (&rown)[16], const i32 (&rowt)[16], u32 na,
                                                 bool colok, i32 ncol, i32 tcol, u32 half, u32& rem, u32& rby,
                                                 std::integer_sequence<int, Rs...>) {
  (newrow_tile_reg<CB, Rs>(acc, rown, rowt, na, colok, ncol, tcol, half, rem, rby), ...);
}
template <int CB>
__device__ __forceinline__ void newrow_tile(const unsigned char* Xs, const SmallLds& S, const i32 (&rown)[16],
                                            const i32 (&rowt)[16], u32 clean, u32 na, u32 total, u32 ksteps, int lane,
                                            u32& rem, u32& rby) {
  const u32 half = (u32)lane >> 5;
  const u32 t = (u32)lane & 31u;
  const u32 ib = 32u * CB + t;
  const u32 ra = clean + (t < na ? t : na - 1u);
  const u32 rb = ib < total ? S.inv[ib] : 0u;
  const unsigned char* pa = Xs + ra * SM_STRIDE + 16u * half;
  const unsigned char* pb = Xs + rb * SM_STRIDE + 16u * half;
  v4i_t av[4], bv[4];
#pragma unroll
  for (u32 ks = 0; ks < 4; ++ks) {
    const u32 kk = ks < ksteps ? ks : ksteps - 1u;
    const v4i_t x = *reinterpret_cast<const v4i_t*>(pa + 32u * kk);
    const v4i_t y = *reinterpret_cast<const v4i_t*>(pb + 32u * kk);
    av[ks] = ks < ksteps ? x : v4i_t{0, 0, 0, 0};
    bv[ks] = y;
  }
  v16i_t acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(av[ks], bv[ks], acc, 0, 0, 0);
  const bool colok = ib < total;
  const i32 ncol = colok ? (i32)S.snrm[ib] : 0;
  const i32 tcol = colok ? S.sthr[ib] : -1;
  newrow_tile_regs<CB>(acc, rown, rowt, na, colok, ncol, tcol, half, rem, rby, std::make_integer_sequence<int, 16>{});
}

// S.uid[0..total) holds the candidate ids (old row entries first), the first `clean` of which
// are the row's clean prefix: sorted, none removing another.  Writes the pruned row and
// returns its length.
template <int KIND, int VEC, int NCH>
__device__ __forceinline__ u32 reprune_small_int(const VecTable& T, const QueryRegs<KIND, VEC, NCH>& Q,
                                                 unsigned char* Xs, SmallLds& S, u32 total, u32 clean, u32 R,
                                                 i64 a16, u32* row, int lane) {
  // every pass of eight candidates is requested before the first is used (a pass is at most
  // four registers here): one trip to memory for the whole list
  constexpr int PB = SM_TMAX / 8;
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
      if (t0 + tt >= npass) break;  // uniform
      const u32 c = 8u * (t0 + tt) + grp;
      const u32 dk = distance_key<KIND, VEC, NCH>(Q, x[tt]);
      i32 nn = 0;
#pragma unroll
      for (int u = 0; u < NCH; ++u) {
        const u32 pc = sub + LPC * u;
        u32 wv[VEC / 4];
#pragma unroll
        for (int i = 0; i < VEC / 4; ++i) {
          wv[i] = pc < T.npieces ? (x[tt][u].w[i] ^ flip) : 0u;
          nn = __builtin_amdgcn_sdot4((i32)wv[i], (i32)wv[i], nn, false);
        }
        if (c < total) {
          unsigned char* dst = Xs + c * SM_STRIDE + pc * VEC;
          if constexpr (VEC == 16) {
            *reinterpret_cast<uint4*>(dst) = make_uint4(wv[0], wv[1], wv[2], wv[3]);
          } else {
#pragma unroll
            for (int i = 0; i < VEC / 4; ++i) *reinterpret_cast<u32*>(dst + 4 * i) = wv[i];
          }
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

  // rank of every candidate under (distance, id); keys are distinct.  With at most 32 entries
  // behind the clean prefix only those are compared against everything: a clean entry's rank is
  // its place in the prefix plus the new entries below it.
  const u32 na = total - clean;
  const bool by_new_rows = na <= 32u;
  {
    const u32 j0 = lane, j1 = lane + 64;
    const u64 k0 = j0 < total ? S.key[j0] : KEY_INF;
    const u64 k1 = j1 < total ? S.key[j1] : KEY_INF;
    u32 r0 = 0, r1 = 0;
    if (by_new_rows) {
      const bool c0 = j0 < clean, c1 = j1 < clean;
      u32 below0 = 0, below1 = 0;  // for a new entry: clean entries below it
      for (u32 k = clean; k < total; ++k) {
        const u64 kk = S.key[k];
        const bool g0 = kk < k0, g1 = kk < k1;
        r0 += g0 ? 1u : 0u;
        r1 += g1 ? 1u : 0u;
        const u32 above = (u32)__builtin_popcountll(ballot(g0 && c0)) + (u32)__builtin_popcountll(ballot(g1 && c1));
        if (j0 == k) below0 = clean - above;
        if (j1 == k) below1 = clean - above;
      }
      r0 += c0 ? j0 : below0;
      r1 += c1 ? j1 : below1;
    } else {
      for (u32 i = 0; i < total; ++i) {
        const u64 ki = S.key[i];
        r0 += ki < k0 ? 1u : 0u;
        r1 += ki < k1 ? 1u : 0u;
      }
    }
    if (j0 < total) {
      const i32 thr = alpha_threshold(int_from_dkey(key_dkey(k0)), a16);
      S.sid[r0] = key_id(k0);
      S.snrm[r0] = S.nrm[j0];
      S.sthr[r0] = thr;
      S.inv[r0] = j0;
      if (by_new_rows && j0 >= clean) {
        S.nnrm[j0 - clean] = S.nrm[j0];
        S.nthr[j0 - clean] = thr;
        S.npos[j0 - clean] = r0;
      }
    }
    if (j1 < total) {
      const i32 thr = alpha_threshold(int_from_dkey(key_dkey(k1)), a16);
      S.sid[r1] = key_id(k1);
      S.snrm[r1] = S.nrm[j1];
      S.sthr[r1] = thr;
      S.inv[r1] = j1;
      if (by_new_rows && j1 >= clean) {
        S.nnrm[j1 - clean] = S.nrm[j1];
        S.nthr[j1 - clean] = thr;
        S.npos[j1 - clean] = r1;
      }
    }
  }
  __syncthreads();

  const u32 nb = (total + 31u) >> 5;
  const u32 ksteps = (u32)((T.row_bytes + 31) / 32);
  if (by_new_rows) {
    // distances between the new entries and everything, reduced at once to two 96-bit masks per
    // new entry (lane t: new entry t)
    u32 REM[3] = {0u, 0u, 0u}, RBY[3] = {0u, 0u, 0u};
    // norm and threshold of the row each accumulator register holds in this lane (the same in
    // every tile); rows that do not exist are never looked at
    i32 rown[16], rowt[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      rown[r] = 0;
      rowt[r] = -1;
      if (na > (u32)(8 * (r / 4))) {  // uniform
        const u32 t = (u32)(8 * (r / 4) + (r % 4)) + 4u * ((u32)lane >> 5);
        rown[r] = (i32)S.nnrm[t];
        rowt[r] = S.nthr[t];
      }
    }
    newrow_tile<0>(Xs, S, rown, rowt, clean, na, total, ksteps, lane, REM[0], RBY[0]);
    if (nb > 1) newrow_tile<1>(Xs, S, rown, rowt, clean, na, total, ksteps, lane, REM[1], RBY[1]);
    if (nb > 2) newrow_tile<2>(Xs, S, rown, rowt, clean, na, total, ksteps, lane, REM[2], RBY[2]);
    const u32 mypos = (u32)lane < na ? S.npos[lane] : 0xFFFFFFFFu;

    // replay of the scan of prune() on positions of the sorted list: the clean entries are all
    // selected until a selected new entry in front of them removes them; the new entries are
    // decided in sorted order
    const u32 nlo = total < 64u ? total : 64u;
    u64 sel_lo = nlo == 64u ? ~0ull : ((1ull << nlo) - 1ull);
    u32 sel_hi = total > 64u ? ((total - 64u) >= 32u ? ~0u : ((1u << (total - 64u)) - 1u)) : 0u;
    u64 new_lo = 0;  // positions held by new entries
    u32 new_hi = 0;
    for (u32 t = 0; t < na; ++t) {
      const u32 p = readlane_u32(mypos, (int)t);
      if (p < 64u)
        new_lo |= 1ull << p;
      else
        new_hi |= 1u << (p - 64u);
    }
    sel_lo &= ~new_lo;
    sel_hi &= ~new_hi;
    u64 todo_lo = new_lo;
    u32 todo_hi = new_hi;
    while (todo_lo != 0 || todo_hi != 0) {
      u32 p;
      if (todo_lo != 0) {
        p = (u32)__builtin_ctzll(todo_lo);
        todo_lo &= todo_lo - 1ull;
      } else {
        p = 64u + (u32)__builtin_ctz(todo_hi);
        todo_hi &= todo_hi - 1u;
      }
      const int t = __builtin_ctzll(ballot(mypos == p));  // the new entry at position p
      const u64 before_lo = p >= 64u ? ~0ull : ((1ull << p) - 1ull);
      const u32 before_hi = p >= 64u ? ((1u << (p - 64u)) - 1u) : 0u;
      const u64 rby_lo = (u64)readlane_u32(RBY[0], t) | ((u64)readlane_u32(RBY[1], t) << 32);
      const u32 rby_hi = readlane_u32(RBY[2], t);
      const bool killed = ((rby_lo & sel_lo & before_lo) | (u64)(rby_hi & sel_hi & before_hi)) != 0;
      if (!killed) {
        const u64 rem_lo = (u64)readlane_u32(REM[0], t) | ((u64)readlane_u32(REM[1], t) << 32);
        const u32 rem_hi = readlane_u32(REM[2], t);
        sel_lo &= ~(rem_lo & ~before_lo);
        sel_hi &= ~(rem_hi & ~before_hi);
        if (p < 64u)
          sel_lo |= 1ull << p;
        else
          sel_hi |= 1u << (p - 64u);
      }
    }
    // the first R selected positions, in order
    const u32 cnt_lo = (u32)__builtin_popcountll(sel_lo);
    const u32 nsel = cnt_lo + (u32)__builtin_popcount(sel_hi);
    const u32 nout = nsel < R ? nsel : R;
    if ((sel_lo >> lane) & 1ull) {
      const u32 at = (u32)__builtin_popcountll(sel_lo & lanemask_lt(lane));
      if (at < R) row[at] = S.sid[lane];
    }
    if (lane < 32 && ((sel_hi >> lane) & 1u)) {
      const u32 at = cnt_lo + (u32)__builtin_popcount(sel_hi & ((1u << lane) - 1u));
      if (at < R) row[at] = S.sid[64 + lane];
    }
    for (u32 j = nout + lane; j < R; j += 64) row[j] = NONE_ID;
    __syncthreads();
    return nout;
  }

  // Gram matrix tile by tile; K0[c] of lane i = bits "sorted candidate i removes candidate 32c+j",
  // K1 the same for candidates 64..95 (only column block 2 matters there)
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
  return nout;
}

// ---------------------------------------------------------------------------------------------
// gram path kernel
// ---------------------------------------------------------------------------------------------
template <int KIND, int VEC, int NCH>
__global__ __launch_bounds__(64) void merge_gram_kernel(MergeArgs a, VecTable T) {
  constexpr bool kOk = KindTraits<KIND>::is_int && SmallPathOk<VEC, NCH>::value;
  if constexpr (kOk) {
    __shared__ __align__(16) unsigned char Xs[SM_TMAX * SM_STRIDE];
    __shared__ SmallLds small;
    const int lane = threadIdx.x;
    const u32 nitems = a.list_count[1];
    unsigned long long n_rep = 0, n_edges = 0, n_pair = 0;
    for (u32 it = blockIdx.x; it < nitems; it += gridDim.x) {
      const MergeItem item = a.list_items[1][it];
      const u32 i0 = item.i0, cnt = item.cnt, b = item.b;
      const u32 deg = meta_deg(item.meta), clean = meta_clean(item.meta);
      const u32 total = deg + cnt;
      u32* row = a.graph + (u64)b * a.R;
      for (u32 j = lane; j < total; j += 64)
        small.uid[j] = j < deg ? row[j] : (u32)(a.keys[i0 + (j - deg)] & 0xFFFFFFFFull);
      __syncthreads();
      const QueryRegs<KIND, VEC, NCH> Qb = load_query<KIND, VEC, NCH>(T.base + (u64)b * T.row_bytes, T.npieces, lane);
      const u32 kept = reprune_small_int<KIND, VEC, NCH>(T, Qb, Xs, small, total, clean, a.R, a.a16, row, lane);
      if (lane == 0) a.meta[b] = make_meta(kept, kept);
      ++n_rep;
      n_edges += cnt;
      // pairs whose distance was formed: all of them, or only those with a new entry in them
      n_pair += total - clean <= 32u ? (unsigned long long)(total - clean) * total : (unsigned long long)total * (total + 1) / 2;
    }
    if (a.counters != nullptr && lane == 0 && n_rep) {
      atomicAdd(&block_counters(a.counters)->reprunes, n_rep);
      atomicAdd(&block_counters(a.counters)->edges, n_edges);
      atomicAdd(&block_counters(a.counters)->prune_evals, n_pair);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// generic path kernel
// ---------------------------------------------------------------------------------------------
// CAP: candidate keys the kernel sorts in LDS.  Two instances: MERGE_SPILL_MIN for the few rows
// with long lists (hub vertices; beyond it the list goes to the arena), and MERGE_MEDIUM_MAX for
// the rows in between, which are many when batches hold millions of points: with the large
// buffer three waves fit a compute unit, with the small one sixteen.
template <int KIND, int VEC, int NCH, u32 CAP>
__global__ __launch_bounds__(64) void merge_generic_kernel(MergeArgs a, VecTable T) {
  constexpr int LIST = CAP == MERGE_SPILL_MIN ? 2 : 3;
  __shared__ u64 cand_lds[CAP];
  extern __shared__ __align__(16) unsigned char smem[];
  u32* out = reinterpret_cast<u32*>(smem);  // R entries
  SelStage st;
  st.stride = stage_stride(T.row_bytes);
  st.xx = out + a.R;
  unsigned char* blk = smem + ((a.R * 8u + 15u) & ~15u);  // 8 rows + 8 norms
  st.vec = a.stage_bytes ? blk + 8u * st.stride + 32u : nullptr;
  constexpr bool kMfma = MfmaPruneOk<KIND, VEC, NCH>::value;
  const MfmaLds M = mfma_lds_carve(smem + ((a.R * 4u + 15u) & ~15u), a.R, T.row_bytes);  // used when a.use_mfma

  const int lane = threadIdx.x;
  const u32 nitems = a.list_count[LIST];
  if (blockIdx.x >= nitems) return;
  const AlphaParam al{a.a16, a.af};
  unsigned long long n_rep = 0, n_edges = 0, n_pair = 0;

  for (u32 it = blockIdx.x; it < nitems; it += gridDim.x) {
    const MergeItem item = a.list_items[LIST][LIST == 3 ? -(long long)it : (long long)it];
    const u32 i0 = item.i0, cnt = item.cnt, b = item.b;
    const u32 deg = meta_deg(item.meta);
    const u32 total = deg + cnt;
    u32* row = a.graph + (u64)b * a.R;

    // candidate list U = N_out(b) followed by the new sources
    u64* cand;
    const bool in_lds = total <= CAP;
    if (in_lds) {
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
    const QueryRegs<KIND, VEC, NCH> Q = load_query<KIND, VEC, NCH>(T.base + (u64)b * T.row_bytes, T.npieces, lane);
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
    u32 kept;
    if (in_lds) {
      u32 n2 = 64;
      while (n2 < total) n2 <<= 1;
      for (u32 j = total + lane; j < n2; j += 64) cand[j] = KEY_INF;
      __syncthreads();
      bitonic_sort_keys(cand, n2, lane);
      bool done = false;
      if constexpr (kMfma) {
        if (a.use_mfma) {
          kept = prune_sorted_mfma<KIND, VEC, NCH>(T, M, cand, total, a.R, a.a16, out, lane, pair_evals);
          done = true;
        }
      }
      if (!done) kept = prune_sorted<KIND, VEC, NCH>(T, st, blk, cand, total, a.R, al, out, lane, pair_evals);
    } else {
      // (the staged-vector areas are laid out for the walk in use; the minimum-search walk reads
      // the selected vectors from device memory when the matrix-core layout is active)
      SelStage st2 = st;
      if (a.use_mfma) st2.vec = nullptr;
      kept = prune_unsorted<KIND, VEC, NCH>(T, st2, cand, total, a.R, al, out, lane, pair_evals);
    }
    __syncthreads();
    for (u32 j = lane; j < a.R; j += 64) row[j] = j < kept ? out[j] : NONE_ID;
    if (lane == 0) a.meta[b] = make_meta(kept, kept);
    __syncthreads();
    ++n_rep;
    n_edges += cnt;
    n_pair += pair_evals;
  }
  if (a.counters != nullptr && lane == 0 && n_rep) {
    atomicAdd(&block_counters(a.counters)->reprunes, n_rep);
    atomicAdd(&block_counters(a.counters)->edges, n_edges);
    atomicAdd(&block_counters(a.counters)->prune_evals, n_pair);
  }
}

// The three kernels work on disjoint rows, so they may run side by side: s_gram and s_generic are
// side streams the caller has already made wait for the planning kernel.
template <int KIND, int VEC, int NCH>
static hipError_t launch_merge_t(const MergeArgs& a, const VecTable& T, u32 grid, hipStream_t s, hipStream_t s_gram,
                                 hipStream_t s_generic, hipStream_t s_medium) {
  // the generic kernel's few, long items first, so that they start at once instead of waiting
  // for LDS that the other two kernels' workgroups hold; a small grid serves its short list
  const u32 lds = a.use_mfma ? ((a.R * 4u + 15u) & ~15u) + mfma_lds_bytes(a.R, T.row_bytes)
                            : ((a.R * 8u + 15u) & ~15u) + 8u * stage_stride(T.row_bytes) + 32u + a.stage_bytes;
  const u32 grid_generic = (grid < 1024u || a.force_prune) ? grid : 1024u;
  hipLaunchKernelGGL((merge_generic_kernel<KIND, VEC, NCH, MERGE_SPILL_MIN>), dim3(grid_generic), dim3(64), lds,
                     s_generic, a, T);
  if (a.medium_max)
    hipLaunchKernelGGL((merge_generic_kernel<KIND, VEC, NCH, MERGE_MEDIUM_MAX>), dim3(grid), dim3(64), lds, s_medium, a,
                       T);
  // the caller's stream takes the kernel that usually ends last, so that its waits for the other
  // two streams are already satisfied when it reaches them
  if (a.gram_ok) {
    hipLaunchKernelGGL((merge_fast_kernel<KIND, VEC, NCH>), dim3(grid), dim3(64), 0, s_gram, a, T);
    hipLaunchKernelGGL((merge_gram_kernel<KIND, VEC, NCH>), dim3(grid), dim3(64), 0, s, a, T);
  } else {
    hipLaunchKernelGGL((merge_fast_kernel<KIND, VEC, NCH>), dim3(grid), dim3(64), 0, s, a, T);
  }
  return hipGetLastError();
}

hipError_t launch_merge(const DistCfg& cfg, const MergeArgs& a, u32 grid, hipStream_t s, hipStream_t s_gram,
                        hipStream_t s_generic, hipStream_t s_medium) {
  if (grid == 0) return hipSuccess;
  VecTable T{a.points, (u32)cfg.row_bytes, cfg.npieces};
  ANN_DISPATCH_CFG(launch_merge_t, a, T, grid, s, s_gram, s_generic, s_medium);
}

bool gram_path_ok(const DistCfg& cfg) { return cfg.kind <= 1 && 8 * cfg.nch * cfg.vec <= 128; }
u32 gram_path_tmax() { return SM_TMAX; }
bool mfma_prune_ok(u32 R, const DistCfg& cfg) {
  return cfg.kind <= 1 && 8 * cfg.nch * cfg.vec <= 128 && mfma_lds_bytes(R, (u32)cfg.row_bytes) <= 24576u;
}
u32 prune_stage_bytes(u32 R, const DistCfg& cfg) { return stage_bytes(R, (u32)cfg.row_bytes, STAGE_BUDGET); }
u32 fast_path_amax(const DistCfg& cfg) { return cfg.nch <= 2 ? 4u : (cfg.nch <= 4 ? 2u : 1u); }

// rows given from outside: degree from the row itself, no clean prefix known
__global__ __launch_bounds__(256) void meta_from_rows_kernel(const u32* graph, u64 n, u32 R, u32* meta) {
  const u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const u32* row = graph + i * R;
  u32 deg = 0;
  while (deg < R && row[deg] != NONE_ID) ++deg;
  meta[i] = make_meta(deg, 0u);
}
__global__ __launch_bounds__(256) void meta_forget_clean_kernel(u64 n, u32* meta) {
  const u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) meta[i] &= 0xFFFFu;
}

hipError_t launch_meta_from_rows(const u32* graph, u64 n, u32 R, u32* meta, hipStream_t s) {
  hipLaunchKernelGGL(meta_from_rows_kernel, dim3((u32)((n + 255) / 256)), dim3(256), 0, s, graph, n, R, meta);
  return hipGetLastError();
}
hipError_t launch_meta_forget_clean(u64 n, u32* meta, hipStream_t s) {
  hipLaunchKernelGGL(meta_forget_clean_kernel, dim3((u32)((n + 255) / 256)), dim3(256), 0, s, n, meta);
  return hipGetLastError();
}

}  // namespace annmi
