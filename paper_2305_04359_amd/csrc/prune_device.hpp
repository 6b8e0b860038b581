// The alpha-prune scan of Sec. 4.1 as a wavefront-wide device routine, shared by step 1 and
// step 2 of BatchInsert.
//
// prune(p, C, R) walks C in order of (distance to p, id); a candidate is selected unless a point
// selected before it removes it (alpha * d(p*, c) <= d(p, c)); the walk ends with R selections.
// The wave follows that walk eight candidates at a time: each group of 8 lanes holds one of the
// next eight candidates in registers and measures it against every point selected so far (the
// same selected vector is broadcast from LDS to all groups) and against the other seven; the
// eight verdicts are then settled in order on bit masks.  Candidates behind the R-th selection
// are never looked at.  The vectors of the selected points (at most R) are kept in LDS when they
// fit, with their squared norms, so the only global traffic is one load per candidate, issued a
// block ahead.
#pragma once

#include <utility>

#include "ann_device.hpp"

namespace annmi {

// In-place ascending bitonic sort of n2 keys (a power of two >= 2) by one wave, every step a trip
// through LDS: for the sizes the register version below does not cover.
__device__ __forceinline__ void bitonic_sort_keys_lds(u64* a, u32 n2, int lane) {
  for (u32 k = 2; k <= n2; k <<= 1) {
    for (u32 j = k >> 1; j > 0; j >>= 1) {
      for (u32 t = lane; t < (n2 >> 1); t += 64) {
        const u32 i = 2u * t - (t & (j - 1u));
        const u32 l = i + j;
        const bool up = (i & k) == 0u;
        const u64 x = a[i], y = a[l];
        if ((x > y) == up) {
          a[i] = y;
          a[l] = x;
        }
      }
      __syncthreads();
    }
  }
}

// The same sort with the keys in registers: key 64 q + lane is v[q] of the lane.  Partners 64
// keys or more apart are two registers of one lane; partners inside a row of 16 lanes are reached
// with data-parallel-primitive moves (quad permutations for 1 and 2 lanes, the row turned by 8,
// and for 4 lanes the row turned by 12 for the banks whose partner is above, by 4 for the others);
// only partners 16 and 32 lanes away go through the LDS crossbar.  No barrier, no LDS round trip.
template <u32 J>
__device__ __forceinline__ u32 lane_partner_word(u32 x, int lane) {
  if constexpr (J == 1) {
    return (u32)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xF, 0xF, true);
  } else if constexpr (J == 2) {
    return (u32)__builtin_amdgcn_update_dpp(0, (int)x, 0x4E, 0xF, 0xF, true);
  } else if constexpr (J == 4) {
    return (u32)__builtin_amdgcn_update_dpp(__builtin_amdgcn_update_dpp(0, (int)x, 0x12C, 0xF, 0x5, false), (int)x, 0x124,
                                            0xF, 0xA, false);
  } else if constexpr (J == 8) {
    return (u32)__builtin_amdgcn_update_dpp(0, (int)x, 0x128, 0xF, 0xF, true);
  } else {
    return (u32)__builtin_amdgcn_ds_bpermute((int)(((u32)lane ^ J) << 2), (int)x);
  }
}

template <int KPL, u32 K, u32 J>
struct BitonicStep {
  static __device__ __forceinline__ void run(u64 (&v)[KPL], int lane) {
    if constexpr (J >= 64) {
      constexpr u32 dq = J / 64;
#pragma unroll
      for (u32 q = 0; q < (u32)KPL; ++q) {
        if ((q & dq) == 0) {
          const bool asc = ((64u * q) & K) == 0;  // (K > J >= 64: the lane bits do not matter)
          const u64 x = v[q], y = v[q | dq];
          const bool swap = (x > y) == asc;
          v[q] = swap ? y : x;
          v[q | dq] = swap ? x : y;
        }
      }
    } else {
      const bool low_side = ((u32)lane & J) == 0;
#pragma unroll
      for (u32 q = 0; q < (u32)KPL; ++q) {
        const bool asc = ((64u * q + (u32)lane) & K) == 0;
        const u64 o = ((u64)lane_partner_word<J>((u32)(v[q] >> 32), lane) << 32) | lane_partner_word<J>((u32)v[q], lane);
        // keeps its own key if that is the one wanted here: the smaller on the low side of an
        // ascending run, the larger on its high side (keys are distinct or equal: either)
        v[q] = ((v[q] < o) == (low_side == asc)) ? v[q] : o;
      }
    }
    if constexpr (J > 1) BitonicStep<KPL, K, J / 2>::run(v, lane);
  }
};

template <int KPL, u32 K>
struct BitonicStage {
  static __device__ __forceinline__ void run(u64 (&v)[KPL], int lane) {
    BitonicStep<KPL, K, K / 2>::run(v, lane);
    if constexpr (K < 64u * KPL) BitonicStage<KPL, 2 * K>::run(v, lane);
  }
};

template <int KPL>
__device__ __forceinline__ void bitonic_sort_regs(u64* a, int lane) {
  u64 v[KPL];
#pragma unroll
  for (int q = 0; q < KPL; ++q) v[q] = a[64 * q + lane];
  BitonicStage<KPL, 2>::run(v, lane);
#pragma unroll
  for (int q = 0; q < KPL; ++q) a[64 * q + lane] = v[q];
}

// In-place ascending sort of n2 keys in LDS (a power of two >= 64) by one wave; the keys must be
// visible to the wave when it is called and are visible to it on return.
__device__ __forceinline__ void bitonic_sort_keys(u64* a, u32 n2, int lane) {
  switch (n2) {
    case 64: bitonic_sort_regs<1>(a, lane); break;
    case 128: bitonic_sort_regs<2>(a, lane); break;
    case 256: bitonic_sort_regs<4>(a, lane); break;
    case 512: bitonic_sort_regs<8>(a, lane); break;
    default: bitonic_sort_keys_lds(a, n2, lane); return;
  }
  __syncthreads();
}

// LDS copy of the selected points' vectors
struct SelStage {
  unsigned char* vec;  // R rows of `stride` bytes, or null: read the vectors from device memory
  u32* xx;             // <x,x> of each selected point (integer kinds)
  u32 stride;
};

// Does a selected point remove candidate c?  Qc holds c's vector, dkey_pc = d(p, c).
template <int KIND, int VEC, int NCH>
__device__ __forceinline__ bool removed_by_selected(const VecTable& T, const SelStage& st,
                                                    const QueryRegs<KIND, VEC, NCH>& Qc, u32 dkey_pc,
                                                    const u32* out, u32 nout, const AlphaParam& al, int lane,
                                                    u32& pair_evals) {
  pair_evals += nout;
  if (st.vec != nullptr) {
    const int sub = lane & (LPC - 1);
    const u32 grp = (u32)lane >> 3;
    bool dom = false;
    const u32 npass = (nout + 7u) >> 3;
    for (u32 t = 0; t < npass; ++t) {
      const u32 idx = 8u * t + grp;
      const bool ok = idx < nout;
      const unsigned char* src = st.vec + (ok ? idx : 0u) * st.stride;
      Piece<VEC> x[NCH];
#pragma unroll
      for (int u = 0; u < NCH; ++u) {
        const u32 pc = sub + LPC * u;
        x[u] = pc < T.npieces ? load_piece<VEC>(reinterpret_cast<const char*>(src) + pc * VEC) : zero_piece<VEC>();
      }
      u32 dk;
      if constexpr (KindTraits<KIND>::is_int) {
        i32 qx = 0;
#pragma unroll
        for (int u = 0; u < NCH; ++u)
#pragma unroll
          for (int i = 0; i < VEC / 4; ++i) {
            if constexpr (KIND == K_U8)
              qx = (i32)__builtin_amdgcn_udot4(Qc.q[u].w[i], x[u].w[i], (u32)qx, false);
            else
              qx = __builtin_amdgcn_sdot4((i32)Qc.q[u].w[i], (i32)x[u].w[i], qx, false);
          }
        dk = dkey_from_int(Qc.qq + (i32)st.xx[ok ? idx : 0u] - 2 * group_sum(qx));
      } else {
        dk = distance_key<KIND, VEC, NCH>(Qc, x);
      }
      dom = dom || (ok && alpha_dominates<KIND>(al, dk, dkey_pc));
    }
    return ballot(dom) != 0;
  }
  for (u32 base = 0; base < nout; base += 64) {
    const u32 cnt = nout - base < 64u ? nout - base : 64u;
    const u32* ob = out + base;
    const u32 dk = eval_up_to_64<KIND, VEC, NCH>(T, Qc, [ob](u32 i) { return ob[i]; }, cnt, lane);
    const bool dom = cand_of_lane(lane) < cnt && alpha_dominates<KIND>(al, dk, dkey_pc);
    if (ballot(dom) != 0) return true;
  }
  return false;
}

template <int KIND, int VEC, int NCH>
__device__ __forceinline__ void stage_selected(const VecTable& T, const SelStage& st,
                                               const QueryRegs<KIND, VEC, NCH>& Qc, u32 slot, int lane) {
  if (st.vec == nullptr) return;
  if (lane < LPC) {
#pragma unroll
    for (int u = 0; u < NCH; ++u) {
      const u32 pc = lane + LPC * u;
      if (pc < T.npieces) {
        unsigned char* dst = st.vec + slot * st.stride + pc * VEC;
#pragma unroll
        for (int i = 0; i < VEC / 4; ++i) reinterpret_cast<u32*>(dst)[i] = Qc.q[u].w[i];
      }
    }
    if (lane == 0) st.xx[slot] = (u32)Qc.qq;
  }
}

// largest D with alpha * D <= d, per kind: integers as floor(d * 2^16 / a16), floats via the product
template <int KIND>
struct RemoveTest {
  i32 thr;    // integer kinds
  float dpc;  // float kinds
  float af;
  __device__ __forceinline__ void set(const AlphaParam& al, u32 dkey_pc) {
    if constexpr (KindTraits<KIND>::is_int) {
      const i32 d = int_from_dkey(dkey_pc);
      // floor(d * 65536 / a16), exact (d >= 0 for squared L2)
      const u64 x = (u64)(u32)d << 16;
      u64 t = (u64)__builtin_floor((double)x / (double)al.a16);
      if (t * (u64)al.a16 > x)
        --t;
      else if ((t + 1) * (u64)al.a16 <= x)
        ++t;
      thr = t > 0x7FFFFFFFull ? 0x7FFFFFFF : (i32)t;
    } else {
      dpc = float_from_dkey(dkey_pc);
      af = al.af;
    }
  }
  // d_sc: distance selected <-> candidate (integer, or float bits)
  __device__ __forceinline__ bool removes_int(i32 d_sc) const { return d_sc <= thr; }
  __device__ __forceinline__ bool removes_float(float d_sc) const { return af * d_sc <= dpc; }
};

// distance between the group's candidate (in Qc) and the row pieces x; xx = <x,x> (integers)
template <int KIND, int VEC, int NCH>
__device__ __forceinline__ bool removes_pieces(const RemoveTest<KIND>& rt, const QueryRegs<KIND, VEC, NCH>& Qc,
                                               const Piece<VEC> (&x)[NCH], i32 xx) {
  if constexpr (KindTraits<KIND>::is_int) {
    i32 qx = 0;
#pragma unroll
    for (int u = 0; u < NCH; ++u)
#pragma unroll
      for (int i = 0; i < VEC / 4; ++i) {
        if constexpr (KIND == K_U8)
          qx = (i32)__builtin_amdgcn_udot4(Qc.q[u].w[i], x[u].w[i], (u32)qx, false);
        else
          qx = __builtin_amdgcn_sdot4((i32)Qc.q[u].w[i], (i32)x[u].w[i], qx, false);
      }
    return rt.removes_int(Qc.qq + xx - 2 * group_sum(qx));
  } else {
    return rt.removes_float(float_from_dkey(distance_key<KIND, VEC, NCH>(Qc, x)));
  }
}

// cand[0..m): keys (distance to p | id), ids distinct, p absent, SORTED ascending.
// Selected ids go to out[0..return) in selection order.  blk: LDS for 8 rows of st.stride bytes
// plus 8 norms (used even when the selected vectors themselves are not staged).
template <int KIND, int VEC, int NCH>
__device__ __forceinline__ u32 prune_sorted(const VecTable& T, const SelStage& st, unsigned char* blk,
                                            const u64* cand, u32 m, u32 R, const AlphaParam& al, u32* out,
                                            int lane, u32& pair_evals) {
  const int sub = lane & (LPC - 1);
  const u32 grp = (u32)lane >> 3;
  u32* blkxx = reinterpret_cast<u32*>(blk + 8u * st.stride);
  u32 nout = 0;
  if (m == 0) return 0;
  const u64 k0 = grp < m ? cand[grp] : KEY_INF;
  u64 nkey = k0;
  QueryRegs<KIND, VEC, NCH> nxt =
      load_query_raw<KIND, VEC, NCH>(T.base + (u64)(grp < m ? key_id(k0) : 0u) * T.row_bytes, T.npieces, lane);
  for (u32 i0 = 0; i0 < m && nout < R; i0 += 8) {
    QueryRegs<KIND, VEC, NCH> cur = nxt;
    const u64 key = nkey;
    const bool valid = i0 + grp < m;
    {  // next block's vectors travel while this block is settled
      const u32 ci = i0 + 8u + grp;
      nkey = ci < m ? cand[ci] : KEY_INF;
      nxt = load_query_raw<KIND, VEC, NCH>(T.base + (u64)(ci < m ? key_id(nkey) : 0u) * T.row_bytes, T.npieces, lane);
    }
    query_finish<KIND, VEC, NCH>(cur);
    RemoveTest<KIND> rt;
    rt.set(al, valid ? key_dkey(key) : dkey_from_int(0));
    const u32 nb = m - i0 < 8u ? m - i0 : 8u;

    // park the block's vectors in LDS for the tests among the eight
#pragma unroll
    for (int u = 0; u < NCH; ++u) {
      const u32 pc = sub + LPC * u;
      if (pc < T.npieces) {
        unsigned char* dst = blk + grp * st.stride + pc * VEC;
#pragma unroll
        for (int i = 0; i < VEC / 4; ++i) reinterpret_cast<u32*>(dst)[i] = cur.q[u].w[i];
      }
    }
    if (sub == 0) blkxx[grp] = (u32)cur.qq;

    // against everything selected before this block
    bool dom = false;
    if (st.vec != nullptr) {
      auto test = [&](u32 t) -> bool {
        const unsigned char* src = st.vec + t * st.stride;
        Piece<VEC> x[NCH];
#pragma unroll
        for (int u = 0; u < NCH; ++u) {
          const u32 pc = sub + LPC * u;
          x[u] = pc < T.npieces ? load_piece<VEC>(reinterpret_cast<const char*>(src) + pc * VEC) : zero_piece<VEC>();
        }
        return removes_pieces<KIND, VEC, NCH>(rt, cur, x, (i32)st.xx[t]);
      };
      // four selected points per trip, written out by hand (loops around cross-lane operations
      // are not unrolled for us), so that their LDS reads overlap
      u32 t = 0;
      for (; t + 4 <= nout; t += 4) {
        const bool r0 = test(t), r1 = test(t + 1), r2 = test(t + 2), r3 = test(t + 3);
        dom = dom | r0 | r1 | r2 | r3;
      }
      for (; t < nout; ++t) {
        const bool r = test(t);
        dom = dom | r;
      }
    } else {
      for (u32 t = 0; t < nout; ++t) {
        const char* src = T.base + (u64)out[t] * T.row_bytes;
        Piece<VEC> x[NCH];
#pragma unroll
        for (int u = 0; u < NCH; ++u) {
          const u32 pc = sub + LPC * u;
          x[u] = pc < T.npieces ? load_piece<VEC>(src + (u64)pc * VEC) : zero_piece<VEC>();
        }
        i32 xx = 0;
        if constexpr (KindTraits<KIND>::is_int) {
#pragma unroll
          for (int u = 0; u < NCH; ++u)
#pragma unroll
            for (int i = 0; i < VEC / 4; ++i) {
              if constexpr (KIND == K_U8)
                xx = (i32)__builtin_amdgcn_udot4(x[u].w[i], x[u].w[i], (u32)xx, false);
              else
                xx = __builtin_amdgcn_sdot4((i32)x[u].w[i], (i32)x[u].w[i], xx, false);
            }
          xx = group_sum(xx);
        }
        const bool r = removes_pieces<KIND, VEC, NCH>(rt, cur, x, xx);
        dom = dom | r;
      }
    }
    pair_evals += nout * nb;
    const u64 dead_before = ballot(dom && valid);
    __syncthreads();

    // among the eight: bit 8g of by[t] says "candidate t of the block removes candidate g"
    u64 by[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      by[t] = 0;
      if ((u32)t < nb) {  // uniform
        const unsigned char* src = blk + t * st.stride;
        Piece<VEC> x[NCH];
#pragma unroll
        for (int u = 0; u < NCH; ++u) {
          const u32 pc = sub + LPC * u;
          x[u] = pc < T.npieces ? load_piece<VEC>(reinterpret_cast<const char*>(src) + pc * VEC) : zero_piece<VEC>();
        }
        const bool r = removes_pieces<KIND, VEC, NCH>(rt, cur, x, (i32)blkxx[t]);
        by[t] = ballot(r && valid && (u32)t < grp);
      }
    }
    pair_evals += nb * (nb - 1) / 2;

    // settle the eight in order
    u32 selmask = 0, nsel = 0;
#pragma unroll
    for (int g = 0; g < 8; ++g) {
      if ((u32)g < nb && nout + nsel < R) {
        bool removed = (dead_before >> (8 * g)) & 1ull;
#pragma unroll
        for (int t = 0; t < g; ++t) removed = removed || (((selmask >> t) & 1u) && ((by[t] >> (8 * g)) & 1ull));
        if (!removed) {
          selmask |= 1u << g;
          ++nsel;
        }
      }
    }
    // commit the selected ones: ids, vectors and norms, in order
    if (valid && ((selmask >> grp) & 1u)) {
      const u32 slot = nout + (u32)__builtin_popcount(selmask & ((1u << grp) - 1u));
      if (sub == 0) out[slot] = key_id(key);
      if (st.vec != nullptr) {
#pragma unroll
        for (int u = 0; u < NCH; ++u) {
          const u32 pc = sub + LPC * u;
          if (pc < T.npieces) {
            unsigned char* dst = st.vec + slot * st.stride + pc * VEC;
#pragma unroll
            for (int i = 0; i < VEC / 4; ++i) reinterpret_cast<u32*>(dst)[i] = cur.q[u].w[i];
          }
        }
        if (sub == 0) st.xx[slot] = (u32)cur.qq;
      }
    }
    nout += nsel;
    __syncthreads();
  }
  return nout;
}

// ---------------------------------------------------------------------------------------------
// The same walk for u8/i8 rows of at most 128 bytes, 32 candidates at a time, with the pair
// distances taken on the matrix cores.
//
// For a block of 32 candidates two small matrix products decide everything: (selected so far) x
// (block) tells which candidates are removed by an earlier selection, and (block) x (block) which
// candidate would remove which later one.  Both are Gram-type products of int8 vectors (u8 data
// is shifted by -128; distances do not change), exact in int32, computed with
// v_mfma_i32_32x32x32_i8 from LDS copies of the vectors: D(i,j) = |x_i|^2 + |x_j|^2 - 2<x_i,x_j>,
// and "i removes j" is D(i,j) <= floor(d(p,j) * 2^16 / a16).  The 32 verdicts are then settled in
// order on bit masks.
// ---------------------------------------------------------------------------------------------
typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef int v16i_t __attribute__((ext_vector_type(16)));

constexpr u32 MM_STRIDE = 144;  // bytes between staged rows (128 + 16: spreads LDS banks)
constexpr u32 MM_BLOCK = 32;    // candidates per block

template <int KIND, int VEC, int NCH>
struct MfmaPruneOk {
  static constexpr bool value = KindTraits<KIND>::is_int && (8 * NCH * VEC <= 128);
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

// LDS areas of the matrix-core walk (all 16-byte aligned)
struct MfmaLds {
  unsigned char* sel;  // roundup(R, 32) rows of MM_STRIDE bytes: vectors of the selected points,
                       // or null: rows are whole multiples of 32 bytes and the matrix operand is
                       // loaded straight from the vectors in device memory (more waves per CU)
  u32* selnorm;        // roundup(R, 32): their squared norms (shifted vectors)
  unsigned char* blk;  // 32 rows: the current block of candidates
  u32* cnorm;          // 32
  i32* cthr;           // 32: removal thresholds of the block's candidates
  u32* cid;            // 32
};
__host__ __device__ inline u32 mfma_rows(u32 R) { return (R + 31u) & ~31u; }
__host__ __device__ inline bool mfma_sel_in_lds(u32 row_bytes) { return (row_bytes % 32u) != 0u; }
__host__ __device__ inline u32 mfma_lds_bytes(u32 R, u32 row_bytes) {
  return (mfma_sel_in_lds(row_bytes) ? mfma_rows(R) * MM_STRIDE : 0u) + mfma_rows(R) * 4u + MM_BLOCK * MM_STRIDE +
         3u * MM_BLOCK * 4u;
}
__device__ __forceinline__ MfmaLds mfma_lds_carve(unsigned char* base, u32 R, u32 row_bytes) {
  MfmaLds M;
  const bool in_lds = mfma_sel_in_lds(row_bytes);
  M.sel = in_lds ? base : nullptr;
  M.blk = base + (in_lds ? mfma_rows(R) * MM_STRIDE : 0u);
  M.selnorm = reinterpret_cast<u32*>(M.blk + MM_BLOCK * MM_STRIDE);
  M.cnorm = M.selnorm + mfma_rows(R);
  M.cthr = reinterpret_cast<i32*>(M.cnorm + MM_BLOCK);
  M.cid = reinterpret_cast<u32*>(M.cthr + MM_BLOCK);
  return M;
}

template <int R_>
__device__ __forceinline__ void mm_block_rows(const v16i_t& acc, const uint4 (&n4)[4], i32 ncol, i32 tcol, u32& by) {
  // accumulator register R_ of lane l is entry (row 8*(R_/4) + 4*(l/32) + R_%4, column l%32)
  constexpr int mlo = 8 * (R_ / 4) + (R_ % 4);
  const u32 nrow = (R_ % 4) == 0 ? n4[R_ / 4].x : (R_ % 4) == 1 ? n4[R_ / 4].y : (R_ % 4) == 2 ? n4[R_ / 4].z : n4[R_ / 4].w;
  const i32 D = (i32)nrow + ncol - 2 * acc[R_];
  const u64 bm = ballot(D <= tcol);
  by = writelane_pair<mlo, mlo + 4>(by, bm);
}
template <int... Rs>
__device__ __forceinline__ void mm_block_rows_all(const v16i_t& acc, const uint4 (&n4)[4], i32 ncol, i32 tcol, u32& by,
                                                  std::integer_sequence<int, Rs...>) {
  (mm_block_rows<Rs>(acc, n4, ncol, tcol, by), ...);
}

template <int KIND, int VEC, int NCH>
__device__ __forceinline__ u32 prune_sorted_mfma(const VecTable& T, const MfmaLds& M, const u64* cand, u32 m, u32 R,
                                                 i64 a16, u32* out, int lane, u32& pair_evals) {
  const int sub = lane & (LPC - 1);
  const u32 grp = (u32)lane >> 3;
  const u32 half = (u32)lane >> 5;
  const u32 col = (u32)lane & 31u;
  const u32 flip = KIND == K_U8 ? 0x80808080u : 0u;
  const u32 ksteps = (T.row_bytes + 31u) / 32u;  // <= 4
  u32 nout = 0;
  if (m == 0) return 0;

  Piece<VEC> nx[4][NCH];  // the next block's vectors, 4 passes of 8 candidates
  auto issue = [&](u32 i0) {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const u32 c = i0 + 8u * p + grp;
      const bool ok = c < m;
      const u32 id = ok ? key_id(cand[c]) : 0u;
      const char* src = T.base + (u64)id * T.row_bytes;
#pragma unroll
      for (int u = 0; u < NCH; ++u) {
        const u32 pc = sub + LPC * u;
        nx[p][u] = (ok && pc < T.npieces) ? load_piece<VEC>(src + (u64)pc * VEC) : zero_piece<VEC>();
      }
    }
  };
  issue(0);

  for (u32 i0 = 0; i0 < m && nout < R; i0 += MM_BLOCK) {
    const u32 nb = m - i0 < MM_BLOCK ? m - i0 : MM_BLOCK;
    // park the block in LDS (as int8), take the norms
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const u32 c = 8u * p + grp;
      const bool ok = c < nb;
      i32 nn = 0;
#pragma unroll
      for (int u = 0; u < NCH; ++u) {
        const u32 pc = sub + LPC * u;
#pragma unroll
        for (int i = 0; i < VEC / 4; ++i) {
          const u32 wv = (ok && pc < T.npieces) ? (nx[p][u].w[i] ^ flip) : 0u;
          nn = __builtin_amdgcn_sdot4((i32)wv, (i32)wv, nn, false);
          *reinterpret_cast<u32*>(M.blk + c * MM_STRIDE + pc * VEC + 4 * i) = wv;
        }
      }
      nn = group_sum(nn);
      if (sub == 0) M.cnorm[c] = (u32)nn;
    }
    if (lane < (int)MM_BLOCK) {
      const bool ok = (u32)lane < nb;
      const u64 key = ok ? cand[i0 + lane] : KEY_INF;
      M.cthr[lane] = ok ? alpha_threshold(int_from_dkey(key_dkey(key)), a16) : -1;
      M.cid[lane] = key_id(key);
    }
    if (i0 + MM_BLOCK < m) issue(i0 + MM_BLOCK);  // travels while this block is settled
    __syncthreads();

    // column operand: candidate `col`, this lane's 16 bytes of every k-step
    v4i_t bv[4];
#pragma unroll
    for (u32 ks = 0; ks < 4; ++ks) {
      const v4i_t v =
          *reinterpret_cast<const v4i_t*>(M.blk + col * MM_STRIDE + 32u * (ks < ksteps ? ks : ksteps - 1u) + 16u * half);
      bv[ks] = ks < ksteps ? v : v4i_t{0, 0, 0, 0};
    }
    const i32 ncol = (i32)M.cnorm[col];
    const i32 tcol = M.cthr[col];

    // removed by a point selected before this block?  The row operand of each 32-point slice is
    // requested in one go, and the next slice's before this one's products are taken, so that a
    // block costs one trip to memory rather than one per instruction.
    bool rem = false;
    const u32 kclamp = ksteps - 1u;
    const u32 aflip = M.sel != nullptr ? 0u : flip;
    auto load_slice = [&](u32 s0, v4i_t (&av)[4]) {
      if (M.sel != nullptr) {
#pragma unroll
        for (u32 ks = 0; ks < 4; ++ks)
          av[ks] = *reinterpret_cast<const v4i_t*>(M.sel + (s0 + col) * MM_STRIDE + 32u * (ks < kclamp ? ks : kclamp) +
                                                   16u * half);
      } else {
        const u32 sid = s0 + col < nout ? out[s0 + col] : out[0];
        const char* src = T.base + (u64)sid * T.row_bytes + 16u * half;
#pragma unroll
        for (u32 ks = 0; ks < 4; ++ks) {
          av[ks] = *reinterpret_cast<const v4i_t*>(src + 32u * (ks < kclamp ? ks : kclamp));
        }
      }
    };
    v4i_t av[4];
    if (nout > 0) load_slice(0, av);
    for (u32 s0 = 0; s0 < nout; s0 += 32) {
      v4i_t cur[4];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
        cur[ks] = (u32)ks < ksteps ? (av[ks] ^ (int)aflip) : v4i_t{0, 0, 0, 0};  // device memory holds u8
      if (s0 + 32 < nout) load_slice(s0 + 32, av);
      v16i_t acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(cur[ks], bv[ks], acc, 0, 0, 0);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const u32 sb = s0 + 8u * q + 4u * half;
        const uint4 n4 = *reinterpret_cast<const uint4*>(M.selnorm + sb);
        rem = rem | (sb + 0 < nout && (i32)n4.x + ncol - 2 * acc[4 * q + 0] <= tcol);
        rem = rem | (sb + 1 < nout && (i32)n4.y + ncol - 2 * acc[4 * q + 1] <= tcol);
        rem = rem | (sb + 2 < nout && (i32)n4.z + ncol - 2 * acc[4 * q + 2] <= tcol);
        rem = rem | (sb + 3 < nout && (i32)n4.w + ncol - 2 * acc[4 * q + 3] <= tcol);
      }
    }
    const u64 rm = ballot(rem);
    const u32 removed_old = (u32)rm | (u32)(rm >> 32);

    // which candidate of the block would remove which: lane t ends up with the mask of row t
    u32 by = 0;
    {
      v16i_t acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(bv[ks], bv[ks], acc, 0, 0, 0);
      uint4 n4[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) n4[q] = *reinterpret_cast<const uint4*>(M.cnorm + 8u * q + 4u * half);
      mm_block_rows_all(acc, n4, ncol, tcol, by, std::make_integer_sequence<int, 16>{});
    }
    pair_evals += nb * nout + nb * (nb - 1) / 2;

    // settle the block in order
    u32 alive = (nb >= 32u ? ~0u : ((1u << nb) - 1u)) & ~removed_old;
    u32 selmask = 0, nsel = 0;
    while (alive != 0 && nout + nsel < R) {
      const int t = __builtin_ctz(alive);
      selmask |= 1u << t;
      ++nsel;
      alive &= ~readlane_u32(by, t);
      alive &= ~(1u << t);
    }
    // commit: ids, norms and vectors of the selected candidates, in order
    if (lane < (int)MM_BLOCK && ((selmask >> lane) & 1u)) {
      const u32 slot = nout + (u32)__builtin_popcount(selmask & ((1u << lane) - 1u));
      out[slot] = M.cid[lane];
      M.selnorm[slot] = M.cnorm[lane];
    }
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const u32 t = 8u * p + grp;
      if (M.sel != nullptr && ((selmask >> t) & 1u)) {
        const u32 slot = nout + (u32)__builtin_popcount(selmask & ((1u << t) - 1u));
        *reinterpret_cast<uint4*>(M.sel + slot * MM_STRIDE + 16u * sub) =
            *reinterpret_cast<const uint4*>(M.blk + t * MM_STRIDE + 16u * sub);
      }
    }
    nout += nsel;
    __syncthreads();
  }
  return nout;
}

// The same walk over an UNSORTED key array that may live in device memory (very long lists):
// the next candidate is found by a minimum search, and taken out by overwriting it.
template <int KIND, int VEC, int NCH>
__device__ __forceinline__ u32 prune_unsorted(const VecTable& T, const SelStage& st, u64* cand, u32 m, u32 R,
                                              const AlphaParam& al, u32* out, int lane, u32& pair_evals) {
  u32 nout = 0;
  for (u32 step = 0; step < m && nout < R; ++step) {
    u64 best = KEY_INF;
    u32 besti = 0;
    for (u32 i = lane; i < m; i += 64) {
      const u64 k = cand[i];
      if (k < best) {
        best = k;
        besti = i;
      }
    }
    const u64 key = wave_min_u64(best);
    if (key == KEY_INF) break;
    if (best == key) cand[besti] = KEY_INF;  // keys are distinct: exactly one lane
    const QueryRegs<KIND, VEC, NCH> cur =
        load_query<KIND, VEC, NCH>(T.base + (u64)key_id(key) * T.row_bytes, T.npieces, lane);
    if (!removed_by_selected<KIND, VEC, NCH>(T, st, cur, key_dkey(key), out, nout, al, lane, pair_evals)) {
      __syncthreads();
      if (lane == 0) out[nout] = key_id(key);
      stage_selected<KIND, VEC, NCH>(T, st, cur, nout, lane);
      ++nout;
    }
    __syncthreads();
  }
  return nout;
}

// LDS bytes of a stage for R selected rows, or 0 if they would not fit the budget
__host__ __device__ inline u32 stage_stride(u32 row_bytes) { return (row_bytes + 15u) & ~15u; }
__host__ inline u32 stage_bytes(u32 R, u32 row_bytes, u32 budget) {
  const u64 need = (u64)R * stage_stride(row_bytes);
  return need <= budget ? (u32)need : 0u;
}

}  // namespace annmi
