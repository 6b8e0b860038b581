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

#include "ann_device.hpp"

namespace annmi {

// In-place ascending bitonic sort of n2 keys (a power of two >= 2) by one wave.
__device__ __forceinline__ void bitonic_sort_keys(u64* a, u32 n2, int lane) {
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
