// Device-side building blocks shared by the search, prune and merge kernels (gfx950, wave64).
//
// Work decomposition used everywhere: one wavefront owns one search / one prune.  Distances from
// one "query" vector to a set of graph vertices are taken eight vertices at a time: the 64 lanes
// split into 8 groups of 8 lanes, group g handles one vertex, and lane `sub` of the group loads
// the 16-byte (or 4-byte) pieces sub, sub+8, sub+16, ... of that vertex' row, so one wave-wide
// load instruction reads whole, contiguous rows.  Partial sums are combined inside each group
// with three DPP steps.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace annmi {

using u32 = uint32_t;
using u64 = uint64_t;
using i32 = int32_t;
using i64 = int64_t;

constexpr u32 NONE_ID = 0xFFFFFFFFu;
constexpr u64 KEY_INF = ~0ull;
constexpr int WAVE = 64;
constexpr int LPC = 8;  // lanes per candidate

// element kind + metric
enum Kind : int { K_U8 = 0, K_I8 = 1, K_F32_L2 = 2, K_F32_IP = 3 };

template <int KIND>
struct KindTraits {
  static constexpr bool is_int = (KIND == K_U8 || KIND == K_I8);
};

// ---------------------------------------------------------------------------------------------
// keys: (order-preserving 32-bit distance) << 32 | id << 1 | flag.  Comparing keys as u64
// compares (distance, id).  The flag marks "processed" in the beam and is 0 elsewhere.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ u32 dkey_from_int(i32 d) { return (u32)d ^ 0x80000000u; }
__device__ __forceinline__ i32 int_from_dkey(u32 k) { return (i32)(k ^ 0x80000000u); }
__device__ __forceinline__ u32 dkey_from_float(float f) {
  u32 u = __float_as_uint(f + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float float_from_dkey(u32 k) {
  u32 u = (k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k;
  return __uint_as_float(u);
}
__device__ __forceinline__ u64 make_key(u32 dkey, u32 id) { return ((u64)dkey << 32) | ((u64)id << 1); }
__device__ __forceinline__ u32 key_id(u64 k) { return (u32)(k & 0xFFFFFFFFull) >> 1; }
__device__ __forceinline__ u32 key_dkey(u64 k) { return (u32)(k >> 32); }

// ---------------------------------------------------------------------------------------------
// wave helpers
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ u64 ballot(bool p) { return __builtin_amdgcn_ballot_w64(p); }
__device__ __forceinline__ u64 lanemask_lt(int lane) { return (1ull << lane) - 1ull; }

__device__ __forceinline__ u32 readlane_u32(u32 v, int lane) {
  return (u32)__builtin_amdgcn_readlane((int)v, lane);
}
__device__ __forceinline__ u64 readlane_u64(u64 v, int lane) {
  u32 lo = readlane_u32((u32)v, lane);
  u32 hi = readlane_u32((u32)(v >> 32), lane);
  return ((u64)hi << 32) | lo;
}

// `old` with lanes LO and HI replaced by the low and high half of the wave-uniform mask `m`.
// The scalar operands usually come straight from a vector compare, and a scalar register written
// by a vector instruction must not be read by a vector instruction in the next few issue slots.
// The compiler pads its own instructions for that, but not the text of an asm statement (with
// the write directly behind the compare the lanes were seen to keep their old value), so the
// wait states are part of the statement: four, what the instruction-set manual asks between a
// vector instruction that writes a scalar register and a lane instruction that reads it.  (This
// compiler offers no writelane builtin, which would leave the counting to it.)
template <int LO, int HI>
__device__ __forceinline__ u32 writelane_pair(u32 old, u64 m) {
  const u32 lo = (u32)m, hi = (u32)(m >> 32);
  asm("s_nop 3\n\tv_writelane_b32 %0, %1, %3\n\tv_writelane_b32 %0, %2, %4"
      : "+v"(old)
      : "s"(lo), "s"(hi), "n"(LO), "n"(HI));
  return old;
}

__device__ __forceinline__ u64 wave_min_u64(u64 v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    u32 lo = (u32)__shfl_xor((int)(u32)v, off, WAVE);
    u32 hi = (u32)__shfl_xor((int)(u32)(v >> 32), off, WAVE);
    u64 o = ((u64)hi << 32) | lo;
    v = o < v ? o : v;
  }
  return v;
}

// Sum over the 8 lanes of a group; every lane of the group receives the same total.
// quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror.
__device__ __forceinline__ i32 group_sum(i32 v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, true);
  v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, true);
  return v;
}
__device__ __forceinline__ float group_sum(float v) {
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true));
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true));
  return v;
}

// ---------------------------------------------------------------------------------------------
// row pieces
// ---------------------------------------------------------------------------------------------
template <int VEC>
struct Piece;
template <>
struct Piece<16> {
  u32 w[4];
};
template <>
struct Piece<4> {
  u32 w[1];
};

template <int VEC>
__device__ __forceinline__ Piece<VEC> load_piece(const char* p) {
  Piece<VEC> r;
  if constexpr (VEC == 16) {
    uint4 t = *reinterpret_cast<const uint4*>(p);
    r.w[0] = t.x;
    r.w[1] = t.y;
    r.w[2] = t.z;
    r.w[3] = t.w;
  } else {
    r.w[0] = *reinterpret_cast<const u32*>(p);
  }
  return r;
}
template <int VEC>
__device__ __forceinline__ Piece<VEC> zero_piece() {
  Piece<VEC> r;
#pragma unroll
  for (int i = 0; i < VEC / 4; ++i) r.w[i] = 0;
  return r;
}

// Where the vectors live.
struct VecTable {
  const char* base;
  u32 row_bytes;
  u32 npieces;  // pieces of VEC bytes per row
};

// The vector every distance is measured from, spread over the 8 lanes of each group (all 8
// groups hold the same copy).
template <int KIND, int VEC, int NCH>
struct QueryRegs {
  Piece<VEC> q[NCH];
  i32 qq;  // <q,q> for the integer kinds
};

// The pieces only (no arithmetic on them, so the loads can stay in flight) ...
template <int KIND, int VEC, int NCH>
__device__ __forceinline__ QueryRegs<KIND, VEC, NCH> load_query_raw(const char* row, u32 npieces, int lane) {
  QueryRegs<KIND, VEC, NCH> Q;
  const int sub = lane & (LPC - 1);
#pragma unroll
  for (int u = 0; u < NCH; ++u) {
    u32 pc = sub + LPC * u;
    Q.q[u] = pc < npieces ? load_piece<VEC>(row + (u64)pc * VEC) : zero_piece<VEC>();
  }
  Q.qq = 0;
  return Q;
}
// ... and <q,q>, needed before the first distance is taken
template <int KIND, int VEC, int NCH>
__device__ __forceinline__ void query_finish(QueryRegs<KIND, VEC, NCH>& Q) {
  i32 acc = 0;
#pragma unroll
  for (int u = 0; u < NCH; ++u) {
    if constexpr (KIND == K_U8) {
#pragma unroll
      for (int i = 0; i < VEC / 4; ++i) acc = (i32)__builtin_amdgcn_udot4(Q.q[u].w[i], Q.q[u].w[i], (u32)acc, false);
    } else if constexpr (KIND == K_I8) {
#pragma unroll
      for (int i = 0; i < VEC / 4; ++i) acc = __builtin_amdgcn_sdot4((i32)Q.q[u].w[i], (i32)Q.q[u].w[i], acc, false);
    }
  }
  Q.qq = KindTraits<KIND>::is_int ? group_sum(acc) : 0;
}

template <int KIND, int VEC, int NCH>
__device__ __forceinline__ QueryRegs<KIND, VEC, NCH> load_query(const char* row, u32 npieces, int lane) {
  QueryRegs<KIND, VEC, NCH> Q = load_query_raw<KIND, VEC, NCH>(row, npieces, lane);
  query_finish<KIND, VEC, NCH>(Q);
  return Q;
}

// Distance key from the lane-local pieces of one row; all 8 lanes of the group get the result.
template <int KIND, int VEC, int NCH>
__device__ __forceinline__ u32 distance_key(const QueryRegs<KIND, VEC, NCH>& Q, const Piece<VEC> (&x)[NCH]) {
  if constexpr (KIND == K_U8) {
    u32 xx = 0, qx = 0;
#pragma unroll
    for (int u = 0; u < NCH; ++u)
#pragma unroll
      for (int i = 0; i < VEC / 4; ++i) {
        xx = __builtin_amdgcn_udot4(x[u].w[i], x[u].w[i], xx, false);
        qx = __builtin_amdgcn_udot4(Q.q[u].w[i], x[u].w[i], qx, false);
      }
    i32 part = (i32)xx - 2 * (i32)qx;
    return dkey_from_int(group_sum(part) + Q.qq);
  } else if constexpr (KIND == K_I8) {
    i32 xx = 0, qx = 0;
#pragma unroll
    for (int u = 0; u < NCH; ++u)
#pragma unroll
      for (int i = 0; i < VEC / 4; ++i) {
        xx = __builtin_amdgcn_sdot4((i32)x[u].w[i], (i32)x[u].w[i], xx, false);
        qx = __builtin_amdgcn_sdot4((i32)Q.q[u].w[i], (i32)x[u].w[i], qx, false);
      }
    return dkey_from_int(group_sum(xx - 2 * qx) + Q.qq);
  } else {
    float acc = 0.0f;
#pragma unroll
    for (int u = 0; u < NCH; ++u)
#pragma unroll
      for (int i = 0; i < VEC / 4; ++i) {
        float a = __uint_as_float(Q.q[u].w[i]);
        float b = __uint_as_float(x[u].w[i]);
        if constexpr (KIND == K_F32_L2) {
          float t = a - b;
          acc = __builtin_fmaf(t, t, acc);
        } else {
          acc = __builtin_fmaf(a, b, acc);
        }
      }
    acc = group_sum(acc);
    return dkey_from_float(KIND == K_F32_IP ? -acc : acc);
  }
}

// How many groups-of-8 candidates are loaded before any arithmetic starts (memory-level
// parallelism against registers).
template <int VEC, int NCH>
struct PassBatch {
  static constexpr int budget = (VEC == 16) ? 8 : 16;
  static constexpr int value = (budget / NCH) < 1 ? 1 : ((budget / NCH) > 8 ? 8 : (budget / NCH));
};

// Distances from Q to the candidates id_at(0..cnt), cnt <= 64.  Lane l ends up with the key of
// candidate cand_of_lane(l) = 8*(l&7) + (l>>3) when that index is < cnt.
__device__ __forceinline__ u32 cand_of_lane(int lane) { return (u32)(8 * (lane & 7) + (lane >> 3)); }

// passes t0 .. t0+PBX-1 (a pass = 8 candidates): all loads first, then the arithmetic.
// FULL: every lane's pieces exist (rows of exactly 8 * NCH pieces), and a group without a
// candidate reads candidate 0's row again (a line the pass fetches anyway) instead of being
// masked off and handed zeros: no compare, branch or register clearing per pass; its result is
// never looked at.
template <int KIND, int VEC, int NCH, int PBX, bool FULL, class IdAt>
__device__ __forceinline__ void eval_passes(const VecTable& T, const QueryRegs<KIND, VEC, NCH>& Q, IdAt id_at,
                                            u32 cnt, u32 t0, int sub, u32 grp, u32& result) {
  Piece<VEC> x[PBX][NCH];
#pragma unroll
  for (int tt = 0; tt < PBX; ++tt) {
    const u32 c = 8u * (t0 + tt) + grp;
    const bool ok = c < cnt;
    if constexpr (FULL) {
      const u32 id = id_at(ok ? c : 0u);
      const char* row = T.base + (u64)id * T.row_bytes;
#pragma unroll
      for (int u = 0; u < NCH; ++u) x[tt][u] = load_piece<VEC>(row + (u64)(sub + LPC * u) * VEC);
    } else {
      const u32 id = ok ? id_at(c) : 0u;
      const char* row = T.base + (u64)id * T.row_bytes;
#pragma unroll
      for (int u = 0; u < NCH; ++u) {
        const u32 pc = sub + LPC * u;
        x[tt][u] = (ok && pc < T.npieces) ? load_piece<VEC>(row + (u64)pc * VEC) : zero_piece<VEC>();
      }
    }
  }
#pragma unroll
  for (int tt = 0; tt < PBX; ++tt) {
    const u32 dk = distance_key<KIND, VEC, NCH>(Q, x[tt]);
    if ((u32)sub == t0 + tt) result = dk;
  }
}

template <int KIND, int VEC, int NCH, bool FULL, class IdAt>
__device__ __forceinline__ u32 eval_up_to_64_impl(const VecTable& T, const QueryRegs<KIND, VEC, NCH>& Q,
                                                  IdAt id_at, u32 cnt, int lane) {
  constexpr int PB = PassBatch<VEC, NCH>::value;
  const int sub = lane & (LPC - 1);
  const u32 grp = (u32)lane >> 3;
  const u32 npass = (cnt + 7u) >> 3;
  u32 result = 0;
  u32 t0 = 0;
  // whole batches, then the remainder with the smallest batch that covers it, so that a short
  // candidate list does not pay for eight passes of arithmetic
  while (npass - t0 >= (u32)PB) {
    eval_passes<KIND, VEC, NCH, PB, FULL>(T, Q, id_at, cnt, t0, sub, grp, result);
    t0 += PB;
  }
  const u32 rem = npass - t0;
  if (rem == 0) return result;
  if constexpr (PB >= 8) {
    if (rem > 4) {
      eval_passes<KIND, VEC, NCH, 8, FULL>(T, Q, id_at, cnt, t0, sub, grp, result);
      return result;
    }
  }
  if constexpr (PB >= 4) {
    if (rem > 2) {
      eval_passes<KIND, VEC, NCH, 4, FULL>(T, Q, id_at, cnt, t0, sub, grp, result);
      return result;
    }
  }
  if constexpr (PB >= 2) {
    if (rem > 1) {
      eval_passes<KIND, VEC, NCH, 2, FULL>(T, Q, id_at, cnt, t0, sub, grp, result);
      return result;
    }
  }
  eval_passes<KIND, VEC, NCH, 1, FULL>(T, Q, id_at, cnt, t0, sub, grp, result);
  return result;
}

template <int KIND, int VEC, int NCH, class IdAt>
__device__ __forceinline__ u32 eval_up_to_64(const VecTable& T, const QueryRegs<KIND, VEC, NCH>& Q,
                                             IdAt id_at, u32 cnt, int lane) {
  return eval_up_to_64_impl<KIND, VEC, NCH, false>(T, Q, id_at, cnt, lane);
}

// The same for callers that pass cnt >= 1 and whose id_at(0) is a vertex: rows that fill every
// lane's pieces take the unmasked passes.
template <int KIND, int VEC, int NCH, class IdAt>
__device__ __forceinline__ u32 eval_up_to_64_full_rows(const VecTable& T, const QueryRegs<KIND, VEC, NCH>& Q,
                                                       IdAt id_at, u32 cnt, int lane) {
  if (T.npieces == (u32)(LPC * NCH)) return eval_up_to_64_impl<KIND, VEC, NCH, true>(T, Q, id_at, cnt, lane);
  return eval_up_to_64_impl<KIND, VEC, NCH, false>(T, Q, id_at, cnt, lane);
}

// alpha * d(p*,p') <= d(p,p')  (Sec. 4.1).  Integer kinds: alpha is held as a16 = round(alpha*2^16)
// and the test is exact in 64-bit integers; float kinds: one fp32 product.
struct AlphaParam {
  i64 a16;
  float af;
};
template <int KIND>
__device__ __forceinline__ bool alpha_dominates(const AlphaParam& A, u32 dkey_star_cand, u32 dkey_p_cand) {
  if constexpr (KindTraits<KIND>::is_int) {
    i64 lhs = A.a16 * (i64)int_from_dkey(dkey_star_cand);
    i64 rhs = (i64)int_from_dkey(dkey_p_cand) * 65536;
    return lhs <= rhs;
  } else {
    float prod = A.af * float_from_dkey(dkey_star_cand);
    return prod <= float_from_dkey(dkey_p_cand);
  }
}

}  // namespace annmi
