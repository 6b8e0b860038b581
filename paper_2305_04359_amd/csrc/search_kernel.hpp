// Batched greedy beam search, one wavefront per search (Alg. 1 of the paper).
//
// The beam (at most L candidates ordered by (distance, id), each with a "processed" flag) lives
// in registers, striped over the wave: entry i is held by lane i % 64 in slot i / 64.  LDS is the
// exchange medium when new candidates are merged in.  The visited filter of Sec. 4.5 (a lossy
// hash of vertex ids with one-sided error) is a per-wave LDS table of 16-byte buckets, newest
// entry first: a lost entry only causes a repeated distance evaluation, and the repeated
// candidate is then recognised as a duplicate of a beam entry or is worse than the beam's last
// entry, so results do not depend on the table.  A bucket holds four 32-bit ids, or, when the
// vertex count allows, eight 16-bit or six 21-bit tags: the id is passed through a bijection y
// of its B bits, bucket = floor(y * buckets / 2^B) (from the top 24 bits of y), tag = the low
// B - floor(log2 buckets) bits of y (at most 15, or 20).  Two ids of one bucket differ by less
// than 2^B / buckets in y, so equal tags mean equal ids: a tag match still identifies the vertex
// exactly while the table remembers up to twice as many vertices.  The bucket count need not be
// a power of two; it is chosen so that the wave's LDS lands on an occupancy step.
#pragma once
#include <cstddef>

#include "ann_device.hpp"
#include "ann_internal.hpp"

namespace annmi {

// a bijection of the low `bits` bits: multiplication by an odd constant modulo 2^bits (its top
// bits, which choose the bucket, depend on all bits of x); the 24-bit multiply serves ids of at
// most 24 bits
__device__ __forceinline__ u32 mix_id(u32 x, u32 mask, u32 bits) {
  return (bits <= 24u ? (u32)__umul24(x, 0x9E3779u) : x * 0x9E3779B1u) & mask;
}

// high 16 bits of the 48-bit product of two 24-bit numbers (both operands in vector registers:
// nothing here reads a scalar register that a vector instruction may just have written)
__device__ __forceinline__ u32 umulhi24(u32 a, u32 b) {
  u32 r;
  asm("v_mul_hi_u32_u24 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}

typedef unsigned short us2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32 pk_min_u16(u32 a, u32 b) {
  return __builtin_bit_cast(u32, __builtin_elementwise_min(__builtin_bit_cast(us2_t, a), __builtin_bit_cast(us2_t, b)));
}

// EPS: the (1 + eps) rule is compiled in.  TAG16: the filter holds 16-bit tags (graphs of up to
// a few million points); the other two layouts share the second variant, so that their code does
// not weigh on the registers of the first.
// OWN: every search has a start vertex of its own and reports the closest vertex it found (the
// layered index); compiled apart so that the flat graph's searches do not carry its arguments.
template <int KIND, int VEC, int NCH, int NSLOT, bool EPS, bool TAG16, bool OWN>
__global__ __launch_bounds__(64) void search_kernel(SearchArgs a, VecTable T) {
  extern __shared__ __align__(16) unsigned char smem[];
  u64* beam = reinterpret_cast<u64*>(smem);
  u64* skeys = beam + NSLOT * 64;  // survivors of one batch of candidates
  u32* cid = reinterpret_cast<u32*>(skeys);  // the batch's ids: dead once its keys are formed
  u32* hash = reinterpret_cast<u32*>(skeys + 64);  // 16-byte aligned

  const int lane = threadIdx.x;
  const u32 qi = blockIdx.x;
  const u32 nb = a.hash_buckets;
  const u32 hsize = 4u * nb;  // table size in 32-bit words
  uint4* bucket = reinterpret_cast<uint4*>(hash);
  constexpr bool compact = TAG16;                     // eight 16-bit tags per bucket
  const bool tags21 = !TAG16 && a.tag_width == 21u;  // six 21-bit tags per bucket
  const bool tagged = compact || tags21;
  const u32 idmask = tagged ? ((1u << a.id_bits) - 1u) : 0u;
  const u32 tagmask = tagged ? ((1u << (a.id_bits - (31u - (u32)__builtin_clz(nb)))) - 1u) : 0u;
  // bucket = floor(y' * nb / 2^24) with y' the top 24 bits of y (y shifted up if it has fewer),
  // as the high part of a 24 x 24-bit product: y' * (nb << 8) >> 32
  const u32 yshl = tagged && a.id_bits < 24u ? 24u - a.id_bits : 0u;
  const u32 yshr = tagged && a.id_bits > 24u ? a.id_bits - 24u : 0u;
  const u32 nb8 = nb << 8;
  auto bucket_of_y = [=](u32 y) { return umulhi24((y << yshl) >> yshr, nb8); };
  auto bucket_of_id = [=](u32 x) { return umulhi24((x * 0x9E3779B1u) >> 8, nb8); };
  const u32 L = a.L;

  const u32 qrow = a.qidx ? a.qidx[qi] : qi;
  const QueryRegs<KIND, VEC, NCH> Q =
      load_query<KIND, VEC, NCH>(a.queries + (u64)qrow * a.qrow_bytes, T.npieces, lane);

  for (u32 i = lane; i < hsize; i += 64) hash[i] = NONE_ID;
  if (a.batch_counters != nullptr && qi == 0 && lane == 0) {
    a.batch_counters[0] = 0;
    a.batch_counters[4] = 0;
    a.batch_counters[5] = 0;
    a.batch_counters[8] = 0;
    a.batch_counters[9] = 0;
    a.batch_counters[10] = 0;
    a.batch_counters[11] = 0;
  }

  u64 A[NSLOT];
#pragma unroll
  for (int s = 0; s < NSLOT; ++s) A[s] = KEY_INF;

  // beam <- {s}
  u32 st = a.start;
  if constexpr (OWN) {
    if (a.starts != nullptr) st = a.starts[a.slot != nullptr ? a.slot[qi] : qi];
  }
  {
    u32 dk = eval_up_to_64<KIND, VEC, NCH>(T, Q, [st](u32) { return st; }, 1u, lane);
    dk = readlane_u32(dk, 0);
    if (lane == 0) {
      A[0] = make_key(dk, st);
      beam[0] = A[0];  // the LDS copy of the beam is kept current (processed flags aside)
    }
  }
  __syncthreads();
  if (lane == 0) {
    if (compact) {
      const u32 y = mix_id(st, idmask, a.id_bits);
      hash[4u * bucket_of_y(y)] = 0xFFFF0000u | (y & tagmask);
    } else if (tags21) {
      const u32 y = mix_id(st, idmask, a.id_bits);
      hash[4u * bucket_of_y(y)] = 0xFFE00000u | (y & tagmask);
    } else {
      hash[4u * bucket_of_id(st)] = st;
    }
  }

  u32 size = 1, nv = 0, evals = 1;
  u32 n_pass = 0, n_surv = 0, n_ins = 0;  // statistics only
  // where the visited list goes: the search's own slot, later perhaps a spill chunk
  u64* vptr = a.vis != nullptr ? a.vis + (u64)qi * a.vis_cap : nullptr;
  u32 vcap = a.vis_cap;
  if (a.vis_where != nullptr && lane == 0) a.vis_where[qi] = ~0ull;

  for (;;) {
    // p* <- closest unprocessed member of the beam
    int pos = -1;
    u64 pk = 0;
#pragma unroll
    for (int s = 0; s < NSLOT; ++s) {
      if (pos < 0) {
        const u64 m = ballot(A[s] != KEY_INF && !(A[s] & 1ull));
        if (m) {
          const int l = __builtin_ctzll(m);
          pos = s * 64 + l;
          pk = readlane_u64(A[s], l);
          if (lane == l) A[s] |= 1ull;
        }
      }
    }
    if (pos < 0) break;
    // (1 + eps) rule of Sec. 4.5: p* is searched only while its distance is within the bound of
    // the beam's k-th entry; the beam is sorted and that entry never moves away, so the first
    // failure ends the search.  Integers: d * 2^16 > d_k * (2^16 + eps16), exact; floats:
    // d > d_k + eps * |d_k|, one fp32 product and one fp32 sum.
    if (EPS && size >= a.k) {  // compiled in only for searches that use the rule
      u64 kk = 0;
#pragma unroll
      for (int s = 0; s < NSLOT; ++s)
        if ((int)((a.k - 1u) >> 6) == s) kk = readlane_u64(A[s], (int)((a.k - 1u) & 63u));
      bool beyond;
      if constexpr (KindTraits<KIND>::is_int) {
        const long long d = int_from_dkey(key_dkey(pk)), dk = int_from_dkey(key_dkey(kk));
        beyond = d * 65536ll > dk * (65536ll + a.eps16);
      } else {
        const float d = float_from_dkey(key_dkey(pk)), dk = float_from_dkey(key_dkey(kk));
        beyond = d > __fadd_rn(dk, __fmul_rn(a.epsf, __builtin_fabsf(dk)));
      }
      if (beyond) break;  // (p* keeps its flag: nothing reads it once the search is over)
    }
    const u32 pstar = key_id(pk);
    // visited list: (vptr, vcap) are wave-uniform; vptr turns null when the list is lost (it fits
    // neither its slot nor a spill chunk: the prune kernel sees nv > room and reports it)
    if (vptr != nullptr) {
      if (nv == vcap) {  // the list is full
        u64* moved = nullptr;
        u32 newcap = 0;
        if (vcap == a.vis_cap && a.spill != nullptr) {  // still in its slot: move to a spill chunk
          const u64 need = (u64)vcap + a.spill_chunk;
          unsigned long long off = 0;
          if (lane == 0) off = atomicAdd(a.spill_top, (unsigned long long)need);
          off = readlane_u64(off, 0);
          if (off + need <= a.spill_cap) {
            __threadfence();
            u64* dst = a.spill + off;
            for (u32 i = lane; i < vcap; i += 64)
              dst[i] = __hip_atomic_load(vptr + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (lane == 0) a.vis_where[qi] = off;
            moved = dst;
            newcap = (u32)need;
          }
        }
        vptr = reinterpret_cast<u64*>(readlane_u64(reinterpret_cast<u64>(moved), 0));
        vcap = readlane_u32(newcap, 0);
      }
      if (vptr != nullptr && lane == 0) vptr[nv] = pk;
    }
    ++nv;

    // beam <- beam U N_out(p*), keep the L closest
    const u32* row = a.graph + (u64)pstar * a.R;
    for (u32 base = 0; base < a.R; base += 64) {
      const u32 j = base + lane;
      const u32 x = j < a.R ? row[j] : NONE_ID;
      bool fresh = x != NONE_ID;
      const u64 present = ballot(fresh);
      if (fresh) {
        if (compact) {
          const u32 y = mix_id(x, idmask, a.id_bits);
          const u32 h = bucket_of_y(y);
          const u32 tag = y & tagmask;
          const u32 tt = tag | (tag << 16);
          const uint4 e = bucket[h];
          // some 16-bit half equal to the tag?  (halves of e ^ tt that are zero)
          const u32 mz = pk_min_u16(pk_min_u16(e.x ^ tt, e.y ^ tt), pk_min_u16(e.z ^ tt, e.w ^ tt));
          if ((mz & 0xFFFFu) == 0u || (mz >> 16) == 0u)
            fresh = false;
          else  // shift the bucket by one tag, newest in front
            bucket[h] = make_uint4((e.x << 16) | tag, (e.y << 16) | (e.x >> 16), (e.z << 16) | (e.y >> 16),
                                   (e.w << 16) | (e.z >> 16));
        } else if (tags21) {
          // a bucket is two 64-bit words of three 21-bit tags each (an empty slot is all ones,
          // which no tag of at most 20 bits equals), newest in front
          constexpr u32 M21 = 0x1FFFFFu;
          const u32 y = mix_id(x, idmask, a.id_bits);
          const u32 h = bucket_of_y(y);
          const u32 tag = y & tagmask;
          const uint4 e = bucket[h];
          const u32 f0 = e.x & M21, f1 = __builtin_amdgcn_alignbit(e.y, e.x, 21) & M21, f2 = (e.y >> 10) & M21;
          const u32 f3 = e.z & M21, f4 = __builtin_amdgcn_alignbit(e.w, e.z, 21) & M21, f5 = (e.w >> 10) & M21;
          const u32 ma = (f0 ^ tag) < (f1 ^ tag) ? (f0 ^ tag) : (f1 ^ tag);
          const u32 mb = (f2 ^ tag) < (f3 ^ tag) ? (f2 ^ tag) : (f3 ^ tag);
          const u32 mc = (f4 ^ tag) < (f5 ^ tag) ? (f4 ^ tag) : (f5 ^ tag);
          const u32 mab = ma < mb ? ma : mb;
          if ((mab < mc ? mab : mc) == 0u)
            fresh = false;
          else
            bucket[h] = make_uint4((e.x << 21) | tag, __builtin_amdgcn_alignbit(e.y, e.x, 11), (e.z << 21) | f2,
                                   __builtin_amdgcn_alignbit(e.w, e.z, 11));
        } else {
          const u32 h = bucket_of_id(x);
          const uint4 e = bucket[h];
          const u32 m01 = (e.x ^ x) < (e.y ^ x) ? (e.x ^ x) : (e.y ^ x);
          const u32 m23 = (e.z ^ x) < (e.w ^ x) ? (e.z ^ x) : (e.w ^ x);
          if ((m01 < m23 ? m01 : m23) == 0u)
            fresh = false;
          else
            bucket[h] = make_uint4(x, e.x, e.y, e.z);
        }
      }
      const u64 fm = ballot(fresh);
      const u32 m = __builtin_popcountll(fm);
      if (m) {
        const u32 rank = __builtin_popcountll(fm & lanemask_lt(lane));
        if (fresh) cid[rank] = x;
        __syncthreads();
        // (the variants with start vertices of their own sit at the register count that eight
        // waves per SIMD allow: the second code path of the full-row passes would cost them a wave)
        u32 dk;
        if constexpr (OWN)
          dk = eval_up_to_64<KIND, VEC, NCH>(T, Q, [cid](u32 c) { return cid[c]; }, m, lane);
        else
          dk = eval_up_to_64_full_rows<KIND, VEC, NCH>(T, Q, [cid](u32 c) { return cid[c]; }, m, lane);
        const u32 c = cand_of_lane(lane);
        u64 mykey = c < m ? make_key(dk, cid[c]) : KEY_INF;
        __syncthreads();
        evals += m;
        n_pass += (m + 7u) >> 3;

        u64 worst = KEY_INF;
        if (size == L) {
#pragma unroll
          for (int s = 0; s < NSLOT; ++s)
            if ((int)((L - 1) >> 6) == s) worst = readlane_u64(A[s], (int)((L - 1) & 63)) | 1ull;
        }
        bool surv = mykey < worst;
        u64 sm = ballot(surv);
        if (sm) {
          u32 myrA = 0, myrB = 0, ns = 0;
          u32 shift[NSLOT];
#pragma unroll
          for (int s = 0; s < NSLOT; ++s) shift[s] = 0;
          if (__builtin_popcountll(sm) >= 4) {
            // many survivors: each finds its rank among the beam entries by bisection in the LDS
            // copy of the beam; a survivor that is already in the beam (the filter lost it) sits
            // exactly at its rank there and is dropped
            // the rank is at most 64 * NSLOT - 1 (a survivor lies below the last entry of a full
            // beam): one step per bit of it, each keeping the bit if that many entries lie below
            // the key; entries past `size` are never counted (the read stays inside the array)
            constexpr int BITS = (NSLOT == 1 ? 6 : NSLOT == 2 ? 7 : NSLOT == 4 ? 8 : NSLOT == 8 ? 9 : NSLOT == 16 ? 10 : 11);
            const u64 sk1 = mykey | 1ull;
            u32 lo = 0;
#pragma unroll
            for (int bit = BITS - 1; bit >= 0; --bit) {
              const u32 t = lo + (1u << bit);
              const u64 v = beam[t - 1u] | 1ull;
              lo = (t <= size && v < sk1) ? t : lo;
            }
            myrA = lo;
            if (surv && lo < size && (beam[lo] | 1ull) == sk1) surv = false;
            sm = ballot(surv);
            ns = (u32)__builtin_popcountll(sm);
            if (surv) skeys[__builtin_popcountll(sm & lanemask_lt(lane))] = mykey;
            __syncthreads();
            // ranks among the survivors, and how far each beam entry moves
            // (a lane without a survivor counts too: its sum is never read)
            for (u32 j = 0; j < ns; ++j) {
              const u64 sj = skeys[j];
              myrB += (sj < mykey) ? 1u : 0u;
#pragma unroll
              for (int s = 0; s < NSLOT; ++s) shift[s] += (sj < A[s]) ? 1u : 0u;
            }
            __syncthreads();
          } else {
            // few survivors: one at a time, ranks from wave-wide compares
            for (u64 it = sm; it; it &= it - 1) {
              const int l = __builtin_ctzll(it);
              const u64 sk = readlane_u64(mykey, l);
              u32 rA = 0;
#pragma unroll
              for (int s = 0; s < NSLOT; ++s) rA += __builtin_popcountll(ballot(A[s] < sk));
              u64 at = KEY_INF;
#pragma unroll
              for (int s = 0; s < NSLOT; ++s)
                if ((int)(rA >> 6) == s) at = readlane_u64(A[s], (int)(rA & 63));
              const bool dup = (at | 1ull) == (sk | 1ull);
              if (lane == l) {
                myrA = rA;
                if (dup) surv = false;
              }
            }
            sm = ballot(surv);
            for (u64 it = sm; it; it &= it - 1) {
              const int l = __builtin_ctzll(it);
              const u64 sk = readlane_u64(mykey, l);
              const u32 rB = __builtin_popcountll(ballot(surv && mykey < sk));
#pragma unroll
              for (int s = 0; s < NSLOT; ++s) shift[s] += (sk < A[s]) ? 1u : 0u;
              if (lane == l) myrB = rB;
              ++ns;
            }
          }
          if (sm) {
#pragma unroll
            for (int s = 0; s < NSLOT; ++s) {
              const u32 np = (u32)(s * 64 + lane) + shift[s];
              if (A[s] != KEY_INF && np < L) beam[np] = A[s];
            }
            if (surv) {
              const u32 np = myrA + myrB;
              if (np < L) beam[np] = mykey;
            }
            n_surv += ns;
            ++n_ins;
            size = size + ns < L ? size + ns : L;
            __syncthreads();
#pragma unroll
            for (int s = 0; s < NSLOT; ++s) {
              const u32 idx = (u32)(s * 64 + lane);
              A[s] = idx < size ? beam[idx] : KEY_INF;
            }
            __syncthreads();
          }
        }
      }
      if (present != ~0ull) break;  // rows are compact: the first gap ends the row
    }
  }

  if (a.nvis != nullptr && lane == 0) a.nvis[qi] = nv;
  if constexpr (OWN) {
    // The three pointers this needs are read from the kernel's argument block here, not through
    // `a`: arguments named in the code are all fetched into scalar registers at the kernel's
    // start and would occupy six of them for the whole search.
    if (lane == 0) {
      const char* kp = (const char*)__builtin_amdgcn_kernarg_segment_ptr();
      u32* next = *reinterpret_cast<u32* const volatile*>(kp + offsetof(SearchArgs, next_start));
      if (next != nullptr) {
        const u32* slot = *reinterpret_cast<const u32* const volatile*>(kp + offsetof(SearchArgs, slot));
        const u32* down = *reinterpret_cast<const u32* const volatile*>(kp + offsetof(SearchArgs, down));
        // the beam's first entry is the closest vertex the search visited (it always holds one)
        const u32 best = key_id(A[0]);
        next[slot != nullptr ? slot[qi] : qi] = down != nullptr ? down[best] : best;
      }
    }
  }
  if (a.out_ids != nullptr) {
#pragma unroll
    for (int s = 0; s < NSLOT; ++s) {
      const u32 idx = (u32)(s * 64 + lane);
      if (idx < a.k) {
        const bool ok = A[s] != KEY_INF;
        const u64 o = (u64)qi * a.k + idx;
        a.out_ids[o] = ok ? key_id(A[s]) : NONE_ID;
        if (a.out_dists != nullptr) {
          if constexpr (KindTraits<KIND>::is_int)
            reinterpret_cast<i32*>(a.out_dists)[o] = ok ? int_from_dkey(key_dkey(A[s])) : 0x7FFFFFFF;
          else
            reinterpret_cast<float*>(a.out_dists)[o] = ok ? float_from_dkey(key_dkey(A[s])) : __builtin_inff();
        }
      }
    }
  }
  if (a.counters != nullptr && lane == 0) {
    atomicAdd(&block_counters(a.counters)->searches, 1ull);
    atomicAdd(&block_counters(a.counters)->hops, (unsigned long long)nv);
    atomicAdd(&block_counters(a.counters)->evals, (unsigned long long)evals);
    atomicAdd(&block_counters(a.counters)->passes, (unsigned long long)n_pass);
    atomicAdd(&block_counters(a.counters)->survivors, (unsigned long long)n_surv);
    atomicAdd(&block_counters(a.counters)->insert_hops, (unsigned long long)n_ins);
  }
}


// launches of the variants that other translation units compile: with the (1 + eps) rule
// (search_eps.hip), with start vertices of their own (search_own.hip), with both (search_own_eps.hip)
hipError_t launch_search_eps(const DistCfg& cfg, const SearchArgs& a, const VecTable& T, hipStream_t s);
hipError_t launch_search_own(const DistCfg& cfg, const SearchArgs& a, const VecTable& T, hipStream_t s);
hipError_t launch_search_own_eps(const DistCfg& cfg, const SearchArgs& a, const VecTable& T, hipStream_t s);

// beam slots per lane: the smallest power of two that holds L entries (beams of up to 2,048)
inline u32 search_nslot_for(u32 L) {
  u32 ns = 1;
  while (ns * 64u < L && ns < 32u) ns *= 2u;
  return ns;
}

// One launch for a fixed choice of EPS and OWN; the beam slots and the filter layout are picked here.
template <int KIND, int VEC, int NCH, bool EPS, bool OWN>
inline hipError_t launch_search_variant(const SearchArgs& a, const VecTable& T, hipStream_t s) {
  const u32 lds = search_lds_bytes(a.L, a.hash_buckets);
  const dim3 grid(a.nq), block(64);
  const bool t16 = a.tag_width == 16u;
#define ANN_LAUNCH_SEARCH(NS)                                                                            \
  if (t16)                                                                                               \
    hipLaunchKernelGGL((search_kernel<KIND, VEC, NCH, NS, EPS, true, OWN>), grid, block, lds, s, a, T);  \
  else                                                                                                   \
    hipLaunchKernelGGL((search_kernel<KIND, VEC, NCH, NS, EPS, false, OWN>), grid, block, lds, s, a, T)
  switch (search_nslot_for(a.L)) {
    case 1: ANN_LAUNCH_SEARCH(1); break;
    case 2: ANN_LAUNCH_SEARCH(2); break;
    case 4: ANN_LAUNCH_SEARCH(4); break;
    case 8: ANN_LAUNCH_SEARCH(8); break;
    case 16: ANN_LAUNCH_SEARCH(16); break;
    default: ANN_LAUNCH_SEARCH(32); break;
  }
#undef ANN_LAUNCH_SEARCH
  return hipGetLastError();
}

}  // namespace annmi
