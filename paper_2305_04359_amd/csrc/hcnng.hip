// The clustering-based builder of Sec. 4.3 (ParlayHCNNG) with the cluster trees of Sec. 3.2.
//
// Per group of trees: the points are split level by level (all splitting nodes of a level in one
// pass: every point takes the side of the nearer of its node's two pivots; a stable two-way split
// from running counts of left points puts the children in place, finished children straight into
// the final order); the leaves' vectors are gathered as int8 into tiles of 32 rows laid out as
// the matrix cores read them; one wavefront per 32 points of a leaf finds their l nearest
// neighbours inside the leaf on the matrix cores (32 x 32 inner products per instruction group,
// every lane keeping the best of the candidates it sees for its own point); one workgroup per
// leaf sorts the leaf's candidate pairs in LDS, and one wavefront per leaf runs Kruskal's scan
// with the degree bound, 64 pairs at a time (a pair that fails once fails for good, so the wave
// tests 64 in parallel and only the survivors are taken in order; the scan is a chain of
// dependent LDS reads, so thousands of leaves are scanned side by side).
// At the end the arcs of all trees are sorted by (point, neighbour), repeated ones dropped, and
// every point's neighbours pruned with the alpha rule of Sec. 4.1 by the re-prune kernel of the
// flat graph's BatchInsert.
#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <type_traits>

#include "ann_device.hpp"
#include "driver_internal.hpp"

using namespace annmi;

namespace annmi {
namespace hcnng {

constexpr u32 HC_MAX_LS = 1024;       // points per leaf
constexpr u32 HC_MAX_L = 16;          // nearest neighbours per point that restrict the tree
constexpr u32 HC_MAX_PAIRS = 16384;   // candidate pairs per leaf (sorted in LDS)
constexpr u32 HC_MAX_DEPTH = 39;      // below this depth a node is cut in the middle of its order
constexpr u32 HC_NONE = 0xFFFFFFFFu;

typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef int v16i_t __attribute__((ext_vector_type(16)));

u64 stream_output(u64 seed, u64 k) {  // the (k+1)-th output of SplitMix64(seed)
  u64 z = seed + (k + 1) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
u64 mulhi64(u64 a, u64 b) { return (u64)(((unsigned __int128)a * (unsigned __int128)b) >> 64); }

u32 bits_to_hold(u64 count) {  // smallest b with 2^b - 1 >= count: indices below count never have all b bits set
  u32 b = 1;
  while (((1ull << b) - 1ull) < count) ++b;
  return b;
}

// A wavefront of the side kernels takes SIDE_PER_WAVE consecutive positions, eight at a time
// (eight lanes per point).  The node of its first position is found once, by a uniform search
// that the scalar unit runs; the later positions step forward from there.
constexpr u32 SIDE_PER_WAVE = 32;
__device__ inline u32 side_first_node(const u32* off, u32 nseg, u64 w0) {
  u32 lo = 0, hi = nseg;
  while (hi - lo > 1) {
    const u32 mid = (lo + hi) >> 1;
    if ((u64)off[mid] <= w0)
      lo = mid;
    else
      hi = mid;
  }
  return lo;
}

// One level of one tree.  keys_in[i] = (anything << 32) | id of the point at position i; the
// nodes of the level are the position ranges off[s]..off[s+1].  A node that splits names the
// positions of its two pivots; its points get child index base[s] (left: at most as far from the
// first pivot as from the second) or base[s] + 1.  Other nodes keep their points under base[s].
// Eight lanes per point.
template <bool SIGNED>
__global__ __launch_bounds__(256) void hc_side_kernel(const unsigned char* pts, u32 row_bytes, const u64* keys_in, u64 n,
                                                      const u32* off, u32 nseg, const u32* pos1, const u32* pos2,
                                                      const u32* base, u64* keys_out) {
  const u32 sub = threadIdx.x & 7u, grp = (threadIdx.x >> 3) & 7u;
  const u64 w0 = ((u64)blockIdx.x * 4u + (u32)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6))) * SIDE_PER_WAVE;
  if (w0 >= n) return;
  u32 seg = side_first_node(off, nseg, w0);
  const bool has_piece = sub < row_bytes / 16;  // a row is at most 128 bytes: one 16-byte piece per lane
  // Four positions of a group at a time, every load of one kind requested for all four before the
  // first answer is used: the kernel waits for memory, and this way four waits overlap.
  constexpr u32 NB = 4;
  for (u32 it0 = 0; it0 < SIDE_PER_WAVE / 8u; it0 += NB) {
    u64 pos[NB];
    bool live[NB];
    u32 id[NB];
#pragma unroll
    for (u32 q = 0; q < NB; ++q) {
      pos[q] = w0 + 8u * (it0 + q) + grp;
      live[q] = pos[q] < n;
      id[q] = live[q] ? (u32)keys_in[pos[q]] : 0u;
    }
    u32 idx[NB], p1[NB], p2[NB];
#pragma unroll
    for (u32 q = 0; q < NB; ++q) {
      if (live[q])
        while ((u64)off[seg + 1] <= pos[q]) ++seg;
      idx[q] = base[seg];
      p1[q] = live[q] ? pos1[seg] : HC_NONE;
      p2[q] = pos2[seg];
    }
    u32 ida[NB], idb[NB];
#pragma unroll
    for (u32 q = 0; q < NB; ++q) {
      const bool split = p1[q] != HC_NONE;
      ida[q] = split ? (u32)keys_in[p1[q]] : 0u;
      idb[q] = split ? (u32)keys_in[p2[q]] : 0u;
    }
    uint4 vx[NB], va[NB], vb[NB];
#pragma unroll
    for (u32 q = 0; q < NB; ++q) {
      vx[q] = va[q] = vb[q] = make_uint4(0, 0, 0, 0);
      if (p1[q] != HC_NONE && has_piece) {
        vx[q] = reinterpret_cast<const uint4*>(pts + (u64)id[q] * row_bytes)[sub];
        va[q] = reinterpret_cast<const uint4*>(pts + (u64)ida[q] * row_bytes)[sub];
        vb[q] = reinterpret_cast<const uint4*>(pts + (u64)idb[q] * row_bytes)[sub];
      }
    }
#pragma unroll
    for (u32 q = 0; q < NB; ++q) {
      const u32 wx[4] = {vx[q].x, vx[q].y, vx[q].z, vx[q].w}, wa[4] = {va[q].x, va[q].y, va[q].z, va[q].w},
                wb[4] = {vb[q].x, vb[q].y, vb[q].z, vb[q].w};
      i32 xa = 0, xb = 0, aa = 0, bb = 0;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if constexpr (SIGNED) {
          xa = __builtin_amdgcn_sdot4((i32)wx[k], (i32)wa[k], xa, false);
          xb = __builtin_amdgcn_sdot4((i32)wx[k], (i32)wb[k], xb, false);
          aa = __builtin_amdgcn_sdot4((i32)wa[k], (i32)wa[k], aa, false);
          bb = __builtin_amdgcn_sdot4((i32)wb[k], (i32)wb[k], bb, false);
        } else {
          xa = (i32)__builtin_amdgcn_udot4(wx[k], wa[k], (u32)xa, false);
          xb = (i32)__builtin_amdgcn_udot4(wx[k], wb[k], (u32)xb, false);
          aa = (i32)__builtin_amdgcn_udot4(wa[k], wa[k], (u32)aa, false);
          bb = (i32)__builtin_amdgcn_udot4(wb[k], wb[k], (u32)bb, false);
        }
      }
      // |x-a|^2 <= |x-b|^2  <=>  |a|^2 - 2<x,a> <= |b|^2 - 2<x,b>  (a node that does not split: 0 <= 0)
      const i32 lhs = group_sum(aa - 2 * xa), rhs = group_sum(bb - 2 * xb);
      if (lhs > rhs) idx[q] += 1;
      if (live[q] && sub == 0) keys_out[pos[q]] = ((u64)idx[q] << 32) | id[q];
    }
  }
}

// Leaf vectors are kept in tiles of 32 consecutive points of ONE leaf (a leaf's tiles follow one
// another from tile_of_leaf[leaf]; the unused rows of its last tile are zero, and nothing that is
// kept is computed from them): inside a tile the 16-byte
// piece c of row r lies at (c * 32 + r) * 16, so that the matrix-core operand of the
// nearest-neighbour kernels -- lane (row, half) takes piece 2 ks + half of its row -- is 1 KB of
// consecutive bytes per load instead of 32 bytes out of each of 32 rows.
__device__ inline u32 leaf_of_tile(const u32* tile_of_leaf, u32 nleaves, u32 tile) {
  u32 lo = 0, hi = nleaves;  // uniform: the scalar unit runs this
  while (hi - lo > 1) {
    const u32 mid = (lo + hi) >> 1;
    if (tile_of_leaf[mid] <= tile)
      lo = mid;
    else
      hi = mid;
  }
  return lo;
}

// The vectors in that layout, as int8 (uint8 data moved down by 128: distances do not change),
// rows of lv_stride bytes (a multiple of 32, zero tail), and their squared norms (times 512) by
// position.  One workgroup per tile, eight lanes per point.
template <bool SIGNED>
__global__ __launch_bounds__(256) void hc_gather_kernel(const unsigned char* pts, u32 row_bytes, const u64* keys,
                                                        const u32* leaf_off, const u32* tile_of_leaf, u32 nleaves,
                                                        u32 lv_stride, unsigned char* leafvec, i32* leafnorm) {
  const u32 tile = blockIdx.x;
  const u32 leaf = leaf_of_tile(tile_of_leaf, nleaves, tile);
  const u32 r = threadIdx.x >> 3, sub = threadIdx.x & 7u;
  const u32 in_leaf = 32u * (tile - tile_of_leaf[leaf]) + r;
  unsigned char* y = leafvec + (u64)tile * 32u * lv_stride;
  if (in_leaf >= leaf_off[leaf + 1] - leaf_off[leaf]) {  // an unused row of the leaf's last tile: zeros
    for (u32 pc = sub; pc < lv_stride / 16; pc += 8)
      *reinterpret_cast<uint4*>(y + ((u64)pc * 32u + r) * 16u) = make_uint4(0, 0, 0, 0);
    return;
  }
  const u64 i = (u64)leaf_off[leaf] + in_leaf;
  const u32 id = (u32)keys[i];
  const uint4* x = reinterpret_cast<const uint4*>(pts + (u64)id * row_bytes);
  i32 nn = 0;
  for (u32 pc = sub; pc < lv_stride / 16; pc += 8) {
    uint4 v = make_uint4(0, 0, 0, 0);
    if (pc < row_bytes / 16) {
      v = x[pc];
      if constexpr (!SIGNED) {
        v.x ^= 0x80808080u;
        v.y ^= 0x80808080u;
        v.z ^= 0x80808080u;
        v.w ^= 0x80808080u;
      }
    }
    *reinterpret_cast<uint4*>(y + ((u64)pc * 32u + r) * 16u) = v;
    nn = __builtin_amdgcn_sdot4((i32)v.x, (i32)v.x, nn, false);
    nn = __builtin_amdgcn_sdot4((i32)v.y, (i32)v.y, nn, false);
    nn = __builtin_amdgcn_sdot4((i32)v.z, (i32)v.z, nn, false);
    nn = __builtin_amdgcn_sdot4((i32)v.w, (i32)v.w, nn, false);
  }
  nn = group_sum(nn);
  if (sub == 0) leafnorm[i] = nn << 9;  // where the nearest-neighbour kernel's keys hold the distance
}

// Which leaf and which 32 queries of it a block of the nearest-neighbour kernels takes.  A leaf's
// blocks all read the whole leaf, so they should run at the same time on one XCD and find it in
// that XCD's L2: blocks go to the XCDs in turn, so block b belongs to XCD b % 8, and the blocks of
// one XCD walk through the query tiles of a leaf before they move to the next leaf.
__device__ inline bool knn_block(u32 nleaves, u32 ny, u32& leaf, u32& q0) {
  const u32 xcd = blockIdx.x & 7u, k = blockIdx.x >> 3;
  leaf = 8u * (k / ny) + xcd;
  q0 = 32u * (k % ny);
  return leaf < nleaves;
}

// The l nearest neighbours, inside its leaf, of each of 32 consecutive points of a leaf (block
// (leaf, 32-point block), one wavefront).  Matrix-core tile: rows = 32 candidates, columns = the
// 32 points; lane (half, col) then holds, for point col, the inner products with 16 of the 32
// candidates, and keeps the LCAP smallest (distance, position) keys it has seen in registers.
// The two lanes of a point merge their lists at the end.  knn_pos / knn_d: l entries per point,
// ascending; positions are relative to the leaf.
template <int LCAP>
__global__ __launch_bounds__(64) void hc_knn_kernel(const unsigned char* leafvec, const i32* leafnorm, u32 lv_stride,
                                                    const u32* leaf_off, const u32* tile_of_leaf, u32 l,
                                                    unsigned short* knn_pos, i32* knn_d, u32 nleaves, u32 ny) {
  u32 leaf, q0;
  if (!knn_block(nleaves, ny, leaf, q0)) return;
  const u32 off = leaf_off[leaf];
  const u32 cnt = leaf_off[leaf + 1] - off;
  if (q0 >= cnt) return;
  const unsigned char* tiles = leafvec + (u64)tile_of_leaf[leaf] * 32u * lv_stride;  // the leaf's first tile
  const int lane = threadIdx.x;
  const u32 half = (u32)lane >> 5, col = (u32)lane & 31u;
  const u32 ksteps = lv_stride / 32u;  // at most 4
  const u32 q = q0 + col;
  const u32 qrow = q < cnt ? q : cnt - 1u;
  const u32 qn = (u32)leafnorm[off + qrow];  // (times 512, like the candidates' norms)
  v4i_t bq[4];
#pragma unroll
  for (u32 ks = 0; ks < 4; ++ks) {
    const u32 kk = ks < ksteps ? ks : ksteps - 1u;
    const v4i_t y = *reinterpret_cast<const v4i_t*>(tiles + (u64)q0 * lv_stride + ((2u * kk + half) * 32u + col) * 16u);
    bq[ks] = ks < ksteps ? y : v4i_t{0, 0, 0, 0};
  }
  // A lane meets the candidates c0 + 8 (r / 4) + 4 half + r % 4: numbered c0 / 2 + r (below 512)
  // they ascend with the candidate's position, and a squared distance of at most 128 bytes is
  // below 2^23, so (distance << 9 | number) orders a lane's candidates like (distance, position)
  // in one 32-bit word: an insertion step is a min and a max.
  constexpr u32 K32_INF = 0xFFFFFFFFu;
  u32 best32[LCAP];
#pragma unroll
  for (int i = 0; i < LCAP; ++i) best32[i] = K32_INF;
  // Candidates below the lane's worst kept key wait in a queue of the lane's own (LDS, one
  // column per lane) and are inserted when some lane's queue is full: the insertion code then
  // runs a few times per wave with most lanes busy, not once per candidate for one lane's sake.
  constexpr u32 QCAP = 24;  // a tile adds at most 16 per lane; drained once above 8
  __shared__ u32 pend[QCAP][64];
  u32 pc = 0;
  u32 worst = K32_INF;
  auto drain = [&]() {
#pragma unroll 1
    for (u32 i = 0; i < QCAP; ++i) {
      if (ballot(i < pc) == 0ull) break;
      u32 key = i < pc ? pend[i][lane] : K32_INF;
#pragma unroll
      for (int t = 0; t < LCAP; ++t) {
        const u32 hi = key > best32[t] ? key : best32[t];
        best32[t] = key < best32[t] ? key : best32[t];
        key = hi;
      }
    }
    pc = 0;
    worst = best32[LCAP - 1];
  };

  // the tile after the current one is requested before the current one is used
  v4i_t av[4], cn[4];
  auto request = [&](u32 c0, v4i_t (&a)[4], v4i_t (&nrm)[4]) {
#pragma unroll
    for (u32 ks = 0; ks < 4; ++ks) {
      const u32 kk = ks < ksteps ? ks : ksteps - 1u;
      a[ks] = *reinterpret_cast<const v4i_t*>(tiles + (u64)c0 * lv_stride + ((2u * kk + half) * 32u + col) * 16u);
    }
    // norms of this lane's 16 candidates: rows 8g + 4 half + 0..3, g = 0..3 (the array has a tail
    // of 64 entries, so reading past the leaf's end stays inside it)
#pragma unroll
    for (u32 g = 0; g < 4; ++g) nrm[g] = *reinterpret_cast<const v4i_t*>(leafnorm + off + c0 + 8u * g + 4u * half);
  };
  request(0, av, cn);
  for (u32 c0 = 0; c0 < cnt; c0 += 32u) {
    v4i_t av_next[4], cn_next[4];
    const u32 cnext = c0 + 32u < cnt ? c0 + 32u : c0;  // (the last tile asks for itself again)
    request(cnext, av_next, cn_next);
    if (ballot(pc > QCAP - 16u) != 0ull) drain();  // room for this tile in every lane's queue
    v16i_t acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(av[ks], bq[ks], acc, 0, 0, 0);
    // only the tile with the queries themselves and the leaf's last tile hold candidates to skip
    const u32 qn_tile = qn + (c0 >> 1);
    const int minus_1024 = -1024;
    auto scan = [&](auto checked) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const u32 cand = c0 + 8u * (r / 4) + 4u * half + (r % 4);
        // (|q|^2 + |c|^2 - 2<q,c>) << 9 | number, from norms that come shifted: an add and a
        // multiply-add
        const u32 base = (u32)cn[r / 4][r % 4] + qn_tile + (u32)r;
        u32 packed;  // base - 1024 * <q,c>: an inner product over 128 bytes fits 24 bits
        asm("v_mad_i32_i24 %0, %1, %2, %3" : "=v"(packed) : "v"(acc[r]), "s"(minus_1024), "v"(base));
        const bool valid = !decltype(checked)::value || (cand < cnt && cand != q);
        const u32 key = valid ? packed : K32_INF;
        // written in any case, kept when the count moves on: no lane is masked, no branch taken
        pend[pc][lane] = key;
        pc += key < worst ? 1u : 0u;
      }
    };
    if (c0 == q0 || c0 + 32u > cnt)
      scan(std::true_type{});
    else
      scan(std::false_type{});
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      av[ks] = av_next[ks];
      cn[ks] = cn_next[ks];
    }
  }
  drain();
  // back to (distance << 32 | position), then the other half of the candidates from the partner lane
  u64 best[LCAP];
#pragma unroll
  for (int i = 0; i < LCAP; ++i) {
    const u32 k = best32[i], nr = k & 511u;
    const u32 cand = 32u * (nr >> 4) + 8u * ((nr & 15u) >> 2) + 4u * half + (nr & 3u);
    best[i] = k == K32_INF ? KEY_INF : (((u64)(k >> 9) << 32) | cand);
  }
  u64 other[LCAP];
#pragma unroll
  for (int i = 0; i < LCAP; ++i) other[i] = (u64)__shfl_xor((unsigned long long)best[i], 32, 64);
#pragma unroll
  for (int j = 0; j < LCAP; ++j) {
    u64 key = other[j];
#pragma unroll
    for (int i = 0; i < LCAP; ++i) {
      const u64 lo = key < best[i] ? key : best[i];
      key = key < best[i] ? best[i] : key;
      best[i] = lo;
    }
  }
  if (half == 0 && q < cnt) {
#pragma unroll
    for (int j = 0; j < LCAP; ++j) {
      if ((u32)j < l) {
        const u64 o = (u64)(off + q) * l + j;
        knn_pos[o] = best[j] == KEY_INF ? (unsigned short)0xFFFF : (unsigned short)(best[j] & 0xFFFFull);
        knn_d[o] = (i32)(best[j] >> 32);
      }
    }
  }
}

// ---- float data ------------------------------------------------------------------------------
// The same three steps for float vectors (squared L2, or the negative inner product).  Sums run in
// fp32 in a fixed order; which of two nearly equal distances is the smaller may come out
// differently from an fp64 computation, and with it a point's side, a neighbour or a tree edge.
typedef float v16f_t __attribute__((ext_vector_type(16)));

template <bool MIPS>
__global__ __launch_bounds__(256) void hc_side_f32_kernel(const unsigned char* pts, u32 row_bytes, const u64* keys_in,
                                                          u64 n, const u32* off, u32 nseg, const u32* pos1,
                                                          const u32* pos2, const u32* base, u64* keys_out) {
  const u32 sub = threadIdx.x & 7u, grp = (threadIdx.x >> 3) & 7u;
  const u64 w0 = ((u64)blockIdx.x * 4u + (u32)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6))) * SIDE_PER_WAVE;
  if (w0 >= n) return;
  u32 seg = side_first_node(off, nseg, w0);
  for (u32 it = 0; it < SIDE_PER_WAVE / 8u; ++it) {
    const u64 i = w0 + 8u * it + grp;
    if (i >= n) break;
    const u32 id = (u32)keys_in[i];
    while ((u64)off[seg + 1] <= i) ++seg;
    u32 idx = base[seg];
    const u32 p1 = pos1[seg];
    if (p1 != HC_NONE) {
      const u32 ida = (u32)keys_in[p1], idb = (u32)keys_in[pos2[seg]];
      const float4* x = reinterpret_cast<const float4*>(pts + (u64)id * row_bytes);
      const float4* a = reinterpret_cast<const float4*>(pts + (u64)ida * row_bytes);
      const float4* b = reinterpret_cast<const float4*>(pts + (u64)idb * row_bytes);
      float da = 0.0f, db = 0.0f;
      for (u32 pc = sub; pc < row_bytes / 16; pc += 8) {
        const float4 vx = x[pc], va = a[pc], vb = b[pc];
        const float fx[4] = {vx.x, vx.y, vx.z, vx.w}, fa[4] = {va.x, va.y, va.z, va.w}, fb[4] = {vb.x, vb.y, vb.z, vb.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          if constexpr (MIPS) {
            da = __builtin_fmaf(-fx[k], fa[k], da);
            db = __builtin_fmaf(-fx[k], fb[k], db);
          } else {
            const float ea = fx[k] - fa[k], eb = fx[k] - fb[k];
            da = __builtin_fmaf(ea, ea, da);
            db = __builtin_fmaf(eb, eb, db);
          }
        }
      }
      da = group_sum(da);
      db = group_sum(db);
      if (da > db) idx += 1;
    }
    if (sub == 0) keys_out[i] = ((u64)idx << 32) | id;
  }
}

// vectors in leaf order (rows of lv_stride bytes, zero tail) and their squared norms
__global__ __launch_bounds__(256) void hc_gather_f32_kernel(const unsigned char* pts, u32 row_bytes, const u64* keys,
                                                            const u32* leaf_off, const u32* tile_of_leaf, u32 nleaves,
                                                            u32 lv_stride, unsigned char* leafvec, float* leafnorm) {
  const u32 tile = blockIdx.x;
  const u32 leaf = leaf_of_tile(tile_of_leaf, nleaves, tile);
  const u32 r = threadIdx.x >> 3, sub = threadIdx.x & 7u;
  const u32 in_leaf = 32u * (tile - tile_of_leaf[leaf]) + r;
  unsigned char* y = leafvec + (u64)tile * 32u * lv_stride;
  if (in_leaf >= leaf_off[leaf + 1] - leaf_off[leaf]) {  // an unused row of the leaf's last tile: zeros
    for (u32 pc = sub; pc < lv_stride / 16; pc += 8)
      *reinterpret_cast<float4*>(y + ((u64)pc * 32u + r) * 16u) = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    return;
  }
  const u64 i = (u64)leaf_off[leaf] + in_leaf;
  const u32 id = (u32)keys[i];
  const float4* x = reinterpret_cast<const float4*>(pts + (u64)id * row_bytes);
  float nn = 0.0f;
  for (u32 pc = sub; pc < lv_stride / 16; pc += 8) {
    float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (pc < row_bytes / 16) v = x[pc];
    *reinterpret_cast<float4*>(y + ((u64)pc * 32u + r) * 16u) = v;
    nn = __builtin_fmaf(v.x, v.x, nn);
    nn = __builtin_fmaf(v.y, v.y, nn);
    nn = __builtin_fmaf(v.z, v.z, nn);
    nn = __builtin_fmaf(v.w, v.w, nn);
  }
  nn = group_sum(nn);
  if (sub == 0) leafnorm[i] = nn;
}

// Nearest neighbours inside the leaf on the fp32 matrix cores (v_mfma_f32_32x32x2f32: two
// elements of the inner product per instruction; a lane feeds it, one after the other, the four
// floats of a 16-byte piece, the lower half-wave taking bytes 0..15 of every 32 and the upper half
// bytes 16..31: a reordering of the sum's terms that both operands share).  Squared L2 comes out
// as |a|^2 + |b|^2 - 2<a,b>, clamped at zero, for the selection (as in the integer kernel); the
// distances of the l candidates selected are then taken again as sum (a - b)^2 (see the end of the
// kernel).  knn_d receives the order-preserving 32-bit image of the distance.
template <int LCAP, bool MIPS>
__global__ __launch_bounds__(64) void hc_knn_f32_kernel(const unsigned char* leafvec, const float* leafnorm,
                                                        u32 lv_stride, const u32* leaf_off, const u32* tile_of_leaf,
                                                        u32 l, unsigned short* knn_pos, i32* knn_d, u32 nleaves,
                                                        u32 ny) {
  u32 leaf, q0;
  if (!knn_block(nleaves, ny, leaf, q0)) return;
  const u32 off = leaf_off[leaf];
  const u32 cnt = leaf_off[leaf + 1] - off;
  if (q0 >= cnt) return;
  const int lane = threadIdx.x;
  const u32 half = (u32)lane >> 5, col = (u32)lane & 31u;
  const u32 ksteps = lv_stride / 32u;
  const u32 q = q0 + col;
  const u32 qrow = q < cnt ? q : cnt - 1u;
  const float qn = leafnorm[off + qrow];
  const unsigned char* tiles = leafvec + (u64)tile_of_leaf[leaf] * 32u * lv_stride;  // the leaf's first tile
  const u32 in_tile = (half * 32u + col) * 16u;  // piece 2 ks + half of row col: at in_tile + ks * 1024
  const unsigned char* qp = tiles + (u64)q0 * lv_stride + in_tile;
  u64 best[LCAP];
#pragma unroll
  for (int i = 0; i < LCAP; ++i) best[i] = KEY_INF;
  constexpr u32 QCAP = 24;  // a tile adds at most 16 per lane; drained once above 8
  __shared__ u64 pend[QCAP][64];
  u32 pc = 0;
  u64 worst = KEY_INF;
  auto drain = [&]() {
#pragma unroll 1
    for (u32 i = 0; i < QCAP; ++i) {
      if (ballot(i < pc) == 0ull) break;
      u64 key = i < pc ? pend[i][lane] : KEY_INF;
#pragma unroll
      for (int t = 0; t < LCAP; ++t) {
        const u64 lo = key < best[t] ? key : best[t];
        key = key < best[t] ? best[t] : key;
        best[t] = lo;
      }
    }
    pc = 0;
    worst = best[LCAP - 1];
  };
  for (u32 c0 = 0; c0 < cnt; c0 += 32u) {
    if (ballot(pc > QCAP - 16u) != 0ull) drain();  // room for this tile in every lane's queue
    const unsigned char* cp = tiles + (u64)c0 * lv_stride + in_tile;
    v16f_t acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    for (u32 ks = 0; ks < ksteps; ++ks) {
      const float4 a = *reinterpret_cast<const float4*>(cp + 1024u * ks);
      const float4 b = *reinterpret_cast<const float4*>(qp + 1024u * ks);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc, 0, 0, 0);
    }
    float cn[16];
#pragma unroll
    for (u32 g = 0; g < 4; ++g) {
      const float4 v = *reinterpret_cast<const float4*>(leafnorm + off + c0 + 8u * g + 4u * half);
      cn[4 * g] = v.x;
      cn[4 * g + 1] = v.y;
      cn[4 * g + 2] = v.z;
      cn[4 * g + 3] = v.w;
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const u32 cand = c0 + 8u * (r / 4) + 4u * half + (r % 4);
      float dd;
      if constexpr (MIPS) {
        dd = -acc[r];
      } else {
        dd = (qn + cn[r]) - 2.0f * acc[r];
        dd = dd < 0.0f ? 0.0f : dd;
      }
      const u64 key = (cand < cnt && cand != q) ? (((u64)dkey_from_float(dd) << 32) | cand) : KEY_INF;
      const bool qual = key < worst;
      if (qual) {
        pend[pc][lane] = key;
        ++pc;
      }
    }
  }
  drain();
  u64 other[LCAP];
#pragma unroll
  for (int i = 0; i < LCAP; ++i) other[i] = (u64)__shfl_xor((unsigned long long)best[i], 32, 64);
#pragma unroll
  for (int j = 0; j < LCAP; ++j) {
    u64 key = other[j];
#pragma unroll
    for (int i = 0; i < LCAP; ++i) {
      const u64 lo = key < best[i] ? key : best[i];
      key = key < best[i] ? best[i] : key;
      best[i] = lo;
    }
  }
  if constexpr (!MIPS) {
    // |a|^2 + |b|^2 - 2<a,b> loses the leading digits of a small distance (unit vectors a hundredth
    // apart: errors of a few 1e-5 of the value), which is fine for picking candidates but not for
    // what the pairs are sorted by, nor for deciding the last places of the list.  So the list
    // kept so far is longer than l (LCAP entries: the launch picks LCAP = 16 for l <= 10 and 24
    // beyond); the distances of all of them are taken again as sum (a - b)^2, a chain of fused
    // multiply-adds in the order of the elements, the list is put in (distance, position) order
    // once more and its first l entries are the result.  Both lanes of a point hold the same
    // merged list by now; each takes every other entry and the two exchange the results.
    const u32 npc = lv_stride / 16u;
    const unsigned char* qbase = tiles + (u64)(qrow >> 5) * 32u * lv_stride + (u64)(qrow & 31u) * 16u;
    u64 fresh[LCAP];
#pragma unroll
    for (int j = 0; j < LCAP; ++j) {
      fresh[j] = KEY_INF;
      if (((u32)j & 1u) == half && best[j] != KEY_INF) {
        const u32 cand = (u32)(best[j] & 0xFFFFull);
        const unsigned char* cbase = tiles + (u64)(cand >> 5) * 32u * lv_stride + (u64)(cand & 31u) * 16u;
        float dd = 0.0f;
        for (u32 c = 0; c < npc; ++c) {
          const float4 a = *reinterpret_cast<const float4*>(qbase + (u64)c * 512u);
          const float4 b = *reinterpret_cast<const float4*>(cbase + (u64)c * 512u);
          float t = a.x - b.x;
          dd = __builtin_fmaf(t, t, dd);
          t = a.y - b.y;
          dd = __builtin_fmaf(t, t, dd);
          t = a.z - b.z;
          dd = __builtin_fmaf(t, t, dd);
          t = a.w - b.w;
          dd = __builtin_fmaf(t, t, dd);
        }
        fresh[j] = ((u64)dkey_from_float(dd) << 32) | cand;
      }
    }
#pragma unroll
    for (int j = 0; j < LCAP; ++j) {
      const u64 o = (u64)__shfl_xor((unsigned long long)fresh[j], 32, 64);
      fresh[j] = ((u32)j & 1u) == half ? fresh[j] : o;
      best[j] = KEY_INF;
    }
#pragma unroll
    for (int j = 0; j < LCAP; ++j) {
      u64 key = fresh[j];
#pragma unroll
      for (int i = 0; i < LCAP; ++i) {
        const u64 lo = key < best[i] ? key : best[i];
        key = key < best[i] ? best[i] : key;
        best[i] = lo;
      }
    }
  }
  if (half == 0 && q < cnt) {
#pragma unroll
    for (int j = 0; j < LCAP; ++j) {
      if ((u32)j < l) {
        const u64 o = (u64)(off + q) * l + j;
        knn_pos[o] = best[j] == KEY_INF ? (unsigned short)0xFFFF : (unsigned short)(best[j] & 0xFFFFull);
        knn_d[o] = (i32)(best[j] >> 32);
      }
    }
  }
}

// NS consecutive steps of a bitonic merge (strides jtop, jtop / 2, ... >= 64) over the P keys in
// LDS, for the stage that builds runs of k2 keys: the keys whose positions differ only in the NS
// stride bits exchange among themselves alone, so one thread reads those 2^NS keys, takes the
// steps in registers and writes them back.
template <int NS>
__device__ __forceinline__ void lds_steps(u64* ek, u32 P, u32 k2, u32 jtop, u32 tid) {
  constexpr u32 NK = 1u << NS;
  const u32 jlow = jtop >> (NS - 1);
  for (u32 g = tid; g < (P >> NS); g += 1024) {
    const u32 i = ((g & ~(jlow - 1u)) << NS) | (g & (jlow - 1u));  // the stride bits clear
    const bool asc = (i & k2) == 0;
    u64 v[NK];
#pragma unroll
    for (u32 m = 0; m < NK; ++m) v[m] = ek[i + m * jlow];
#pragma unroll
    for (u32 bit = NK >> 1; bit > 0; bit >>= 1) {
#pragma unroll
      for (u32 m = 0; m < NK; ++m) {
        if ((m & bit) == 0) {
          const u64 a = v[m], b = v[m | bit];
          const bool swap = (a > b) == asc;
          v[m] = swap ? b : a;
          v[m | bit] = swap ? a : b;
        }
      }
    }
#pragma unroll
    for (u32 m = 0; m < NK; ++m) ek[i + m * jlow] = v[m];
  }
}

// One leaf, first half: its candidate pairs (every point with its k = min(l, cnt-1) nearest),
// each once (the entry of the larger end is dropped when the smaller end lists the pair too),
// sorted by (distance, smaller position, larger position) in LDS.  The sorted pairs, as
// (smaller << 16 | larger), replace the head of the leaf's part of knn_d (from knn_d[off * l]);
// their number goes to pair_cnt[leaf].
__global__ __launch_bounds__(1024) void hc_pairs_kernel(const u32* leaf_list, const u32* leaf_off, u32 l,
                                                       const unsigned short* knn_pos, i32* knn_d, u32* pair_cnt) {
  extern __shared__ __align__(16) unsigned char hc_smem[];
  __shared__ u32 kept;
  u64* ek = reinterpret_cast<u64*>(hc_smem);
  const u32 leaf = leaf_list[blockIdx.x];  // the launch's leaves: those of one size class
  const u32 off = leaf_off[leaf];
  const u32 cnt = leaf_off[leaf + 1] - off;
  if (cnt < 2) {
    if (threadIdx.x == 0) pair_cnt[leaf] = 0;
    return;
  }
  const u32 tid = threadIdx.x;
  const int lane = (int)(tid & 63u);
  const u32 k = l < cnt - 1u ? l : cnt - 1u;
  const u32 E = cnt * k;
  if (tid == 0) kept = 0;
  __syncthreads();
  for (u32 e0 = tid - (u32)lane; e0 < E; e0 += 1024) {  // whole waves: the ballot below needs every lane
    const u32 e = e0 + (u32)lane;
    bool keep = false;
    u64 key = KEY_INF;
    if (e < E) {
      const u32 a = e / k, j = e - a * k;
      const u64 o = (u64)(off + a) * l + j;
      const u32 b = knn_pos[o];
      keep = true;
      if (a > b) {
        // does b list a?  Eight entries of b's list at a time, all requested before the first is
        // looked at (entries past the list's end repeat its last one)
        const unsigned short* lb = knn_pos + (u64)(off + b) * l;
        for (u32 t0 = 0; t0 < k; t0 += 8) {
          unsigned short w[8];
#pragma unroll
          for (u32 t = 0; t < 8; ++t) w[t] = lb[t0 + t < k ? t0 + t : k - 1u];
#pragma unroll
          for (u32 t = 0; t < 8; ++t) keep = keep && w[t] != a;
        }
      }
      const u32 u = a < b ? a : b, v = a < b ? b : a;
      key = ((u64)(u32)knn_d[o] << 32) | (u << 16) | v;
    }
    const u64 m = ballot(keep);
    u32 base = 0;
    if (lane == 0 && m != 0ull) base = atomicAdd(&kept, (u32)__builtin_popcountll(m));
    base = readlane_u32(base, 0);
    if (keep) ek[base + (u32)__builtin_popcountll(m & lanemask_lt(lane))] = key;
  }
  __syncthreads();
  const u32 M = kept;
  u32 P = 64;
  while (P < M) P <<= 1;  // within the launch's LDS: the host sized it for the largest leaf
  for (u32 e = M + tid; e < P; e += 1024) ek[e] = KEY_INF;
  __syncthreads();
  // bitonic sort; the steps whose partners lie within 64 consecutive keys (more than half of all
  // steps) run in registers, one wavefront per 64 keys, with lane exchanges instead of LDS trips
  // and workgroup barriers
  for (u32 k2 = 2; k2 <= P; k2 <<= 1) {
    u32 j = k2 >> 1;
    // the steps across 64 keys or more, up to three in one trip through LDS: a thread takes the 2,
    // 4 or 8 keys that those steps exchange among themselves
    while (j >= 64) {
      if (j >= 256) {
        lds_steps<3>(ek, P, k2, j, tid);
        j >>= 3;
      } else if (j >= 128) {
        lds_steps<2>(ek, P, k2, j, tid);
        j >>= 2;
      } else {
        lds_steps<1>(ek, P, k2, j, tid);
        j >>= 1;
      }
      __syncthreads();
    }
    // four keys of a thread at a time, so that the lane exchanges of one do not wait for another's
    for (u32 i0 = tid; i0 < P; i0 += 4096) {
      u64 v[4];
      bool keep_low[4];  // this position keeps the smaller key of an exchange across bit jj ...
#pragma unroll
      for (u32 q = 0; q < 4; ++q) {
        const u32 i = i0 + 1024u * q;
        v[q] = i < P ? ek[i] : KEY_INF;
        keep_low[q] = (i & k2) == 0;  // ... when its own bit jj is clear; the other way round otherwise
      }
      // keeps its own key if that is the one wanted here: the smaller on the low side of an
      // ascending run and on the high side of a descending one (equal keys: either)
      auto settle = [&](u32 q, u32 jj, u32 olo, u32 ohi) {
        const u64 o = ((u64)ohi << 32) | olo;
        const bool want_low = (((u32)lane & jj) == 0) == keep_low[q];
        v[q] = ((v[q] < o) == want_low) ? v[q] : o;
      };
      for (u32 jj = j; jj >= 16; jj >>= 1) {  // partners 16 or 32 lanes away: through the LDS crossbar
        const int src = (int)(((u32)lane ^ jj) << 2);
#pragma unroll
        for (u32 q = 0; q < 4; ++q)
          settle(q, jj, (u32)__builtin_amdgcn_ds_bpermute(src, (int)(u32)v[q]),
                 (u32)__builtin_amdgcn_ds_bpermute(src, (int)(u32)(v[q] >> 32)));
      }
      // partners inside a row of 16 lanes: data-parallel-primitive moves.  8 away: the row turned
      // by 8.  4 away: the row turned by 12 for the lanes whose partner is above (banks 0 and 2),
      // by 4 for those whose partner is below (banks 1 and 3).
      if (j >= 8) {
#pragma unroll
        for (u32 q = 0; q < 4; ++q)
          settle(q, 8u, (u32)__builtin_amdgcn_update_dpp(0, (int)(u32)v[q], 0x128, 0xF, 0xF, true),
                 (u32)__builtin_amdgcn_update_dpp(0, (int)(u32)(v[q] >> 32), 0x128, 0xF, 0xF, true));
      }
      if (j >= 4) {
#pragma unroll
        for (u32 q = 0; q < 4; ++q) {
          const int lo = (int)(u32)v[q], hi = (int)(u32)(v[q] >> 32);
          const int olo = __builtin_amdgcn_update_dpp(__builtin_amdgcn_update_dpp(0, lo, 0x12C, 0xF, 0x5, false), lo,
                                                      0x124, 0xF, 0xA, false);
          const int ohi = __builtin_amdgcn_update_dpp(__builtin_amdgcn_update_dpp(0, hi, 0x12C, 0xF, 0x5, false), hi,
                                                      0x124, 0xF, 0xA, false);
          settle(q, 4u, (u32)olo, (u32)ohi);
        }
      }
      if (j >= 2) {  // partners inside a group of four lanes: quad_perm [2,3,0,1], then [1,0,3,2]
#pragma unroll
        for (u32 q = 0; q < 4; ++q)
          settle(q, 2u, (u32)__builtin_amdgcn_update_dpp(0, (int)(u32)v[q], 0x4E, 0xF, 0xF, true),
                 (u32)__builtin_amdgcn_update_dpp(0, (int)(u32)(v[q] >> 32), 0x4E, 0xF, 0xF, true));
      }
#pragma unroll
      for (u32 q = 0; q < 4; ++q)
        settle(q, 1u, (u32)__builtin_amdgcn_update_dpp(0, (int)(u32)v[q], 0xB1, 0xF, 0xF, true),
               (u32)__builtin_amdgcn_update_dpp(0, (int)(u32)(v[q] >> 32), 0xB1, 0xF, 0xF, true));
#pragma unroll
      for (u32 q = 0; q < 4; ++q) {
        const u32 i = i0 + 1024u * q;
        if (i < P) ek[i] = v[q];
      }
    }
    __syncthreads();
  }
  u32* out = reinterpret_cast<u32*>(knn_d) + (u64)off * l;
  for (u32 e = tid; e < M; e += 1024) out[e] = (u32)ek[e];
  if (tid == 0) pair_cnt[leaf] = M;
}

// Second half, one wavefront per leaf: Kruskal's scan over the sorted pairs with the degree bound
// s.  A pair whose ends are connected, or one of whose ends is full, stays so: the wave tests 64
// pairs at once against the state so far and walks through the survivors in order.  Accepted
// pairs go, as two arcs (point << 32 | neighbour), to arcs[2 * (off - leaf) ...] (a leaf of cnt
// points accepts at most cnt - 1; unused entries keep what they hold).
__global__ __launch_bounds__(64) void hc_kruskal_kernel(const u64* keys, const u32* leaf_off, u32 l, u32 s,
                                                        const i32* knn_d, const u32* pair_cnt, u64* arcs) {
  __shared__ unsigned short parent_lds[HC_MAX_LS];
  __shared__ unsigned char deg_lds[HC_MAX_LS];
  volatile unsigned short* parent = parent_lds;
  volatile unsigned char* deg = deg_lds;
  const u32 leaf = blockIdx.x;
  const u32 off = leaf_off[leaf];
  const u32 cnt = leaf_off[leaf + 1] - off;
  if (cnt < 2) return;
  const int lane = threadIdx.x;
  const u32 E = pair_cnt[leaf];
  const u32* pairs = reinterpret_cast<const u32*>(knn_d) + (u64)off * l;
  for (u32 i = (u32)lane; i < cnt; i += 64) {
    parent[i] = (unsigned short)i;
    deg[i] = 0;
  }
  __builtin_amdgcn_wave_barrier();
  u64* out = arcs + 2ull * (off - leaf);
  u32 accepted = 0;
  // The accepted pairs wait in the lanes' registers, one per lane, and leave 64 at a time: the
  // ids' loads then overlap, and none of them sits in the chain of dependent steps.
  u32 mine = 0;
  auto write_out = [&](u32 first, u32 count) {
    if ((u32)lane < count) {
      const u64 gu = keys[off + (mine >> 16)] & 0xFFFFFFFFull, gv = keys[off + (mine & 0xFFFFu)] & 0xFFFFFFFFull;
      out[2 * (first + (u32)lane)] = (gu << 32) | gv;
      out[2 * (first + (u32)lane) + 1] = (gv << 32) | gu;
    }
  };
  bool flat = true;  // every point stands directly under its root
  for (u32 c = 0; c < E && accepted < cnt - 1u; c += 64) {
    if (!flat) {
      // the links made while the last 64 pairs were scanned are the only ones a search has to
      // follow afterwards (without this the chains grow as long as the leaf)
      for (u32 i = (u32)lane; i < cnt; i += 64) {
        u32 r = i;
        while (parent[r] != r) r = parent[r];
        __builtin_amdgcn_wave_barrier();
        parent[i] = (unsigned short)r;
      }
      __builtin_amdgcn_wave_barrier();
      flat = true;
    }
    const u32 e = c + (u32)lane;
    const u32 pr = e < E ? pairs[e] : 0u;
    const bool dup = e > 0 && e < E && pr == pairs[e - 1];
    const u32 u = pr >> 16, v = pr & 0xFFFFu;
    bool ok = e < E && !dup;
    if (ok) ok = deg[u] < s && deg[v] < s;
    u32 pu = 0, pv = 0;  // the ends' roots as the chunk starts (flat: parents are roots)
    if (ok) {
      pu = parent[u];
      pv = parent[v];
      ok = pu != pv;
    }
    u64 mask = ballot(ok);
    while (mask != 0ull) {
      const int j = __builtin_ctzll(mask);
      mask &= mask - 1ull;
      // every lane repeats the same step on the same LDS words; the four reads a step starts
      // with do not wait for one another, and only links made within this chunk add to them
      const u32 uu = readlane_u32(u, j), vv = readlane_u32(v, j);
      u32 ru = readlane_u32(pu, j), rv = readlane_u32(pv, j);
      const unsigned char du = deg[uu], dv = deg[vv];
      u32 nu = parent[ru], nv = parent[rv];
      if (du < s && dv < s) {
        while (nu != ru) {
          ru = nu;
          nu = parent[ru];
        }
        while (nv != rv) {
          rv = nv;
          nv = parent[rv];
        }
        if (ru != rv) {
          __builtin_amdgcn_wave_barrier();  // every lane has read before any lane writes
          parent[ru] = (unsigned short)rv;
          deg[uu] = du + 1;
          deg[vv] = dv + 1;
          if (lane == (int)(accepted & 63u)) mine = (uu << 16) | vv;
          ++accepted;
          if ((accepted & 63u) == 0) write_out(accepted - 64u, 64u);
          flat = false;
        }
      }
      __builtin_amdgcn_wave_barrier();
    }
  }
  write_out(accepted & ~63u, accepted & 63u);
}

// ---- repeated keys out of a sorted array --------------------------------------------------
constexpr u32 UQ_TILE = 2048;  // keys per workgroup of 256 threads

__device__ __forceinline__ bool uq_keep(const u64* keys, u64 i, u64 n) {
  return i < n && keys[i] != KEY_INF && (i == 0 || keys[i] != keys[i - 1]);
}

__global__ __launch_bounds__(256) void uq_count_kernel(const u64* keys, u64 n, u32* counts) {
  __shared__ u32 total;
  if (threadIdx.x == 0) total = 0;
  __syncthreads();
  const u64 base = (u64)blockIdx.x * UQ_TILE + threadIdx.x * 8u;
  u32 c = 0;
  for (u32 k = 0; k < 8; ++k) c += uq_keep(keys, base + k, n) ? 1u : 0u;
  atomicAdd(&total, c);
  __syncthreads();
  if (threadIdx.x == 0) counts[blockIdx.x] = total;
}

// counts[0..m) -> exclusive prefix sums in place, the grand total in counts[m]
__global__ __launch_bounds__(1024) void uq_scan_kernel(u32* counts, u32 m) {
  __shared__ unsigned long long part[1024];
  const u32 t = threadIdx.x;
  const u32 per = (m + 1023u) / 1024u;
  const u32 lo = t * per < m ? t * per : m, hi = lo + per < m ? lo + per : m;
  unsigned long long s = 0;
  for (u32 i = lo; i < hi; ++i) s += counts[i];
  part[t] = s;
  __syncthreads();
  for (u32 o = 1; o < 1024; o <<= 1) {
    const unsigned long long v = t >= o ? part[t - o] : 0ull;
    __syncthreads();
    part[t] += v;
    __syncthreads();
  }
  unsigned long long run = t ? part[t - 1] : 0ull;
  for (u32 i = lo; i < hi; ++i) {
    const u32 v = counts[i];
    counts[i] = (u32)run;
    run += v;
  }
  if (t == 1023) counts[m] = (u32)part[1023];
}

__global__ __launch_bounds__(256) void uq_scatter_kernel(const u64* keys, u64 n, const u32* offsets, u64* out) {
  __shared__ u32 pre[256];
  const u32 t = threadIdx.x;
  const u64 base = (u64)blockIdx.x * UQ_TILE + t * 8u;
  bool keep[8];
  u32 c = 0;
  for (u32 k = 0; k < 8; ++k) {
    keep[k] = uq_keep(keys, base + k, n);
    c += keep[k] ? 1u : 0u;
  }
  pre[t] = c;
  __syncthreads();
  for (u32 o = 1; o < 256; o <<= 1) {
    const u32 v = t >= o ? pre[t - o] : 0u;
    __syncthreads();
    pre[t] += v;
    __syncthreads();
  }
  u64 w = (u64)offsets[blockIdx.x] + (t ? pre[t - 1] : 0u);
  for (u32 k = 0; k < 8; ++k)
    if (keep[k]) out[w++] = keys[base + k];
}

// ---- a stable two-way split of every node, without a sort -------------------------------------
// keys[i] = (side << 32) | id, side 0 = left.  With L(i) = number of left points before position
// i, a point of the node [a, b) with nl = L(b) - L(a) left points goes to a + (L(i) - L(a)) if it
// is a left point and to a + nl + (i - a) - (L(i) - L(a)) otherwise.
constexpr u32 SP_TILE = 2048;  // positions per workgroup of 256 threads

__global__ __launch_bounds__(256) void hc_count_left_kernel(const u64* keys, u64 m, u32* tile_cnt) {
  __shared__ u32 total;
  if (threadIdx.x == 0) total = 0;
  __syncthreads();
  const u64 base = (u64)blockIdx.x * SP_TILE + threadIdx.x;  // neighbouring lanes, neighbouring keys
  u32 c = 0;
#pragma unroll
  for (u32 k = 0; k < 8; ++k)
    if (base + 256u * k < m && (u32)(keys[base + 256u * k] >> 32) == 0u) ++c;
  atomicAdd(&total, c);
  __syncthreads();
  if (threadIdx.x == 0) tile_cnt[blockIdx.x] = total;
}

// Lb[j] = L(woff[j]) for the nact + 1 node boundaries; one wavefront each
__global__ __launch_bounds__(64) void hc_seg_left_kernel(const u64* keys, u64 m, const u32* woff, const u32* tile_off,
                                                         u32* Lb) {
  const u64 a = woff[blockIdx.x];
  const u64 t = a / SP_TILE;
  u32 c = 0;
  for (u64 i = t * SP_TILE + threadIdx.x; i < a; i += 64)
    if ((u32)(keys[i] >> 32) == 0u) ++c;
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) c += (u32)__shfl_xor((int)c, o, 64);
  if (threadIdx.x == 0) Lb[blockIdx.x] = tile_off[t] + c;
}

// Every point to its place: the split position sp inside its node as above, then the child that
// covers sp (children 2 seg and 2 seg + 1 start at cstart[..]) and from there either the final
// order (a finished child, dest = its first final position) or the next level's work array (top
// bit of dest set).
__global__ __launch_bounds__(256) void hc_split_route_kernel(const u64* keys, u64 m, const u32* woff, u32 nact,
                                                             const u32* Lb, const u32* tile_off, const u32* cstart,
                                                             const u32* dest, u64* final_keys, u64* next_work) {
  // The tile's 2,048 positions in eight rows of 256: a wavefront reads 64 neighbouring keys at a
  // time and writes the left ones (and the right ones) of a node to neighbouring places.
  __shared__ u32 before[32];  // left points of the tile before row k's quarter w, at [4 k + w]
  const u32 t = threadIdx.x, w = t >> 6;
  const int lane = (int)(t & 63u);
  const u64 tile0 = (u64)blockIdx.x * SP_TILE;
  u64 key[8], lefts[8];
#pragma unroll
  for (u32 k = 0; k < 8; ++k) {
    const u64 i = tile0 + 256u * k + t;
    key[k] = i < m ? keys[i] : ~0ull;
    lefts[k] = ballot((u32)(key[k] >> 32) == 0u);
    if (lane == 0) before[4 * k + w] = (u32)__builtin_popcountll(lefts[k]);
  }
  __syncthreads();
  if (t < 32) {  // exclusive running sums of the 32 counts
    const u32 own = before[t];
    u32 v = own;
#pragma unroll
    for (int o = 1; o < 32; o <<= 1) {
      const u32 up = (u32)__shfl_up((int)v, o, 64);
      if ((int)t >= o) v += up;
    }
    before[t] = v - own;
  }
  __syncthreads();
  const u64 first = tile0 + 64u * w;  // the wavefront's first position: its node by a uniform search
  if (first >= m) return;
  u32 lo = side_first_node(woff, nact, first);
  const u32 tile_left = tile_off[blockIdx.x];
#pragma unroll
  for (u32 k = 0; k < 8; ++k) {
    const u64 i = tile0 + 256u * k + t;
    if (i >= m) break;
    const bool left = (u32)(key[k] >> 32) == 0u;
    const u32 L = tile_left + before[4 * k + w] + (u32)__builtin_popcountll(lefts[k] & lanemask_lt(lane));
    while ((u64)woff[lo + 1] <= i) ++lo;
    const u32 a = woff[lo], La = Lb[lo], nl = Lb[lo + 1] - La;
    const u32 lr = L - La;  // left points of the node before this one
    const u32 sp = left ? a + lr : a + nl + ((u32)i - a - lr);
    const u32 r = sp >= cstart[2 * lo + 1] ? 2 * lo + 1 : 2 * lo;
    const u32 d = dest[r];
    const u64 kk = sp - cstart[r];
    const u64 id = key[k] & 0xFFFFFFFFull;
    if (d & 0x80000000u)
      next_work[(u64)(d & 0x7FFFFFFFu) + kk] = id;
    else
      final_keys[(u64)d + kk] = id;
  }
}

__global__ __launch_bounds__(256) void hc_iota_mod_kernel(u64* keys, u64 n, u64 total) {
  const u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < total) keys[i] = i % n;
}

struct Seg {
  u64 goff, cnt, node, woff;  // place in the final order, size, heap number, place in the work array
  u32 depth, tree;
};
struct Leaf {
  u64 goff, cnt;
};

// Everything one group of trees needs on the device.  The trees of a group are cut side by side:
// tree g of the group owns the positions g*n .. (g+1)*n of every array.
struct HcCtx {
  u64 n = 0, N = 0;  // points; positions of a full group
  u32 G = 1;
  u32 row_bytes = 0, lv_stride = 0;
  bool is_signed = false;
  bool is_f32 = false, is_mips = false;
  const unsigned char* pts = nullptr;
  u32 Ls = 0, s = 0, l = 0;
  u64 seed = 0;
  DevBuf final_keys, work[2], segbuf, routebuf, tilebuf, first, leafvec, leafnorm, leaf_off, knn_pos, knn_d, pair_cnt, leaf_list;
  u64 pair_cnt_cap = 0;
  u64 leaf_tiles = 0;  // tiles of 32 rows that leafvec holds
  u64 seg_words = 0;
  HostBuf h_up, h_route, h_first;  // a level's node table, its routing table, the left counts read back
  // test hook (ann_hcnng_leaf_knn): host arrays that receive every point's neighbour positions
  // and distance keys as the nearest-neighbour kernel leaves them
  unsigned short* dump_pos = nullptr;
  i32* dump_d = nullptr;
  int alloc() {
    HIP_TRY(final_keys.alloc(N * 8));
    for (auto& k : work) HIP_TRY(k.alloc(N * 8));
    // nodes that split at one level: each holds more than Ls points
    const u64 nact = N / ((u64)Ls + 1) + G + 1;
    seg_words = 8 * nact + 16;
    HIP_TRY(segbuf.alloc(seg_words * 4));
    HIP_TRY(routebuf.alloc(seg_words * 4));
    HIP_TRY(h_up.alloc(seg_words * 4));
    HIP_TRY(h_route.alloc(seg_words * 4));
    HIP_TRY(h_first.alloc((2 * nact + 2) * 4));
    HIP_TRY(tilebuf.alloc((N / SP_TILE + 4) * 4));
    HIP_TRY(first.alloc((2 * nact + 2) * 4));
    // every leaf but a tree's smallest few is well above 32 points: room for one partly used tile
    // per Ls / 4 positions (hc_leaves allocates again if a group needs more)
    leaf_tiles = N / 32 + 4 * (N / Ls) + G + 64;
    // test-only option of ann_hcnng_build (see ann.h): start with one tile, so that hc_leaves
    // takes the path that allocates the buffer again
    if (getenv("ANN_HCNNG_FEW_TILES") != nullptr) leaf_tiles = 1;
    HIP_TRY(leafvec.alloc(leaf_tiles * 32 * lv_stride));
    HIP_TRY(leafnorm.alloc((N + 64) * 4));
    HIP_TRY(hipMemset(leafnorm.p, 0, (N + 64) * 4));
    HIP_TRY(leaf_off.alloc(2 * (N + 1) * 4));
    HIP_TRY(knn_pos.alloc(N * l * 2));
    HIP_TRY(knn_d.alloc(N * l * 4));
    return ANN_OK;
  }
};

// The cluster trees tree0 .. tree0+G-1, level by level, all of them in the same launches.  Only
// the points of nodes that still split are worked on: a node's place in the final order is known
// when it is made (children share their parent's range), so finished nodes are copied there and
// the rest is packed for the next level.  On return final_keys holds the point ids (low words),
// tree after tree, leaf after leaf, and `leaves` the leaves in that order.
int hc_partition(HcCtx& X, u32 tree0, u32 G, std::vector<Leaf>& leaves, hipStream_t st) {
  const u64 n = X.n, N = (u64)G * n;
  leaves.clear();
  if (n <= X.Ls) {
    hipLaunchKernelGGL(hc_iota_mod_kernel, dim3((u32)((N + 255) / 256)), dim3(256), 0, st, X.final_keys.as<u64>(), n, N);
    HIP_TRY(hipGetLastError());
    for (u32 g = 0; g < G; ++g) leaves.push_back(Leaf{(u64)g * n, n});
    return ANN_OK;
  }
  hipLaunchKernelGGL(hc_iota_mod_kernel, dim3((u32)((N + 255) / 256)), dim3(256), 0, st, X.work[0].as<u64>(), n, N);
  HIP_TRY(hipGetLastError());
  std::vector<Seg> act, next;
  for (u32 g = 0; g < G; ++g) act.push_back(Seg{(u64)g * n, n, 1, (u64)g * n, 0, tree0 + g});
  u64 m = N;
  while (!act.empty()) {
    const u32 nact = (u32)act.size();
    if (8ull * nact + 16 > X.seg_words) return fail(ANN_EINTERNAL, "more splitting nodes than planned for");
    // woff[nact+1] | pos1[nact] | pos2[nact] | base[nact]
    // (the host tables are free again: the wait in the middle of the previous level came after
    // this table's copy, and the routing table is not written before this level's wait)
    u32* woff = X.h_up.as<u32>();
    std::fill(woff, woff + (size_t)4 * nact + 1, HC_NONE);
    u32* pos1 = woff + nact + 1;
    u32* pos2 = pos1 + nact;
    u32* base = pos2 + nact;
    for (u32 j = 0; j < nact; ++j) {
      const Seg& sg = act[j];
      woff[j] = (u32)sg.woff;
      base[j] = 0;  // the side is all the key carries: 0 left, 1 right
      if (sg.depth < HC_MAX_DEPTH) {
        const u64 k = 2 * (((u64)sg.tree << 40) + sg.node);
        const u64 i1 = mulhi64(stream_output(X.seed, k), sg.cnt);
        u64 i2 = mulhi64(stream_output(X.seed, k + 1), sg.cnt - 1);
        if (i2 >= i1) ++i2;
        pos1[j] = (u32)(sg.woff + i1);
        pos2[j] = (u32)(sg.woff + i2);
      }
    }
    woff[nact] = (u32)m;
    u32* d_seg = X.segbuf.as<u32>();
    HIP_TRY(hipMemcpyAsync(d_seg, woff, ((size_t)4 * nact + 1) * 4, hipMemcpyHostToDevice, st));
    const u32 grid_side = (u32)((m + 4 * SIDE_PER_WAVE - 1) / (4 * SIDE_PER_WAVE));
#define HC_SIDE(KERNEL)                                                                                                  \
  hipLaunchKernelGGL(KERNEL, dim3(grid_side), dim3(256), 0, st, X.pts, X.row_bytes, X.work[0].as<u64>(), m, d_seg, nact, \
                     d_seg + nact + 1, d_seg + 2 * nact + 1, d_seg + 3 * nact + 1, X.work[1].as<u64>())
    if (X.is_f32 && X.is_mips)
      HC_SIDE(hc_side_f32_kernel<true>);
    else if (X.is_f32)
      HC_SIDE(hc_side_f32_kernel<false>);
    else if (X.is_signed)
      HC_SIDE(hc_side_kernel<true>);
    else
      HC_SIDE(hc_side_kernel<false>);
#undef HC_SIDE
    HIP_TRY(hipGetLastError());
    // left points per tile, their running sums, and L at every node boundary
    const u32 ntiles = (u32)((m + SP_TILE - 1) / SP_TILE);
    u32* d_tile = X.tilebuf.as<u32>();
    u32* d_Lb = X.first.as<u32>();
    hipLaunchKernelGGL(hc_count_left_kernel, dim3(ntiles), dim3(256), 0, st, X.work[1].as<u64>(), m, d_tile);
    hipLaunchKernelGGL(uq_scan_kernel, dim3(1), dim3(1024), 0, st, d_tile, ntiles);
    hipLaunchKernelGGL(hc_seg_left_kernel, dim3(nact + 1), dim3(64), 0, st, X.work[1].as<u64>(), m, d_seg, d_tile, d_Lb);
    HIP_TRY(hipGetLastError());
    const u32* h_first = X.h_first.as<u32>();
    HIP_TRY(hipMemcpyAsync(X.h_first.p, d_Lb, ((size_t)nact + 1) * 4, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    // the children: the split leaves every node in its range of the work array
    next.clear();
    u32* cstart = X.h_route.as<u32>();  // cstart[2 nact + 1] | dest[2 nact]
    u32* dest = cstart + 2 * nact + 1;
    u64 nm = 0;
    for (u32 j = 0; j < nact; ++j) {
      const Seg& sg = act[j];
      u64 cl;
      const u64 nl = h_first[j + 1] - h_first[j];
      if (pos1[j] == HC_NONE || nl == 0 || nl == sg.cnt)
        cl = (sg.cnt + 1) / 2;  // too deep, or nothing separated: the order is cut in the middle
      else
        cl = nl;
      const u64 ccnt[2] = {cl, sg.cnt - cl};
      const u64 cgo[2] = {sg.goff, sg.goff + cl};
      const u64 cws[2] = {sg.woff, sg.woff + cl};
      for (int c = 0; c < 2; ++c) {
        cstart[2 * j + c] = (u32)cws[c];
        if (ccnt[c] <= X.Ls) {
          dest[2 * j + c] = (u32)cgo[c];
          leaves.push_back(Leaf{cgo[c], ccnt[c]});
        } else {
          dest[2 * j + c] = 0x80000000u | (u32)nm;
          next.push_back(Seg{cgo[c], ccnt[c], 2 * sg.node + (u64)c, nm, sg.depth + 1, sg.tree});
          nm += ccnt[c];
        }
      }
    }
    cstart[2 * nact] = (u32)m;
    u32* d_route = X.routebuf.as<u32>();
    HIP_TRY(hipMemcpyAsync(d_route, cstart, ((size_t)4 * nact + 1) * 4, hipMemcpyHostToDevice, st));
    hipLaunchKernelGGL(hc_split_route_kernel, dim3(ntiles), dim3(256), 0, st, X.work[1].as<u64>(), m, d_seg, nact, d_Lb,
                       d_tile, d_route, d_route + 2 * nact + 1, X.final_keys.as<u64>(), X.work[0].as<u64>());
    HIP_TRY(hipGetLastError());
    act.swap(next);
    m = nm;
  }
  HIP_TRY(hipStreamSynchronize(st));  // the host tables may be written again
  std::sort(leaves.begin(), leaves.end(), [](const Leaf& a, const Leaf& b) { return a.goff < b.goff; });
  return ANN_OK;
}

// Leaves -> nearest neighbours -> degree-bounded trees, for a whole group; the accepted pairs of
// the group's j-th leaf land, as arcs, at arcs[2 * (goff_j - j) ...].
int hc_leaves(HcCtx& X, u32 G, const std::vector<Leaf>& leaves, u64* arcs, hipStream_t st) {
  const u64 N = (u64)G * X.n;
  const u32 nleaves = (u32)leaves.size();
  // leaf_off[nleaves + 1] | tile_of_leaf[nleaves + 1]: where a leaf's points and its tiles of 32 begin
  std::vector<u32> lo(2 * ((size_t)nleaves + 1));
  u32* lt = lo.data() + nleaves + 1;
  u64 maxc = 0, ntile = 0;
  for (u32 j = 0; j < nleaves; ++j) {
    lo[j] = (u32)leaves[j].goff;
    lt[j] = (u32)ntile;
    ntile += (leaves[j].cnt + 31) / 32;
    maxc = std::max(maxc, leaves[j].cnt);
  }
  lo[nleaves] = (u32)N;
  lt[nleaves] = (u32)ntile;
  if (ntile > X.leaf_tiles) {  // many small leaves: more partly used tiles than planned for
    HIP_TRY(hipStreamSynchronize(st));
    HIP_TRY(X.leafvec.alloc(ntile * 32 * X.lv_stride));
    X.leaf_tiles = ntile;
  }
  HIP_TRY(hipMemcpyAsync(X.leaf_off.p, lo.data(), lo.size() * 4, hipMemcpyHostToDevice, st));
  HIP_TRY(hipStreamSynchronize(st));  // lo goes out of scope
  const u32* d_leaf_off = X.leaf_off.as<u32>();
  const u32* d_tile_of_leaf = d_leaf_off + nleaves + 1;
  if (X.is_f32)
    hipLaunchKernelGGL(hc_gather_f32_kernel, dim3((u32)ntile), dim3(256), 0, st, X.pts, X.row_bytes, X.final_keys.as<u64>(),
                       d_leaf_off, d_tile_of_leaf, nleaves, X.lv_stride, X.leafvec.as<unsigned char>(),
                       X.leafnorm.as<float>());
  else if (X.is_signed)
    hipLaunchKernelGGL(hc_gather_kernel<true>, dim3((u32)ntile), dim3(256), 0, st, X.pts, X.row_bytes,
                       X.final_keys.as<u64>(), d_leaf_off, d_tile_of_leaf, nleaves, X.lv_stride,
                       X.leafvec.as<unsigned char>(), X.leafnorm.as<i32>());
  else
    hipLaunchKernelGGL(hc_gather_kernel<false>, dim3((u32)ntile), dim3(256), 0, st, X.pts, X.row_bytes,
                       X.final_keys.as<u64>(), d_leaf_off, d_tile_of_leaf, nleaves, X.lv_stride,
                       X.leafvec.as<unsigned char>(), X.leafnorm.as<i32>());
  HIP_TRY(hipGetLastError());
  const u32 kny = (u32)((maxc + 31) / 32);
  const dim3 kgrid((u32)(((u64)nleaves + 7) / 8 * 8 * kny));
#define HC_KNN(KERNEL, NORMT)                                                                                       \
  hipLaunchKernelGGL(KERNEL, kgrid, dim3(64), 0, st, X.leafvec.as<unsigned char>(), X.leafnorm.as<NORMT>(), X.lv_stride, \
                     d_leaf_off, d_tile_of_leaf, X.l, X.knn_pos.as<unsigned short>(), X.knn_d.as<i32>(), (u32)nleaves, kny)
  if (X.is_f32 && X.is_mips) {
    if (X.l <= 10)
      HC_KNN((hc_knn_f32_kernel<10, true>), float);
    else
      HC_KNN((hc_knn_f32_kernel<16, true>), float);
  } else if (X.is_f32) {
    // squared L2: a few more candidates than l are kept, see the end of the kernel
    if (X.l <= 10)
      HC_KNN((hc_knn_f32_kernel<16, false>), float);
    else
      HC_KNN((hc_knn_f32_kernel<24, false>), float);
  } else if (X.l <= 4) {
    HC_KNN(hc_knn_kernel<4>, i32);
  } else if (X.l <= 8) {
    HC_KNN(hc_knn_kernel<8>, i32);
  } else if (X.l <= 10) {
    HC_KNN(hc_knn_kernel<10>, i32);
  } else {
    HC_KNN(hc_knn_kernel<16>, i32);
  }
#undef HC_KNN
  HIP_TRY(hipGetLastError());
  if (X.dump_pos != nullptr) {
    HIP_TRY(hipMemcpyAsync(X.dump_pos, X.knn_pos.p, N * X.l * 2, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipMemcpyAsync(X.dump_d, X.knn_d.p, N * X.l * 4, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
  }
  if (X.pair_cnt_cap < nleaves) {
    HIP_TRY(hipStreamSynchronize(st));
    HIP_TRY(X.pair_cnt.alloc(((size_t)nleaves + 1) * 4));
    HIP_TRY(X.leaf_list.alloc(((size_t)nleaves + 1) * 4));
    X.pair_cnt_cap = nleaves;
  }
  // the pair sort by size class: a leaf's LDS follows from its size, and the smaller the
  // allocation the more leaves a compute unit sorts at a time
  {
    std::vector<u32> order;
    order.reserve(nleaves);
    u32 first_of[4] = {0, 0, 0, 0};
    const u32 limit[3] = {4096, 8192, HC_MAX_PAIRS};
    for (int c = 0; c < 3; ++c) {
      first_of[c] = (u32)order.size();
      for (u32 j = 0; j < nleaves; ++j) {
        const u64 cj = leaves[j].cnt;
        const u64 e = cj * (X.l < cj - 1 ? X.l : (cj > 1 ? cj - 1 : 1));
        if (e <= limit[c] && (c == 0 || e > limit[c - 1])) order.push_back(j);
      }
    }
    first_of[3] = (u32)order.size();
    HIP_TRY(hipMemcpyAsync(X.leaf_list.p, order.data(), order.size() * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(hipStreamSynchronize(st));  // `order` goes out of scope
    for (int c = 0; c < 3; ++c) {
      const u32 cntc = first_of[c + 1] - first_of[c];
      if (!cntc) continue;
      const u32 lds = limit[c] * 8;
      HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(hc_pairs_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
      hipLaunchKernelGGL(hc_pairs_kernel, dim3(cntc), dim3(1024), lds, st, X.leaf_list.as<u32>() + first_of[c],
                         X.leaf_off.as<u32>(), X.l, X.knn_pos.as<unsigned short>(), X.knn_d.as<i32>(),
                         X.pair_cnt.as<u32>());
    }
  }
  hipLaunchKernelGGL(hc_kruskal_kernel, dim3(nleaves), dim3(64), 0, st, X.final_keys.as<u64>(), X.leaf_off.as<u32>(), X.l,
                     X.s, X.knn_d.as<i32>(), X.pair_cnt.as<u32>(), arcs);
  HIP_TRY(hipGetLastError());
  return ANN_OK;
}

int hc_check(uint64_t n, uint32_t d, ann_dtype dtype, ann_metric metric, uint32_t Ls, uint32_t s, uint32_t l) {
  if (dtype != ANN_U8 && dtype != ANN_I8 && dtype != ANN_F32) return fail(ANN_EINVAL, "unknown dtype");
  if (metric != ANN_L2SQ && !(metric == ANN_MIPS && dtype == ANN_F32))
    return fail(ANN_EINVAL, "ANN_MIPS is supported for ANN_F32 only");
  if (n < 1 || n >= (1ull << 31)) return fail(ANN_EINVAL, "n must be in [1, 2^31)");
  if (dtype == ANN_F32 ? (d < 4 || d > 256) : (d < 1 || d > 128))
    return fail(ANN_EINVAL, "the clustering-based builder takes rows of at most 128 bytes (1024 for ANN_F32)");
  if (Ls < 2 || Ls > HC_MAX_LS) return fail(ANN_EINVAL, "leaf size must be in [2, 1024]");
  if (l < 1 || l > HC_MAX_L) return fail(ANN_EINVAL, "l must be in [1, 16]");
  if ((u64)Ls * l > HC_MAX_PAIRS) return fail(ANN_EINVAL, "leaf size times l must be at most 16384");
  if (s < 1 || s > 255) return fail(ANN_EINVAL, "s must be in [1, 255]");
  return ANN_OK;
}

int hc_setup(HcCtx& X, const ann_graph* g, const void* pts, uint32_t Ls, uint32_t s, uint32_t l, uint64_t seed,
             u32 G) {
  X.n = g->n;
  X.G = G;
  X.N = (u64)G * g->n;
  X.row_bytes = (u32)g->cfg.row_bytes;
  X.lv_stride = (X.row_bytes + 31u) / 32u * 32u;
  X.is_signed = g->dtype == ANN_I8;
  X.is_f32 = g->dtype == ANN_F32;
  X.is_mips = g->metric == ANN_MIPS;
  X.pts = static_cast<const unsigned char*>(pts);
  X.Ls = Ls;
  X.s = s;
  X.l = l;
  X.seed = seed;
  return X.alloc();
}

}  // namespace hcnng
}  // namespace annmi
using namespace annmi::hcnng;

extern "C" {

}  // extern "C"

// One tree: the order of its leaves, their accepted pairs and (when knn_ids is given) every
// point's nearest neighbours inside its leaf with their distances, as the kernels left them.
static int hc_one_tree(const void* points_dev, uint64_t n, uint32_t d, ann_dtype dtype, ann_metric metric,
                       uint32_t Ls, uint32_t s, uint32_t l, uint64_t seed, uint32_t tree, void* stream, uint32_t* perm_host,
                       uint64_t* leaf_off_host, uint64_t* nleaves, uint32_t* pairs_host, uint64_t* npairs,
                       uint32_t* knn_ids, void* knn_dists) {
  if (!points_dev || !perm_host || !leaf_off_host || !nleaves || (!pairs_host && !knn_ids) || (pairs_host && !npairs) ||
      (knn_ids && !knn_dists))
    return fail(ANN_EINVAL, "null argument");
  int rc = hc_check(n, d, dtype, metric, Ls, s, l);
  if (rc) return rc;
  if (tree >= (1u << 20)) return fail(ANN_EINVAL, "tree index must be below 2^20");
  hipStream_t st = static_cast<hipStream_t>(stream);
  ann_graph* g = nullptr;
  rc = new_graph(n, d, dtype, metric, 1, &g);
  if (rc) return rc;
  struct Guard {
    ann_graph* g;
    ~Guard() { ann_graph_free(g); }
  } guard{g};
  const void* pts = nullptr;
  rc = resolve_points(g, points_dev, st, &pts);
  if (rc) return rc;
  HcCtx X;
  rc = hc_setup(X, g, pts, Ls, s, l, seed, 1);
  if (rc) return rc;
  DevBuf arcs;
  HIP_TRY(arcs.alloc(2 * n * 8));
  HIP_TRY(hipMemsetAsync(arcs.p, 0xFF, 2 * n * 8, st));
  std::vector<unsigned short> kpos;
  std::vector<i32> kd;
  if (knn_ids) {
    kpos.resize(n * l);
    kd.resize(n * l);
    X.dump_pos = kpos.data();
    X.dump_d = kd.data();
  }
  std::vector<Leaf> leaves;
  rc = hc_partition(X, tree, 1, leaves, st);
  if (rc) return rc;
  rc = hc_leaves(X, 1, leaves, arcs.as<u64>(), st);
  if (rc) return rc;
  std::vector<u64> hk(n), ha(2 * n);
  HIP_TRY(hipMemcpyAsync(hk.data(), X.final_keys.p, n * 8, hipMemcpyDeviceToHost, st));
  HIP_TRY(hipMemcpyAsync(ha.data(), arcs.p, 2 * n * 8, hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  for (u64 i = 0; i < n; ++i) perm_host[i] = (u32)hk[i];
  for (size_t j = 0; j < leaves.size(); ++j) leaf_off_host[j] = leaves[j].goff;
  leaf_off_host[leaves.size()] = n;
  *nleaves = leaves.size();
  if (pairs_host) {
    u64 np = 0;
    for (u64 i = 0; i + 1 < 2 * n; i += 2)
      if (ha[i] != ~0ull) {
        pairs_host[2 * np] = (u32)(ha[i] >> 32);
        pairs_host[2 * np + 1] = (u32)ha[i];
        ++np;
      }
    *npairs = np;
  }
  if (knn_ids) {
    // positions inside the leaf -> point ids; distance keys -> distances
    for (size_t j = 0; j < leaves.size(); ++j) {
      const u64 lo = leaves[j].goff;
      for (u64 i = lo; i < lo + leaves[j].cnt; ++i)
        for (u32 t = 0; t < l; ++t) {
          const u64 o = i * l + t;
          const bool none = kpos[o] == 0xFFFFu;
          knn_ids[o] = none ? ANN_NONE : perm_host[lo + kpos[o]];
          const u32 key = (u32)kd[o];
          if (dtype == ANN_F32) {
            const u32 bits = (key & 0x80000000u) ? (key & 0x7FFFFFFFu) : ~key;  // inverse of the order-preserving image
            float f;
            memcpy(&f, &bits, 4);
            static_cast<float*>(knn_dists)[o] = none ? INFINITY : f;
          } else {
            static_cast<int32_t*>(knn_dists)[o] = none ? INT32_MAX : (int32_t)key;
          }
        }
    }
  }
  return ANN_OK;
}

extern "C" {

int ann_hcnng_tree_edges(const void* points_dev, uint64_t n, uint32_t d, ann_dtype dtype, ann_metric metric,
                         uint32_t Ls, uint32_t s, uint32_t l, uint64_t seed, uint32_t tree, void* stream, uint32_t* perm_host,
                         uint64_t* leaf_off_host, uint64_t* nleaves, uint32_t* pairs_host, uint64_t* npairs) try {
  if (!pairs_host || !npairs) return fail(ANN_EINVAL, "null argument");
  return hc_one_tree(points_dev, n, d, dtype, metric, Ls, s, l, seed, tree, stream, perm_host, leaf_off_host, nleaves,
                     pairs_host, npairs, nullptr, nullptr);
} catch (...) {
  return annmi::on_exception();
}

int ann_hcnng_leaf_knn(const void* points_dev, uint64_t n, uint32_t d, ann_dtype dtype, ann_metric metric, uint32_t Ls,
                       uint32_t l, uint64_t seed, uint32_t tree, void* stream, uint32_t* perm_host,
                       uint64_t* leaf_off_host, uint64_t* nleaves, uint32_t* knn_ids_host, void* knn_dists_host) try {
  if (!knn_ids_host || !knn_dists_host) return fail(ANN_EINVAL, "null argument");
  return hc_one_tree(points_dev, n, d, dtype, metric, Ls, 1, l, seed, tree, stream, perm_host, leaf_off_host, nleaves,
                     nullptr, nullptr, knn_ids_host, knn_dists_host);
} catch (...) {
  return annmi::on_exception();
}

int ann_hcnng_build(const void* points_dev, uint64_t n, uint32_t d, ann_dtype dtype, ann_metric metric, uint32_t T,
                    uint32_t Ls, uint32_t s, uint32_t l, uint32_t R, float alpha, uint64_t seed, void* stream,
                    ann_graph** out) try {
  if (out) *out = nullptr;
  if (!points_dev || !out) return fail(ANN_EINVAL, "null argument");
  int rc = hc_check(n, d, dtype, metric, Ls, s, l);
  if (rc) return rc;
  if (T < 1 || T >= (1u << 20)) return fail(ANN_EINVAL, "the number of trees must be in [1, 2^20)");
  if ((u64)T * 2 * n >= (1ull << 32)) return fail(ANN_EINVAL, "trees times points must stay below 2^31");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const bool trace = getenv("ANN_TRACE_BUILD") != nullptr;  // wall-clock breakdown on stderr
  auto t_last = std::chrono::steady_clock::now();
  auto mark = [&](const char* what) {
    if (!trace) return;
    (void)hipStreamSynchronize(st);
    const auto now = std::chrono::steady_clock::now();
    fprintf(stderr, "[hcnng] %-28s %8.3f ms\n", what, std::chrono::duration<double, std::milli>(now - t_last).count());
    t_last = now;
  };
  ann_graph* g = nullptr;
  rc = new_graph(n, d, dtype, metric, R, &g);
  if (rc) return rc;
  struct Guard {
    ann_graph* g;
    ~Guard() {
      if (g) ann_graph_free(g);
    }
  } guard{g};
  rc = check_insert_params(g, 1, alpha);
  if (rc) return rc;
  HIP_TRY(hipMemsetAsync(g->rows, 0xFF, (size_t)n * R * sizeof(u32), st));
  const void* pts = nullptr;
  rc = resolve_points(g, points_dev, st, &pts);
  if (rc) return rc;
  {
    u32 sv = 0;
    HIP_TRY(start_vertex_device(points_dev, n, d, dtype, st, &sv));
    g->start = sv;
  }
  // trees are cut in groups, as many at a time as keep a group within 32 million positions
  u32 G = (u32)std::max<u64>(1, (32ull << 20) / n);
  if (G > T) G = T;
  mark("graph, points, start vertex");
  HcCtx X;
  rc = hc_setup(X, g, pts, Ls, s, l, seed, G);
  if (rc) return rc;
  mark("buffers of a tree group");
  const u64 total = (u64)T * 2 * n;
  DevBuf arcs, arcs_tmp, big_hist, uq_counts, lists, small, arena;
  HIP_TRY(arcs.alloc(total * 8));
  HIP_TRY(arcs_tmp.alloc(total * 8));
  HIP_TRY(hipMemsetAsync(arcs.p, 0xFF, total * 8, st));
  mark("arc buffers");
  std::vector<Leaf> leaves;
  for (u32 t = 0; t < T; t += G) {
    const u32 Gc = T - t < G ? T - t : G;
    rc = hc_partition(X, t, Gc, leaves, st);
    if (rc) return rc;
    mark("cluster trees");
    rc = hc_leaves(X, Gc, leaves, arcs.as<u64>() + (u64)t * 2 * n, st);
    if (rc) return rc;
    mark("leaves");
    g->stats.rounds += Gc;
  }
  // all arcs by (point, neighbour): the neighbour bits first, then, stably, the point bits; the
  // unused entries (all ones) end up behind every point
  const u64 he = radix_hist_entries(total);
  HIP_TRY(big_hist.alloc(he * 4));
  const u32 idb = bits_to_hold(n);
  HIP_TRY(radix_sort_edges(arcs.as<u64>(), arcs_tmp.as<u64>(), big_hist.as<u32>(), he, total, idb, st, 0));
  HIP_TRY(radix_sort_edges(arcs.as<u64>(), arcs_tmp.as<u64>(), big_hist.as<u32>(), he, total, idb, st, 32));
  // each (point, neighbour) once
  const u32 ntiles = (u32)((total + UQ_TILE - 1) / UQ_TILE);
  HIP_TRY(uq_counts.alloc(((size_t)ntiles + 1) * 4));
  hipLaunchKernelGGL(uq_count_kernel, dim3(ntiles), dim3(256), 0, st, arcs.as<u64>(), total, uq_counts.as<u32>());
  hipLaunchKernelGGL(uq_scan_kernel, dim3(1), dim3(1024), 0, st, uq_counts.as<u32>(), ntiles);
  hipLaunchKernelGGL(uq_scatter_kernel, dim3(ntiles), dim3(256), 0, st, arcs.as<u64>(), total, uq_counts.as<u32>(),
                     arcs_tmp.as<u64>());
  HIP_TRY(hipGetLastError());
  u32 nuniq = 0;
  HIP_TRY(hipMemcpyAsync(&nuniq, uq_counts.as<u32>() + ntiles, 4, hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  mark("arcs sorted, each once");
  // prune(p, neighbours, R) for every point: the re-prune kernel of BatchInsert on empty rows
  HIP_TRY(hipMemsetAsync(g->meta, 0, (size_t)n * sizeof(u32), st));
  HIP_TRY(lists.alloc(3 * n * sizeof(MergeItem)));
  HIP_TRY(small.alloc(64));
  HIP_TRY(hipMemsetAsync(small.p, 0, 64, st));
  const u64 longest = (u64)s * T;  // neighbours of one point, at most
  const u64 arena_cap = longest > MERGE_SPILL_MIN ? (u64)nuniq : 16;
  HIP_TRY(arena.alloc(arena_cap * 8));
  MergeArgs ma{};
  ma.points = static_cast<const char*>(pts);
  ma.graph = g->rows;
  ma.meta = g->meta;
  ma.R = R;
  ma.keys = arcs_tmp.as<u64>();
  ma.nkeys = nuniq;
  u32* sm = small.as<u32>();
  ma.list_count = sm + 8;
  for (int c = 0; c < 3; ++c) ma.list_items[c] = lists.as<MergeItem>() + (u64)c * n;
  ma.list_items[3] = ma.list_items[2] + (n - 1);  // (not filled here: every list is pruned by the large instance)
  ma.fast_amax = fast_path_amax(g->cfg);
  ma.gram_ok = gram_path_ok(g->cfg) ? 1u : 0u;
  ma.gram_tmax = gram_path_tmax();
  ma.stage_bytes = prune_stage_bytes(R, g->cfg);
  ma.use_mfma = mfma_prune_ok(R, g->cfg) ? 1u : 0u;
  ma.arena = arena.as<u64>();
  ma.arena_cap = arena_cap;
  ma.arena_top = reinterpret_cast<unsigned long long*>(sm + 4);
  ma.error_flag = sm + 2;
  ma.a16 = llround((double)alpha * 65536.0);
  ma.af = alpha;
  ma.counters = nullptr;
  ma.force_prune = 1;
  g->clean_alpha = alpha;
  HIP_TRY(launch_plan(ma, st));
  const u64 want = nuniq < 8192 ? nuniq : 8192;
  HIP_TRY(launch_merge(g->cfg, ma, (u32)(want ? want : 1), st, st, st, st));
  u32 flags[4] = {0, 0, 0, 0};
  HIP_TRY(hipMemcpyAsync(flags, small.p, 16, hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  if (flags[2] != 0) return fail(ANN_EINTERNAL, "merge spill arena exhausted");
  mark("prune");
  g->stats.edges = nuniq;
  guard.g = nullptr;
  *out = g;
  return ANN_OK;
} catch (...) {
  return annmi::on_exception();
}

}  // extern "C"
