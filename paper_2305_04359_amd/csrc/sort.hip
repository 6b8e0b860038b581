// Grouping of reversed edges by destination: a stable least-significant-digit radix sort of
// 64-bit keys (destination << 32 | source) on the destination bits only (by default; a caller
// may name another run of key bits).  It takes the place of
// the semisort in BatchInsert (Alg. 3): equal destinations become consecutive, and, the sort
// being stable, the sources of one destination stay in the order they were emitted (batch order).
//
// One wavefront owns a tile of consecutive keys and walks it 64 keys at a time, so ranking inside
// a tile needs no cross-wave coordination: a key's rank among equal digits of its 64-key row is
// a popcount over a match mask built from one ballot per digit bit.  Digits are up to 10 bits
// wide, so 20 destination bits (a million points) take two passes.
#include "ann_device.hpp"
#include "ann_internal.hpp"

namespace annmi {

constexpr u32 RS_DIGIT_BITS = 10;  // at most this many key bits per pass
constexpr u32 RS_RADIX = 1u << RS_DIGIT_BITS;

static u64 rs_tile_keys(u64 count) {
  // at least 1024 keys per tile, at most 8192 tiles
  u64 t = (count + 8191) / 8192;
  if (t < 1024) t = 1024;
  return (t + 63) / 64 * 64;
}
static u64 rs_tiles(u64 count) { return (count + rs_tile_keys(count) - 1) / rs_tile_keys(count); }

// RS_RADIX x tiles counters and RS_RADIX digit totals, enough for any sort of AT MOST `count`
// keys.  (The number of tiles is not monotone in the key count: 8,192 x 1,024 keys make 8,192
// tiles, a few more keys make tiles of 1,088 keys and fewer of them.)
u64 radix_hist_entries(u64 count) {
  u64 tiles = (count + 1023) / 1024 + 1;
  if (tiles > 8192) tiles = 8192;
  return RS_RADIX * (tiles + 1);
}

__global__ __launch_bounds__(64) void rs_hist_kernel(const u64* keys, u64 count, u64 tile_keys, u32 tiles,
                                                     u32 shift, u32 mask, u32* hist) {
  __shared__ u32 cnt[RS_RADIX];
  const int lane = threadIdx.x;
  for (u32 i = lane; i < RS_RADIX; i += 64) cnt[i] = 0;
  __syncthreads();
  const u64 lo = (u64)blockIdx.x * tile_keys;
  const u64 hi = lo + tile_keys < count ? lo + tile_keys : count;
  // four rows of 64 keys requested at a time: the walk waits for memory, not for arithmetic
  for (u64 i0 = lo + lane; i0 < hi; i0 += 256) {
    u64 k4[4];
#pragma unroll
    for (u32 q = 0; q < 4; ++q) k4[q] = i0 + 64u * q < hi ? keys[i0 + 64u * q] : 0ull;
#pragma unroll
    for (u32 q = 0; q < 4; ++q)
      if (i0 + 64u * q < hi) atomicAdd(&cnt[(u32)(k4[q] >> shift) & mask], 1u);
  }
  __syncthreads();
  for (u32 i = lane; i < RS_RADIX; i += 64) hist[(u64)i * tiles + blockIdx.x] = cnt[i];
}

// hist is a RS_RADIX x tiles table.  One workgroup per digit turns its row into an exclusive
// prefix over the tiles and leaves the row total in digit_total[digit] ...
__global__ __launch_bounds__(256) void rs_rowscan_kernel(u32* hist, u32 tiles, u32* digit_total) {
  __shared__ u32 part[256];
  const u32 t = threadIdx.x;
  u32* row = hist + (u64)blockIdx.x * tiles;
  const u32 per = (tiles + 255) / 256;
  const u32 lo = t * per < tiles ? t * per : tiles;
  const u32 hi = lo + per < tiles ? lo + per : tiles;
  u32 s = 0;
  for (u32 i = lo; i < hi; ++i) s += row[i];
  part[t] = s;
  __syncthreads();
  for (u32 off = 1; off < 256; off <<= 1) {
    const u32 v = t >= off ? part[t - off] : 0u;
    __syncthreads();
    part[t] += v;
    __syncthreads();
  }
  u32 run = t ? part[t - 1] : 0u;
  for (u32 i = lo; i < hi; ++i) {
    const u32 v = row[i];
    row[i] = run;
    run += v;
  }
  if (t == 255) digit_total[blockIdx.x] = part[255];
}

// ... and every scatter workgroup turns the RS_RADIX totals into the first output index of each
// digit for itself (an exclusive scan of 1,024 numbers in LDS costs a microsecond; a kernel of
// its own for it cost six, and a "last workgroup does it" ticket inside the row scan more still:
// RS_RADIX atomics on one address).
__global__ __launch_bounds__(64) void rs_scatter_kernel(const u64* keys, u64* out, u64 count, u64 tile_keys,
                                                        u32 tiles, u32 shift, u32 mask, u32 nbits,
                                                        const u32* hist, const u32* digit_total) {
  __shared__ u32 base[RS_RADIX];
  const int lane = threadIdx.x;
  {
    // exclusive scan of the digit totals: lane l owns digits [PL*l, PL*(l+1))
    constexpr u32 PL = RS_RADIX / 64;
    u32 v[PL], sum = 0;
#pragma unroll
    for (u32 k = 0; k < PL; ++k) {
      v[k] = digit_total[PL * lane + k];
      sum += v[k];
    }
    u32 incl = sum;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const u32 o = (u32)__shfl_up((int)incl, off, 64);
      if (lane >= off) incl += o;
    }
    u32 run = incl - sum;
#pragma unroll
    for (u32 k = 0; k < PL; ++k) {
      const u32 dgt = PL * lane + k;
      base[dgt] = run + hist[(u64)dgt * tiles + blockIdx.x];
      run += v[k];
    }
  }
  __syncthreads();
  const u64 lo = (u64)blockIdx.x * tile_keys;
  const u64 hi = lo + tile_keys < count ? lo + tile_keys : count;
  for (u64 i4 = lo; i4 < hi; i4 += 256) {
    u64 k4[4];  // four rows requested before the first is ranked
#pragma unroll
    for (u32 q = 0; q < 4; ++q) k4[q] = i4 + 64u * q + lane < hi ? keys[i4 + 64u * q + lane] : 0ull;
#pragma unroll
    for (u32 q = 0; q < 4; ++q) {
      const u64 i0 = i4 + 64u * q;
      if (i0 >= hi) break;  // uniform
      const u64 i = i0 + lane;
      const bool valid = i < hi;
      const u64 key = k4[q];
      const u32 dg = (u32)(key >> shift) & mask;
      u64 match = ballot(valid);
      for (u32 b = 0; b < nbits; ++b) {
        const bool bit = (dg >> b) & 1u;
        const u64 bm = ballot(bit);
        match &= bit ? bm : ~bm;
      }
      const u32 rank = (u32)__builtin_popcountll(match & lanemask_lt(lane));
      u32 dst = 0;
      if (valid) dst = base[dg] + rank;
      __syncthreads();
      // the highest lane of each group of equal digits advances the group's counter
      if (valid && (match >> lane) == 1ull) base[dg] += (u32)__builtin_popcountll(match);
      __syncthreads();
      if (valid) out[dst] = key;
    }
  }
}

hipError_t radix_sort_edges(u64* keys, u64* tmp, u32* hist, u64 hist_entries, u64 count, u32 key_bits,
                            hipStream_t s, u32 first_bit) {
  if (count < 2 || key_bits == 0) return hipSuccess;
  if ((u64)RS_RADIX * (rs_tiles(count) + 1) > hist_entries) return hipErrorInvalidValue;  // histogram too small
  if (first_bit + key_bits > 64) key_bits = 64 - first_bit;  // (callers sort within the key)
  const u64 tile_keys = rs_tile_keys(count);
  const u32 tiles = (u32)rs_tiles(count);
  const u32 npass = (key_bits + RS_DIGIT_BITS - 1) / RS_DIGIT_BITS;
  const u32 per = (key_bits + npass - 1) / npass;
  u64* src = keys;
  u64* dst = tmp;
  u32 done = 0;
  for (u32 p = 0; p < npass; ++p) {
    const u32 nb = key_bits - done < per ? key_bits - done : per;
    const u32 shift = first_bit + done;
    const u32 mask = (1u << nb) - 1u;
    hipLaunchKernelGGL(rs_hist_kernel, dim3(tiles), dim3(64), 0, s, src, count, tile_keys, tiles, shift, mask, hist);
    u32* digit_total = hist + (u64)RS_RADIX * tiles;
    hipLaunchKernelGGL(rs_rowscan_kernel, dim3(RS_RADIX), dim3(256), 0, s, hist, tiles, digit_total);
    hipLaunchKernelGGL(rs_scatter_kernel, dim3(tiles), dim3(64), 0, s, src, dst, count, tile_keys, tiles, shift,
                       mask, nb, hist, digit_total);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    u64* t = src;
    src = dst;
    dst = t;
    done += nb;
  }
  if (src != keys) return hipMemcpyAsync(keys, src, count * sizeof(u64), hipMemcpyDeviceToDevice, s);
  return hipSuccess;
}

}  // namespace annmi
