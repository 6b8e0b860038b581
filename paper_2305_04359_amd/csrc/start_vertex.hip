// Start vertex of the build: the point nearest (squared L2) to the mean, smallest id on ties.
// The paper takes s as an input of batchBuild (Alg. 3) and leaves its choice open; this is the
// usual medoid approximation.
//
// Integer vectors: argmin ||x - S/n||^2 = argmin n*||x||^2 - 2<x,S> with S the column sums, all
// in exact 64-bit integers.  Float vectors: column sums, mean and scores in fp64, with every
// sum taken in a fixed order so that repeated runs agree bit for bit.
#include "ann_device.hpp"
#include "ann_internal.hpp"

namespace annmi {

template <typename T>
struct SumType {
  using type = long long;
};
template <>
struct SumType<float> {
  using type = double;
};

// partial[block][col] = sum of the block's rows
template <typename T>
__global__ __launch_bounds__(256) void colsum_partial_kernel(const T* x, u64 n, u32 d, u64 rows_per_block,
                                                             typename SumType<T>::type* partial) {
  using S = typename SumType<T>::type;
  __shared__ S red[256];
  const u32 t = threadIdx.x;
  const u64 r0 = (u64)blockIdx.x * rows_per_block;
  const u64 r1 = r0 + rows_per_block < n ? r0 + rows_per_block : n;
  const u32 cpb = d < 256u ? d : 256u;  // columns per pass
  const u32 rpi = 256u / cpb;           // rows per iteration
  const u32 roff = t / cpb;
  for (u32 col0 = 0; col0 < d; col0 += cpb) {
    const u32 col = col0 + t % cpb;
    S acc = 0;
    if (roff < rpi && col < d)
      for (u64 r = r0 + roff; r < r1; r += rpi) acc += (S)x[r * d + col];
    red[t] = acc;
    __syncthreads();
    if (roff == 0 && col < d) {
      S tot = 0;
      for (u32 k = 0; k < rpi; ++k) tot += red[k * cpb + (t % cpb)];
      partial[(u64)blockIdx.x * d + col] = tot;
    }
    __syncthreads();
  }
}

template <typename S>
__global__ void colsum_final_kernel(const S* partial, u32 nblocks, u32 d, S* colsum) {
  const u32 col = blockIdx.x * blockDim.x + threadIdx.x;
  if (col >= d) return;
  S tot = 0;
  for (u32 b = 0; b < nblocks; ++b) tot += partial[(u64)b * d + col];
  colsum[col] = tot;
}

__device__ __forceinline__ u64 score_bits(long long s) { return (u64)s ^ 0x8000000000000000ull; }
__device__ __forceinline__ u64 score_bits(double s) { return (u64)__double_as_longlong(s); }  // s >= 0

template <typename T>
__device__ __forceinline__ u64 point_score(const T* row, u32 d, u64 n, const typename SumType<T>::type* colsum) {
  if constexpr (sizeof(T) == 1) {
    long long nn = 0, xs = 0;
    for (u32 j = 0; j < d; ++j) {
      const long long v = (long long)row[j];
      nn += v * v;
      xs += v * colsum[j];
    }
    return score_bits((long long)n * nn - 2 * xs);
  } else {
    double s = 0.0;
    for (u32 j = 0; j < d; ++j) {
      const double t = (double)row[j] - colsum[j] / (double)n;
      s += t * t;
    }
    return score_bits(s);
  }
}

// Byte vectors with d % 4 == 0: eight lanes per point, each taking every eighth 4-byte word of
// the row (coalesced reads), the exact 64-bit partial scores summed across the eight lanes.
template <typename T>
__global__ __launch_bounds__(256) void score8_kernel(const T* x, u64 n, u32 d, const long long* colsum,
                                                     unsigned long long* best, u32* best_id, int pass) {
  extern __shared__ long long cs[];  // column sums
  for (u32 j = threadIdx.x; j < d; j += blockDim.x) cs[j] = colsum[j];
  __syncthreads();
  const u64 i = ((u64)blockIdx.x * blockDim.x + threadIdx.x) >> 3;
  const u32 sub = threadIdx.x & 7u;
  long long nn = 0, xs = 0;
  if (i < n) {
    const u32* row = reinterpret_cast<const u32*>(x + i * d);
    for (u32 wd = sub; wd < d / 4; wd += 8) {
      const u32 v4 = row[wd];
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const long long v = sizeof(T) == 1 && T(-1) < T(0) ? (long long)(signed char)(v4 >> (8 * b))
                                                           : (long long)((v4 >> (8 * b)) & 0xFFu);
        nn += v * v;
        xs += v * cs[4 * wd + b];
      }
    }
  }
#pragma unroll
  for (int off = 1; off < 8; off <<= 1) {
    nn += __shfl_xor(nn, off, 64);
    xs += __shfl_xor(xs, off, 64);
  }
  // one atomic per workgroup: thousands of atomics on one address queue up at a single channel
  __shared__ unsigned long long red[4];
  const bool mine = i < n && sub == 0;
  const u64 sc = mine ? score_bits((long long)n * nn - 2 * xs) : ~0ull;
  unsigned long long v = pass == 0 ? sc : ((mine && sc == *best) ? (unsigned long long)i : ~0ull);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const unsigned long long o = __shfl_xor(v, off, 64);
    v = o < v ? o : v;
  }
  if ((threadIdx.x & 63u) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) v = red[w] < v ? red[w] : v;
    if (v != ~0ull) {
      if (pass == 0)
        atomicMin(best, v);
      else
        atomicMin(best_id, (u32)v);
    }
  }
}

// pass 0: best score; pass 1: smallest id that attains it
template <typename T>
__global__ __launch_bounds__(256) void score_kernel(const T* x, u64 n, u32 d, const typename SumType<T>::type* colsum,
                                                    unsigned long long* best, u32* best_id, int pass) {
  const u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
  const bool mine = i < n;
  const u64 sc = mine ? point_score<T>(x + i * d, d, n, colsum) : ~0ull;
  unsigned long long v = pass == 0 ? sc : ((mine && sc == *best) ? (unsigned long long)i : ~0ull);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {  // one atomic per wavefront
    const unsigned long long o = __shfl_xor(v, off, 64);
    v = o < v ? o : v;
  }
  if ((threadIdx.x & 63u) == 0 && v != ~0ull) {
    if (pass == 0)
      atomicMin(best, v);
    else
      atomicMin(best_id, (u32)v);
  }
}

template <typename T>
static hipError_t start_vertex_t(const T* x, u64 n, u32 d, hipStream_t s, u32* start_out) {
  using S = typename SumType<T>::type;
  const u32 nblocks = (u32)(n < 2048 ? 1 : (n + 2047) / 2048 > 4096 ? 4096 : (n + 2047) / 2048);
  const u64 rpb = (n + nblocks - 1) / nblocks;
  S* partial = nullptr;
  S* colsum = nullptr;
  unsigned long long* best = nullptr;
  u32* best_id = nullptr;
  hipError_t e;
  if ((e = hipMalloc(&partial, (size_t)nblocks * d * sizeof(S))) != hipSuccess) return e;
  if ((e = hipMalloc(&colsum, (size_t)d * sizeof(S) + 16)) != hipSuccess) {
    (void)hipFree(partial);
    return e;
  }
  best = reinterpret_cast<unsigned long long*>(reinterpret_cast<char*>(colsum) + (size_t)d * sizeof(S));
  best_id = reinterpret_cast<u32*>(best + 1);
  hipLaunchKernelGGL((colsum_partial_kernel<T>), dim3(nblocks), dim3(256), 0, s, x, n, d, rpb, partial);
  hipLaunchKernelGGL((colsum_final_kernel<S>), dim3((d + 63) / 64), dim3(64), 0, s, partial, nblocks, d, colsum);
  (void)hipMemsetAsync(best, 0xFF, 12, s);
  if constexpr (sizeof(T) == 1) {
    if (d % 4 == 0 && d <= 4096) {
      const u32 grid8 = (u32)((n * 8 + 255) / 256);
      hipLaunchKernelGGL((score8_kernel<T>), dim3(grid8), dim3(256), d * sizeof(long long), s, x, n, d, colsum, best,
                         best_id, 0);
      hipLaunchKernelGGL((score8_kernel<T>), dim3(grid8), dim3(256), d * sizeof(long long), s, x, n, d, colsum, best,
                         best_id, 1);
    } else {
      const u32 grid = (u32)((n + 255) / 256);
      hipLaunchKernelGGL((score_kernel<T>), dim3(grid), dim3(256), 0, s, x, n, d, colsum, best, best_id, 0);
      hipLaunchKernelGGL((score_kernel<T>), dim3(grid), dim3(256), 0, s, x, n, d, colsum, best, best_id, 1);
    }
  } else {
    const u32 grid = (u32)((n + 255) / 256);
    hipLaunchKernelGGL((score_kernel<T>), dim3(grid), dim3(256), 0, s, x, n, d, colsum, best, best_id, 0);
    hipLaunchKernelGGL((score_kernel<T>), dim3(grid), dim3(256), 0, s, x, n, d, colsum, best, best_id, 1);
  }
  e = hipGetLastError();
  if (e == hipSuccess) e = hipMemcpyAsync(start_out, best_id, sizeof(u32), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  (void)hipFree(partial);
  (void)hipFree(colsum);
  return e;
}

hipError_t start_vertex_device(const void* points, u64 n, u32 d, int dtype, hipStream_t s, u32* start_out) {
  switch (dtype) {
    case 0: return start_vertex_t<uint8_t>(static_cast<const uint8_t*>(points), n, d, s, start_out);
    case 1: return start_vertex_t<int8_t>(static_cast<const int8_t*>(points), n, d, s, start_out);
    case 2: return start_vertex_t<float>(static_cast<const float*>(points), n, d, s, start_out);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace annmi
