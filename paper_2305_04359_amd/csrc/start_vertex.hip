// Start vertex of the build: the point nearest (squared L2) to the mean, smallest id on ties.
// The paper takes s as an input of batchBuild (Alg. 3) and leaves its choice open; this is the
// usual medoid approximation.
//
// Integer vectors: argmin ||x - S/n||^2 = argmin n*||x||^2 - 2<x,S> with S the column sums, all
// in exact 64-bit integers.  Float vectors: column sums, mean and scores in fp64, with every
// sum taken in a fixed order so that repeated runs agree bit for bit.
#include "ann_device.hpp"
#include "ann_internal.hpp"
#include "driver_internal.hpp"

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

// Byte rows with d % 4 == 0: a thread reads 4-byte words (four columns at once), 256 / (d/4)
// rows per step of the workgroup; per-thread sums fit 32 bits (at most 2,048 rows per workgroup).
template <typename T>
__global__ __launch_bounds__(256) void colsum4_partial_kernel(const T* x, u64 n, u32 d, u64 rows_per_block,
                                                              long long* partial) {
  extern __shared__ int red4[];  // 256 x 4
  const u32 t = threadIdx.x;
  const u32 wpr = d / 4;                       // words per row
  const u32 cw = wpr < 256u ? wpr : 256u;      // words per pass
  const u32 rpi = 256u / cw;                   // rows per step
  const u32 roff = t / cw;
  const u64 r0 = (u64)blockIdx.x * rows_per_block;
  const u64 r1 = r0 + rows_per_block < n ? r0 + rows_per_block : n;
  for (u32 w0 = 0; w0 < wpr; w0 += cw) {
    const u32 w = w0 + t % cw;
    int a0 = 0, a1 = 0, a2 = 0, a3 = 0;
    if (roff < rpi && w < wpr) {
      for (u64 r = r0 + roff; r < r1; r += rpi) {
        const u32 v = reinterpret_cast<const u32*>(x + r * d)[w];
        if (T(-1) < T(0)) {
          a0 += (int)(signed char)v;
          a1 += (int)(signed char)(v >> 8);
          a2 += (int)(signed char)(v >> 16);
          a3 += (int)(signed char)(v >> 24);
        } else {
          a0 += (int)(v & 0xFFu);
          a1 += (int)((v >> 8) & 0xFFu);
          a2 += (int)((v >> 16) & 0xFFu);
          a3 += (int)(v >> 24);
        }
      }
    }
    red4[4 * t + 0] = a0;
    red4[4 * t + 1] = a1;
    red4[4 * t + 2] = a2;
    red4[4 * t + 3] = a3;
    __syncthreads();
    if (roff == 0 && w < wpr) {
      long long s0 = 0, s1 = 0, s2 = 0, s3 = 0;
      for (u32 k = 0; k < rpi; ++k) {
        const int* p = red4 + 4 * (k * cw + (t % cw));
        s0 += p[0];
        s1 += p[1];
        s2 += p[2];
        s3 += p[3];
      }
      long long* o = partial + (u64)blockIdx.x * d + 4 * w;
      o[0] = s0;
      o[1] = s1;
      o[2] = s2;
      o[3] = s3;
    }
    __syncthreads();
  }
}

// colsum[col] = sum over the workgroups' partial rows; one workgroup per column
template <typename S>
__global__ __launch_bounds__(256) void colsum_final_kernel(const S* partial, u32 nblocks, u32 d, S* colsum) {
  __shared__ S red[256];
  const u32 col = blockIdx.x;
  S tot = 0;
  for (u32 b = threadIdx.x; b < nblocks; b += 256) tot += partial[(u64)b * d + col];
  red[threadIdx.x] = tot;
  __syncthreads();
  // fixed order: the sum does not depend on timing
  for (u32 off = 128; off > 0; off >>= 1) {
    if (threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) colsum[col] = red[0];
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

__device__ __forceinline__ unsigned long long wave_min64(unsigned long long v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const unsigned long long o = __shfl_xor(v, off, 64);
    v = o < v ? o : v;
  }
  return v;
}

// Workgroup of 256 threads: the best (smallest) score among the threads' points and the smallest
// id that attains it go to wg_score / wg_id [blockIdx.x]; (~0, ~0) stands for "no point".  No
// atomics: thousands of them on one address queue up at a single memory channel.
__device__ __forceinline__ void block_best(unsigned long long sc, unsigned long long id, unsigned long long* wg_score,
                                           unsigned long long* wg_id) {
  __shared__ unsigned long long red[4];
  __shared__ unsigned long long best_s;
  const u32 t = threadIdx.x;
  unsigned long long v = wave_min64(sc);
  if ((t & 63u) == 0) red[t >> 6] = v;
  __syncthreads();
  if (t == 0) {
    for (int w = 1; w < 4; ++w) v = red[w] < v ? red[w] : v;
    best_s = v;
  }
  __syncthreads();
  const unsigned long long bs = best_s;
  unsigned long long cand = wave_min64(sc == bs ? id : ~0ull);
  __syncthreads();
  if ((t & 63u) == 0) red[t >> 6] = cand;
  __syncthreads();
  if (t == 0) {
    for (int w = 1; w < 4; ++w) cand = red[w] < cand ? red[w] : cand;
    wg_score[blockIdx.x] = bs;
    wg_id[blockIdx.x] = cand;
  }
}

// Byte vectors with d % 4 == 0: eight lanes per point, each taking every eighth 4-byte word of
// the row (coalesced reads), the exact 64-bit partial scores summed across the eight lanes.
template <typename T>
__global__ __launch_bounds__(256) void score8_kernel(const T* x, u64 n, u32 d, const long long* colsum,
                                                     unsigned long long* wg_score, unsigned long long* wg_id) {
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
  const bool mine = i < n && sub == 0;
  const u64 sc = mine ? score_bits((long long)n * nn - 2 * xs) : ~0ull;
  block_best(sc, mine ? i : ~0ull, wg_score, wg_id);
}

// the same with one thread per point (any element type, any d)
template <typename T>
__global__ __launch_bounds__(256) void score_kernel(const T* x, u64 n, u32 d, const typename SumType<T>::type* colsum,
                                                    unsigned long long* wg_score, unsigned long long* wg_id) {
  const u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
  const bool mine = i < n;
  const u64 sc = mine ? point_score<T>(x + i * d, d, n, colsum) : ~0ull;
  block_best(sc, mine ? i : ~0ull, wg_score, wg_id);
}

// best score over the workgroups' results, smallest id among those that attain it
__global__ __launch_bounds__(1024) void best_final_kernel(const unsigned long long* wg_score,
                                                          const unsigned long long* wg_id, u32 nwg, u32* best_id) {
  __shared__ unsigned long long red[16];
  __shared__ unsigned long long best_s;
  const u32 t = threadIdx.x;
  unsigned long long v = ~0ull;
  for (u32 k = t; k < nwg; k += 1024) v = wg_score[k] < v ? wg_score[k] : v;
  v = wave_min64(v);
  if ((t & 63u) == 0) red[t >> 6] = v;
  __syncthreads();
  if (t == 0) {
    for (int w = 1; w < 16; ++w) v = red[w] < v ? red[w] : v;
    best_s = v;
  }
  __syncthreads();
  const unsigned long long bs = best_s;
  unsigned long long id = ~0ull;
  for (u32 k = t; k < nwg; k += 1024)
    if (wg_score[k] == bs && wg_id[k] < id) id = wg_id[k];
  id = wave_min64(id);
  __syncthreads();
  if ((t & 63u) == 0) red[t >> 6] = id;
  __syncthreads();
  if (t == 0) {
    for (int w = 1; w < 16; ++w) id = red[w] < id ? red[w] : id;
    *best_id = (u32)id;
  }
}

template <typename T>
static hipError_t start_vertex_t(const T* x, u64 n, u32 d, hipStream_t s, u32* start_out) {
  using S = typename SumType<T>::type;
  const u32 nblocks = (u32)(n < 2048 ? 1 : (n + 2047) / 2048 > 4096 ? 4096 : (n + 2047) / 2048);
  const u64 rpb = (n + nblocks - 1) / nblocks;
  const bool byte_words = sizeof(T) == 1 && d % 4 == 0 && d <= 4096;
  const u32 nwg = byte_words ? (u32)((n * 8 + 255) / 256) : (u32)((n + 255) / 256);
  DevBuf partial_b, colsum_b, wg_b;  // (from the calling thread's allocator)
  hipError_t e;
  if ((e = partial_b.alloc((size_t)nblocks * d * sizeof(S))) != hipSuccess) return e;
  if ((e = colsum_b.alloc((size_t)d * sizeof(S))) != hipSuccess) return e;
  if ((e = wg_b.alloc(((size_t)2 * nwg + 1) * sizeof(unsigned long long))) != hipSuccess) return e;
  S* partial = partial_b.as<S>();
  S* colsum = colsum_b.as<S>();
  unsigned long long* wg = wg_b.as<unsigned long long>();  // nwg scores, nwg ids, then the result
  u32* best_id = reinterpret_cast<u32*>(wg + 2 * (size_t)nwg);
  if constexpr (sizeof(T) == 1) {
    if (byte_words)
      hipLaunchKernelGGL((colsum4_partial_kernel<T>), dim3(nblocks), dim3(256), 256 * 4 * sizeof(int), s, x, n, d, rpb,
                         partial);
    else
      hipLaunchKernelGGL((colsum_partial_kernel<T>), dim3(nblocks), dim3(256), 0, s, x, n, d, rpb, partial);
  } else {
    hipLaunchKernelGGL((colsum_partial_kernel<T>), dim3(nblocks), dim3(256), 0, s, x, n, d, rpb, partial);
  }
  hipLaunchKernelGGL((colsum_final_kernel<S>), dim3(d), dim3(256), 0, s, partial, nblocks, d, colsum);
  bool done = false;
  if constexpr (sizeof(T) == 1) {
    if (byte_words) {
      hipLaunchKernelGGL((score8_kernel<T>), dim3(nwg), dim3(256), d * sizeof(long long), s, x, n, d, colsum, wg,
                         wg + nwg);
      done = true;
    }
  }
  if (!done) hipLaunchKernelGGL((score_kernel<T>), dim3(nwg), dim3(256), 0, s, x, n, d, colsum, wg, wg + nwg);
  hipLaunchKernelGGL(best_final_kernel, dim3(1), dim3(1024), 0, s, wg, wg + nwg, nwg, best_id);
  e = hipGetLastError();
  if (e == hipSuccess) e = hipMemcpyAsync(start_out, best_id, sizeof(u32), hipMemcpyDeviceToHost, s);
  const hipError_t e2 = hipStreamSynchronize(s);  // also before the buffers go back
  return e != hipSuccess ? e : e2;
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
