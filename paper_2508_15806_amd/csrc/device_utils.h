// Block-level building blocks (wave64): scans, reductions and the digit search of the radix select.
#ifndef SLKV_DEVICE_UTILS_H
#define SLKV_DEVICE_UTILS_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace slkv {

constexpr int kWave = 64;
constexpr int kHistBins = 2048;

template <typename T>
__device__ __forceinline__ T wave_incl_scan(T v) {
  const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
  for (int dlt = 1; dlt < kWave; dlt <<= 1) {
    T o = __shfl_up(v, dlt, kWave);
    if (lane >= dlt) v += o;
  }
  return v;
}

template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
  for (int dlt = kWave / 2; dlt > 0; dlt >>= 1) v += __shfl_xor(v, dlt, kWave);
  return v;
}

// Inclusive scan over the NT threads of the block in thread order.  `sh` holds NT/64 values.
// Ends with a barrier, so `sh` may be reused at once.
template <int NT, typename T>
__device__ __forceinline__ T block_incl_scan(T v, T* sh) {
  constexpr int NW = NT / kWave;
  const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
  T s = wave_incl_scan(v);
  if (lane == kWave - 1) sh[wv] = s;
  __syncthreads();
  if (wv == 0) {
    T t = lane < NW ? sh[lane] : T(0);
    t = wave_incl_scan(t);
    if (lane < NW) sh[lane] = t;
  }
  __syncthreads();
  T base = wv ? sh[wv - 1] : T(0);
  __syncthreads();
  return s + base;
}

// Sum over the block in a fixed order (wave tree, then waves in order); result to all threads.
template <int NT, typename T>
__device__ __forceinline__ T block_sum(T v, T* sh) {
  constexpr int NW = NT / kWave;
  const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
  T s = wave_sum(v);
  if (lane == 0) sh[wv] = s;
  __syncthreads();
  T tot = T(0);
#pragma unroll
  for (int i = 0; i < NW; ++i) tot += sh[i];
  __syncthreads();
  return tot;
}

// hist[kHistBins] holds counts per digit.  Finds the digit holding the k-th largest element
// (k >= 1, k <= total count) and how many elements of that digit are still wanted:
// res[0] = digit, res[1] = k - (count in larger digits).  Ends with a barrier.
template <int NT>
__device__ __forceinline__ void select_bin(const uint32_t* hist, uint32_t k, uint32_t* sh_scan, uint32_t* res) {
  constexpr int BPT = kHistBins / NT;
  const int t = NT - 1 - (int)threadIdx.x;       // thread 0 owns the largest digits
  uint32_t c[BPT];
  uint32_t sum = 0;
#pragma unroll
  for (int i = 0; i < BPT; ++i) {
    c[i] = hist[t * BPT + i];
    sum += c[i];
  }
  const uint32_t incl = block_incl_scan<NT, uint32_t>(sum, sh_scan);
  uint32_t above = incl - sum;
  if (above < k && incl >= k) {
#pragma unroll
    for (int i = BPT - 1; i >= 0; --i) {
      if (above < k && above + c[i] >= k) {
        res[0] = (uint32_t)(t * BPT + i);
        res[1] = k - above;
      }
      above += c[i];
    }
  }
  __syncthreads();
}

// Order-preserving map from fp32 bit patterns to unsigned integers (larger float -> larger key).
__device__ __forceinline__ uint32_t float_key(float f) {
  uint32_t u = f == 0.f ? 0u : __float_as_uint(f);   // -0 and +0 rank as equal
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

}  // namespace slkv
#endif
