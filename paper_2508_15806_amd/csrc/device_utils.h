// Block-level building blocks (wave64): scans, reductions and the digit search of the radix select.
#ifndef SLKV_DEVICE_UTILS_H
#define SLKV_DEVICE_UTILS_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace slkv {

constexpr int kWave = 64;
constexpr int kHistBins = 2048;

// One cross-lane move inside the wave (DPP): every lane reads `src` of the lane that the control
// word CTRL names; a lane whose source lies outside its row of 16, or whose row ROW_MASK leaves
// out, gets `old` instead.
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ uint32_t dpp_move(uint32_t old, uint32_t src) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)old, (int)src, CTRL, ROW_MASK, 0xf, false);
}
constexpr int kDppRowShr = 0x110;       // + n: lane l reads lane l - n of its row
constexpr int kDppRowBcast15 = 0x142;   // lane 15 of a row goes to every lane of the next row
constexpr int kDppRowBcast31 = 0x143;   // lane 31 goes to every lane of rows 2 and 3

// Inclusive prefix sums inside each row of 16 lanes.
__device__ __forceinline__ uint32_t row_incl_scan(uint32_t v) {
  v += dpp_move<kDppRowShr + 1>(0u, v);
  v += dpp_move<kDppRowShr + 2>(0u, v);
  v += dpp_move<kDppRowShr + 4>(0u, v);
  v += dpp_move<kDppRowShr + 8>(0u, v);
  return v;
}

// Inclusive prefix sums over the 64 lanes: the rows first, then the last lane of row 0 and of
// row 2 is added to the row after it, then the last lane of row 1 to rows 2 and 3.
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
  v = row_incl_scan(v);
  v += dpp_move<kDppRowBcast15, 0xa>(0u, v);
  v += dpp_move<kDppRowBcast31, 0xc>(0u, v);
  return v;
}

// op over the 64 lanes for an idempotent op (min, max): the result is valid in lane 63 only.
template <class OP>
__device__ __forceinline__ uint32_t wave_reduce_to_last(uint32_t v, OP op) {
  v = op(v, dpp_move<kDppRowShr + 1>(v, v));
  v = op(v, dpp_move<kDppRowShr + 2>(v, v));
  v = op(v, dpp_move<kDppRowShr + 4>(v, v));
  v = op(v, dpp_move<kDppRowShr + 8>(v, v));
  v = op(v, dpp_move<kDppRowBcast15, 0xa>(v, v));
  v = op(v, dpp_move<kDppRowBcast31, 0xc>(v, v));
  return v;
}

template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
  for (int dlt = kWave / 2; dlt > 0; dlt >>= 1) v += __shfl_xor(v, dlt, kWave);
  return v;
}

// Inclusive scan over the NT threads of the block in thread order.  `sh` holds NT/64 values.
// Every wave adds up the totals of the waves before it by itself.  With TRAIL the call ends
// with a barrier, so `sh` may be reused at once; without, the caller places that barrier.
template <int NT, bool TRAIL = true>
__device__ __forceinline__ uint32_t block_incl_scan(uint32_t v, uint32_t* sh) {
  constexpr int NW = NT / kWave;
  static_assert(NW <= 16, "the wave totals are scanned inside one row of 16 lanes");
  const int lane = threadIdx.x & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const uint32_t s = wave_incl_scan(v);
  if (lane == kWave - 1) sh[wv] = s;
  __syncthreads();
  const uint32_t t = row_incl_scan(lane < NW ? sh[lane] : 0u);
  const uint32_t base = wv ? (uint32_t)__builtin_amdgcn_readlane((int)t, wv - 1) : 0u;
  if (TRAIL) __syncthreads();
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
  const uint32_t incl = block_incl_scan<NT, false>(sum, sh_scan);   // the barrier below covers sh_scan
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
