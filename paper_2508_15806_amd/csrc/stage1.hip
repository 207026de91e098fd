// Stage 1 of SurfaceLogicKV (Section 3.2, Algorithm 1) on gfx950: for every attention row,
// the top-K set by radix select and the four weight cells; then a fixed-order reduction over
// the rows of each head and the SF / LG / INF scores.
#include <hip/hip_runtime.h>

#include <cmath>

#include "device_utils.h"
#include "slkv_internal.h"

namespace slkv {

constexpr int kS1Threads = 256;
constexpr int kS1Resident = 64;   // elements per thread held in registers (rows up to 16384)
constexpr int kS1Cand = 512;      // weights at or above the bound that the exact ranking can hold

// One workgroup per row.  RESIDENT: the row (n % 4 == 0, n <= 256*64, K <= 64) is read once with
// 16-byte loads and kept in registers for the small-K path; the general radix select re-reads
// the row in every sweep.
// cells[row] = (WO, WD, WS, Wide).
template <bool RESIDENT>
__global__ __launch_bounds__(kS1Threads, 4) void row_cells_kernel(const float* __restrict__ rows, int32_t n,
                                                                  int32_t needle_start, int32_t needle_len, int32_t topk,
                                                               double* __restrict__ cells) {
  constexpr int NT = kS1Threads;
  __shared__ uint32_t hist[kHistBins];
  __shared__ uint32_t sh_scan[NT / 64];
  __shared__ uint32_t res[2];
  __shared__ double sh_d[NT / 64];
  __shared__ uint32_t sh_u[NT / 64];

  const int tid = threadIdx.x;
  const float* W = rows + (int64_t)blockIdx.x * n;
  const int32_t ne = needle_start + needle_len;

  float v[RESIDENT ? kS1Resident : 1];
  // element e of the resident copy: position ((e/4)*NT + tid)*4 + e%4
  if (RESIDENT) {
#pragma unroll
    for (int i = 0; i < kS1Resident / 4; ++i) {
      const int32_t j = (i * NT + tid) * 4;
      const float4 x = *reinterpret_cast<const float4*>(W + (j < n ? j : n - 4));   // past the end: ignored below
      v[4 * i + 0] = x.x;
      v[4 * i + 1] = x.y;
      v[4 * i + 2] = x.z;
      v[4 * i + 3] = x.w;
    }
  }
  auto pos_of = [&](int e) -> int32_t { return ((e >> 2) * NT + tid) * 4 + (e & 3); };

  // sweep helper of the general path: f(position, value) over the row, re-read from memory
  auto sweep = [&](auto f) {
    for (int32_t j = tid; j < n; j += NT) f(j, W[j]);
  };

  // row sum and needle sum in double
  double tot = 0.0, tnw = 0.0;
  if (RESIDENT) {
#pragma unroll
    for (int e = 0; e < kS1Resident; ++e)
      if (pos_of(e) < n) tot += (double)v[e];
  } else {
    sweep([&](int32_t, float x) { tot += (double)x; });
  }
  for (int32_t j = needle_start + tid; j < ne; j += NT) tnw += (double)W[j];
  tot = block_sum<NT, double>(tot, sh_d);
  tnw = block_sum<NT, double>(tnw, sh_d);

  // Small K on a resident row: a lower bound of the K-th largest weight comes from the lane
  // maxima of each wave (K distinct elements); the few weights at or above the bound are
  // collected in LDS and ranked exactly (larger first, equal weights by lower position).
  if (RESIDENT && topk <= kWave) {
    __shared__ float sh_bound[NT / 64];
    __shared__ uint32_t cand_cnt;
    __shared__ float cand_val[kS1Cand];
    __shared__ int32_t cand_pos[kS1Cand];
    __shared__ float slot_val[kWave];
    __shared__ int32_t slot_in[kWave];
    const int lane = tid & 63, wv = tid >> 6;
    float mx = -INFINITY;
#pragma unroll
    for (int e = 0; e < kS1Resident; ++e)
      if (pos_of(e) < n) mx = fmaxf(mx, v[e]);
    // Each wave finds the ceil(K/4)-th largest of its 64 lane maxima (bisection on the key bits
    // with ballots).  At least K weights are >= the smallest of the four values, so that value
    // bounds the K-th largest weight from below.
    const int want = (topk + NT / 64 - 1) / (NT / 64);
    const uint32_t mkey = float_key(mx);
    uint32_t tkey = 0;
    for (int b = 31; b >= 0; --b) {
      const uint32_t trial = tkey | (1u << b);
      if (__popcll(__ballot(mkey >= trial)) >= want) tkey = trial;
    }
    // tkey is now the want-th largest key of the wave; recover its float from a lane holding it
    const unsigned long long hit = __ballot(mkey == tkey);
    const float bound_w = __shfl(mx, __ffsll((long long)hit) - 1, kWave);
    if (lane == 0) sh_bound[wv] = bound_w;
    if (tid == 0) cand_cnt = 0;
    __syncthreads();
    float bound = sh_bound[0];
#pragma unroll
    for (int i = 1; i < NT / 64; ++i) bound = fminf(bound, sh_bound[i]);
#pragma unroll
    for (int e = 0; e < kS1Resident; ++e) {
      const int32_t j = pos_of(e);
      if (j < n && v[e] >= bound) {
        const uint32_t slot = atomicAdd(&cand_cnt, 1u);
        if (slot < (uint32_t)kS1Cand) {
          cand_val[slot] = v[e];
          cand_pos[slot] = j;
        }
      }
    }
    __syncthreads();
    const uint32_t nc = cand_cnt;
    if (nc <= (uint32_t)kS1Cand) {
      for (uint32_t i = tid; i < nc; i += NT) {
        const float x = cand_val[i];
        const int32_t px = cand_pos[i];
        int r = 0;
        for (uint32_t o = 0; o < nc; ++o) {
          const float y = cand_val[o];
          r += (y > x || (y == x && cand_pos[o] < px)) ? 1 : 0;
        }
        if (r < topk) {
          slot_val[r] = x;
          slot_in[r] = (px >= needle_start && px < ne) ? 1 : 0;
        }
      }
      __syncthreads();
      if (wv == 0) {
        const bool on = lane < topk;
        const double x = on ? (double)slot_val[lane] : 0.0;
        const bool inn = on && slot_in[lane];
        const double WO = wave_sum<double>(inn ? x : 0.0);
        const double WD = wave_sum<double>(inn ? 0.0 : x);
        if (lane == 0) {
          const double WS = fmax(0.0, tnw - WO);
          double* c = cells + (int64_t)blockIdx.x * 4;
          c[0] = WO;
          c[1] = WD;
          c[2] = WS;
          c[3] = tot - WO - WD - WS;
        }
      }
      return;
    }
    __syncthreads();   // too many ties at the bound: fall through to the general select
  }

  // K-th largest weight: three histogram levels over the order-preserving key
  uint32_t prefix = 0, k = (uint32_t)topk;
#pragma unroll 1
  for (int level = 0; level < 3; ++level) {
    const int shift = level == 0 ? 21 : (level == 1 ? 10 : 0);
    const int bits = level == 2 ? 10 : 11;
    for (int i = tid; i < kHistBins; i += NT) hist[i] = 0;
    __syncthreads();
    sweep([&](int32_t, float x) {
      const uint32_t key = float_key(x);
      if (level == 0 || (key >> (shift + bits)) == prefix) atomicAdd(&hist[(key >> shift) & ((1u << bits) - 1u)], 1u);
    });
    __syncthreads();
    select_bin<NT>(hist, k, sh_scan, res);
    prefix = (prefix << bits) | res[0];
    k = res[1];
    __syncthreads();
  }
  const uint32_t tau = prefix;
  const uint32_t need_eq = k;            // elements equal to the K-th value that are inside T_k

  // mass above the threshold, inside / outside the needle; census of the ties
  double wo = 0.0, wd = 0.0;
  uint32_t eq_all = 0, eq_needle = 0;
  float tau_val = 0.f;
  sweep([&](int32_t j, float x) {
    const uint32_t key = float_key(x);
    const bool inn = j >= needle_start && j < ne;
    if (key > tau) {
      if (inn) wo += (double)x; else wd += (double)x;
    } else if (key == tau) {
      eq_all += 1;
      eq_needle += inn ? 1u : 0u;
      tau_val = x;
    }
  });
  wo = block_sum<NT, double>(wo, sh_d);
  wd = block_sum<NT, double>(wd, sh_d);
  eq_all = block_sum<NT, uint32_t>(eq_all, sh_u);
  eq_needle = block_sum<NT, uint32_t>(eq_needle, sh_u);
  // every tie has the same value; fetch it from any thread that saw one
  {
    __shared__ float sh_tau;
    if (tid == 0) sh_tau = 0.f;
    __syncthreads();
    if (float_key(tau_val) == tau) sh_tau = tau_val;
    __syncthreads();
    tau_val = sh_tau;
  }

  uint32_t take_needle;                  // ties inside the needle that belong to T_k
  if (need_eq == eq_all) {
    take_needle = eq_needle;
  } else {
    // ties are cut: T_k takes the need_eq ties of lowest position.  Find that position bound
    // by a radix select on the inverted position among the ties, then count.
    uint32_t p2 = 0, k2 = need_eq;
#pragma unroll 1
    for (int level = 0; level < 3; ++level) {
      const int shift = level == 0 ? 21 : (level == 1 ? 10 : 0);
      const int bits = level == 2 ? 10 : 11;
      for (int i = tid; i < kHistBins; i += NT) hist[i] = 0;
      __syncthreads();
      sweep([&](int32_t j, float x) {
        if (float_key(x) != tau) return;
        const uint32_t key = ~(uint32_t)j;
        if (level == 0 || (key >> (shift + bits)) == p2) atomicAdd(&hist[(key >> shift) & ((1u << bits) - 1u)], 1u);
      });
      __syncthreads();
      select_bin<NT>(hist, k2, sh_scan, res);
      p2 = (p2 << bits) | res[0];
      k2 = res[1];
      __syncthreads();
    }
    const int32_t last_pos = (int32_t)(~p2);
    uint32_t cntn = 0;
    sweep([&](int32_t j, float x) {
      if (float_key(x) == tau && j <= last_pos && j >= needle_start && j < ne) cntn += 1;
    });
    take_needle = block_sum<NT, uint32_t>(cntn, sh_u);
  }
  if (tid == 0) {
    const double WO = wo + (double)tau_val * (double)take_needle;
    const double WD = wd + (double)tau_val * (double)(need_eq - take_needle);
    const double WS = fmax(0.0, tnw - WO);
    double* c = cells + (int64_t)blockIdx.x * 4;
    c[0] = WO;
    c[1] = WD;
    c[2] = WS;
    c[3] = tot - WO - WD - WS;
  }
}

// One thread per head: adds the head's T rows (in order) into the accumulators and
// finalises SF, LG, INF (Algorithm 1, steps 5-7; 0/0 = 0).
__global__ void head_reduce_kernel(const double* __restrict__ cells, int32_t heads, int32_t T,
                                   double* __restrict__ acc, double* __restrict__ scores) {
  const int hd = blockIdx.x * blockDim.x + threadIdx.x;
  if (hd >= heads) return;
  double a[4] = {0.0, 0.0, 0.0, 0.0};
  for (int t = 0; t < T; ++t)
    for (int c = 0; c < 4; ++c) a[c] += cells[((int64_t)hd * T + t) * 4 + c];
  double* A = acc + (int64_t)hd * 5;
  for (int c = 0; c < 4; ++c) A[c] += a[c];
  A[4] += (double)T;
  if (scores) {
    const double WO = A[0], WD = A[1], WS = A[2];
    const double SF = (WO + WD) > 0.0 ? WO / (WO + WD) : 0.0;
    const double LG = (WO + WS) > 0.0 ? WO / (WO + WS) : 0.0;
    const double INF = (SF + LG) > 0.0 ? 2.0 * SF * LG / (SF + LG) : 0.0;
    scores[(int64_t)hd * 3 + 0] = SF;
    scores[(int64_t)hd * 3 + 1] = LG;
    scores[(int64_t)hd * 3 + 2] = INF;
  }
}

}  // namespace slkv

using namespace slkv;

extern "C" size_t slkv_score_heads_workspace_bytes(int32_t L, int32_t H, int32_t T, int64_t n) {
  (void)n;
  if (L < 1 || H < 1 || T < 1) return 0;
  return (size_t)L * H * T * 4 * sizeof(double);
}

extern "C" slkv_status slkv_score_heads(const float* d_rows, int32_t L, int32_t H, int32_t T, int64_t n,
                                        int64_t needle_start, int32_t needle_len, int32_t topk, double* d_acc,
                                        double* d_scores, void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  clear_error();
  if (!d_rows || !d_acc || !d_workspace) return fail(SLKV_ERR_NULL, "d_rows, d_acc and d_workspace are required");
  if (L < 1 || H < 1 || T < 1 || n < 1) return fail(SLKV_ERR_BAD_ARG, "L, H, T, n must be >= 1");
  if (n >= (int64_t(1) << 31)) return fail(SLKV_ERR_BAD_ARG, "n >= 2^31");
  const int64_t nrows = (int64_t)L * H * T;
  if (nrows >= (int64_t(1) << 31)) return fail(SLKV_ERR_BAD_ARG, "L*H*T >= 2^31");
  if (needle_len < 1 || needle_start < 0 || needle_start + needle_len > n)
    return fail(SLKV_ERR_BAD_ARG, "needle [%lld, +%d) outside [0, %lld)", (long long)needle_start, needle_len, (long long)n);
  if (topk < 1 || topk > n) return fail(SLKV_ERR_BAD_ARG, "topk %d outside 1..n", topk);
  const void* ptrs[] = {d_rows, d_acc, d_scores, d_workspace};
  for (const void* ptr : ptrs)
    if (reinterpret_cast<uintptr_t>(ptr) % 16) return fail(SLKV_ERR_BAD_ARG, "device pointer %p not 16-byte aligned", ptr);
  const size_t need = slkv_score_heads_workspace_bytes(L, H, T, n);
  if (workspace_bytes < need) return fail(SLKV_ERR_WORKSPACE, "workspace %zu < %zu bytes", workspace_bytes, need);

  hipStream_t st = (hipStream_t)hip_stream;
  double* cells = (double*)d_workspace;
  const bool resident = (n % 4 == 0) && n >= 4 && n <= (int64_t)kS1Threads * kS1Resident && topk <= kWave;
  {
  ScopedKernelTimer tm(SLKV_K_ROW_CELLS, st);
  if (resident)
    hipLaunchKernelGGL(row_cells_kernel<true>, dim3((unsigned)nrows), dim3(kS1Threads), 0, st, d_rows, (int32_t)n,
                       (int32_t)needle_start, needle_len, topk, cells);
  else
    hipLaunchKernelGGL(row_cells_kernel<false>, dim3((unsigned)nrows), dim3(kS1Threads), 0, st, d_rows, (int32_t)n,
                       (int32_t)needle_start, needle_len, topk, cells);
  }
  const int heads = L * H;
  {
    ScopedKernelTimer tm(SLKV_K_HEAD_REDUCE, st);
    hipLaunchKernelGGL(head_reduce_kernel, dim3((heads + 127) / 128), dim3(128), 0, st, cells, heads, T, d_acc, d_scores);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(SLKV_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(e));
  return SLKV_OK;
}
