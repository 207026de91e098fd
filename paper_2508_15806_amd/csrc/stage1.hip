// Stage 1 of SurfaceLogicKV (Section 3.2, Algorithm 1) on gfx950: for every attention row,
// the top-K set by radix select and the four weight cells; then a fixed-order reduction over
// the rows of each head and the SF / LG / INF scores.
#include <hip/hip_runtime.h>

#include <cmath>

#include "device_utils.h"
#include "launch.h"
#include "slkv_internal.h"

namespace slkv {

constexpr int kS1Threads = 256;
constexpr int kS1Resident = 64;   // elements per thread held in registers (rows up to 16384)
constexpr int kS1Cand = 512;      // weights at or above the bound that the exact ranking can hold

// One workgroup per row.  RESIDENT (n % 4 == 0, n <= 256*64, K <= 64): the row is read once with
// 16-byte loads and stays in registers for the small-K path.  The general radix select reads
// the row from memory in every sweep.
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

  // sweep helper of the general path: f(position, value) over the row, re-read from memory
  auto sweep = [&](auto f) {
    for (int32_t j = tid; j < n; j += NT) f(j, W[j]);
  };

  double tot = 0.0, tnw = 0.0;           // row sum and needle sum, in double
  if (RESIDENT) {
    // Small K on a row held in registers.  A lower bound of the K-th largest weight comes from
    // the lane maxima of each wave (K distinct elements); the few weights at or above the bound
    // are collected in LDS and ranked exactly (larger first, equal weights by lower position).
    constexpr int NW = NT / kWave;
    constexpr int kWaveCand = kS1Cand / NW;
    __shared__ double sh_tot[NW], sh_tnw[NW];
    __shared__ float sh_bound[NW];
    __shared__ uint32_t sh_cnt[NW];
    __shared__ float cand_val[kS1Cand];
    __shared__ uint64_t cand_key[kS1Cand];   // (order-preserving key of the weight) << 32 | ~position
    const int lane = tid & 63, wv = tid >> 6;
    const int32_t ngroups = n >> 2;      // n % 4 == 0: the row is whole 16-byte groups

    // group i of this thread: positions 4 * (i * NT + tid) .. + 3; all loads are issued first
    // The rows are read exactly once: non-temporal loads (they do not displace anything in the
    // caches) stream about 13 % faster than plain ones on this part.
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const f32x4* W4 = reinterpret_cast<const f32x4*>(W);
    float4 v[kS1Resident / 4];
#pragma unroll
    for (int i = 0; i < kS1Resident / 4; ++i) {
      const int32_t g = i * NT + tid;
      const f32x4 x = __builtin_nontemporal_load(W4 + (g < ngroups ? g : ngroups - 1));   // past the end: loaded again, never used
      v[i] = make_float4(x.x, x.y, x.z, x.w);
    }
    const int32_t jn = needle_start + tid;
    const float nd = W[jn < ne ? jn : needle_start];

    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < kS1Resident / 4; ++i) {
      if (i * NT + tid < ngroups) {
        tot += (double)v[i].x;
        tot += (double)v[i].y;
        tot += (double)v[i].z;
        tot += (double)v[i].w;
        mx = fmaxf(fmaxf(mx, fmaxf(v[i].x, v[i].y)), fmaxf(v[i].z, v[i].w));
      }
    }
    if (jn < ne) tnw = (double)nd;
    for (int32_t j = jn + NT; j < ne; j += NT) tnw += (double)W[j];
    tot = wave_sum<double>(tot);
    tnw = wave_sum<double>(tnw);

    // Each wave finds a value at or below the ceil(K/4)-th largest of its 64 lane maxima
    // (bisection on the upper 20 bits of the order-preserving key, with ballots).  At least K
    // weights are >= the smallest of the four values, so it bounds the K-th largest from below.
    const uint32_t want = (uint32_t)(topk + NW - 1) / NW;
    const uint32_t mkey = tid < ngroups ? float_key(mx) : 0u;   // lanes without data never count
    uint32_t tkey = 0;
#pragma unroll
    for (int b = 31; b >= 12; --b) {
      const uint32_t trial = tkey | (1u << b);
      if ((uint32_t)__popcll(__ballot(mkey >= trial)) >= want) tkey = trial;
    }
    // the float whose key is tkey (low bits cleared: not above the value found); 0 keys: -inf
    const float bound_w = tkey == 0 ? -INFINITY
                                    : __uint_as_float((tkey & 0x80000000u) ? (tkey ^ 0x80000000u) : ~tkey);
    if (lane == 0) {
      sh_tot[wv] = tot;
      sh_tnw[wv] = tnw;
      sh_bound[wv] = bound_w;
    }
    __syncthreads();
    tot = sh_tot[0];
    tnw = sh_tnw[0];
    float bound = sh_bound[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) {
      tot += sh_tot[i];
      tnw += sh_tnw[i];
      bound = fminf(bound, sh_bound[i]);
    }

    // Candidates of this wave go to its own part of the list; the slot of a lane is the number
    // of candidates found so far plus the candidates of the same element in lower lanes.
    uint32_t base = 0;                   // wave-uniform
    float* my_val = cand_val + wv * kWaveCand;
    uint64_t* my_key = cand_key + wv * kWaveCand;
#pragma unroll
    for (int i = 0; i < kS1Resident / 4; ++i) {
      const int32_t g = i * NT + tid;
      const float bnd = g < ngroups ? bound : INFINITY;
      const float x[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bool is = x[c] >= bnd;
        const unsigned long long mask = __ballot(is);
        if (mask) {
          const uint32_t slot = base + __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                                                 __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
          if (is && slot < (uint32_t)kWaveCand) {
            my_val[slot] = x[c];
            my_key[slot] = ((uint64_t)float_key(x[c]) << 32) | (uint32_t)(~(uint32_t)(4 * g + c));
          }
          base += (uint32_t)__popcll(mask);
        }
      }
    }
    if (lane == 0) sh_cnt[wv] = base;
    __syncthreads();
    uint32_t cnt[NW], nc = 0;
    bool fits = true;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
      cnt[i] = sh_cnt[i];
      nc += cnt[i];
      fits = fits && cnt[i] <= (uint32_t)kWaveCand;
    }
    if (fits && nc >= (uint32_t)topk) {
      // A candidate belongs to T_k if fewer than K candidates are ahead of it (larger, or equal
      // at a lower position: one comparison of the packed keys).  Up to 256 candidates are handled
      // by the first wave alone, each lane counting for up to four of them; the other waves retire.
      constexpr int kPerLane = 4;
      const bool one_wave = nc <= (uint32_t)(kWave * kPerLane);
      if (one_wave && wv != 0) return;
      double wo = 0.0, wd = 0.0;
      const uint32_t stride = one_wave ? kWave : NT;
      const uint32_t per_thread = (nc + stride - 1) / stride;    // uniform over the workgroup
      for (uint32_t c0 = 0; c0 < per_thread; c0 += kPerLane) {
        uint64_t mine[kPerLane];
        float xval[kPerLane];
        uint32_t ahead[kPerLane];
#pragma unroll
        for (int q = 0; q < kPerLane; ++q) {
          const uint32_t c = (c0 + q) * stride + (one_wave ? lane : tid);
          uint32_t part = 0, idx = c;
#pragma unroll
          for (int i = 0; i < NW - 1; ++i)
            if (part == (uint32_t)i && idx >= cnt[i]) {
              idx -= cnt[i];
              part = i + 1;
            }
          const bool have = c < nc;
          mine[q] = have ? cand_key[part * kWaveCand + idx] : ~0ull;   // nothing is ahead of the filler, and it is never summed
          xval[q] = have ? cand_val[part * kWaveCand + idx] : 0.f;
          ahead[q] = have ? 0u : (uint32_t)topk;
        }
#pragma unroll
        for (int p = 0; p < NW; ++p)
          for (uint32_t o = 0; o < cnt[p]; ++o) {
            const uint64_t ko = cand_key[p * kWaveCand + o];
#pragma unroll
            for (int q = 0; q < kPerLane; ++q) ahead[q] += ko > mine[q] ? 1u : 0u;
          }
#pragma unroll
        for (int q = 0; q < kPerLane; ++q)
          if (ahead[q] < (uint32_t)topk) {
            const int32_t px = (int32_t)(~(uint32_t)mine[q]);
            if (px >= needle_start && px < ne) wo += (double)xval[q]; else wd += (double)xval[q];
          }
      }
      if (one_wave) {
        wo = wave_sum<double>(wo);
        wd = wave_sum<double>(wd);
      } else {
        wo = block_sum<NT, double>(wo, sh_d);
        wd = block_sum<NT, double>(wd, sh_d);
      }
      if (tid == 0) {
        const double WS = fmax(0.0, tnw - wo);
        double* c = cells + (int64_t)blockIdx.x * 4;
        c[0] = wo;
        c[1] = wd;
        c[2] = WS;
        c[3] = tot - wo - wd - WS;
      }
      return;
    }
    // too many ties at the bound: the general select below re-reads the row
  } else {
    sweep([&](int32_t, float x) { tot += (double)x; });
    for (int32_t j = needle_start + tid; j < ne; j += NT) tnw += (double)W[j];
    tot = block_sum<NT, double>(tot, sh_d);
    tnw = block_sum<NT, double>(tnw, sh_d);
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

// Steps 5-7 of Algorithm 1 (0/0 = 0); a component that is switched off enters as 0.
__device__ __forceinline__ void sf_lg(double WO, double WD, double WS, int use_wo, int use_wd, int use_ws, double& SF,
                                      double& LG) {
  WO = use_wo ? WO : 0.0;
  WD = use_wd ? WD : 0.0;
  WS = use_ws ? WS : 0.0;
  SF = (WO + WD) > 0.0 ? WO / (WO + WD) : 0.0;
  LG = (WO + WS) > 0.0 ? WO / (WO + WS) : 0.0;
}

// One thread per head: adds the head's T rows (in order) into the accumulators and finalises
// SF, LG, INF (Algorithm 1, steps 5-7).  STRIDE 5: the accumulators of slkv_score_heads;
// STRIDE 8: those of slkv_score_heads_ex, which also carry the sums of the per-row SF and LG.
template <int STRIDE>
__global__ void head_reduce_kernel(const double* __restrict__ cells, int32_t heads, int32_t T, double* __restrict__ acc,
                                   double* __restrict__ scores, int macro, int use_wo, int use_wd, int use_ws) {
  const int hd = blockIdx.x * blockDim.x + threadIdx.x;
  if (hd >= heads) return;
  double a[4] = {0.0, 0.0, 0.0, 0.0}, sf_sum = 0.0, lg_sum = 0.0;
  for (int t = 0; t < T; ++t) {
    const double* c = cells + ((int64_t)hd * T + t) * 4;
    for (int i = 0; i < 4; ++i) a[i] += c[i];
    if (STRIDE == 8) {
      double sf, lg;
      sf_lg(c[0], c[1], c[2], use_wo, use_wd, use_ws, sf, lg);
      sf_sum += sf;
      lg_sum += lg;
    }
  }
  double* A = acc + (int64_t)hd * STRIDE;
  for (int i = 0; i < 4; ++i) A[i] += a[i];
  A[4] += (double)T;
  if (STRIDE == 8) {
    A[5] += sf_sum;
    A[6] += lg_sum;
  }
  if (scores) {
    double SF, LG;
    if (STRIDE == 8 && macro) {
      SF = A[4] > 0.0 ? A[5] / A[4] : 0.0;
      LG = A[4] > 0.0 ? A[6] / A[4] : 0.0;
    } else {
      sf_lg(A[0], A[1], A[2], use_wo, use_wd, use_ws, SF, LG);
    }
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

namespace {

slkv_status run_score_heads(const float* d_rows, int32_t L, int32_t H, int32_t T, int64_t n, int64_t needle_start,
                            int32_t needle_len, int32_t topk, double* d_acc, double* d_scores, void* d_workspace,
                            size_t workspace_bytes, void* hip_stream, const slkv_score_params* prm) {
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
      SLKV_LAUNCH(row_cells_kernel<true>, dim3((unsigned)nrows), dim3(kS1Threads), 0, st, d_rows, (int32_t)n,
                  (int32_t)needle_start, needle_len, topk, cells);
    else
      SLKV_LAUNCH(row_cells_kernel<false>, dim3((unsigned)nrows), dim3(kS1Threads), 0, st, d_rows, (int32_t)n,
                  (int32_t)needle_start, needle_len, topk, cells);
  }
  const int heads = L * H;
  {
    ScopedKernelTimer tm(SLKV_K_HEAD_REDUCE, st);
    if (prm)
      SLKV_LAUNCH(head_reduce_kernel<8>, dim3((heads + 127) / 128), dim3(128), 0, st, (const double*)cells, heads, T, d_acc,
                  d_scores, (int)(prm->aggregation == SLKV_AGG_MACRO), prm->use_wo, prm->use_wd, prm->use_ws);
    else
      SLKV_LAUNCH(head_reduce_kernel<5>, dim3((heads + 127) / 128), dim3(128), 0, st, (const double*)cells, heads, T, d_acc,
                  d_scores, 0, 1, 1, 1);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(SLKV_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(e));
  return SLKV_OK;
}

}  // namespace

extern "C" slkv_status slkv_score_heads(const float* d_rows, int32_t L, int32_t H, int32_t T, int64_t n,
                                        int64_t needle_start, int32_t needle_len, int32_t topk, double* d_acc,
                                        double* d_scores, void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  clear_error();
  return run_score_heads(d_rows, L, H, T, n, needle_start, needle_len, topk, d_acc, d_scores, d_workspace, workspace_bytes,
                         hip_stream, nullptr);
}

extern "C" slkv_status slkv_score_heads_ex(const slkv_score_params* params, const float* d_rows, int32_t L, int32_t H,
                                           int32_t T, int64_t n, int64_t needle_start, int32_t needle_len, int32_t topk,
                                           double* d_acc, double* d_scores, void* d_workspace, size_t workspace_bytes,
                                           void* hip_stream) {
  clear_error();
  if (!params) return fail(SLKV_ERR_NULL, "params is NULL");
  if (params->struct_size != sizeof(slkv_score_params))
    return fail(SLKV_ERR_BAD_ARG, "params.struct_size %u != %zu", params->struct_size, sizeof(slkv_score_params));
  if (params->aggregation != SLKV_AGG_MICRO && params->aggregation != SLKV_AGG_MACRO)
    return fail(SLKV_ERR_BAD_ARG, "unknown aggregation %d", params->aggregation);
  const int32_t flags[3] = {params->use_wo, params->use_wd, params->use_ws};
  for (int32_t f : flags)
    if (f != 0 && f != 1) return fail(SLKV_ERR_BAD_ARG, "use_wo / use_wd / use_ws must be 0 or 1");
  if (params->reserved != 0) return fail(SLKV_ERR_BAD_ARG, "params.reserved must be 0");
  return run_score_heads(d_rows, L, H, T, n, needle_start, needle_len, topk, d_acc, d_scores, d_workspace, workspace_bytes,
                         hip_stream, params);
}
