// Stage 1 of SurfaceLogicKV (Section 3.2, Algorithm 1) on gfx950: for every attention row,
// the top-K set by radix select and the four weight cells; then a fixed-order reduction over
// the rows of each head and the SF / LG / INF scores.
#include <hip/hip_runtime.h>

#include <cmath>
#include <mutex>

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
__device__ __forceinline__ void row_cells_impl(const float* __restrict__ W, int32_t n, int32_t needle_start,
                                               int32_t needle_len, int32_t topk, double* __restrict__ c_out) {
  constexpr int NT = kS1Threads;
  __shared__ uint32_t hist[kHistBins];
  __shared__ uint32_t sh_scan[NT / 64];
  __shared__ uint32_t res[2];
  __shared__ double sh_d[NT / 64];
  __shared__ uint32_t sh_u[NT / 64];

  const int tid = threadIdx.x;
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
        double* c = c_out;
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
    double* c = c_out;
    c[0] = WO;
    c[1] = WD;
    c[2] = WS;
    c[3] = tot - WO - WD - WS;
  }
}

template <bool RESIDENT>
__global__ __launch_bounds__(kS1Threads, 4) void row_cells_kernel(const float* __restrict__ rows, int32_t n,
                                                                  int32_t needle_start, int32_t needle_len, int32_t topk,
                                                                  double* __restrict__ cells) {
  row_cells_impl<RESIDENT>(rows + (int64_t)blockIdx.x * n, n, needle_start, needle_len, topk, cells + (int64_t)blockIdx.x * 4);
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

// ------------------------------------------------------------------------------------------
// Stage 1 straight from the decode queries and the context keys (Section 3.1, Eq. 2-4 feeding
// Algorithm 1): the attention rows are never written anywhere.  One workgroup owns 64 query rows
// of one KV head (the T decode steps of its G query heads) and all n keys.
//
// With 64 rows per key the work is bound by reading the keys (64 flop per byte), so the kernel is
// built as a stream: each of the 8 waves takes every 8th sub-tile of 32 keys, loads it straight
// from memory into the operand registers of the 32x32x16 bf16 MFMA (a lane: 16 bytes of one key
// row per load; nothing is staged in LDS and the waves never wait for each other inside a chunk),
// keeps two sub-tiles in flight, and multiplies it with both 32-row tiles of the queries, which
// stay in registers.  A lane owns two query rows (one per row tile) and, per sub-tile, 16 keys of
// each: it keeps the running softmax statistics and the needle mass of its rows.
// Logits at or above the row's bound are appended to the row's candidate list in LDS.  The keys
// are cut into chunks: the first kQkFirst keys, then chunks half as long as everything before
// them.  After every chunk the waves meet, the bound of a row becomes the K-th largest entry of
// its list (the K-th largest logit so far, resolved to its leading bits) and the list is cut back
// to the entries at or above it; since a chunk holds at most half as many keys as came before, about K/2 new entries
// join the K carried ones.  Only the first chunk, which has no bound to start from, is walked
// twice: its first walk tracks 8 running maxima per lane and row, the 16 lanes of a row give 128
// maxima of disjoint key subsets, and their K-th largest is a lower bound of the row's K-th
// largest logit; its second walk collects.  So the keys are read 1 + kQkFirst/n times.
// At the end a wave per row ranks its candidates exactly (larger logit first, equal logits by
// lower position), turns the K winners into weights with the row's log-sum-exp and splits them
// into WO / WD by needle membership.  A row whose list overflows (many equal logits at the top,
// or logits that keep rising along the context) is flagged and redone by qk_fallback_kernel.
constexpr int kQkThreads = 512;      // 8 waves
constexpr int kQkWaves = kQkThreads / 64;
constexpr int kQkRows = 64;          // two row tiles of 32
constexpr int kQkStripe = 32 * kQkWaves;   // keys the waves take together: chunk ends are multiples of it
constexpr int kQkFirst = 4 * kQkStripe;    // keys of the first chunk
constexpr int kQkSubsets = kQkWaves * 2 * 8;    // key subsets per row whose maxima are tracked in the first walk
constexpr int kQkCand = 128;
constexpr int kQkBoundBits = 18;     // leading key bits that the bound of a row is resolved to between chunks
constexpr int kQkFallbackWGs = 128;

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 qk_bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float qk_f32x16;
typedef uint32_t qk_u32x4 __attribute__((ext_vector_type(4)));
union QkPack16 {
  qk_u32x4 u;
  qk_bf16x8 b;
};

template <int DK>
struct QkLds {
  float cand_x[kQkRows][kQkCand];                           // first walk: the subset maxima [row][(wave, half, i)]
  int32_t cand_p[kQkRows][kQkCand];
  float st_m[kQkRows][2 * kQkWaves], st_s[kQkRows][2 * kQkWaves], st_t[kQkRows][2 * kQkWaves];
  float bound[kQkRows];
  uint32_t cnt[kQkRows];
  uint32_t ovf[kQkRows];
};

__device__ __forceinline__ float key_to_float(uint32_t key) {
  return __uint_as_float((key & 0x80000000u) ? (key ^ 0x80000000u) : ~key);
}
// a key whose low bits were cleared, as a bound: a value at or below the one the key came from
// (a truncated key of -inf reads as a NaN pattern: -inf then)
__device__ __forceinline__ float bound_from_key(uint32_t key) {
  const float f = key_to_float(key);
  return f != f ? -INFINITY : f;
}

template <int DK>
__global__ __launch_bounds__(kQkThreads) void qk_cells_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ kmat,
                                                                 int Hq, int Hkv, int T, int n, int rowgroups,
                                                                 int needle_start, int needle_len, int topk, float c_log2,
                                                                 double* __restrict__ cells, unsigned char* __restrict__ overflow) {
  constexpr int KK = DK / 16;
  extern __shared__ __attribute__((aligned(16))) unsigned char qk_smem[];
  QkLds<DK>& S = *reinterpret_cast<QkLds<DK>*>(qk_smem);

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  static_assert(sizeof(float) * kQkSubsets <= sizeof(S.cand_x[0]) + sizeof(S.cand_p[0]) &&
                    offsetof(QkLds<DK>, cand_p) == sizeof(S.cand_x),
                "the subset maxima of the first walk live in the (still empty) candidate lists");
  static_assert(kQkSubsets == 128 && kQkCand == 128 && kQkRows % kQkWaves == 0, "eight lanes hold the maxima / candidates of a row, 16 each");
  float (*mxl)[kQkSubsets] = reinterpret_cast<float (*)[kQkSubsets]>(&S.cand_x[0][0]);
  constexpr int RPW = kQkRows / kQkWaves;            // rows a wave looks after between the chunks
  const int G = Hq / Hkv, R = G * T;
  const int rg = blockIdx.x % rowgroups, seg = blockIdx.x / rowgroups;   // seg = l * Hkv + kvh
  const int l = seg / Hkv, kvh = seg % Hkv;
  const int row0 = rg * kQkRows;
  const int nrows = min(kQkRows, R - row0);
  const int64_t rowid0 = ((int64_t)l * Hq + (int64_t)kvh * G) * T + row0;   // first global row of this workgroup
  const uint16_t* qbase = q + rowid0 * DK;
  const unsigned char* kbase = reinterpret_cast<const unsigned char*>(kmat + (int64_t)seg * n * DK);
  const int ne = needle_start + needle_len;

  for (int i = tid; i < kQkRows; i += kQkThreads) {
    S.cnt[i] = 0;
    S.ovf[i] = 0;
    S.bound[i] = INFINITY;
  }
  // this lane's rows inside the workgroup: l32 and 32 + l32
  qk_bf16x8 qreg[2][KK];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      QkPack16 p;
      p.u = *reinterpret_cast<const qk_u32x4*>(qbase + (int64_t)min(mt * 32 + l32, nrows - 1) * DK + kk * 16 + half * 8);
      qreg[mt][kk] = p.b;
    }
  float m_run[2] = {-INFINITY, -INFINITY}, s_run[2] = {0.f, 0.f}, t_run[2] = {0.f, 0.f};   // running maximum, sum of exp2(x - max), the same over the needle
  float bound[2] = {INFINITY, INFINITY}, bound_raw[2] = {INFINITY, INFINITY};
  __syncthreads();

  // one sub-tile of 32 keys starting at key_s: 16 bytes of key row (key_s + l32) per load (clamped at the end of the keys)
  auto issue = [&](int key_s, qk_u32x4 (&kf)[KK]) __attribute__((always_inline)) {
    const uint32_t off = (uint32_t)min(key_s + l32, n - 1) * (uint32_t)(DK * 2) + (uint32_t)half * 16u;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) kf[kk] = *reinterpret_cast<const qk_u32x4*>(kbase + (off + (uint32_t)kk * 32u));
  };
  // MFMAs of one sub-tile against both row tiles: acc[mt][i] = q(row mt*32 + l32) . k(key_s + 8*(i/4) + 4*half + i%4),
  // not yet scaled by log2(e)/sqrt(d)
  auto mfma_sub = [&](const qk_u32x4 (&kf)[KK], qk_f32x16 (&acc)[2]) __attribute__((always_inline)) {
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      QkPack16 p;
      p.u = kf[kk];
      if (kk == 0) {
        qk_f32x16 z;
#pragma unroll
        for (int i = 0; i < 16; ++i) z[i] = 0.f;
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p.b, qreg[0][kk], z, 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p.b, qreg[1][kk], z, 0, 0, 0);
      } else {
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p.b, qreg[0][kk], acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(p.b, qreg[1][kk], acc[1], 0, 0, 0);
      }
    }
  };
  // the last sub-tile of the keys: what lies beyond them counts as -inf
  auto mask_sub = [&](int key_s, qk_f32x16 (&acc)[2]) __attribute__((always_inline)) {
    if (key_s + 32 > n) {
      const int key0 = key_s + 4 * half;
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (key0 + 8 * (i >> 2) + (i & 3) >= n) acc[mt][i] = -INFINITY;
    }
  };
  // softmax statistics of the 16 unscaled logits a of row tile mt; returns their maximum.  Straight-line
  // code (it is scheduled among the MFMAs of the next sub-tile); the needle mass of the few sub-tiles
  // that touch the needle is added by needle_mass() afterwards.
  auto stats = [&](int mt, const qk_f32x16& a) __attribute__((always_inline)) {
    float mxr = fmaxf(a[0], a[1]);
#pragma unroll
    for (int i = 2; i < 16; i += 2) mxr = fmaxf(mxr, fmaxf(a[i], a[i + 1]));
    const float mn = fmaxf(m_run[mt], mxr * c_log2);
    const float mu = mn == -INFINITY ? 0.f : mn;
    const float scale = __builtin_amdgcn_exp2f(m_run[mt] - mu);
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) sum += __builtin_amdgcn_exp2f(fmaf(a[i], c_log2, -mu));
    s_run[mt] = s_run[mt] * scale + sum;
    t_run[mt] = t_run[mt] * scale;
    m_run[mt] = mn;
    return mxr;
  };
  // after stats(): the weights of the sub-tile's needle keys, against the same (updated) reference
  auto needle_mass = [&](int mt, int key0, const qk_f32x16& a) __attribute__((always_inline)) {
    if (key0 + 32 > needle_start && key0 < ne) {
      const float mu = m_run[mt] == -INFINITY ? 0.f : m_run[mt];
      float tsum = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = key0 + 8 * (i >> 2) + (i & 3);
        if (key >= needle_start && key < ne) tsum += __builtin_amdgcn_exp2f(fmaf(a[i], c_log2, -mu));
      }
      t_run[mt] += tsum;
    }
  };
  // the logits at or above the bound join the row's list (mxr: the largest unscaled logit of the 16;
  // bound_raw: the bound in unscaled units, rounded down, so the first test never misses one)
  auto collect = [&](int mt, int key0, const qk_f32x16& a, float mxr) __attribute__((always_inline)) {
    if (mxr >= bound_raw[mt]) {
      const int r = mt * 32 + l32;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float x = a[i] * c_log2;
        if (x >= bound[mt]) {
          const uint32_t slot = atomicAdd(&S.cnt[r], 1u);
          if (slot < (uint32_t)kQkCand) {
            S.cand_x[r][slot] = x;
            S.cand_p[r][slot] = key0 + 8 * (i >> 2) + (i & 3);
          }
        }
      }
    }
  };
  // This wave's sub-tiles of [key_lo, key_hi) (multiples of kQkStripe, key_hi clipped to n) as a
  // software pipeline: the MFMAs of a sub-tile are issued among the statistics of the sub-tile
  // before it (the two sets of accumulators alternate), and the loads of the sub-tile after it are
  // in flight.  front(mt, key0, a) runs inside that mix and returns a value that back(mt, key0, a, v)
  // receives afterwards (back may branch).
  // (preloaded: the wave's first sub-tile is already on its way into kfA, requested by prefetch())
  qk_u32x4 kfA[KK], kfB[KK];
  auto prefetch = [&](int key_lo, int key_hi) __attribute__((always_inline)) {
    if (key_lo + wv * 32 < key_hi) issue(key_lo + wv * 32, kfA);
  };
  auto walk = [&](int key_lo, int key_hi, bool preloaded, auto front, auto back) __attribute__((always_inline)) {
    int ks = key_lo + wv * 32;
    if (ks >= key_hi) return;
    if (!preloaded) issue(ks, kfA);
    qk_f32x16 accA[2], accB[2];
    if (ks + kQkStripe < key_hi) issue(ks + kQkStripe, kfB);
    mfma_sub(kfA, accA);
    // one pipelined step: the sub-tile at ks is in `cur`; the next one goes from kn into `nxt`, and kc is refilled
    auto pstep = [&](qk_f32x16 (&cur)[2], qk_f32x16 (&nxt)[2], qk_u32x4 (&kc)[KK], qk_u32x4 (&kn)[KK]) __attribute__((always_inline)) {
      const int key0 = ks + 4 * half;
      float v[2];
      // kc held the current sub-tile, whose MFMAs have been issued: refill it with the sub-tile after the next
      if (ks + 2 * kQkStripe < key_hi) issue(ks + 2 * kQkStripe, kc);
      mfma_sub(kn, nxt);
      v[0] = front(0, key0, cur[0]);
      v[1] = front(1, key0, cur[1]);
#pragma unroll
      for (int g = 0; g < 2 * KK; ++g) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
        __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);   // eight vector instructions of the statistics
      }
      // the statistics are complete here (they must not sink below the branches that follow)
      asm volatile("" ::"v"(v[0]), "v"(v[1]), "v"(s_run[0]), "v"(s_run[1]), "v"(m_run[0]), "v"(m_run[1]));
      back(0, key0, cur[0], v[0]);
      back(1, key0, cur[1], v[1]);
      ks += kQkStripe;
    };
    // the wave's last sub-tile of the walk (the only one that can reach past the end of the keys)
    auto last = [&](qk_f32x16 (&cur)[2]) __attribute__((always_inline)) {
      const int key0 = ks + 4 * half;
      mask_sub(ks, cur);
      const float v0 = front(0, key0, cur[0]), v1 = front(1, key0, cur[1]);
      back(0, key0, cur[0], v0);
      back(1, key0, cur[1], v1);
    };
    int rem = (key_hi - ks + kQkStripe - 1) / kQkStripe;   // sub-tiles of this wave still to finish (>= 1); the current one is in accA
    while (rem >= 3) {
      pstep(accA, accB, kfA, kfB);
      pstep(accB, accA, kfB, kfA);
      rem -= 2;
    }
    if (rem == 2) {
      pstep(accA, accB, kfA, kfB);
      last(accB);
    } else {
      last(accA);
    }
  };
  // Bounds of the wave's RPW = 8 rows at once: 8 lanes per row, NE keys per lane (0 = no entry).
  // Bisection on the leading kQkBoundBits bits of the keys: the result (the same in the 8 lanes
  // of a row) is the largest value with the remaining bits clear that at least K keys reach, so
  // it lies at or below the K-th largest key and within 2^-(kQkBoundBits - 9) of it (relative, in
  // the logit).  All on the vector unit: no lane-mask round trips through scalar registers.
  auto group_kth = [&](auto& keys, auto ne_c) __attribute__((always_inline)) {
    constexpr int NE = decltype(ne_c)::value;
    uint32_t tkey = 0;
#pragma unroll 1
    for (int b = 31; b >= 32 - kQkBoundBits; --b) {
      const uint32_t trial = tkey | (1u << b);
      uint32_t c = 0;
#pragma unroll
      for (int j = 0; j < NE; ++j) c += keys[j] >= trial ? 1u : 0u;
      // sum over the 8 lanes of the row: neighbours in the quad, then the other quad (DPP, no LDS crossbar)
      c += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)c, 0xB1, 0xF, 0xF, false);    // quad_perm [1,0,3,2]
      c += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)c, 0x4E, 0xF, 0xF, false);    // quad_perm [2,3,0,1]
      c += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)c, 0x141, 0xF, 0xF, false);   // row_half_mirror
      if (c >= (uint32_t)topk) tkey = trial;
    }
    return tkey;
  };
  // A wave sets the new bound nb of row rr and drops the list entries below it (an overflowed
  // list sends the row to the fallback).
  auto refilter = [&](int rr, float nb) __attribute__((always_inline)) {
    const uint32_t c = S.cnt[rr];
    if (c > (uint32_t)kQkCand) {
      if (lane == 0) {
        S.ovf[rr] = 1;
        S.cnt[rr] = 0;
        S.bound[rr] = INFINITY;
      }
    } else {
      const float x0 = lane < (int)c ? S.cand_x[rr][lane] : -INFINITY, x1 = lane + 64 < (int)c ? S.cand_x[rr][lane + 64] : -INFINITY;
      const int32_t p0 = S.cand_p[rr][lane], p1 = S.cand_p[rr][lane + 64];
      const bool k0 = lane < (int)c && x0 >= nb, k1 = lane + 64 < (int)c && x1 >= nb;
      const unsigned long long m0 = __ballot(k0), m1 = __ballot(k1);
      const uint32_t n0 = (uint32_t)__popcll(m0);
      const uint32_t lb0 = __builtin_amdgcn_mbcnt_hi((uint32_t)(m0 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m0, 0u));
      const uint32_t lb1 = __builtin_amdgcn_mbcnt_hi((uint32_t)(m1 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m1, 0u));
      if (k0) {
        S.cand_x[rr][lb0] = x0;
        S.cand_p[rr][lb0] = p0;
      }
      if (k1) {
        S.cand_x[rr][n0 + lb1] = x1;
        S.cand_p[rr][n0 + lb1] = p1;
      }
      if (lane == 0) {
        S.cnt[rr] = n0 + (uint32_t)__popcll(m1);
        if (!S.ovf[rr]) S.bound[rr] = nb;
      }
    }
  };

  // this lane's bounds from the rows' bounds in LDS; the unscaled form is lowered by a few ulps so
  // that a logit whose scaled value reaches the bound never fails the first test
  auto load_bounds = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      bound[mt] = mt * 32 + l32 < nrows ? S.bound[mt * 32 + l32] : INFINITY;
      const float raw = bound[mt] / c_log2;
      bound_raw[mt] = fabsf(raw) == INFINITY ? raw : raw - fabsf(raw) * 4.8e-7f;
    }
  };
  auto no_front = [&](int, int, const qk_f32x16&) __attribute__((always_inline)) { return 0.f; };

  int c_lo = 0, c_hi = min(n, kQkFirst);
  {
    // The first chunk, first walk: statistics and 8 running maxima (of pairs of keys) per lane and row
    float mxs[2][8];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int i = 0; i < 8; ++i) mxs[mt][i] = -INFINITY;
    walk(c_lo, c_hi, false,
         [&](int mt, int, const qk_f32x16& a) __attribute__((always_inline)) { return stats(mt, a); },
         [&](int mt, int key0, const qk_f32x16& a, float) __attribute__((always_inline)) {
           needle_mass(mt, key0, a);
#pragma unroll
           for (int i = 0; i < 8; ++i) mxs[mt][i] = fmaxf(mxs[mt][i], fmaxf(a[2 * i], a[2 * i + 1]));
         });
    prefetch(c_lo, c_hi);                             // the second walk starts where the first did
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int i = 0; i < 8; ++i) mxl[mt * 32 + l32][(wv * 2 + half) * 8 + i] = mxs[mt][i] * c_log2;
    __syncthreads();
    const int grow = wv * RPW + (lane >> 3), gl = lane & 7;   // between chunks: 8 lanes look after one row
    float nb0;
    {
      uint32_t keys[kQkSubsets / 8];
#pragma unroll
      for (int j = 0; j < kQkSubsets / 8; ++j) keys[j] = float_key(mxl[grow][gl + 8 * j]);
      nb0 = grow < nrows ? bound_from_key(group_kth(keys, std::integral_constant<int, kQkSubsets / 8>{})) : INFINITY;
    }
    __syncthreads();                                  // the maxima have been read: the lists may fill
    if (gl == 0) S.bound[grow] = nb0;
    __syncthreads();
    load_bounds();
    // second walk: collect
    walk(c_lo, c_hi, true, no_front,
         [&](int mt, int key0, const qk_f32x16& a, float) __attribute__((always_inline)) {
           float mxr = fmaxf(a[0], a[1]);
#pragma unroll
           for (int i = 2; i < 16; i += 2) mxr = fmaxf(mxr, fmaxf(a[i], a[i + 1]));
           collect(mt, key0, a, mxr);
         });
  }
  for (;;) {
    // the next chunk: at most half as many keys as came before, in whole stripes; its first
    // sub-tile is requested before the waves meet
    const int n_lo = c_hi, n_hi = min(n, n_lo + max(kQkStripe, n_lo / 2 / kQkStripe * kQkStripe));
    if (n_lo < n) prefetch(n_lo, n_hi);
    // every list now holds all logits so far that are at or above the row's bound, hence the K
    // largest: their K-th largest is the new bound, and the entries below it are dropped
    __syncthreads();
    {
      const int grow = wv * RPW + (lane >> 3), gl = lane & 7;
      const uint32_t c = min(S.cnt[grow], (uint32_t)kQkCand);
      uint32_t keys[kQkCand / 8];
#pragma unroll
      for (int j = 0; j < kQkCand / 8; ++j) keys[j] = gl + 8 * j < (int)c ? float_key(S.cand_x[grow][gl + 8 * j]) : 0u;
      const uint32_t tkey = group_kth(keys, std::integral_constant<int, kQkCand / 8>{});
      // (a list shorter than K cannot happen for a row of finite logits; -inf keeps everything)
      const float nbg = grow < nrows ? (c >= (uint32_t)topk ? bound_from_key(tkey) : -INFINITY) : INFINITY;
      for (int j = 0; j < RPW; ++j) refilter(wv * RPW + j, __shfl(nbg, 8 * j, 64));
    }
    __syncthreads();
    if (c_hi >= n) break;
    load_bounds();
    c_lo = n_lo;
    c_hi = n_hi;
    walk(c_lo, c_hi, true,
         [&](int mt, int, const qk_f32x16& a) __attribute__((always_inline)) { return stats(mt, a); },
         [&](int mt, int key0, const qk_f32x16& a, float mxr) __attribute__((always_inline)) {
           needle_mass(mt, key0, a);
           collect(mt, key0, a, mxr);
         });
  }

  // statistics of a row: its 16 lanes -> log-sum-exp and needle mass
#pragma unroll
  for (int mt = 0; mt < 2; ++mt) {
    S.st_m[mt * 32 + l32][wv * 2 + half] = m_run[mt];
    S.st_s[mt * 32 + l32][wv * 2 + half] = s_run[mt];
    S.st_t[mt * 32 + l32][wv * 2 + half] = t_run[mt];
  }
  __syncthreads();
  for (int rr = wv * RPW; rr < min(wv * RPW + RPW, nrows); ++rr) {
    float M = S.st_m[rr][0];
#pragma unroll
    for (int j = 1; j < 2 * kQkWaves; ++j) M = fmaxf(M, S.st_m[rr][j]);
    float ssum = 0.f, tsum = 0.f;
#pragma unroll
    for (int j = 0; j < 2 * kQkWaves; ++j) {
      const float f = __builtin_amdgcn_exp2f(S.st_m[rr][j] - M);
      ssum += S.st_s[rr][j] * f;
      tsum += S.st_t[rr][j] * f;
    }
    const float lse = M + log2f(ssum);
    const double tnw = (double)tsum / (double)ssum;
    const uint32_t c = S.cnt[rr];
    const bool over = S.ovf[rr] || c > (uint32_t)kQkCand;
    if (lane == 0) overflow[rowid0 + rr] = over ? 1 : 0;
    if (over) continue;
    // exact rank of the candidates: larger logit first, equal logits by lower position
    const float x0 = lane < (int)c ? S.cand_x[rr][lane] : -INFINITY, x1 = lane + 64 < (int)c ? S.cand_x[rr][lane + 64] : -INFINITY;
    const int32_t p0 = S.cand_p[rr][lane], p1 = S.cand_p[rr][lane + 64];
    uint32_t a0 = 0, a1 = 0;
    for (uint32_t j = 0; j < c; ++j) {
      const float xj = S.cand_x[rr][j];
      const int32_t pj = S.cand_p[rr][j];
      a0 += (xj > x0 || (xj == x0 && pj < p0)) ? 1u : 0u;
      a1 += (xj > x1 || (xj == x1 && pj < p1)) ? 1u : 0u;
    }
    double wo = 0.0, wd = 0.0;
    if (lane < (int)c && a0 < (uint32_t)topk) {
      const double wgt = (double)__builtin_amdgcn_exp2f(x0 - lse);
      if (p0 >= needle_start && p0 < ne) wo += wgt; else wd += wgt;
    }
    if (lane + 64 < (int)c && a1 < (uint32_t)topk) {
      const double wgt = (double)__builtin_amdgcn_exp2f(x1 - lse);
      if (p1 >= needle_start && p1 < ne) wo += wgt; else wd += wgt;
    }
    wo = wave_sum<double>(wo);
    wd = wave_sum<double>(wd);
    if (lane == 0) {
      const double WS = fmax(0.0, tnw - wo);
      double* cdst = cells + (rowid0 + rr) * 4;
      cdst[0] = wo;
      cdst[1] = wd;
      cdst[2] = WS;
      cdst[3] = 1.0 - wo - wd - WS;                  // a softmax row sums to one
    }
  }
}

// Rows flagged by qk_cells_kernel: the row's weights are written to this workgroup's slot of the
// workspace (plain dot products, softmax in three sweeps) and go through the general path of the
// row kernel, which handles any number of equal weights.
template <int DK>
__global__ __launch_bounds__(kS1Threads) void qk_fallback_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ kmat,
                                                                 int Hq, int Hkv, int T, int n, int64_t nrows_total,
                                                                 int needle_start, int needle_len, int topk, float c_log2,
                                                                 const unsigned char* __restrict__ overflow, float* __restrict__ slots,
                                                                 double* __restrict__ cells) {
  __shared__ float qs[DK];
  __shared__ float red[kS1Threads / 64];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int G = Hq / Hkv;
  float* W = slots + (int64_t)blockIdx.x * n;
  auto block_max = [&](float v) {
#pragma unroll
    for (int dlt = 32; dlt > 0; dlt >>= 1) v = fmaxf(v, __shfl_xor(v, dlt, 64));
    __syncthreads();
    if (lane == 0) red[wv] = v;
    __syncthreads();
    float o = red[0];
    for (int i = 1; i < kS1Threads / 64; ++i) o = fmaxf(o, red[i]);
    return o;
  };
  auto block_add = [&](float v) {
    v = wave_sum<float>(v);
    __syncthreads();
    if (lane == 0) red[wv] = v;
    __syncthreads();
    float o = red[0];
    for (int i = 1; i < kS1Threads / 64; ++i) o += red[i];
    return o;
  };
  // rows blockIdx.x, blockIdx.x + gridDim.x, ... are this workgroup's; their flags are read 256 at a time
  __shared__ int64_t todo[kS1Threads];
  __shared__ uint32_t ntodo;
  for (int64_t base = blockIdx.x; base < nrows_total; base += (int64_t)gridDim.x * kS1Threads) {
    __syncthreads();
    if (tid == 0) ntodo = 0;
    __syncthreads();
    const int64_t mine = base + (int64_t)tid * gridDim.x;
    if (mine < nrows_total && overflow[mine]) todo[atomicAdd(&ntodo, 1u)] = mine;
    __syncthreads();
    const uint32_t cnt = ntodo;
  for (uint32_t it = 0; it < cnt; ++it) {
    const int64_t row = todo[it];
    const int64_t hq_l = row / T;                     // l * Hq + hq
    const int l = (int)(hq_l / Hq), hq = (int)(hq_l % Hq);
    const uint16_t* kb = kmat + ((int64_t)l * Hkv + hq / G) * n * DK;
    __syncthreads();
    for (int p = tid; p < DK; p += kS1Threads) qs[p] = __uint_as_float((uint32_t)q[row * DK + p] << 16);
    __syncthreads();
    float mx = -INFINITY;
    for (int j = tid; j < n; j += kS1Threads) {
      float acc = 0.f;
      for (int p = 0; p < DK; p += 2) {
        const uint32_t pr = *reinterpret_cast<const uint32_t*>(kb + (int64_t)j * DK + p);
        acc = fmaf(qs[p], __uint_as_float(pr << 16), acc);
        acc = fmaf(qs[p + 1], __uint_as_float(pr & 0xffff0000u), acc);
      }
      const float x = acc * c_log2;
      W[j] = x;
      mx = fmaxf(mx, x);
    }
    mx = block_max(mx);
    float sum = 0.f;
    for (int j = tid; j < n; j += kS1Threads) {
      const float e = __builtin_amdgcn_exp2f(W[j] - mx);
      W[j] = e;
      sum += e;
    }
    sum = block_add(sum);
    const float inv = 1.f / sum;
    for (int j = tid; j < n; j += kS1Threads) W[j] *= inv;
    __threadfence_block();
    __syncthreads();
    row_cells_impl<false>(W, n, needle_start, needle_len, topk, cells + row * 4);
    __syncthreads();
  }
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

// ------------------------------------------------------------------ Stage 1 from queries and keys

namespace {

struct QkLayout {
  size_t cells_bytes, flags_bytes, slots_bytes, off_flags, off_slots, total;
};

QkLayout qk_layout(int64_t rows, int64_t n) {
  auto align = [](size_t x) { return (x + 255) / 256 * 256; };
  QkLayout w;
  w.cells_bytes = align((size_t)rows * 4 * sizeof(double));
  w.flags_bytes = align((size_t)rows);
  w.slots_bytes = align((size_t)kQkFallbackWGs * (size_t)n * sizeof(float));
  w.off_flags = w.cells_bytes;
  w.off_slots = w.off_flags + w.flags_bytes;
  w.total = w.off_slots + w.slots_bytes;
  return w;
}

// LDS above the default limit is requested once per kernel instance and device.
template <int DK>
hipError_t qk_prepare() {
  static std::mutex mu;
  static uint64_t done = 0;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  std::lock_guard<std::mutex> lk(mu);
  const uint64_t bit = dev >= 0 && dev < 64 ? (uint64_t(1) << dev) : 0;
  if (!(done & bit)) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&qk_cells_kernel<DK>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)sizeof(QkLds<DK>));
    if (e != hipSuccess) return e;
    done |= bit;
  }
  return hipSuccess;
}

template <int DK>
slkv_status qk_launch(const uint16_t* q, const uint16_t* k, int32_t L, int32_t Hq, int32_t Hkv, int32_t T, int32_t n,
                      int32_t needle_start, int32_t needle_len, int32_t topk, double* d_acc, double* d_scores,
                      unsigned char* ws, const QkLayout& w, hipStream_t st) {
  hipError_t pe = qk_prepare<DK>();
  if (pe != hipSuccess) return fail(SLKV_ERR_HIP, "kernel set-up failed: %s", hipGetErrorString(pe));
  const int G = Hq / Hkv, R = G * T, rowgroups = (R + kQkRows - 1) / kQkRows;
  const int64_t rows = (int64_t)L * Hq * T;
  double* cells = (double*)ws;
  unsigned char* flags = ws + w.off_flags;
  float* slots = (float*)(ws + w.off_slots);
  const float c_log2 = (float)(1.4426950408889634 / std::sqrt((double)DK));
  {
    ScopedKernelTimer tm(SLKV_K_QK_CELLS, st);
    SLKV_LAUNCH(qk_cells_kernel<DK>, dim3((unsigned)(L * Hkv * rowgroups)), dim3(kQkThreads), sizeof(QkLds<DK>), st, q, k, Hq, Hkv,
                T, n, rowgroups, needle_start, needle_len, topk, c_log2, cells, flags);
  }
  {
    ScopedKernelTimer tm(SLKV_K_QK_FALLBACK, st);
    SLKV_LAUNCH(qk_fallback_kernel<DK>, dim3(kQkFallbackWGs), dim3(kS1Threads), 0, st, q, k, Hq, Hkv, T, n, rows, needle_start,
                needle_len, topk, c_log2, (const unsigned char*)flags, slots, cells);
  }
  const int heads = L * Hq;
  {
    ScopedKernelTimer tm(SLKV_K_HEAD_REDUCE, st);
    SLKV_LAUNCH(head_reduce_kernel<5>, dim3((heads + 127) / 128), dim3(128), 0, st, (const double*)cells, heads, T, d_acc,
                d_scores, 0, 1, 1, 1);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(SLKV_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(e));
  return SLKV_OK;
}

}  // namespace

extern "C" size_t slkv_score_heads_qk_workspace_bytes(int32_t L, int32_t Hq, int32_t T, int64_t n) {
  if (L < 1 || Hq < 1 || T < 1 || n < 1) return 0;
  return qk_layout((int64_t)L * Hq * T, n).total;
}

extern "C" slkv_status slkv_score_heads_qk(const void* d_q, const void* d_k, int32_t L, int32_t Hq, int32_t Hkv, int32_t T,
                                           int64_t n, int32_t d, int64_t needle_start, int32_t needle_len, int32_t topk,
                                           double* d_acc, double* d_scores, void* d_workspace, size_t workspace_bytes,
                                           void* hip_stream) {
  clear_error();
  if (!d_q || !d_k || !d_acc || !d_workspace) return fail(SLKV_ERR_NULL, "d_q, d_k, d_acc and d_workspace are required");
  if (L < 1 || Hq < 1 || Hkv < 1 || T < 1 || n < 1) return fail(SLKV_ERR_BAD_ARG, "L, Hq, Hkv, T, n must be >= 1");
  if (Hq % Hkv) return fail(SLKV_ERR_BAD_ARG, "Hq %% Hkv != 0");
  if (d != 64 && d != 128) return fail(SLKV_ERR_UNSUPPORTED, "head_dim %d (supported: 64, 128)", d);
  if (n * d * 2 >= (int64_t(1) << 31)) return fail(SLKV_ERR_UNSUPPORTED, "one head's keys span 2 GiB or more");
  const int64_t rows = (int64_t)L * Hq * T;
  if (rows >= (int64_t(1) << 31) || (int64_t)L * Hkv * (((int64_t)(Hq / Hkv) * T + kQkRows - 1) / kQkRows) >= (int64_t(1) << 31))
    return fail(SLKV_ERR_BAD_ARG, "too many rows");
  if (needle_len < 1 || needle_start < 0 || needle_start + needle_len > n)
    return fail(SLKV_ERR_BAD_ARG, "needle [%lld, +%d) outside [0, %lld)", (long long)needle_start, needle_len, (long long)n);
  if (topk < 1 || topk > n) return fail(SLKV_ERR_BAD_ARG, "topk %d outside 1..n", topk);
  if (topk > 64) return fail(SLKV_ERR_UNSUPPORTED, "topk %d > 64 (use slkv_score_heads on materialised rows)", topk);
  const void* ptrs[] = {d_q, d_k, d_acc, d_scores, d_workspace};
  for (const void* ptr : ptrs)
    if (reinterpret_cast<uintptr_t>(ptr) % 16) return fail(SLKV_ERR_BAD_ARG, "device pointer %p not 16-byte aligned", ptr);
  const QkLayout w = qk_layout(rows, n);
  if (workspace_bytes < w.total) return fail(SLKV_ERR_WORKSPACE, "workspace %zu < %zu bytes", workspace_bytes, w.total);
  hipStream_t st = (hipStream_t)hip_stream;
  if (d == 128)
    return qk_launch<128>((const uint16_t*)d_q, (const uint16_t*)d_k, L, Hq, Hkv, T, (int32_t)n, (int32_t)needle_start, needle_len,
                          topk, d_acc, d_scores, (unsigned char*)d_workspace, w, st);
  return qk_launch<64>((const uint16_t*)d_q, (const uint16_t*)d_k, L, Hq, Hkv, T, (int32_t)n, (int32_t)needle_start, needle_len, topk,
                       d_acc, d_scores, (unsigned char*)d_workspace, w, st);
}
