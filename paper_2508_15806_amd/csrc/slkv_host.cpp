// Host-only part of libslkv: status strings, error detail, budget allocation (Eq. 6 /
// Algorithm 2) and the size helpers.  No GPU call is made from this file.
#include "slkv_internal.h"

#include <algorithm>
#include <climits>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

namespace {
thread_local char g_err[512] = "";
}

namespace slkv {

slkv_status fail(slkv_status s, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return s;
}

void clear_error() { g_err[0] = '\0'; }

int64_t kept_rows(int64_t n, int64_t w, int64_t cap) {
  // Algorithm 3: a segment no longer than its capacity (or than the window) is kept whole;
  // otherwise C - w history rows (not below zero) plus the window.
  if (n <= w || n <= cap) return n;
  return std::max<int64_t>(cap, w);
}

// Checks of the shape parameters the two descriptors share.
static slkv_status validate_shape(int32_t dtype, int32_t B, int32_t Hq, int32_t Hkv, int32_t dd, int32_t w,
                                  int32_t pool_kernel, int32_t pool, int32_t reserved, const int32_t* h_budgets) {
  if (dtype != SLKV_F32 && dtype != SLKV_BF16 && dtype != SLKV_F16 && dtype != SLKV_BF16_KV_FP8) return fail(SLKV_ERR_BAD_ARG, "unknown dtype %d", dtype);
  if (B < 1 || Hq < 1 || Hkv < 1 || w < 1) return fail(SLKV_ERR_BAD_ARG, "B, Hq, Hkv, w must be >= 1");
  if (B > (1 << 20) || Hkv > (1 << 16) || Hq > (1 << 16)) return fail(SLKV_ERR_BAD_ARG, "B, Hq or Hkv too large");
  if (Hq % Hkv) return fail(SLKV_ERR_BAD_ARG, "Hq %% Hkv != 0");
  if (dd != 64 && dd != 128) return fail(SLKV_ERR_UNSUPPORTED, "head_dim %d (supported: 64, 128)", dd);
  int64_t rows = (int64_t)(Hq / Hkv) * w;
  if (rows > kMaxRows) return fail(SLKV_ERR_UNSUPPORTED, "(Hq/Hkv)*w = %lld rows > %d", (long long)rows, kMaxRows);
  if (pool != SLKV_POOL_NONE && pool != SLKV_POOL_MAX && pool != SLKV_POOL_AVG)
    return fail(SLKV_ERR_BAD_ARG, "unknown pool mode %d", pool);
  if (pool_kernel < 1 || pool_kernel > kMaxPool || pool_kernel % 2 == 0)
    return fail(SLKV_ERR_BAD_ARG, "pool_kernel %d must be odd and in 1..%d", pool_kernel, kMaxPool);
  if (reserved != 0) return fail(SLKV_ERR_BAD_ARG, "desc.reserved must be 0");
  if (!h_budgets) return fail(SLKV_ERR_NULL, "h_budgets is NULL");
  for (int h = 0; h < Hkv; ++h)
    if (h_budgets[h] < 0) return fail(SLKV_ERR_BAD_ARG, "budget[%d] < 0", h);
  return SLKV_OK;
}

slkv_status validate_desc(const slkv_layer_desc* d) {
  if (!d) return fail(SLKV_ERR_NULL, "desc is NULL");
  if (d->struct_size != sizeof(slkv_layer_desc))
    return fail(SLKV_ERR_BAD_ARG, "desc.struct_size %u != %zu", d->struct_size, sizeof(slkv_layer_desc));
  slkv_status st = validate_shape(d->dtype, d->B, d->Hq, d->Hkv, d->d, d->w, d->pool_kernel, d->pool, d->reserved,
                                  d->h_budgets);
  if (st != SLKV_OK) return st;
  if (!d->h_cu_seqlens) return fail(SLKV_ERR_NULL, "h_cu_seqlens is NULL");
  if (d->h_cu_seqlens[0] < 0) return fail(SLKV_ERR_BAD_ARG, "cu_seqlens[0] < 0");
  for (int b = 0; b < d->B; ++b)
    if (d->h_cu_seqlens[b + 1] < d->h_cu_seqlens[b]) return fail(SLKV_ERR_BAD_ARG, "cu_seqlens not monotone at %d", b);
  if (d->h_cu_seqlens[d->B] >= (int64_t(1) << 31)) return fail(SLKV_ERR_BAD_ARG, "cu_seqlens[B] >= 2^31");
  const int64_t strides[4] = {d->k_stride_tok, d->k_stride_head, d->v_stride_tok, d->v_stride_head};
  const int64_t align_elems = d->dtype == SLKV_F32 ? 4 : (d->dtype == SLKV_BF16_KV_FP8 ? 16 : 8);   // 16 bytes
  for (int i = 0; i < 4; ++i) {
    if (strides[i] < 0 || strides[i] % align_elems) return fail(SLKV_ERR_BAD_ARG, "stride %d not a non-negative multiple of %lld elements", i, (long long)align_elems);
  }
  if (d->k_stride_tok < d->d || d->v_stride_tok < d->d) return fail(SLKV_ERR_BAD_ARG, "token stride < head_dim");
  int64_t total = (int64_t)d->Hkv * d->h_cu_seqlens[d->B];
  if (total >= (int64_t(1) << 31)) return fail(SLKV_ERR_BAD_ARG, "Hkv * tokens >= 2^31");
  return SLKV_OK;
}

slkv_status validate_ragged_desc(const slkv_ragged_desc* d) {
  if (!d) return fail(SLKV_ERR_NULL, "desc is NULL");
  if (d->struct_size != sizeof(slkv_ragged_desc))
    return fail(SLKV_ERR_BAD_ARG, "desc.struct_size %u != %zu", d->struct_size, sizeof(slkv_ragged_desc));
  slkv_status st = validate_shape(d->dtype, d->B, d->Hq, d->Hkv, d->d, d->w, d->pool_kernel, d->pool, d->reserved,
                                  d->h_budgets);
  if (st != SLKV_OK) return st;
  if (!d->h_in_offsets) return fail(SLKV_ERR_NULL, "h_in_offsets is NULL");
  if (d->h_in_offsets[0] < 0) return fail(SLKV_ERR_BAD_ARG, "in_offsets[0] < 0");
  const int64_t S = (int64_t)d->B * d->Hkv;
  for (int64_t s = 0; s < S; ++s)
    if (d->h_in_offsets[s + 1] < d->h_in_offsets[s]) return fail(SLKV_ERR_BAD_ARG, "in_offsets not monotone at %lld", (long long)s);
  if (d->h_in_offsets[S] >= (int64_t(1) << 31)) return fail(SLKV_ERR_BAD_ARG, "in_offsets[B*Hkv] >= 2^31");
  return SLKV_OK;
}

}  // namespace slkv

using namespace slkv;

extern "C" {

const char* slkv_status_str(slkv_status s) {
  switch (s) {
    case SLKV_OK: return "ok";
    case SLKV_ERR_NULL: return "null pointer";
    case SLKV_ERR_BAD_ARG: return "bad argument";
    case SLKV_ERR_BAD_VALUE: return "bad value";
    case SLKV_ERR_UNSUPPORTED: return "unsupported configuration";
    case SLKV_ERR_WORKSPACE: return "workspace too small";
    case SLKV_ERR_CAPACITY: return "output capacity too small";
    case SLKV_ERR_HIP: return "HIP error";
  }
  return "unknown status";
}

const char* slkv_last_error(void) { return g_err; }

int32_t slkv_version(void) { return 1005; }

int32_t slkv_fixed_from_beta(int32_t avg_budget, double beta) {
  if (avg_budget < 0 || !(beta >= 1.0)) return -1;
  return (int32_t)std::floor((double)avg_budget * (1.0 - 1.0 / beta) + 0.5);
}

}  // extern "C"

namespace {

typedef unsigned __int128 u128;

// Largest-remainder split of `total` over integer weights: floor of the exact quota, leftover
// units to the largest remainders, ties to the lower index.  All-zero weights count as equal.
void largest_remainder(int64_t total, const std::vector<u128>& w_in, std::vector<int64_t>& seats) {
  const size_t n = w_in.size();
  std::vector<u128> w(w_in);
  u128 wsum = 0;
  for (u128 v : w) wsum += v;
  if (wsum == 0) {
    for (auto& v : w) v = 1;
    wsum = n;
  }
  seats.assign(n, 0);
  std::vector<u128> rem(n);
  int64_t used = 0;
  for (size_t i = 0; i < n; ++i) {
    u128 prod = (u128)total * w[i];
    seats[i] = (int64_t)(prod / wsum);
    rem[i] = prod % wsum;
    used += seats[i];
  }
  int64_t left = total - used;
  std::vector<size_t> order(n);
  for (size_t i = 0; i < n; ++i) order[i] = i;
  std::stable_sort(order.begin(), order.end(), [&](size_t a, size_t b) { return rem[a] > rem[b]; });
  for (int64_t i = 0; i < left; ++i) seats[order[(size_t)i]] += 1;
}

}  // namespace

extern "C" slkv_status slkv_allocate_budgets(const double* h_inf, int32_t L, int32_t Hq, int32_t Hkv,
                                             int32_t avg_budget, int32_t fixed_budget, int32_t mode,
                                             int32_t* h_budgets) {
  clear_error();
  if (!h_inf) return fail(SLKV_ERR_NULL, "h_inf is NULL");
  if (!h_budgets) return fail(SLKV_ERR_NULL, "h_budgets is NULL");
  if (L < 1 || Hq < 1 || Hkv < 1) return fail(SLKV_ERR_BAD_ARG, "L, Hq, Hkv must be >= 1");
  if (Hq % Hkv) return fail(SLKV_ERR_BAD_ARG, "Hq %% Hkv != 0");
  if ((int64_t)L * Hkv > (1 << 20)) return fail(SLKV_ERR_BAD_ARG, "L * Hkv > 2^20");
  if (avg_budget < 0 || avg_budget > (1 << 24)) return fail(SLKV_ERR_BAD_ARG, "avg_budget outside 0..2^24");
  if (fixed_budget < 0 || fixed_budget > avg_budget) return fail(SLKV_ERR_BAD_ARG, "need 0 <= fixed <= avg");
  if (mode != SLKV_BUDGET_EXACT && mode != SLKV_BUDGET_PAPER_LITERAL && mode != SLKV_BUDGET_EXACT_PER_QUERY_HEAD)
    return fail(SLKV_ERR_BAD_ARG, "unknown mode %d", mode);
  for (int64_t i = 0; i < (int64_t)L * Hq; ++i) {
    double v = h_inf[i];
    if (!(v >= 0.0 && v <= 1.0)) return fail(SLKV_ERR_BAD_VALUE, "INF_sc[%lld] = %g outside [0,1]", (long long)i, v);
  }
  if (mode == SLKV_BUDGET_EXACT_PER_QUERY_HEAD) {
    // Algorithm 2 over the query heads (exact rule), then a KV head keeps the sum of its group
    if ((int64_t)L * Hq > (1 << 20)) return fail(SLKV_ERR_BAD_ARG, "L * Hq > 2^20");
    std::vector<int32_t> per_q((size_t)L * Hq);
    slkv_status st = slkv_allocate_budgets(h_inf, L, Hq, Hq, avg_budget, fixed_budget, SLKV_BUDGET_EXACT, per_q.data());
    if (st != SLKV_OK) return st;
    const int Gq = Hq / Hkv;
    for (int l = 0; l < L; ++l)
      for (int g = 0; g < Hkv; ++g) {
        int64_t acc = 0;
        for (int t = 0; t < Gq; ++t) acc += per_q[(size_t)l * Hq + (size_t)g * Gq + t];
        if (acc > INT32_MAX) return fail(SLKV_ERR_BAD_ARG, "capacity overflow");
        h_budgets[(size_t)l * Hkv + g] = (int32_t)acc;
      }
    return SLKV_OK;
  }
  const int G = Hq / Hkv;
  // group mean: the INF_sc of the G query heads sharing a KV head, summed left to right, / G
  std::vector<double> mean((size_t)L * Hkv);
  for (int l = 0; l < L; ++l)
    for (int g = 0; g < Hkv; ++g) {
      double acc = 0.0;
      for (int t = 0; t < G; ++t) acc = acc + h_inf[(size_t)l * Hq + (size_t)g * G + t];
      mean[(size_t)l * Hkv + g] = acc / (double)G;
    }

  if (mode == SLKV_BUDGET_PAPER_LITERAL) {
    // Algorithm 2 as printed, float64, beta = avg / (avg - fixed)
    if (avg_budget == fixed_budget) {
      for (int64_t i = 0; i < (int64_t)L * Hkv; ++i) h_budgets[i] = fixed_budget;
      return SLKV_OK;
    }
    const double b_c = (double)avg_budget;
    const double beta = b_c / (double)(avg_budget - fixed_budget);
    const double b_fixed = b_c * (1.0 - 1.0 / beta);
    const double B_total = b_c / beta * (double)L * (double)Hkv;
    std::vector<double> layer_sum(L);
    double L_s = 0.0;
    for (int l = 0; l < L; ++l) {
      double s = 0.0;
      for (int g = 0; g < Hkv; ++g) s = s + mean[(size_t)l * Hkv + g];
      layer_sum[l] = s;
    }
    for (int l = 0; l < L; ++l) L_s = L_s + layer_sum[l];
    for (int l = 0; l < L; ++l)
      for (int g = 0; g < Hkv; ++g) {
        double S = 0.0, Li = 0.0;
        if (L_s > 0.0) {
          S = mean[(size_t)l * Hkv + g] / L_s;
          Li = layer_sum[l] / L_s;
        }
        double b = b_fixed + B_total * (0.01 + Li) * S;
        h_budgets[(size_t)l * Hkv + g] = (int32_t)std::floor(std::max(0.0, b) + 0.5);
      }
    return SLKV_OK;
  }

  // EXACT: quantise to 2^-30, then two levels of largest-remainder apportionment
  std::vector<u128> x((size_t)L * Hkv);
  std::vector<u128> A(L, 0);
  u128 T = 0;
  for (int l = 0; l < L; ++l)
    for (int g = 0; g < Hkv; ++g) {
      int64_t q = (int64_t)std::floor(mean[(size_t)l * Hkv + g] * 1073741824.0 + 0.5);
      x[(size_t)l * Hkv + g] = (u128)q;
      A[l] += (u128)q;
      T += (u128)q;
    }
  const int64_t pool = (int64_t)(avg_budget - fixed_budget) * L * Hkv;
  std::vector<u128> layer_w(L);
  for (int l = 0; l < L; ++l) layer_w[l] = T > 0 ? T + 100 * A[l] : (u128)1;   // ~ 0.01 + A_l / T
  std::vector<int64_t> layer_pool, dyn;
  largest_remainder(pool, layer_w, layer_pool);
  for (int l = 0; l < L; ++l) {
    std::vector<u128> hw(x.begin() + (size_t)l * Hkv, x.begin() + (size_t)(l + 1) * Hkv);
    largest_remainder(layer_pool[l], hw, dyn);
    for (int g = 0; g < Hkv; ++g) h_budgets[(size_t)l * Hkv + g] = (int32_t)(fixed_budget + dyn[g]);
  }
  return SLKV_OK;
}

extern "C" slkv_status slkv_compacted_sizes(const slkv_layer_desc* desc, int64_t* h_out_offsets, int64_t* total_kept) {
  clear_error();
  slkv_status st = validate_desc(desc);
  if (st != SLKV_OK) return st;
  int64_t run = 0;
  for (int b = 0; b < desc->B; ++b) {
    int64_t n = desc->h_cu_seqlens[b + 1] - desc->h_cu_seqlens[b];
    for (int h = 0; h < desc->Hkv; ++h) {
      if (h_out_offsets) h_out_offsets[(size_t)b * desc->Hkv + h] = run;
      run += kept_rows(n, desc->w, desc->h_budgets[h]);
    }
  }
  if (h_out_offsets) h_out_offsets[(size_t)desc->B * desc->Hkv] = run;
  if (total_kept) *total_kept = run;
  return SLKV_OK;
}

slkv_status slkv_recompress_sizes(const slkv_ragged_desc* desc, int64_t* h_out_offsets, int64_t* total_kept) {
  clear_error();
  slkv_status st = validate_ragged_desc(desc);
  if (st != SLKV_OK) return st;
  int64_t run = 0;
  const int64_t S = (int64_t)desc->B * desc->Hkv;
  for (int64_t s = 0; s < S; ++s) {
    if (h_out_offsets) h_out_offsets[s] = run;
    run += kept_rows(desc->h_in_offsets[s + 1] - desc->h_in_offsets[s], desc->w, desc->h_budgets[s % desc->Hkv]);
  }
  if (h_out_offsets) h_out_offsets[S] = run;
  if (total_kept) *total_kept = run;
  return SLKV_OK;
}
