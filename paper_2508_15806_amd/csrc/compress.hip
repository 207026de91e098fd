// Stage 2b of SurfaceLogicKV (Section 3.4, Eq. 7-8, Algorithm 3) on gfx950:
//   pass 1  score_*<.., 1>  window-query x history-key logits, per-row log-sum-exp of every key chunk;
//                            the chunk of a segment that finishes last folds them into the row's log-sum-exp
//   pass 2  score_*<.., 2>  logits again, exp(logit - lse) summed down the G*w rows -> importance
//   select                   1-D pooling + per-head top-k (radix select, ordered compaction)
//   gather                   kept K/V rows -> compacted ragged cache
// bf16 inputs use the 32x32x16 bf16 MFMA with Q held in registers and K tiles staged in LDS;
// fp32 inputs use plain FMA kernels.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <type_traits>
#include <vector>

#include "device_utils.h"
#include "launch.h"
#include "slkv_internal.h"

// Development aid, compiled only with -DSLKV_TRACE: clock stamps of chosen workgroups.
#ifdef SLKV_TRACE
__device__ long long slkv_trace_buf[64 * 1024];
#define SLKV_STAMP(wg, slot) do { if (threadIdx.x == 0 && (wg) < 1024) slkv_trace_buf[(wg) * 16 + (slot)] = wall_clock64(); } while (0)
extern "C" int slkv_trace_read(long long* h, int n) {
  return (int)hipMemcpyFromSymbol(h, HIP_SYMBOL(slkv_trace_buf), (size_t)n * sizeof(long long));
}
#else
#define SLKV_STAMP(wg, slot) do {} while (0)
#endif

namespace slkv {

// Per-launch table of (sequence, KV head) segments, passed by value as a kernel argument.
struct SegTable {
  int32_t nseg;
  int32_t total_chunks;
  int32_t tok_begin[kMaxSegPerLaunch];   // first token of the sequence in the packed K/V
  int32_t n[kMaxSegPerLaunch];           // tokens in the sequence
  int32_t kkeep[kMaxSegPerLaunch];       // history rows to keep; -1 = keep every token
  int32_t out_off[kMaxSegPerLaunch + 1]; // first output row of the segment
  int32_t head[kMaxSegPerLaunch];        // KV head
  int32_t qrow_off[kMaxSegPerLaunch];    // first row of the segment's [G*w][d] query block
  int32_t score_off[kMaxSegPerLaunch];   // offset of the segment in the importance / pooled arrays
  int32_t chunk_begin[kMaxSegPerLaunch + 1];  // prefix of key-chunk counts (0 chunks when not ranked)
  int32_t seg_global[kMaxSegPerLaunch];  // index b*Hkv + h
  int32_t blk_begin[kMaxSegPerLaunch + 1];    // prefix of selection-block counts (no block when not ranked)
  int32_t hblk[kMaxSegPerLaunch];        // first block histogram of the segment
  int32_t tick[kMaxSegPerLaunch];        // ticket slot of the segment (segments of several key chunks)
};

// The same table in device memory, for calls with more segments than fit a kernel argument.
// chunk_begin, blk_begin and out_off are prefixes over all segments of the call.
struct SegTableDev {
  int32_t nseg;
  int32_t total_chunks;
  int32_t *tok_begin, *n, *kkeep, *out_off, *head, *qrow_off, *score_off, *chunk_begin, *seg_global, *blk_begin, *hblk, *tick;
};

// The workspace starts with ticket words (zero between calls): slot t counts the key chunks of a
// segment that have finished the statistics pass.
constexpr int kTicketSlots = 16384;
constexpr size_t kTicketBytes = (size_t)kTicketSlots * sizeof(uint32_t);

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // native 16-byte vector (register friendly)

union Pack16 {
  u32x4 u;
  bf16x8 b;
};

// 32x32x16 MFMA on eight 16-bit elements per lane and operand: bfloat16, or IEEE half when F16
// (the registers are typed bf16x8 either way; only the instruction reads them differently).
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
template <bool F16>
__device__ __forceinline__ f32x16 mfma16(bf16x8 a, bf16x8 b, f32x16 c) {
  if constexpr (F16)
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Segment of a block / row: the largest s with prefix[s] <= x (prefix non-decreasing, prefix[nseg] > x).
__device__ __forceinline__ int find_segment(const int32_t* prefix, int nseg, int x) {
  int lo = 0, hi = nseg - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (prefix[mid] <= x) lo = mid; else hi = mid - 1;
  }
  return lo;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Merge two (max, sum) pairs of a running softmax in the log2 domain.
__device__ __forceinline__ void merge_stats(float& m, float& s, float m2, float s2) {
  float mn = fmaxf(m, m2);
  float mu = mn == -INFINITY ? 0.f : mn;
  s = s * fast_exp2(m - mu) + s2 * fast_exp2(m2 - mu);
  m = mn;
}

// Data that one workgroup writes and another workgroup of the SAME kernel reads (after a ticket
// tells it that the writers are done) moves with device-scope accesses: the stores are written
// through to memory and the loads do not take a line that another XCD's L2 may hold newer, so no
// L2 write-back / invalidate (a device-scope fence costs tens of microseconds per kernel here) is
// needed.  The writer waits for its stores (workgroup release fence + barrier) before one thread
// takes the ticket.
__device__ __forceinline__ void st_dev(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_dev(uint32_t* p, uint32_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float ld_dev(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ uint32_t ld_dev(const uint32_t* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// Takes a ticket of `count` arrivals after the workgroup's device-scope stores have completed.
// Returns true in the workgroup that arrives last (its ticket word is zero again afterwards).
// `flag` is one word of LDS.  Every thread of the workgroup must call it.
__device__ __forceinline__ bool last_arrival(uint32_t* ticket, uint32_t count, uint32_t* flag) {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // the stores above have been performed
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t old = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old == count - 1u) __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *flag = old;
  }
  __syncthreads();
  const bool last = *flag == count - 1u;
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  return last;
}

// Per-row log-sum-exp (log2 domain) of a segment from the log-sum-exp of its key chunks
// (part[chunk][row]; -inf for a chunk without keys for the row), one thread per row.  The loads
// of a batch are all in flight together and the exponentials are independent of each other;
// only the additions run in chunk order, so the result does not depend on timing.
__device__ __forceinline__ void segment_lse(int c0, int c1, int seg, int Rpad, const float* __restrict__ part,
                                            float* __restrict__ lse) {
  constexpr int NB = 64;   // as many loads as a wave can have in flight
  for (int row = threadIdx.x; row < Rpad; row += blockDim.x) {
    float mm = -INFINITY, ss = 0.f;
    for (int c = c0; c < c1; c += NB) {
      float v[NB];
#pragma unroll
      for (int u = 0; u < NB; ++u) v[u] = c + u < c1 ? ld_dev(part + (int64_t)(c + u) * Rpad + row) : -INFINITY;
      float bm = v[0];
#pragma unroll
      for (int u = 1; u < NB; ++u) bm = fmaxf(bm, v[u]);
      const float mn = fmaxf(mm, bm);
      const float mu = mn == -INFINITY ? 0.f : mn;
      float e[NB];
#pragma unroll
      for (int u = 0; u < NB; ++u) e[u] = fast_exp2(v[u] - mu);
      ss *= fast_exp2(mm - mu);
#pragma unroll
      for (int u = 0; u < NB; ++u) ss += e[u];
      mm = mn;
    }
    lse[seg * Rpad + row] = ss > 0.f ? mm + log2f(ss) : INFINITY;
  }
}

// End of the statistics pass of one key chunk (its pairs are written): the chunk that arrives
// last at the segment's ticket folds all chunks into the segment's log-sum-exp and clears the
// ticket for the next call.  `flag` is one word of LDS.
template <class TAB>
__device__ __forceinline__ void finish_stats_chunk(const TAB& tab, int seg, int Rpad, const float* __restrict__ part,
                                                   float* __restrict__ lse, uint32_t* __restrict__ tickets, uint32_t* flag) {
  const int c0 = tab.chunk_begin[seg], c1 = tab.chunk_begin[seg + 1];
  if (c1 - c0 > 1) {
    if (!last_arrival(tickets + tab.tick[seg], (uint32_t)(c1 - c0), flag)) return;
    SLKV_STAMP(256 + blockIdx.x, 3);
  } else {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __syncthreads();
  }
  segment_lse(c0, c1, seg, Rpad, part, lse);
}

// The two workgroups that share a CU would otherwise run one after the other: the scheduler
// favours the older waves, the older workgroup finishes a third earlier and the younger one spends
// the end of the kernel alone on the CU, one wave per SIMD, with nothing to overlap with.  Waves
// raise their priority on even tiles and drop it on odd ones, so the workgroup that is a tile behind
// wins the issue slots for a tile.  (Measured: -0.7 us per pass on the 32K-prefix shape; the older
// workgroup still ends its loop about 5 us before the younger one.  Four priority levels falling
// with the tile index made pass 1 slower.)
__device__ __forceinline__ void tile_priority(int t) {
  if (t & 1) __builtin_amdgcn_s_setprio(0);
  else __builtin_amdgcn_s_setprio(1);
}

// ------------------------------------------------------------------------------------------
// MFMA scoring of 16-bit inputs (bfloat16, or half when F16).  One workgroup (4 waves) owns one chunk of history keys of one segment.
// K is staged in LDS in tiles of 64 keys (two buffers); up to kPrefetch further tiles are in
// flight from HBM into registers.  Wave (rb, ks) holds rows [rb*32*MT, (rb+1)*32*MT) of the
// G*w query rows in registers for the whole chunk and works on the 32-key sub-tiles
// ks, ks+KS, .. of every tile.  The 32x32x16 MFMA takes, per lane, 8 consecutive k-elements of
// row (lane%32) at k offset 8*(lane/32) for both operands, and returns in result register i the
// element at row 8*(i/4) + 4*(lane/32) + i%4, column lane%32.
//   PASS 1: D[key][qrow]: a lane owns one query row per MFMA tile -> sum of exp2(x - reference).
//   PASS 2: D[qrow][key]: a lane owns one key column -> sum over rows of exp2(x - lse[row]).
// Rows beyond R and keys beyond the chunk are loaded from a clamped (valid) address and masked.
constexpr int kTileKeys = 64;
constexpr int kPrefetch = 2;

template <int DK, int MT, int RB, int PASS, int KIND, class TAB>   // KIND: 0 bf16, 1 fp16, 2 bf16 queries with E4M3 keys
__global__ __launch_bounds__(256, (MT <= 2 ? 2 : 1)) void score_bf16_kernel(const TAB tab, const uint16_t* __restrict__ q,
                                                         const void* __restrict__ kmat_v, int64_t k_stride_tok,
                                                         int64_t k_stride_head, int R, int Rpad, int w, int CH,
                                                         float c_log2, float* __restrict__ part,
                                                         const float* __restrict__ lse, float* __restrict__ imp,
                                                         float* __restrict__ lse_out, uint32_t* __restrict__ tickets,
                                                         int grid2d) {
  constexpr int KS = 4 / RB;               // waves along the keys
  constexpr int TK = kTileKeys;
  constexpr int NSUB = TK / 32 / KS;       // 32-key sub-tiles per wave per tile
  constexpr int KK = DK / 16;
  constexpr int ROWB = DK * 2 + 16;        // padded LDS row (bf16 / fp16 elements): conflict-free 16-byte reads down a column
  constexpr bool KF8 = KIND == 2;          // keys arrive as E4M3 bytes and are widened to bf16 on their way into LDS
  constexpr int EB = KF8 ? 1 : 2;          // bytes per key element in memory
  constexpr int CPR = DK * EB / 16;        // 16-byte pieces per key row in memory
  constexpr int LPT = TK * CPR / 256;      // pieces per thread per tile
  constexpr int NPF = kPrefetch;
  static_assert(TK * CPR % 256 == 0 && LPT < 16, "tile must divide over the workgroup; LPT is or-ed into a wait count");
  __shared__ __attribute__((aligned(16))) unsigned char ktile[2][TK * ROWB];
  __shared__ float red[2][RB][TK];
  __shared__ float2 comb[KS][RB * 32 * MT];
  __shared__ uint32_t sh_flag;

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int rb = wv % RB, ks = wv / RB;
  const int l32 = lane & 31, half = lane >> 5;

  // Which chunk of which segment.  With a two-dimensional grid (grid2d; the host chooses it when the
  // segments' chunk counts are alike enough) blockIdx.y is the segment and blockIdx.x the chunk, and
  // workgroups past a segment's last chunk leave at once; otherwise blockIdx.x counts the chunks of
  // all segments and the segment is searched in the table.  The table is read through the scalar
  // cache, cold at every launch, so each dependent lookup costs a memory round trip before the
  // first key can be requested: the entries of segment blockIdx.y are therefore fetched before it
  // is known which case applies (y is 0 with a one-dimensional grid: a valid entry either way).
  struct SegEntry {
    int32_t n, tok_begin, head, qrow_off, chunk0, chunk1;
  };
  auto entry_of = [&](int s) {
    return SegEntry{tab.n[s], tab.tok_begin[s], tab.head[s], tab.qrow_off[s], tab.chunk_begin[s], tab.chunk_begin[s + 1]};
  };
  int seg = (int)blockIdx.y;
  SegEntry se = entry_of(seg);
  asm volatile("" :: "s"(se.n), "s"(se.tok_begin), "s"(se.head), "s"(se.qrow_off), "s"(se.chunk0), "s"(se.chunk1));   // fetched here, not behind the branch
  int bid;
  if (grid2d) {
    bid = se.chunk0 + (int)blockIdx.x;
    if (bid >= se.chunk1) return;
  } else {
    bid = blockIdx.x;
    seg = find_segment(tab.chunk_begin, tab.nseg, bid);
    se = entry_of(seg);
  }
  if (PASS == 1) SLKV_STAMP(256 + bid, 0);
  const int chunk = bid - se.chunk0;
  const int m = se.n - w;
  const int key_begin = chunk * CH;
  const int key_end = min(m, key_begin + CH);
  // tiles are processed in pairs (one per register slot); a surplus tile is fully masked
  const int ntiles = ((key_end - key_begin + TK - 1) / TK + 1) & ~1;
  // uniform 64-bit base of the segment's keys + 32-bit byte offsets (the host checks the range)
  const unsigned char* kbase = reinterpret_cast<const unsigned char*>(kmat_v) +
      ((int64_t)se.head * k_stride_head + (int64_t)se.tok_begin * k_stride_tok) * EB;
  const uint32_t row_bytes = (uint32_t)k_stride_tok * (uint32_t)EB;
  const uint32_t piece_off = (uint32_t)(tid % CPR) * 16u;
  const int piece_row = tid / CPR;

  u32x4 pf0[LPT], pf1[LPT];
  auto issue_tile = [&](int t, u32x4 (&pf)[LPT]) __attribute__((always_inline)) {
    const int key0 = key_begin + t * TK + piece_row;
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
      const int key = min(key0 + i * (256 / CPR), key_end - 1);
      // non-temporal: a workgroup reads its keys once (plain loads measured the same in either pass)
      pf[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kbase + ((uint32_t)key * row_bytes + piece_off)));
    }
  };
  auto store_tile = [&](const u32x4 (&pf)[LPT], int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
      const int idx = i * 256 + tid;
      if constexpr (KF8) {
        // 16 E4M3 bytes -> 16 bf16: the hardware converter gives exact fp32 values (checked against the
        // format's definition for all 256 codes), whose upper halves are the bf16 patterns
        u32x4 lo, hi;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)pf[i][j], false);
          const f32x2 b = __builtin_amdgcn_cvt_pk_f32_fp8((int)pf[i][j], true);
          const uint32_t p0 = __builtin_amdgcn_perm(__float_as_uint(a[1]), __float_as_uint(a[0]), 0x07060302u);
          const uint32_t p1 = __builtin_amdgcn_perm(__float_as_uint(b[1]), __float_as_uint(b[0]), 0x07060302u);
          if (j < 2) {
            lo[2 * j] = p0;
            lo[2 * j + 1] = p1;
          } else {
            hi[2 * (j - 2)] = p0;
            hi[2 * (j - 2) + 1] = p1;
          }
        }
        unsigned char* dst = &ktile[buf][(idx / CPR) * ROWB + (idx % CPR) * 32];
        *reinterpret_cast<u32x4*>(dst) = lo;
        *reinterpret_cast<u32x4*>(dst + 16) = hi;
      } else {
        *reinterpret_cast<u32x4*>(&ktile[buf][(idx / CPR) * ROWB + (idx % CPR) * 16]) = pf[i];
      }
    }
  };
  static_assert(NPF == 2, "the tile loop below is written out for two register slots");
  issue_tile(0, pf0);   // the second tile is requested after the queries: the loop can start without it

  // query rows of this wave, kept in registers for the whole chunk
  bf16x8 qreg[MT][KK];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int row = min(rb * 32 * MT + mt * 32 + l32, R - 1);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      Pack16 p;
      p.u = *reinterpret_cast<const u32x4*>(q + ((int64_t)se.qrow_off + row) * DK + kk * 16 + half * 8);
      qreg[mt][kk] = p.b;
    }
  }
  // pass 2: the log-sum-exp of the workgroup's rows, one coalesced load per thread here, handed
  // to the lanes through LDS once the loads have landed
  constexpr int NLSE = (RB * 32 * MT + 255) / 256;
  float lse_ld[PASS == 2 ? NLSE : 1];
  float lse_r[PASS == 2 ? MT : 1][16];
  if (PASS == 2) {
#pragma unroll
    for (int j = 0; j < NLSE; ++j) lse_ld[j] = lse[seg * Rpad + min(tid + j * 256, Rpad - 1)];
  }
  float m_run[MT], s_run[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    m_run[mt] = -INFINITY;
    s_run[mt] = 0.f;
  }

  // one tile: registers -> LDS, refill the register slot, barrier, MFMAs + epilogue
  auto do_tile = [&](int t, u32x4 (&pf)[LPT], auto masked_c, auto online_c, auto first_c) __attribute__((always_inline)) {
    constexpr bool MASKED = decltype(masked_c)::value;   // the tile may reach past key_end
    constexpr bool ONLINE = decltype(online_c)::value;   // pass 1: running maximum instead of a fixed reference
    constexpr bool FIRST = decltype(first_c)::value;     // pass 1: the chunk's first tile (fixes the reference)
    const int buf = t & 1;
    tile_priority(t);
    store_tile(pf, buf);
    if (!ONLINE) issue_tile(t + NPF, pf);   // past the chunk end every piece comes from one clamped row
    __syncthreads();
    if (PASS == 2 && t > 0 && tid < TK) {          // column sums of the previous tile
      float v = 0.f;
#pragma unroll
      for (int r = 0; r < RB; ++r) v += red[buf ^ 1][r][tid];
      const int key = key_begin + (t - 1) * TK + tid;
      if (key < key_end) imp[tab.score_off[seg] + key] = v;
    }
#pragma unroll
    for (int sb = 0; sb < NSUB; ++sb) {
      __builtin_amdgcn_sched_barrier(0);   // keep one sub-tile's operands live at a time
      const int sub = ks + sb * KS;
      const int key0 = key_begin + t * TK + sub * 32;   // first key of this sub-tile
      bf16x8 kreg[KK];
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        Pack16 p;
        p.u = *reinterpret_cast<const u32x4*>(&ktile[buf][(sub * 32 + l32) * ROWB + kk * 32 + half * 16]);
        kreg[kk] = p.b;
      }
      float colsum = 0.f;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          if (PASS == 1)
            acc = mfma16<KIND == 1>(kreg[kk], qreg[mt][kk], acc);
          else
            acc = mfma16<KIND == 1>(qreg[mt][kk], kreg[kk], acc);
        }
        if (PASS == 1) {
          // lane: query row mt*32 + l32, keys key0 + 8*(i/4) + 4*half + i%4
          if (MASKED && key0 + 32 > key_end) {
#pragma unroll
            for (int i = 0; i < 16; ++i)
              if (key0 + 8 * (i >> 2) + 4 * half + (i & 3) >= key_end) acc[i] = -INFINITY;
          }
          if (ONLINE) {
            float mx = fmaxf(acc[0], acc[1]);
#pragma unroll
            for (int i = 2; i < 16; i += 2) mx = fmaxf(mx, fmaxf(acc[i], acc[i + 1]));
            const float mn = fmaxf(m_run[mt], mx * c_log2);
            const float mu = mn == -INFINITY ? 0.f : mn;
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) sum += fast_exp2(fmaf(acc[i], c_log2, -mu));
            s_run[mt] = s_run[mt] * fast_exp2(m_run[mt] - mu) + sum;
            m_run[mt] = mn;
          } else {
            // The reference of the exponentials is fixed by the lane's first 16 logits of the chunk
            // (any finite reference gives the same log-sum-exp); later logits may exceed it by up to
            // ~2^100 before the sum overflows, which the caller detects and repeats ONLINE.
            if (FIRST && sb == 0) {
              float mx = fmaxf(acc[0], acc[1]);
#pragma unroll
              for (int i = 2; i < 16; i += 2) mx = fmaxf(mx, fmaxf(acc[i], acc[i + 1]));
              const float mn = mx * c_log2;
              m_run[mt] = mn == -INFINITY ? 0.f : mn;
            }
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) sum += fast_exp2(fmaf(acc[i], c_log2, -m_run[mt]));
            s_run[mt] += sum;
          }
        } else {
          // lane: key key0 + l32, query rows mt*32 + 8*(i/4) + 4*half + i%4
#pragma unroll
          for (int i = 0; i < 16; ++i) colsum += fast_exp2(fmaf(acc[i], c_log2, -lse_r[mt][i]));
        }
      }
      if (PASS == 2) {
        colsum += __shfl_xor(colsum, 32, 64);
        if (half == 0) red[buf][rb][sub * 32 + l32] = colsum;
      }
    }
  };

  // The first tile, Q and lse have to be complete here (loads return in order; the LPT loads of
  // the second tile, issued last, may still be in flight); inside the loop only the two tile slots
  // stay in flight, so the waits there can be partial.
  __builtin_amdgcn_sched_barrier(0);          // keep every earlier load ahead of the second tile's
  issue_tile(1, pf1);
  __builtin_amdgcn_s_waitcnt(0x0F70 | LPT);   // vmcnt(LPT)
  __builtin_amdgcn_sched_barrier(0);
  if (PASS == 2) {
    float* lse_s = reinterpret_cast<float*>(&comb[0][0]);   // comb is used by pass 1 only
    static_assert(sizeof(comb) >= NLSE * 256 * sizeof(float), "comb holds one value per thread and load");
#pragma unroll
    for (int j = 0; j < NLSE; ++j) lse_s[tid + j * 256] = tid + j * 256 < R ? lse_ld[j] : INFINITY;
    __syncthreads();
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i)
        lse_r[mt][i] = lse_s[rb * 32 * MT + mt * 32 + 8 * (i >> 2) + 4 * half + (i & 3)];
  }
  using T = std::true_type;
  using F = std::false_type;
  // Pass 1 with both sub-tiles of a tile in one wave (RB == 4; up to 64 rows per wave): software pipeline over sub-tiles.
  // The MFMAs of sub-tile s (two interleaved chains, one per row tile) are issued one per slot,
  // each slot also carrying the exponentials of two logits of sub-tile s-1 (read from the other
  // accumulator set), so the matrix pipe works in the shadow of the exponentials; the key operand
  // of the tile's second sub-tile is read from LDS during the first one's MFMAs.
  if constexpr (PASS == 1 && NSUB == 2 && MT <= 2) {
    constexpr int NSLOT = KK * MT, EPS = (16 * MT + NSLOT - 1) / NSLOT;
    f32x16 accA[MT], accB[MT];
    bf16x8 kA[KK], kB[KK];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int i = 0; i < 16; ++i) accA[mt][i] = accB[mt][i] = -INFINITY;   // exp2 of "the sub-tile before the first" is 0
    auto lds_read = [&](bf16x8& dst, int buf, int sub, int kk) __attribute__((always_inline)) {
      Pack16 pk;
      pk.u = *reinterpret_cast<const u32x4*>(&ktile[buf][(sub * 32 + l32) * ROWB + kk * 32 + half * 16]);
      dst = pk.b;
    };
    // keys past the chunk end count as -inf (pkey0 = first key of the accumulators' sub-tile)
    auto mask_tail = [&](f32x16 (&a)[MT], int pkey0) __attribute__((always_inline)) {
      if (pkey0 + 32 > key_end) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (pkey0 + 8 * (i >> 2) + 4 * half + (i & 3) >= key_end) a[mt][i] = -INFINITY;
      }
    };
    // one sub-tile: MFMAs into cur from operand kc, exponentials of prev; kn is filled for sub-tile nsub
    auto step = [&](f32x16 (&cur)[MT], f32x16 (&prev)[MT], bf16x8 (&kc)[KK], bf16x8 (&kn)[KK], auto prefetch_c, int buf,
                    int nsub) __attribute__((always_inline)) {
      constexpr bool PREFETCH = decltype(prefetch_c)::value;
#pragma unroll
      for (int sl = 0; sl < NSLOT; ++sl) {
        const int kk = sl / MT, mt = sl % MT;
#pragma unroll
        for (int j = 0; j < EPS; ++j) {
          const int e = sl * EPS + j;
          if (e < 16 * MT) s_run[e / 16] += fast_exp2(fmaf(prev[e / 16][e % 16], c_log2, -m_run[e / 16]));
        }
        if (kk == 0) {
          f32x16 z;
#pragma unroll
          for (int i = 0; i < 16; ++i) z[i] = 0.f;
          cur[mt] = mfma16<KIND == 1>(kc[kk], qreg[mt][kk], z);
        } else {
          cur[mt] = mfma16<KIND == 1>(kc[kk], qreg[mt][kk], cur[mt]);
        }
        if (PREFETCH && mt == MT - 1) lds_read(kn[kk], buf, nsub, kk);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    auto pipe_tile = [&](int t, u32x4 (&pf)[LPT], auto masked_c, auto first_c) __attribute__((always_inline)) {
      constexpr bool MASKED = decltype(masked_c)::value;   // this tile or the one before may reach past key_end
      constexpr bool FIRST = decltype(first_c)::value;
      const int buf = t & 1;
      const int key0 = key_begin + t * TK;
      tile_priority(t);
      store_tile(pf, buf);
      issue_tile(t + NPF, pf);
      __syncthreads();
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) lds_read(kA[kk], buf, 0, kk);
      if (MASKED) mask_tail(accB, key0 - 32);            // second sub-tile of the tile before
      step(accA, accB, kA, kB, T{}, buf, 1);
      if (FIRST || MASKED) mask_tail(accA, key0);
      if (FIRST) {
        // The reference of the exponentials is fixed by the lane's first 16 logits of the chunk (any
        // finite reference gives the same log-sum-exp); later logits may exceed it by up to ~2^100
        // before the sum overflows, which is detected below and repeated with a running maximum.
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          float mx = fmaxf(accA[mt][0], accA[mt][1]);
#pragma unroll
          for (int i = 2; i < 16; i += 2) mx = fmaxf(mx, fmaxf(accA[mt][i], accA[mt][i + 1]));
          const float mn = mx * c_log2;
          m_run[mt] = mn == -INFINITY ? 0.f : mn;
        }
      }
      step(accB, accA, kB, kA, F{}, buf, 0);
    };
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) m_run[mt] = 0.f;
    if (ntiles > NPF) {
      pipe_tile(0, pf0, F{}, T{});
      pipe_tile(1, pf1, F{}, F{});
      for (int t0 = NPF; t0 < ntiles - NPF; t0 += NPF) {
        pipe_tile(t0, pf0, F{}, F{});
        pipe_tile(t0 + 1, pf1, F{}, F{});
      }
      pipe_tile(ntiles - 2, pf0, T{}, F{});
      pipe_tile(ntiles - 1, pf1, T{}, F{});
    } else {
      pipe_tile(0, pf0, T{}, T{});
      pipe_tile(1, pf1, T{}, F{});
    }
    // the exponentials of the last sub-tile
    mask_tail(accB, key_begin + (ntiles - 1) * TK + 32);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      float sum = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) sum += fast_exp2(fmaf(accB[mt][i], c_log2, -m_run[mt]));
      s_run[mt] += sum;
    }
  } else if (PASS == 1) {
    // the first tile fixes the reference of the exponentials; only the last pair can reach past the chunk end
    if (ntiles > NPF) {
      do_tile(0, pf0, F{}, F{}, T{});
      do_tile(1, pf1, F{}, F{}, F{});
      for (int t0 = NPF; t0 < ntiles - NPF; t0 += NPF) {
        do_tile(t0, pf0, F{}, F{}, F{});
        do_tile(t0 + 1, pf1, F{}, F{}, F{});
      }
      do_tile(ntiles - 2, pf0, T{}, F{}, F{});
      do_tile(ntiles - 1, pf1, T{}, F{}, F{});
    } else {
      do_tile(0, pf0, T{}, F{}, T{});
      do_tile(1, pf1, T{}, F{}, F{});
    }
  } else {
    for (int t0 = 0; t0 < ntiles - NPF; t0 += NPF) {
      do_tile(t0, pf0, F{}, F{}, F{});
      do_tile(t0 + 1, pf1, F{}, F{}, F{});
    }
    do_tile(ntiles - 2, pf0, T{}, F{}, F{});
    do_tile(ntiles - 1, pf1, T{}, F{}, F{});
  }

  if (PASS == 1) SLKV_STAMP(256 + bid, 1);
  if (PASS == 1) {
    // A sum that left the fp32 range (logits far above the chunk's first ones): the whole
    // workgroup repeats the chunk with the running maximum.  Not taken for ordinary inputs.
    bool bad = false;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) bad = bad || !(s_run[mt] < INFINITY);
    if (__syncthreads_or(bad ? 1 : 0)) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        m_run[mt] = -INFINITY;
        s_run[mt] = 0.f;
      }
      for (int t = 0; t < ntiles; ++t) {          // plain loop, one tile in flight: this path is rare
        issue_tile(t, pf0);
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        do_tile(t, pf0, T{}, T{}, F{});
      }
    }
  }

  if (PASS == 2) {
    __syncthreads();
    if (tid < TK) {
      const int t = ntiles - 1;
      float v = 0.f;
#pragma unroll
      for (int r = 0; r < RB; ++r) v += red[t & 1][r][tid];
      const int key = key_begin + t * TK + tid;
      if (key < key_end) imp[tab.score_off[seg] + key] = v;
    }
  } else {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      // (reference, sum) -> (log-sum-exp, 1): a sum referenced to early logits can be very large
      // or small, and merging such pairs directly could lose it to an underflowing factor
      m_run[mt] = s_run[mt] > 0.f ? m_run[mt] + __builtin_amdgcn_logf(s_run[mt]) : -INFINITY;
      s_run[mt] = 1.f;
      float m2 = __shfl_xor(m_run[mt], 32, 64);
      float s2 = __shfl_xor(s_run[mt], 32, 64);
      merge_stats(m_run[mt], s_run[mt], m2, s2);
      if (half == 0) comb[ks][rb * 32 * MT + mt * 32 + l32] = make_float2(m_run[mt], s_run[mt]);
    }
    __syncthreads();
    for (int row = tid; row < RB * 32 * MT; row += 256) {
      float mm = comb[0][row].x, ss = comb[0][row].y;
#pragma unroll
      for (int k2 = 1; k2 < KS; ++k2) merge_stats(mm, ss, comb[k2][row].x, comb[k2][row].y);
      // the chunk's log-sum-exp of the row (-inf: no key)
      if (row < Rpad) st_dev(part + (int64_t)bid * Rpad + row, ss > 0.f ? mm + __builtin_amdgcn_logf(ss) : -INFINITY);
    }
    SLKV_STAMP(256 + bid, 2);
    finish_stats_chunk(tab, seg, Rpad, part, lse_out, tickets, &sh_flag);
    SLKV_STAMP(256 + bid, 4);
  }
}

// ------------------------------------------------------------------------------------------
// fp32 scoring with plain FMAs (small shapes).  Same chunking and outputs as the bf16 kernels.
// PASS 1: thread = query row, K tile in LDS (broadcast reads).  PASS 2: thread = key, Q rows in LDS.
template <int DK, int PASS, class TAB>
__global__ __launch_bounds__(256) void score_f32_kernel(const TAB tab, const float* __restrict__ q,
                                                        const float* __restrict__ kmat, int64_t k_stride_tok,
                                                        int64_t k_stride_head, int R, int Rpad, int w, int CH,
                                                        float c_log2, float* __restrict__ part,
                                                        const float* __restrict__ lse, float* __restrict__ imp,
                                                        float* __restrict__ lse_out, uint32_t* __restrict__ tickets) {
  constexpr int TROWS = 32;                 // keys (pass 1) or query rows (pass 2) per LDS tile
  constexpr int NSUB = 256 / TROWS;         // thread = (lane32, sub): 32 rows x 8 key subsets, or 32 keys x 8 row subsets
  __shared__ __attribute__((aligned(16))) float tile[TROWS][DK];
  __shared__ float lse_s[TROWS];
  __shared__ float2 red[NSUB][TROWS];
  __shared__ uint32_t sh_flag;
  const int tid = threadIdx.x;
  const int l32 = tid & (TROWS - 1), sub = tid / TROWS;
  const int bid = blockIdx.x;
  const int seg = find_segment(tab.chunk_begin, tab.nseg, bid);
  const int chunk = bid - tab.chunk_begin[seg];
  const int m = tab.n[seg] - w;
  const int key_begin = chunk * CH;
  const int key_end = min(m, key_begin + CH);
  const float* kbase = kmat + (int64_t)tab.head[seg] * k_stride_head + (int64_t)tab.tok_begin[seg] * k_stride_tok;
  const float* qbase = q + (int64_t)tab.qrow_off[seg] * DK;

  if (PASS == 1) {
    // 32 query rows at a time; the thread's key subset is keys sub, sub + 8, ... of every tile
    for (int r0 = 0; r0 < Rpad; r0 += TROWS) {
      const int row = r0 + l32;
      float qr[DK];
#pragma unroll
      for (int p = 0; p < DK; ++p) qr[p] = row < R ? qbase[(int64_t)row * DK + p] : 0.f;
      float mm = -INFINITY, ss = 0.f;
      for (int k0 = key_begin; k0 < key_end; k0 += TROWS) {
        __syncthreads();
        for (int idx = tid; idx < TROWS * DK; idx += 256) {
          const int kr = idx / DK, p = idx % DK;
          tile[kr][p] = k0 + kr < key_end ? kbase[(int64_t)(k0 + kr) * k_stride_tok + p] : 0.f;
        }
        __syncthreads();
        float x[TROWS / NSUB];
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < TROWS / NSUB; ++i) {
          const int kr = sub + i * NSUB;
          float acc = 0.f;
#pragma unroll
          for (int p = 0; p < DK; ++p) acc = fmaf(qr[p], tile[kr][p], acc);
          x[i] = k0 + kr < key_end ? acc * c_log2 : -INFINITY;
          mx = fmaxf(mx, x[i]);
        }
        const float mn = fmaxf(mm, mx);
        const float mu = mn == -INFINITY ? 0.f : mn;
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < TROWS / NSUB; ++i) sum += fast_exp2(x[i] - mu);
        ss = ss * fast_exp2(mm - mu) + sum;
        mm = mn;
      }
      __syncthreads();
      red[sub][l32] = make_float2(mm, ss);
      __syncthreads();
      if (sub == 0) {
#pragma unroll
        for (int k2 = 1; k2 < NSUB; ++k2) merge_stats(mm, ss, red[k2][l32].x, red[k2][l32].y);
        st_dev(part + (int64_t)bid * Rpad + row, (row < R && ss > 0.f) ? mm + __builtin_amdgcn_logf(ss) : -INFINITY);
      }
    }
    finish_stats_chunk(tab, seg, Rpad, part, lse_out, tickets, &sh_flag);
  } else {
    // 32 keys at a time; the thread's row subset is rows sub, sub + 8, ... of every query tile
    for (int k0 = key_begin; k0 < key_end; k0 += TROWS) {
      const int key = k0 + l32;
      float kr[DK];
#pragma unroll
      for (int p = 0; p < DK; ++p) kr[p] = key < key_end ? kbase[(int64_t)key * k_stride_tok + p] : 0.f;
      float colsum = 0.f;
      for (int r0 = 0; r0 < R; r0 += TROWS) {
        __syncthreads();
        for (int idx = tid; idx < TROWS * DK; idx += 256) {
          const int rr = idx / DK, p = idx % DK;
          tile[rr][p] = r0 + rr < R ? qbase[(int64_t)(r0 + rr) * DK + p] : 0.f;
        }
        if (tid < TROWS) lse_s[tid] = r0 + tid < R ? lse[seg * Rpad + r0 + tid] : INFINITY;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < TROWS / NSUB; ++i) {
          const int rr = sub + i * NSUB;
          float acc = 0.f;
#pragma unroll
          for (int p = 0; p < DK; ++p) acc = fmaf(tile[rr][p], kr[p], acc);
          colsum += fast_exp2(fmaf(acc, c_log2, -lse_s[rr]));   // rows past R: exp2(-inf) = 0
        }
      }
      __syncthreads();
      red[sub][l32].x = colsum;
      __syncthreads();
      if (sub == 0) {
#pragma unroll
        for (int k2 = 1; k2 < NSUB; ++k2) colsum += red[k2][l32].x;
        if (key < key_end) imp[tab.score_off[seg] + key] = colsum;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Pooling + top-k (Algorithm 3, steps 7-8).  Writes the kept positions: history positions
// ascending, then the window.
//
// Histories longer than one round of kSelRound positions take six launches; whatever touches every
// position runs with one workgroup per block of kSelBlock positions, only the digit searches run
// per segment (the block-wise kernels are described where they are defined):
//   select_pool_kernel: pool the block's importance scores (halo from the neighbours), write the
//     pooled scores, histogram their leading 11 key bits, write the block's histogram;
//   select_rank_kernel, phase 0: one workgroup per segment adds the block histograms and picks
//     the digit that holds the k-th largest score;
//   select_collect_kernel: the blocks copy their scores of that digit to the segment's list;
//   select_rank_kernel, phase 1: narrows the list down to the exact k-th largest value tau and
//     the number of scores equal to tau that belong to the top k (ties go to lower positions);
//     it also writes the window's positions and those of segments that are not ranked;
//   select_count_kernel, select_emit_kernel: the kept history positions, block by block: those
//     with score > tau, or == tau among the first `need_eq`.
// (One kernel with a per-segment ticket, the last block doing the ranking, was measured and
// dropped: with 1024-thread workgroups at one per CU, the blocks of later segments queue behind
// ranking workgroups and start tens of microseconds late.)
// Keys are the bit patterns of the pooled scores (>= 0, so monotone).  While ranking, a wave owns
// 2048 consecutive positions of a round, lane l the positions 64*j + l (j < 32).
constexpr int kInlineGatherRows = 256;    // segments up to this many kept rows are gathered by the selection kernel

struct GatherArgs {
  const unsigned char* k;
  const unsigned char* v;
  unsigned char* k_out;
  unsigned char* v_out;
  int64_t k_stride_tok, k_stride_head, v_stride_tok, v_stride_head;   // elements
  int lanes_per_row, elt_bytes;
  const int32_t* pos_in;   // optional: original position of every input row (ragged input)
  int32_t* pos_out;        // optional: pos_in at the kept rows
};

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelBlock = 4096;           // history positions per phase-A block
constexpr int kSelEmitThreads = 256;      // workgroup of the block-wise count / emit kernels (16 positions per thread)
constexpr int kSelEPT = 32;
constexpr int kSelEPTMid = 8, kSelEPTSmall = 2;   // shorter histories: fewer positions per thread in the one-workgroup kernel
constexpr int kSelRound = kSelThreads * kSelEPT;
constexpr int kSelHaloMax = kMaxPool / 2;
constexpr int kSelRankMax = 256;          // lists up to this length are ranked by direct counting
constexpr int kSelTieGroups = 512;        // this many group maxima in the bound's digit switch the histograms to the pile-aware step
constexpr int kSelTrackMax = 512;         // up to this many wanted keys the first level also tracks the largest and smallest key of every digit
constexpr int kSelCandidates = 12288;     // scores of one first-level digit that the LDS list can hold
constexpr int kDigitShift = 20;           // first-level digit = key >> 20: sign (0), 8 exponent and 3 mantissa bits
constexpr uint32_t kKeyNone = 0xffffffffu;
static_assert(kTicketBytes == SLKV_WORKSPACE_HEADER_BYTES, "the header documents the size of the ticket area");
static_assert((0x7f800000u >> kDigitShift) < (uint32_t)kHistBins, "every key has a first-level digit inside the histogram");

// Key of a pooled score: its bit pattern; anything that is not a non-negative number (cannot
// come out of finite inputs) ranks as +infinity, so that both phases count it the same way.
__device__ __forceinline__ uint32_t score_key(float v) {
  const uint32_t u = __float_as_uint(v);
  return u > 0x7f800000u ? 0x7f800000u : u;
}

__device__ __forceinline__ uint32_t lanes_below(unsigned long long mask) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

template <int RADIUS, class TAB>   // pooling radius known at compile time (0..3), or -1: any radius
__global__ __launch_bounds__(kSelThreads) void select_pool_kernel(const TAB tab, int w, int pool_kernel, int pool_mode,
                                                                  const float* __restrict__ imp, float* __restrict__ pooled,
                                                                  uint32_t* __restrict__ blockhist) {
  constexpr int NT = kSelThreads;
  __shared__ uint32_t hist[kHistBins];
  __shared__ float stage[kSelBlock + 2 * kSelHaloMax];
  const int tid = threadIdx.x;
  const int bid = blockIdx.x;
  const int seg = find_segment(tab.blk_begin, tab.nseg, bid);
  const int blk = bid - tab.blk_begin[seg];
  const int n = tab.n[seg];
  const int kk = tab.kkeep[seg];
  const int m = n - w;
  if (!(kk > 0 && kk < m)) return;                    // not ranked: nothing to pool (such segments have no block)
  SLKV_STAMP(bid, 0);
  const float* I = imp + tab.score_off[seg];
  float* P = pooled + tab.score_off[seg];
  const int radius = RADIUS >= 0 ? RADIUS : pool_kernel / 2;
  const bool is_max = pool_mode != SLKV_POOL_AVG;
  const float fill = is_max ? -INFINITY : 0.f;
  const float inv_p = 1.f / (float)pool_kernel;
  const int p0 = blk * kSelBlock;
  const int cnt = min(kSelBlock, m - p0);
  for (int s = tid; s < cnt + 2 * radius; s += NT) {   // stage[s] = importance at position p0 - radius + s
    const int j = p0 - radius + s;
    stage[s] = (j >= 0 && j < m) ? I[j] : fill;
  }
  for (int i = tid; i < kHistBins; i += NT) hist[i] = 0;
  __syncthreads();
#pragma unroll
  for (int e = 0; e < kSelBlock / NT; ++e) {
    const int s = e * NT + tid;
    if (s < cnt) {
      float a = stage[s];
      if (RADIUS >= 0) {
#pragma unroll
        for (int t = 1; t <= 2 * (RADIUS >= 0 ? RADIUS : 0); ++t) a = is_max ? fmaxf(a, stage[s + t]) : a + stage[s + t];
      } else {
        for (int t = 1; t <= 2 * radius; ++t) a = is_max ? fmaxf(a, stage[s + t]) : a + stage[s + t];
      }
      if (!is_max) a *= inv_p;
      P[p0 + s] = a;
      atomicAdd(&hist[score_key(a) >> kDigitShift], 1u);
    }
  }
  __syncthreads();
  uint32_t* bh = blockhist + (size_t)(tab.hblk[seg] + blk) * kHistBins;
  for (int i = tid; i < kHistBins; i += NT) bh[i] = hist[i];
  SLKV_STAMP(bid, 1);
}

// Phase B: one workgroup per segment (unranked segments only write their positions).
template <class TAB>
__global__ __launch_bounds__(kSelThreads) void select_rank_kernel(const TAB tab, int w, const float* __restrict__ pooled,
                                                                  uint32_t* __restrict__ blockhist,
                                                                  int32_t* __restrict__ kept_idx, int64_t* __restrict__ d_out_offsets,
                                                                  const GatherArgs ga, int split_emit,
                                                                  const uint32_t* __restrict__ lists, int phase) {
  constexpr int NT = kSelThreads, NW = kSelWaves, EPT = kSelEPT, ROUND = kSelRound;
  __shared__ uint32_t hist[kHistBins];
  __shared__ uint32_t cand[kSelCandidates];
  __shared__ uint32_t small_list[kSelRankMax];
  __shared__ int32_t sh_pos[kInlineGatherRows];
  __shared__ uint32_t sh_scan[NW];
  __shared__ uint32_t res[4];

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int seg = blockIdx.x;
  const int bid = seg;
  (void)bid;                                           // (only the development stamps use it)
  const int nblk = tab.blk_begin[seg + 1] - tab.blk_begin[seg];
  const int n = tab.n[seg];
  const int kk = tab.kkeep[seg];
  const int m = n - w;
  const int kept = tab.out_off[seg + 1] - tab.out_off[seg];
  const bool small_seg = !split_emit && kept <= kInlineGatherRows;   // (split_emit: the launch has ranked segments, and gather_kernel copies every row)
  int32_t* out = kept_idx + tab.out_off[seg];
  if (d_out_offsets && tid == 0 && phase != 0) {
    d_out_offsets[tab.seg_global[seg]] = tab.out_off[seg];
    if (seg == tab.nseg - 1) d_out_offsets[tab.seg_global[seg] + 1] = tab.out_off[tab.nseg];
  }
  auto emit = [&](int pos, int j) __attribute__((always_inline)) {   // kept position j goes to output slot pos
    if ((uint32_t)pos < (uint32_t)kept) {
      out[pos] = j;
      if (small_seg) sh_pos[pos] = j;
    }
  };
  SLKV_STAMP(bid, 2);
  if (small_seg)
    for (int i = tid; i < kInlineGatherRows; i += NT) sh_pos[i] = 0;
  __syncthreads();
  const bool ranked = kk > 0 && kk < m;
  // Ranked segments take two launches of this kernel with select_collect_kernel between them
  // (words 4.. of the segment's first histogram row carry the state across):
  //   phase 0: add up the block histograms, find the first-level digit of the k-th largest score;
  //   (collect: the blocks copy their scores of that digit to the segment's list in memory)
  //   phase 1: rank the list, or, if the digit holds more scores than the LDS list, narrow it by
  //            sweeps over the pooled array; write the window's positions.
  if (phase == 0 && !ranked) return;
  uint32_t* const hdr = blockhist + (size_t)tab.hblk[seg] * kHistBins;   // (used for ranked segments only)
  if (!ranked) {
    if (kk < 0) {
      for (int j = tid; j < n; j += NT) emit(j, j);
    } else {
      for (int j = tid; j < w; j += NT) emit(j, m + j);   // kk == 0: the window alone
    }
  } else {
    const float* P = pooled + tab.score_off[seg];
    if (phase == 0) {
      // first-level histogram of the segment: the sum of its blocks' histograms
      static_assert(kHistBins == 2 * NT, "a thread adds up two bins");
      const uint32_t* bh0 = blockhist + (size_t)tab.hblk[seg] * kHistBins;
      uint32_t a0 = 0, a1 = 0;
      for (int b0 = 0; b0 < nblk; b0 += 24) {             // 48 loads in flight
        uint32_t v0[24], v1[24];
#pragma unroll
        for (int u = 0; u < 24; ++u) {
          const int b = min(b0 + u, nblk - 1);
          v0[u] = bh0[(size_t)b * kHistBins + tid];
          v1[u] = bh0[(size_t)b * kHistBins + NT + tid];
        }
#pragma unroll
        for (int u = 0; u < 24; ++u)
          if (b0 + u < nblk) {
            a0 += v0[u];
            a1 += v1[u];
          }
      }
      hist[tid] = a0;
      hist[NT + tid] = a1;
      __syncthreads();
      SLKV_STAMP(bid, 3);
      select_bin<NT>(hist, (uint32_t)kk, sh_scan, res);
      if (tid == 0) {
        const uint32_t in_range = hist[res[0]];
        hdr[4] = res[0] << kDigitShift;                    // [lo, hi]: the keys of the chosen digit
        hdr[5] = (res[0] << kDigitShift) + ((1u << kDigitShift) - 1u);
        hdr[6] = res[1];                                  // rank of the wanted key inside the digit
        hdr[7] = 0;                                       // length of the list (filled by the blocks)
        hdr[8] = in_range;
        hdr[9] = in_range <= (uint32_t)kSelCandidates ? 1u : 0u;   // 1: the blocks list the digit's scores
      }
      SLKV_STAMP(bid, 5);
      return;
    }
    // ---------------- the k-th largest pooled score of the segment
    const int rounds = (m + ROUND - 1) / ROUND;
    const bool multi = rounds > 1;
    uint32_t key[EPT];
    auto load_round = [&](int r) __attribute__((always_inline)) {
      const int base = r * ROUND + wv * (64 * EPT) + lane;
      float ld[EPT];
#pragma unroll
      for (int j = 0; j < EPT; ++j) ld[j] = P[min(base + j * 64, m - 1)];
#pragma unroll
      for (int j = 0; j < EPT; ++j) key[j] = base + j * 64 < m ? score_key(ld[j]) : kKeyNone;
    };
    // f(key) over every score of the segment (rounds beyond the first re-read the pooled array)
    auto sweep = [&](auto f) __attribute__((always_inline)) {
      for (int r = 0; r < rounds; ++r) {
        if (multi) load_round(r);
#pragma unroll
        for (int j = 0; j < EPT; ++j) f(key[j]);
      }
    };
    uint32_t lo = hdr[4], hi = hdr[5], k = hdr[6], in_range = hdr[8];
    const bool use_list = hdr[9] != 0u;
    const uint32_t ncand = min(hdr[7], (uint32_t)kSelCandidates);   // (== in_range when the list is used)
    if (use_list) {
      // the scores of the chosen digit, listed by the blocks: into LDS
      const uint32_t* L = lists + tab.score_off[seg];
      for (uint32_t i = tid; i < ncand; i += NT) cand[i] = L[i];
      __syncthreads();
    } else if (!multi) {
      load_round(0);
    }
    SLKV_STAMP(bid, 4);
    SLKV_STAMP(bid, 6);
    // narrow [lo, hi] down to one value: 11 bits per level over what is left of the range
    for (;;) {
      if (in_range <= (uint32_t)kSelRankMax && (use_list || lo == hi)) {
        if (lo == hi) break;                              // every score left equals lo
        // short list: gather the scores still in range, then the k-th largest by counting
        if (tid == 0) res[3] = 0;
        __syncthreads();
        for (uint32_t i = tid; i < ncand; i += NT) {
          const uint32_t kv = cand[i];
          if (kv >= lo && kv <= hi) {
            const uint32_t slot = atomicAdd(&res[3], 1u);
            if (slot < (uint32_t)kSelRankMax) small_list[slot] = kv;
          }
        }
        __syncthreads();
        const uint32_t ns = min(res[3], (uint32_t)kSelRankMax);
        if ((uint32_t)tid < ns) {
          const uint32_t kv = small_list[tid];
          uint32_t gt = 0, ge = 0;
          for (uint32_t i = 0; i < ns; ++i) {
            const uint32_t o = small_list[i];
            gt += o > kv ? 1u : 0u;
            ge += o >= kv ? 1u : 0u;
          }
          if (gt < k && k <= ge) {   // every thread holding the k-th largest value writes the same pair
            res[0] = kv;
            res[1] = k - gt;
          }
        }
        __syncthreads();
        lo = hi = res[0];
        k = res[1];
        __syncthreads();
        break;
      }
      const uint32_t span1 = hi - lo;
      const int nbits = span1 ? 32 - __clz(span1) : 0;
      const int shift = nbits > 11 ? nbits - 11 : 0;
      for (int i = tid; i < kHistBins; i += NT) hist[i] = 0;
      __syncthreads();
      if (use_list) {
        for (uint32_t i = tid; i < ncand; i += NT) {
          const uint32_t kv = cand[i];
          if (kv >= lo && kv <= hi) atomicAdd(&hist[(kv - lo) >> shift], 1u);
        }
      } else {
        sweep([&](uint32_t kv) {
          if (kv >= lo && kv <= hi) atomicAdd(&hist[(kv - lo) >> shift], 1u);
        });
      }
      __syncthreads();
      select_bin<NT>(hist, k, sh_scan, res);
      in_range = hist[res[0]];
      k = res[1];
      lo = lo + (res[0] << shift);
      hi = min(hi, lo + ((1u << shift) - 1u));
      __syncthreads();
      if (shift == 0) break;
    }
    const uint32_t tau = lo, need_eq = k;
    SLKV_STAMP(bid, 7);

    // The kept history positions are written by select_count_kernel + select_emit_kernel, one
    // workgroup per block of the history: they find the threshold in words 2 and 3 of the segment's
    // first block histogram (read in full above, not needed again in this call).
    if (tid == 0) {
      hdr[2] = tau;
      hdr[3] = need_eq;
    }
    for (int j = tid; j < w; j += NT) emit(kk + j, m + j);
    SLKV_STAMP(bid, 8);
  }

  // Small segments copy their K/V rows here (saves the gather launch); larger ones are left
  // to gather_kernel, which skips the segments handled here.
  if (kept > 0 && small_seg) {
    __syncthreads();                                // sh_pos is complete
    const int64_t tok0 = tab.tok_begin[seg], h = tab.head[seg], row0 = tab.out_off[seg];
    const int pieces = kept * ga.lanes_per_row;
    for (int idx = tid; idx < pieces; idx += NT) {
      const int row = idx / ga.lanes_per_row, c = idx % ga.lanes_per_row;
      const int64_t tok = tok0 + sh_pos[row];
      const uint4 kv = *reinterpret_cast<const uint4*>(ga.k + (h * ga.k_stride_head + tok * ga.k_stride_tok) * ga.elt_bytes + c * 16);
      const uint4 vv = *reinterpret_cast<const uint4*>(ga.v + (h * ga.v_stride_head + tok * ga.v_stride_tok) * ga.elt_bytes + c * 16);
      const int64_t o = ((row0 + row) * ga.lanes_per_row + c) * 16;
      *reinterpret_cast<uint4*>(ga.k_out + o) = kv;
      *reinterpret_cast<uint4*>(ga.v_out + o) = vv;
      if (ga.pos_out && c == 0) ga.pos_out[row0 + row] = ga.pos_in[tok];
    }
  }
  SLKV_STAMP(bid, 9);
}

// Between the two phases of select_rank_kernel: every block copies its scores of the digit chosen
// for its segment (keys in [lo, hi], words 4 and 5 of the segment's first histogram row) to the
// segment's list in memory, in any order: one atomic on the list's length (word 7) per wave.
// Nothing is listed when the digit holds more scores than the ranking workgroup's LDS list (word 9).
template <class TAB>
__global__ __launch_bounds__(kSelEmitThreads) void select_collect_kernel(const TAB tab, int w, const float* __restrict__ pooled,
                                                                     uint32_t* __restrict__ blockhist,
                                                                     uint32_t* __restrict__ lists, int seg0) {
  constexpr int NT = kSelEmitThreads, PER = kSelBlock / NT;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  int seg, blk;
  if (seg0 >= 0) {
    seg = seg0 + (int)blockIdx.y;
    blk = blockIdx.x;
    if (blk >= tab.blk_begin[seg + 1] - tab.blk_begin[seg]) return;
  } else {
    seg = find_segment(tab.blk_begin, tab.nseg, (int)blockIdx.x);
    blk = (int)blockIdx.x - tab.blk_begin[seg];
  }
  const int m = tab.n[seg] - w;
  const int kk = tab.kkeep[seg];
  if (!(kk > 0 && kk < m)) return;
  uint32_t* hdr = blockhist + (size_t)tab.hblk[seg] * kHistBins;
  const float* P = pooled + tab.score_off[seg];
  const int p0 = blk * kSelBlock + wv * (64 * PER) + lane;
  float pv[PER];
#pragma unroll
  for (int j = 0; j < PER; ++j) pv[j] = P[min(p0 + j * 64, m - 1)];
  if (hdr[9] == 0u) return;
  const uint32_t lo = hdr[4], span = hdr[5] - lo;
  uint32_t* L = lists + tab.score_off[seg];         // as long as the history: every list fits
  uint32_t key[PER];
  uint32_t c = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    key[j] = p0 + j * 64 < m ? score_key(pv[j]) : kKeyNone;
    c += (uint32_t)__popcll(__ballot(key[j] - lo <= span));   // (kKeyNone - lo exceeds every span)
  }
  if (c) {
    uint32_t base = 0;
    if (lane == 0) base = atomicAdd(&hdr[7], c);
    base = (uint32_t)__shfl((int)base, 0, 64);
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      const bool in = key[j] - lo <= span;
      const unsigned long long mask = __ballot(in);
      if (in) L[base + lanes_below(mask)] = key[j];
      base += (uint32_t)__popcll(mask);
    }
  }
}

// Ordered compaction of long histories, spread over the blocks of select_pool_kernel (one
// workgroup per kSelBlock positions) once select_rank_kernel has left the threshold tau and the
// number need_eq of positions equal to tau that are kept (the first ones in position order):
//   select_count_kernel: positions of the block above tau / equal to tau -> words 0, 1 of the
//     block's histogram row (free by now);
//   select_emit_kernel: sums the counts of the segment's earlier blocks, scans its own positions
//     (a wave owns 1024 consecutive ones) and writes the kept ones to their output slots:
//     slot = (#greater before) + min(#equal before, need_eq).
template <class TAB>
__global__ __launch_bounds__(kSelEmitThreads) void select_count_kernel(const TAB tab, int w, const float* __restrict__ pooled,
                                                                   uint32_t* __restrict__ blockhist, int seg0) {
  constexpr int NT = kSelEmitThreads, PER = kSelBlock / NT;
  __shared__ uint32_t sh[NT / 64];
  const int tid = threadIdx.x;
  // seg0 >= 0: one grid row per segment (no search in the table; blocks past the segment's last
  // one leave at once); seg0 < 0: one row over all blocks
  int seg, blk;
  if (seg0 >= 0) {
    seg = seg0 + (int)blockIdx.y;
    blk = blockIdx.x;
    if (blk >= tab.blk_begin[seg + 1] - tab.blk_begin[seg]) return;
  } else {
    seg = find_segment(tab.blk_begin, tab.nseg, (int)blockIdx.x);
    blk = (int)blockIdx.x - tab.blk_begin[seg];
  }
  const int m = tab.n[seg] - w;
  const int kk = tab.kkeep[seg];
  if (!(kk > 0 && kk < m)) return;                    // (such segments have no block)
  uint32_t* row0 = blockhist + (size_t)tab.hblk[seg] * kHistBins;
  const uint32_t tau = row0[2];
  const float* P = pooled + tab.score_off[seg];
  const int p0 = blk * kSelBlock + tid;               // (which thread counts which position does not matter here)
  uint32_t cg = 0, ce = 0;
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const int j = p0 + e * NT;
    const uint32_t kv = score_key(P[min(j, m - 1)]);
    if (j < m) {
      cg += kv > tau ? 1u : 0u;
      ce += kv == tau ? 1u : 0u;
    }
  }
  const uint32_t tot = block_sum<NT, uint32_t>((ce << 16) | cg, sh);   // a block holds 4096 positions: 13 bits each
  if (tid == 0) {
    uint32_t* row = row0 + (size_t)blk * kHistBins;
    row[0] = tot & 0xffffu;
    row[1] = tot >> 16;
  }
}

template <class TAB>
__global__ __launch_bounds__(kSelEmitThreads) void select_emit_kernel(const TAB tab, int w, const float* __restrict__ pooled,
                                                                  const uint32_t* __restrict__ blockhist,
                                                                  int32_t* __restrict__ kept_idx, int seg0) {
  constexpr int NT = kSelEmitThreads, PER = kSelBlock / NT;
  __shared__ uint32_t sh[NT / 64];
  const int tid = threadIdx.x;
  // seg0 >= 0: one grid row per segment (no search in the table; blocks past the segment's last
  // one leave at once); seg0 < 0: one row over all blocks
  int seg, blk;
  if (seg0 >= 0) {
    seg = seg0 + (int)blockIdx.y;
    blk = blockIdx.x;
    if (blk >= tab.blk_begin[seg + 1] - tab.blk_begin[seg]) return;
  } else {
    seg = find_segment(tab.blk_begin, tab.nseg, (int)blockIdx.x);
    blk = (int)blockIdx.x - tab.blk_begin[seg];
  }
  const int m = tab.n[seg] - w;
  const int kk = tab.kkeep[seg];
  if (!(kk > 0 && kk < m)) return;
  const uint32_t* row0 = blockhist + (size_t)tab.hblk[seg] * kHistBins;
  const uint32_t tau = row0[2], need_eq = row0[3];
  const int kept = tab.out_off[seg + 1] - tab.out_off[seg];
  int32_t* out = kept_idx + tab.out_off[seg];
  const float* P = pooled + tab.score_off[seg];
  // this block's own positions first (the loads fly while the earlier blocks are added up): a wave
  // owns 64 * PER consecutive positions, lane l the positions 64 j + l, so that loads are coalesced
  // and ballots are in position order
  const int lane = tid & 63, wv = tid >> 6;
  const int p0 = blk * kSelBlock + wv * (64 * PER) + lane;
  float pv[PER];
#pragma unroll
  for (int j = 0; j < PER; ++j) pv[j] = P[min(p0 + j * 64, m - 1)];
  // kept positions before this block: greater, and equal (capped at need_eq when they are used)
  uint32_t pg = 0, pe = 0;
  for (int b = tid; b < blk; b += NT) {
    pg += row0[(size_t)b * kHistBins];
    pe += row0[(size_t)b * kHistBins + 1];
  }
  // (a segment has at most 2^31 / kSelBlock blocks of at most 4096 positions: the sums fit 32 bits each)
  const uint32_t g0 = block_sum<NT, uint32_t>(pg, sh);
  const uint32_t e0 = block_sum<NT, uint32_t>(pe, sh);
  uint32_t key[PER];
  uint32_t wg = 0, we = 0;
#pragma unroll
  for (int j = 0; j < PER; ++j) {
    key[j] = p0 + j * 64 < m ? score_key(pv[j]) : kKeyNone;
    wg += (uint32_t)__popcll(__ballot(key[j] > tau && key[j] != kKeyNone));
    we += (uint32_t)__popcll(__ballot(key[j] == tau));
  }
  __shared__ uint32_t sh_wg[NT / 64], sh_we[NT / 64];
  if (lane == 0) {
    sh_wg[wv] = wg;
    sh_we[wv] = we;
  }
  __syncthreads();
  uint32_t g = g0, q = e0;                            // greater / equal before this wave's positions
#pragma unroll
  for (int v2 = 0; v2 < NT / 64; ++v2)
    if (v2 < wv) {
      g += sh_wg[v2];
      q += sh_we[v2];
    }
  if (wg + we) {
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      const bool isg = key[j] > tau && key[j] != kKeyNone;
      const bool ise = key[j] == tau;
      const unsigned long long mg = __ballot(isg), me = __ballot(ise);
      if (mg | me) {
        const uint32_t my_g = g + lanes_below(mg);
        const uint32_t my_e = q + lanes_below(me);    // ties are taken in position order
        uint32_t pos = 0xffffffffu;
        if (isg) pos = my_g + min(my_e, need_eq);
        else if (ise && my_e < need_eq) pos = my_g + my_e;
        if (pos < (uint32_t)kept) out[pos] = p0 + j * 64;
        g += (uint32_t)__popcll(mg);
        q += (uint32_t)__popcll(me);
      }
    }
  }
}

// The same selection for launches whose histories all fit one round of kSelRound positions: one
// workgroup per segment does everything, and the scores never leave its registers between the
// first load and the last store (no second workgroup to wait for, no re-read).  Thread t owns 32
// consecutive positions (values reach it through an LDS transposition of coalesced loads), so
// pooling is a sliding window in registers and the ordered compaction is one block scan of
// packed (greater, equal) counts plus per-thread bit masks.  The radix levels take their 11-bit
// digits relative to the range of keys still in question, which spreads the LDS histogram over
// nearly all bins and leaves few scores in the chosen one; where k allows, the range is first cut
// from below by the k-th largest of per-group maxima (see the search in the kernel).
constexpr int kResStageFloats = kSelRound + 2 * kSelHaloMax + ((kSelRound + 2 * kSelHaloMax) >> 5) + 8;
constexpr int kResCandidates = 3072;   // keys that the list behind the staging array can hold
constexpr int kResAuxWords = 3 * kHistBins;   // second histogram, largest and smallest key per digit: the start of the staging array, once the scores are in registers
constexpr size_t kResLdsBytes = (size_t)(kResStageFloats + kResCandidates) * sizeof(float);

// index into the staging array: one word of padding per thread's positions, so that the threads
// of a wave read their consecutive positions from different banks
template <int EPT>
__device__ __forceinline__ int pad_idx(int i) { return i + i / EPT; }

template <int RADIUS, int EPT_, class TAB>   // pooling radius known at compile time (0..3), or -1: any radius, window read from LDS;
                                             // EPT_: positions per thread (the history is at most 1024 * EPT_ positions)
__global__ __launch_bounds__(kSelThreads) void select_resident_kernel(const TAB tab, int w, int pool_kernel, int pool_mode,
                                                                      int write_pooled, const float* __restrict__ imp,
                                                                      float* __restrict__ pooled, int32_t* __restrict__ kept_idx,
                                                                      int64_t* __restrict__ d_out_offsets, const GatherArgs ga) {
  constexpr int NT = kSelThreads, EPT = EPT_, ROUND = NT * EPT_;   // the history is at most ROUND positions
  extern __shared__ float stage[];
  __shared__ uint32_t hist[kHistBins];
  __shared__ int32_t sh_pos[kInlineGatherRows];
  __shared__ uint32_t sh_scan[NT / 64];
  __shared__ uint32_t res[4];                      // [0], [1]: digit search and ranking results; [2], [3]: list lengths, in turn
  __shared__ uint32_t sh_mm[2 * (NT / 64)];

  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int seg = blockIdx.x;
  const int n = tab.n[seg];
  const int kk = tab.kkeep[seg];
  const int m = n - w;
  const int kept = tab.out_off[seg + 1] - tab.out_off[seg];
  const bool small_seg = kept <= kInlineGatherRows;
  int32_t* out = kept_idx + tab.out_off[seg];
  if (d_out_offsets && tid == 0) {
    d_out_offsets[tab.seg_global[seg]] = tab.out_off[seg];
    if (seg == tab.nseg - 1) d_out_offsets[tab.seg_global[seg] + 1] = tab.out_off[tab.nseg];
  }
  auto emit = [&](int pos, int j) __attribute__((always_inline)) {   // kept position j goes to output slot pos
    if ((uint32_t)pos < (uint32_t)kept) {
      out[pos] = j;
      if (small_seg) sh_pos[pos] = j;
    }
  };
  SLKV_STAMP(128 + seg, 0);
  if (small_seg)
    for (int i = tid; i < kInlineGatherRows; i += NT) sh_pos[i] = 0;
  __syncthreads();
  // The observation window is kept whatever the scores say: where this kernel also copies the rows
  // (small segments) and the window is one 16-byte piece per thread at most, the pieces are
  // fetched right behind the scores and stored at the end, off the critical path.
  const int lpr = ga.lanes_per_row;
  const bool win_early = small_seg && w * lpr <= NT;
  const bool win_mine = win_early && tid < w * lpr;
  const int win_piece = min(tid, max(w * lpr - 1, 0));           // (threads past the window's pieces fetch its last one again: a load
  const int win_row = win_piece / lpr, win_c = win_piece % lpr;  //  under a condition would have to be waited for where the branches meet)
  u32x4 win_k, win_v;
  const bool ranked = kk > 0 && kk < m;
  if (!ranked) {
    if (kk < 0) {
      for (int j = tid; j < n; j += NT) emit(j, j);
    } else {
      for (int j = tid; j < w; j += NT) emit(j, m + j);   // kk == 0: the window alone
    }
  }
  if (ranked) {
  const float* I = imp + tab.score_off[seg];
  float* P = pooled + tab.score_off[seg];
  const int radius = RADIUS >= 0 ? RADIUS : pool_kernel / 2;
  const bool is_max = pool_mode != SLKV_POOL_AVG;
  const float fill = 0.f;                          // scores are >= 0, so zero padding leaves window maxima as they are
  const float inv_p = 1.f / (float)pool_kernel;

  // Keys: bit patterns of the pooled scores (>= 0, so monotone as unsigned integers); positions
  // past the end of the history get a key above every score.
  uint32_t key[EPT];
  const int j0 = EPT * tid;

  // keys of the pooled scores from the importance array.  Window maxima are taken on the keys
  // themselves (integer maxima, three operands at a time); averages in floating point.
  auto pool_all = [&]() {
    const int base = 0;
    // all loads first (clamped addresses, so none depends on a branch), then the LDS writes
    float ld[EPT + 1];
#pragma unroll
    for (int c = 0; c <= EPT; ++c) {
      const int j = base - radius + (c < EPT ? c * NT + tid : ROUND + min(tid, 2 * radius));
      ld[c] = I[min(max(j, 0), m - 1)];
    }
#pragma unroll
    for (int c = 0; c < EPT; ++c) {
      const int s = c * NT + tid, j = base - radius + s;
      stage[pad_idx<EPT>(s)] = (j >= 0 && j < m) ? ld[c] : fill;
    }
    if (tid < 2 * radius) {
      const int s = ROUND + tid, j = base - radius + s;
      stage[pad_idx<EPT>(s)] = (j >= 0 && j < m) ? ld[EPT] : fill;
    }
    __syncthreads();
    // (behind the barrier: every score has arrived, and nothing waits for these loads before the end)
    {
      const int64_t tok = (int64_t)tab.tok_begin[seg] + m + win_row, h = tab.head[seg];
      win_k = *reinterpret_cast<const u32x4*>(ga.k + (h * ga.k_stride_head + tok * ga.k_stride_tok) * ga.elt_bytes + win_c * 16);
      win_v = *reinterpret_cast<const u32x4*>(ga.v + (h * ga.v_stride_head + tok * ga.v_stride_tok) * ga.elt_bytes + win_c * 16);
    }
    if (RADIUS >= 0) {
      constexpr int RR = RADIUS >= 0 ? RADIUS : 0;
      float v[EPT + 2 * RR];
#pragma unroll
      for (int e = 0; e < EPT + 2 * RR; ++e) v[e] = stage[pad_idx<EPT>(EPT * tid + e)];
      if (is_max) {
        uint32_t kv[EPT + 2 * RR], t3[EPT + 3];
#pragma unroll
        for (int e = 0; e < EPT + 2 * RR; ++e) kv[e] = score_key(v[e]);
        if (RR >= 2) {
#pragma unroll
          for (int e = 0; e < EPT + RR; ++e) t3[e] = max(max(kv[e], kv[e + 1]), kv[e + 2]);   // RR == 2 reads t3 up to EPT + 1, RR == 3 up to EPT + 2
        }
#pragma unroll
        for (int e = 0; e < EPT; ++e)
          key[e] = RR == 0 ? kv[e] : RR == 1 ? max(max(kv[e], kv[e + 1]), kv[e + 2]) : RR == 2 ? max(t3[e], t3[e + 2]) : max(max(t3[e], t3[e + 3]), kv[e + 6]);
      } else {
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
          float a = v[e];
#pragma unroll
          for (int t = 1; t <= 2 * RR; ++t) a += v[e + t];
          key[e] = score_key(a * inv_p);
        }
      }
    } else {
#pragma unroll 1
      for (int e = 0; e < EPT; ++e) {
        float a = stage[pad_idx<EPT>(EPT * tid + e)];
        for (int t = 1; t <= 2 * radius; ++t) {
          const float x = stage[pad_idx<EPT>(EPT * tid + e + t)];
          a = is_max ? fmaxf(a, x) : a + x;
        }
        key[e] = score_key(is_max ? a : a * inv_p);
      }
    }
    __syncthreads();
  };

  // pass 1: keys of the pooled scores, the largest key of each group of GS consecutive positions
  // (NQ groups per thread), the range of the keys over the segment, and (if asked) the pooled array
  constexpr int NQ = EPT < 4 ? EPT : 4, GS = EPT / NQ;
  uint32_t kmin = 0xffffffffu, kmax = 0u;
  uint32_t gmax[NQ];
  pool_all();
  SLKV_STAMP(128 + seg, 1);
#pragma unroll
  for (int q = 0; q < NQ; ++q) gmax[q] = 0u;
  if (j0 + EPT <= m) {                             // every thread but the last ones with positions
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      kmin = min(kmin, key[e]);
      gmax[e / GS] = max(gmax[e / GS], key[e]);
    }
  } else {
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      if (j0 + e < m) {
        kmin = min(kmin, key[e]);
        gmax[e / GS] = max(gmax[e / GS], key[e]);
      } else {
        key[e] = kKeyNone;
      }
    }
  }
#pragma unroll
  for (int q = 0; q < NQ; ++q) kmax = max(kmax, gmax[q]);
  if (write_pooled) {
#pragma unroll
    for (int e = 0; e < EPT; ++e)
      if (j0 + e < m) P[j0 + e] = __uint_as_float(key[e]);
  }
  kmin = wave_reduce_to_last(kmin, [](uint32_t a, uint32_t b) { return min(a, b); });
  kmax = wave_reduce_to_last(kmax, [](uint32_t a, uint32_t b) { return max(a, b); });
  if (lane == 63) {
    sh_mm[wv] = kmin;
    sh_mm[NT / 64 + wv] = kmax;
  }
  // histograms for the levels below, cleared here under the same barrier; the second one and the
  // digits' largest and smallest keys live at the start of the staging array, which is free now
  uint32_t* const aux_hist = reinterpret_cast<uint32_t*>(stage);
  uint32_t* const aux_max = aux_hist + kHistBins;
  uint32_t* const aux_min = aux_max + kHistBins;
  for (int i = tid; i < kHistBins; i += NT) {
    hist[i] = 0;
    aux_hist[i] = 0;
    aux_max[i] = 0;
    aux_min[i] = 0xffffffffu;
  }
  if (tid == 0) res[2] = 0;                        // counter of the first list (see below)
  __syncthreads();
  kmin = sh_mm[0];
  kmax = sh_mm[NT / 64];
#pragma unroll
  for (int i = 1; i < NT / 64; ++i) {
    kmin = min(kmin, sh_mm[i]);
    kmax = max(kmax, sh_mm[NT / 64 + i]);
  }

  SLKV_STAMP(128 + seg, 2);
  // The k-th largest key: radix select on (key - lo) >> shift with 11-bit digits taken relative to
  // the range [lo, hi] still in question.  After a digit search the keys of the chosen digit are
  // copied to a list in LDS (two areas in turn), the next level histograms that list, and a list of
  // at most kSelRankMax keys is ranked by direct counting.
  // Where at least k groups hold positions, two shortcuts come first.  The k-th largest of the
  // groups' maxima bounds the k-th largest key from below: its digit is found from a histogram of
  // one key per group, and the first level over all keys then counts only those from that digit's
  // lower edge upwards (a few times k, as a rule), in finer digits.  That level also keeps the
  // largest and smallest key of every digit: if the chosen digit holds one value only (with max
  // pooling a run of equal scores, as a rule), or its largest key is the one wanted, the search
  // ends there.
  uint32_t lo = kmin, hi = kmax, k = (uint32_t)kk;
  auto list_at = [&](int i) { return reinterpret_cast<uint32_t*>(stage) + (i ? kResStageFloats : kResAuxWords); };
  auto list_cap = [](int i) { return (uint32_t)(i ? kResCandidates : kSelRound - kResAuxWords); };
  int cur = -1;                                    // the list that holds the candidates; -1: the keys in registers
  uint32_t nlist = 0;
  int ncollect = 0;                                // lists made so far; list i counts its entries in res[2 + (i & 1)]
  bool hist_clean = true, unsynced = false;        // unsynced: results of a digit search read, no barrier since
  bool pending = false;                            // a digit has been chosen whose keys are not listed yet
  bool found = false;
  uint32_t cnt_sel = 0;
  const bool full = j0 + EPT <= m;                 // this thread holds no key of a position past the end
  auto shift_of = [](uint32_t span) {
    const int nbits = span ? 32 - __clz(span) : 0;
    return nbits > 11 ? nbits - 11 : 0;
  };
  // a list is made between two barriers: the counter of the one after it is cleared meanwhile
  auto begin_list = [&]() {
    if (tid == 0) res[2 + ((ncollect + 1) & 1)] = 0;
  };
  auto push = [&](int dst, uint32_t kv) __attribute__((always_inline)) {
    const uint32_t slot = atomicAdd(&res[2 + (ncollect & 1)], 1u);
    if (slot < list_cap(dst)) list_at(dst)[slot] = kv;
  };
  auto end_list = [&](int dst) {
    __syncthreads();
    nlist = min(res[2 + (ncollect & 1)], list_cap(dst));
    ++ncollect;
    cur = dst;
    unsynced = false;
  };
  // Histogram step for segments with piles of equal keys (thousands of LDS atomics on one address
  // would serialise): the lanes of the wave whose key equals that of the first counted lane are
  // added by that lane in one atomic, likewise those equal to the first counted lane left over;
  // the other counted lanes add themselves.
  bool ties = false;
  auto count_pile = [&](bool in, uint32_t kv, uint32_t d, uint32_t* h, bool with_range) __attribute__((always_inline)) {
    const unsigned long long act = __builtin_amdgcn_ballot_w64(in);
    if (act) {                                     // (the same for the whole wave, like `rest` below)
      const int first = __builtin_ctzll(act);
      const bool same = in && kv == (uint32_t)__builtin_amdgcn_readlane((int)kv, first);
      const unsigned long long sm = __builtin_amdgcn_ballot_w64(same);
      bool mine = in;
      uint32_t add = 1u;
      if (same) {
        mine = lane == first;
        add = (uint32_t)__popcll(sm);
      }
      const unsigned long long rest = act & ~sm;
      if (rest) {
        const int second = __builtin_ctzll(rest);
        const bool same2 = in && kv == (uint32_t)__builtin_amdgcn_readlane((int)kv, second);
        if (same2) {
          mine = lane == second;
          add = (uint32_t)__popcll(__builtin_amdgcn_ballot_w64(same2));
        }
      }
      if (mine) {
        atomicAdd(&h[d], add);
        if (with_range) {
          atomicMax(&aux_max[d], kv);
          atomicMin(&aux_min[d], kv);
        }
      }
    }
  };
  const uint32_t groups = (uint32_t)((m + GS - 1) / GS);     // groups that hold at least one position
  if (k <= groups) {
    {
      const int shift = shift_of(hi - lo);
#pragma unroll
      for (int q = 0; q < NQ; ++q)
        if (j0 + q * GS < m) atomicAdd(&hist[(gmax[q] - lo) >> shift], 1u);
      __syncthreads();
      SLKV_STAMP(128 + seg, 3);
      select_bin<NT>(hist, k, sh_scan, res);
      SLKV_STAMP(128 + seg, 4);
      ties = hist[res[0]] >= (uint32_t)kSelTieGroups;   // many groups share one digit: expect piles of equal keys
      lo += res[0] << shift;                       // k groups hold a key >= lo, so the k-th largest key is >= lo
      hist_clean = false;
    }
    const uint32_t span1 = hi - lo;
    const int shift = shift_of(span1);
    if (span1 == 0u) {
      found = true;                                // k groups or more hold the largest key (all scores equal, for one): it is the threshold
    } else {
    const bool track = ties || k <= (uint32_t)kSelTrackMax;   // (with many keys wanted the two extra atomics per counted key cost more than they save)
    if (ties) {
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        const uint32_t dk = key[e] - lo;
        count_pile(dk <= span1, key[e], dk >> shift, aux_hist, true);
      }
    } else if (track) {
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        const uint32_t dk = key[e] - lo;             // (a key below lo wraps to a difference above any span)
        if (dk <= span1) {
          const uint32_t d = dk >> shift;
          atomicAdd(&aux_hist[d], 1u);
          atomicMax(&aux_max[d], key[e]);
          atomicMin(&aux_min[d], key[e]);
        }
      }
    } else {
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        const uint32_t dk = key[e] - lo;
        if (dk <= span1) atomicAdd(&aux_hist[dk >> shift], 1u);
      }
    }
    __syncthreads();
    select_bin<NT>(aux_hist, k, sh_scan, res);
    const uint32_t bsel = res[0];
    const uint32_t top = aux_max[bsel], bottom = aux_min[bsel];
    cnt_sel = aux_hist[bsel];
    k = res[1];
    unsynced = true;
    lo = lo + (bsel << shift);
    hi = min(hi, lo + ((1u << shift) - 1u));
    if (track && (top == bottom || k == 1u)) {
      lo = top;                                    // one value in the digit, or the largest of the digit is wanted
      found = true;
    } else if (shift == 0) {
      found = true;                                // the digit is the key
    } else {
      pending = true;
    }
    }
  }
  while (!found) {
    if (pending) {
      // the keys of the chosen digit go to the other list (their order does not matter for counting)
      pending = false;
      const int dst = cur == 0 ? 1 : 0;
      if (cnt_sel <= (cur >= 0 ? list_cap(dst) : (uint32_t)kResCandidates)) {   // (from registers every copied key costs an LDS atomic with its latency)
        begin_list();
        const uint32_t span2 = hi - lo;
        if (cur >= 0) {
          const uint32_t* cand = list_at(cur);
          for (uint32_t i = tid; i < nlist; i += NT) {
            const uint32_t kv = cand[i];
            if (kv - lo <= span2) push(dst, kv);
          }
        } else {
#pragma unroll
          for (int e = 0; e < EPT; ++e)
            if (key[e] - lo <= span2) push(dst, key[e]);
        }
        end_list(dst);
      }
    }
    const uint32_t span1 = hi - lo;
    const int shift = shift_of(span1);
    if (cur >= 0 && nlist <= (uint32_t)kSelRankMax) {
      // short list: the k-th largest by counting, for each entry, the entries above it (four
      // entries a step; both list areas are longer than any index read here)
      const uint32_t* cand = list_at(cur);
      if ((uint32_t)tid < nlist) {
        const uint32_t kv = cand[tid];
        uint32_t gt = 0, ge = 0;
        for (uint32_t i = 0; i < nlist; i += 4) {
#pragma unroll
          for (uint32_t u = 0; u < 4; ++u) {
            const uint32_t o = cand[i + u];
            const bool live = i + u < nlist;
            gt += (live && o > kv) ? 1u : 0u;
            ge += (live && o >= kv) ? 1u : 0u;
          }
        }
        if (gt < k && k <= ge) {   // every thread holding the k-th largest value writes the same pair
          res[0] = kv;
          res[1] = k - gt;
        }
      }
      __syncthreads();
      lo = res[0];
      k = res[1];
      break;
    }
    if (!hist_clean) {
      if (unsynced) __syncthreads();               // every thread has read the counts and results of the level before
      for (int i = tid; i < kHistBins; i += NT) hist[i] = 0;
      __syncthreads();
    }
    if (cur >= 0) {
      const uint32_t* cand = list_at(cur);
      for (uint32_t i = tid; i < nlist; i += NT) {
        const uint32_t dk = cand[i] - lo;
        if (dk <= span1) atomicAdd(&hist[dk >> shift], 1u);
      }
    } else if (ties) {
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        const uint32_t dk = key[e] - lo;
        count_pile(dk <= span1, key[e], dk >> shift, hist, false);
      }
    } else if (hist_clean && full) {
      // lo and hi are the smallest and largest key of the segment: nothing to test
#pragma unroll
      for (int e = 0; e < EPT; ++e) atomicAdd(&hist[(key[e] - lo) >> shift], 1u);
    } else {
      // in [lo, hi] <=> key - lo <= hi - lo: a key below lo wraps to a difference above any span,
      // and kKeyNone lies above every hi
#pragma unroll
      for (int e = 0; e < EPT; ++e) {
        const uint32_t dk = key[e] - lo;
        if (dk <= span1) atomicAdd(&hist[dk >> shift], 1u);
      }
    }
    __syncthreads();
    if (hist_clean) SLKV_STAMP(128 + seg, 3);
    select_bin<NT>(hist, k, sh_scan, res);
    if (hist_clean) SLKV_STAMP(128 + seg, 4);
    const uint32_t bsel = res[0];
    cnt_sel = hist[bsel];
    k = res[1];
    hist_clean = false;
    unsynced = true;
    lo = lo + (bsel << shift);
    hi = min(hi, lo + ((1u << shift) - 1u));
    if (shift == 0) break;
    pending = true;
  }
  const uint32_t tau = lo, need_eq = k;
  SLKV_STAMP(128 + seg, 5);

  // ordered compaction: slot = (#greater before) + min(#equal before, need_eq)
  {
    uint32_t gmask = 0, emask = 0;                 // bit e: element e is above / equal to the threshold
    const uint32_t upto = kKeyNone - tau;           // tau <= key < kKeyNone <=> key - tau < upto
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      const uint32_t dk = key[e] - tau;
      const bool in = dk < upto;
      if (__builtin_amdgcn_ballot_w64(in)) {        // few positions are kept: most waves skip most steps
        gmask |= (in && dk != 0u) ? (1u << e) : 0u;
        emask |= dk == 0u ? (1u << e) : 0u;
      }
    }
    const uint32_t cg = __popc(gmask), ce = __popc(emask);
    const uint32_t packed = (ce << 16) | cg;       // the round holds at most 32768 of either
    const uint32_t incl = block_incl_scan<NT, false>(packed, sh_scan);   // sh_scan is not used again
    const uint32_t excl = incl - packed;
    const uint32_t g_before = excl & 0xffffu, e_before = excl >> 16;
    // ties are taken in position order: this thread keeps its first `take` equal elements
    uint32_t take = 0;
    if (e_before < need_eq) take = (need_eq - e_before) < ce ? (need_eq - e_before) : ce;
    uint32_t sel = gmask;
    for (uint32_t em = emask; take > 0; --take) {
      sel |= em & (0u - em);                       // lowest set bit
      em &= em - 1u;
    }
    uint32_t pos = g_before + (e_before < need_eq ? e_before : need_eq);
    while (sel) {
      const int e = __ffs(sel) - 1;
      emit((int)pos++, j0 + e);
      sel &= sel - 1u;
    }
  }
  for (int j = tid; j < w; j += NT) emit(kk + j, m + j);
  SLKV_STAMP(128 + seg, 6);
  }  // ranked

  // Small segments copy their K/V rows here (saves the gather launch); larger ones are left
  // to gather_kernel, which skips the segments handled here.  Four pieces per thread are in
  // flight at a time.
  if (kept > 0 && small_seg) {
    __syncthreads();                                // sh_pos is complete
    const int64_t tok0 = tab.tok_begin[seg], h = tab.head[seg], row0 = tab.out_off[seg];
    const bool win_done = ranked && win_early;      // the window's pieces are in registers
    const int pieces = (win_done ? kk : kept) * lpr;
    const uint32_t magic = 0xffffffffu / (uint32_t)lpr + 1u;   // idx / lpr == umulhi(idx, magic) for idx < 2^16 (lpr > 1)
    struct Piece {
      u32x4 kq, vq;
      int row, c;
      int64_t tok;
    };
    auto fetch = [&](int idx, Piece& q) __attribute__((always_inline)) {
      q.row = lpr == 1 ? idx : (int)__umulhi((uint32_t)idx, magic);
      q.c = idx - q.row * lpr;
      if (idx < pieces) {
        q.tok = tok0 + sh_pos[q.row];
        q.kq = *reinterpret_cast<const u32x4*>(ga.k + (h * ga.k_stride_head + q.tok * ga.k_stride_tok) * ga.elt_bytes + q.c * 16);
        q.vq = *reinterpret_cast<const u32x4*>(ga.v + (h * ga.v_stride_head + q.tok * ga.v_stride_tok) * ga.elt_bytes + q.c * 16);
      }
    };
    auto put = [&](int idx, const Piece& q) __attribute__((always_inline)) {
      if (idx < pieces) {
        const int64_t o = ((row0 + q.row) * lpr + q.c) * 16;
        *reinterpret_cast<u32x4*>(ga.k_out + o) = q.kq;
        *reinterpret_cast<u32x4*>(ga.v_out + o) = q.vq;
        if (ga.pos_out && q.c == 0) ga.pos_out[row0 + q.row] = ga.pos_in[q.tok];
      }
    };
    for (int base = tid; base < pieces; base += 4 * NT) {
      Piece q0, q1, q2, q3;
      fetch(base, q0);
      fetch(base + NT, q1);
      fetch(base + 2 * NT, q2);
      fetch(base + 3 * NT, q3);
      put(base, q0);
      put(base + NT, q1);
      put(base + 2 * NT, q2);
      put(base + 3 * NT, q3);
    }
    if (win_done && win_mine) {
      const int64_t o = ((row0 + kk + win_row) * lpr + win_c) * 16;
      *reinterpret_cast<u32x4*>(ga.k_out + o) = win_k;
      *reinterpret_cast<u32x4*>(ga.v_out + o) = win_v;
      if (ga.pos_out && win_c == 0) ga.pos_out[row0 + kk + win_row] = ga.pos_in[tok0 + m + win_row];
    }
  }
  SLKV_STAMP(128 + seg, 7);
}

// Copies kept rows of K and V (bit copies) into the packed output; one 16-byte lane per piece.
template <class TAB>
__global__ __launch_bounds__(256) void gather_kernel(const TAB tab, const GatherArgs ga,
                                                     const int32_t* __restrict__ kept_idx, int all_segments) {
  const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t rel = g / ga.lanes_per_row;
  const int c = (int)(g % ga.lanes_per_row);
  const int64_t row0 = tab.out_off[0], row1 = tab.out_off[tab.nseg];
  const int64_t row = row0 + rel;
  if (row >= row1) return;
  const int seg = find_segment(tab.out_off, tab.nseg, (int)row);
  if (!all_segments && tab.out_off[seg + 1] - tab.out_off[seg] <= kInlineGatherRows) return;   // done by the selection kernel
  // (a position outside the segment cannot come out of the selection; clamped all the same, so
  // that no input can turn into an out-of-bounds read here)
  const int64_t tok = (int64_t)tab.tok_begin[seg] + min(max(kept_idx[row], 0), max(tab.n[seg] - 1, 0));
  const int64_t h = tab.head[seg];
  const uint4 kv = *reinterpret_cast<const uint4*>(ga.k + (h * ga.k_stride_head + tok * ga.k_stride_tok) * ga.elt_bytes + c * 16);
  const uint4 vv = *reinterpret_cast<const uint4*>(ga.v + (h * ga.v_stride_head + tok * ga.v_stride_tok) * ga.elt_bytes + c * 16);
  const int64_t o = (row * ga.lanes_per_row + c) * 16;
  *reinterpret_cast<uint4*>(ga.k_out + o) = kv;
  *reinterpret_cast<uint4*>(ga.v_out + o) = vv;
  if (ga.pos_out && c == 0) ga.pos_out[row] = ga.pos_in[tok];
}

// Copies one kernel-argument table (up to kMaxSegPerLaunch segments starting at segment s0) into
// the device-resident table.  The prefix arrays get one entry more.
__global__ void table_write_kernel(const SegTable part, int s0, const SegTableDev dst) {
  const int i = threadIdx.x;
  if (i < part.nseg) {
    dst.tok_begin[s0 + i] = part.tok_begin[i];
    dst.n[s0 + i] = part.n[i];
    dst.kkeep[s0 + i] = part.kkeep[i];
    dst.head[s0 + i] = part.head[i];
    dst.qrow_off[s0 + i] = part.qrow_off[i];
    dst.score_off[s0 + i] = part.score_off[i];
    dst.seg_global[s0 + i] = part.seg_global[i];
    dst.hblk[s0 + i] = part.hblk[i];
    dst.tick[s0 + i] = part.tick[i];
  }
  if (i <= part.nseg) {
    dst.out_off[s0 + i] = part.out_off[i];
    dst.chunk_begin[s0 + i] = part.chunk_begin[i];
    dst.blk_begin[s0 + i] = part.blk_begin[i];
  }
}

// ------------------------------------------------------------------------------------------
// Host side: planning, validation, launches.

// One (sequence, KV head) segment as the kernels see it.
struct Seg {
  int64_t row_begin;   // first token row of the segment (multiplied by the token stride)
  int64_t n;           // rows in the segment; the last w are the window
  int64_t cap;         // capacity C of its head
  int32_t head;        // multiplied by the head stride (0 for a ragged cache)
  int64_t qrow_off;    // first row of the segment's [G*w][d] query block
  int64_t score_off;   // offset of the segment in the importance / pooled arrays
};

// What both entry points reduce to: common shape parameters plus the list of segments.
struct Geometry {
  int dtype, Hq, Hkv, d, w, pool_kernel, pool;
  int64_t k_stride_tok, k_stride_head, v_stride_tok, v_stride_head;
  int64_t score_elems;   // length of the importance / pooled arrays
  std::vector<Seg> segs;
};

struct Plan {
  int R, Rpad, CH;
  int64_t hist_blocks;   // block histograms of the selection
  int64_t ticketed;      // segments that need a ticket slot
  size_t part_bytes, lse_bytes, score_bytes, hist_bytes, table_bytes;
  size_t off_part, off_lse, off_imp, off_pooled, off_hist, off_table, total_bytes;
};

static bool seg_ranked(int64_t n, int64_t w, int64_t cap) { return n > w && n > cap && cap > w; }
// key chunks of the scoring passes and blocks of the selection for one segment
static int64_t seg_chunks(const Seg& s, int w, int64_t ch) { return seg_ranked(s.n, w, s.cap) ? (s.n - w + ch - 1) / ch : 0; }
static int64_t seg_blocks(const Seg& s, int w) { return seg_ranked(s.n, w, s.cap) ? (s.n - w + kSelBlock - 1) / kSelBlock : 0; }

static void make_plan(const Geometry& g, Plan& p) {
  p.R = (g.Hq / g.Hkv) * g.w;
  p.Rpad = (p.R + 31) / 32 * 32;
  // keys to score over all ranked segments -> chunk length giving about 512 workgroups
  int64_t keys = 0;
  for (const Seg& s : g.segs)
    if (seg_ranked(s.n, g.w, s.cap)) keys += s.n - g.w;
  int64_t ch = (keys + 511) / 512;
  if (g.dtype != SLKV_F32) {                  // MFMA kernels: pairs of 64-key tiles
    ch = (ch + 127) / 128 * 128;
    ch = std::max<int64_t>(256, std::min<int64_t>(ch, 1 << 16));
  } else {                                    // fp32 kernels: 32-key tiles
    ch = (ch + 31) / 32 * 32;
    ch = std::max<int64_t>(32, std::min<int64_t>(ch, 1 << 16));
  }
  // All chunks should be resident at once (two 256-thread workgroups per CU on 256 CUs): the
  // partial last chunk of every segment can push the count a little over that, and the surplus
  // workgroups would then run alone in a second round that doubles the kernel's time.  Lengthen
  // the chunk, by up to a quarter, until the count fits.
  {
    constexpr int64_t kSlots = 512;
    const int64_t granule = g.dtype != SLKV_F32 ? 128 : 32;
    auto count = [&](int64_t c) {
      int64_t total = 0;
      for (const Seg& s : g.segs)
        if (seg_ranked(s.n, g.w, s.cap)) total += (s.n - g.w + c - 1) / c;
      return total;
    };
    if (count(ch) > kSlots)
      for (int64_t c = ch + granule; c <= ch + ch / 4 && c <= (1 << 16); c += granule)
        if (count(c) <= kSlots) {
          ch = c;
          break;
        }
  }
  p.CH = (int)ch;
  int64_t chunks = 0;
  p.hist_blocks = 0;
  p.ticketed = 0;
  for (const Seg& s : g.segs) {
    const int64_t nc = seg_chunks(s, g.w, ch), nb = seg_blocks(s, g.w);
    chunks += nc;
    p.hist_blocks += nb;
    if (nc > 1) p.ticketed += 1;
  }
  auto align = [](size_t x) { return (x + 255) / 256 * 256; };
  p.part_bytes = align((size_t)std::max<int64_t>(chunks, 1) * p.Rpad * sizeof(float));
  p.lse_bytes = align(std::max<size_t>(g.segs.size(), 1) * p.Rpad * sizeof(float));
  p.score_bytes = align((size_t)std::max<int64_t>(1, g.score_elems) * sizeof(float));
  p.hist_bytes = align((size_t)p.hist_blocks * kHistBins * sizeof(uint32_t));
  p.off_part = kTicketBytes;                   // the ticket words come first
  p.off_lse = p.off_part + p.part_bytes;
  p.off_imp = p.off_lse + p.lse_bytes;
  p.off_pooled = p.off_imp + p.score_bytes;
  p.off_hist = p.off_pooled + p.score_bytes;
  p.off_table = p.off_hist + p.hist_bytes;
  // device-resident segment table: only for calls with more segments than one kernel argument holds
  const size_t S = g.segs.size();
  p.table_bytes = S > (size_t)kMaxSegPerLaunch ? align((12 * S + 3) * sizeof(int32_t)) : 0;
  p.total_bytes = p.off_table + p.table_bytes;
}

static void layer_geometry(const slkv_layer_desc* d, Geometry& g) {
  g.dtype = d->dtype; g.Hq = d->Hq; g.Hkv = d->Hkv; g.d = d->d; g.w = d->w;
  g.pool_kernel = d->pool_kernel; g.pool = d->pool;
  g.k_stride_tok = d->k_stride_tok; g.k_stride_head = d->k_stride_head;
  g.v_stride_tok = d->v_stride_tok; g.v_stride_head = d->v_stride_head;
  g.score_elems = (int64_t)d->Hkv * d->h_cu_seqlens[d->B];
  const int G = d->Hq / d->Hkv;
  g.segs.resize((size_t)d->B * d->Hkv);
  for (int b = 0; b < d->B; ++b) {
    const int64_t n = d->h_cu_seqlens[b + 1] - d->h_cu_seqlens[b];
    for (int h = 0; h < d->Hkv; ++h) {
      Seg& s = g.segs[(size_t)b * d->Hkv + h];
      s.row_begin = d->h_cu_seqlens[b];
      s.n = n;
      s.cap = d->h_budgets[h];
      s.head = h;
      s.qrow_off = ((int64_t)b * d->Hq + (int64_t)h * G) * d->w;
      s.score_off = (int64_t)d->Hkv * d->h_cu_seqlens[b] + (int64_t)h * n;
    }
  }
}

static void ragged_geometry(const slkv_ragged_desc* d, Geometry& g) {
  g.dtype = d->dtype; g.Hq = d->Hq; g.Hkv = d->Hkv; g.d = d->d; g.w = d->w;
  g.pool_kernel = d->pool_kernel; g.pool = d->pool;
  g.k_stride_tok = g.v_stride_tok = d->d;     // packed rows
  g.k_stride_head = g.v_stride_head = 0;      // a segment's rows are addressed by row_begin alone
  const int S = d->B * d->Hkv;
  g.score_elems = d->h_in_offsets[S] - d->h_in_offsets[0];
  const int G = d->Hq / d->Hkv;
  g.segs.resize((size_t)S);
  for (int i = 0; i < S; ++i) {
    const int b = i / d->Hkv, h = i % d->Hkv;
    Seg& s = g.segs[(size_t)i];
    s.row_begin = d->h_in_offsets[i];
    s.n = d->h_in_offsets[i + 1] - d->h_in_offsets[i];
    s.cap = d->h_budgets[h];
    s.head = 0;
    s.qrow_off = ((int64_t)b * d->Hq + (int64_t)h * G) * d->w;
    s.score_off = d->h_in_offsets[i] - d->h_in_offsets[0];
  }
}

// Grid of a scoring launch: `chunks` workgroups in a row, or (rows > 0) one row of `per_row`
// workgroups per segment.
struct ScoreGrid {
  int chunks, per_row, rows;
};

template <int DK, int MT, int RB, int KIND, class TAB>
static void launch_bf16(int pass, ScoreGrid grid, hipStream_t st, const TAB& tab, const void* q, const void* k,
                        const Geometry& g, const Plan& p, float c_log2, float* part, float* lse, float* imp,
                        uint32_t* tickets) {
  // segments with like chunk counts: one grid row per segment (see the kernel's first lines)
  const bool two = grid.rows > 0;
  const dim3 gr = two ? dim3((unsigned)grid.per_row, (unsigned)grid.rows) : dim3((unsigned)grid.chunks);
  if (pass == 1)
    SLKV_LAUNCH((score_bf16_kernel<DK, MT, RB, 1, KIND, TAB>), gr, dim3(256), 0, st, tab, (const uint16_t*)q,
                       k, g.k_stride_tok, g.k_stride_head, p.R, p.Rpad, g.w, p.CH, c_log2, part, lse, imp,
                       lse, tickets, two ? 1 : 0);
  else
    SLKV_LAUNCH((score_bf16_kernel<DK, MT, RB, 2, KIND, TAB>), gr, dim3(256), 0, st, tab, (const uint16_t*)q,
                       k, g.k_stride_tok, g.k_stride_head, p.R, p.Rpad, g.w, p.CH, c_log2, part, lse, imp,
                       lse, tickets, two ? 1 : 0);
}

template <int DK, int KIND, class TAB>
static void launch_bf16_rows(int pass, ScoreGrid grid, hipStream_t st, const TAB& tab, const void* q, const void* k,
                             const Geometry& g, const Plan& p, float c_log2, float* part, float* lse, float* imp,
                             uint32_t* tickets) {
  if (p.R <= 64) launch_bf16<DK, 1, 2, KIND>(pass, grid, st, tab, q, k, g, p, c_log2, part, lse, imp, tickets);
  else if (p.R <= 128) launch_bf16<DK, 2, 2, KIND>(pass, grid, st, tab, q, k, g, p, c_log2, part, lse, imp, tickets);
  else if (p.R <= 256) launch_bf16<DK, 2, 4, KIND>(pass, grid, st, tab, q, k, g, p, c_log2, part, lse, imp, tickets);
  else launch_bf16<DK, 4, 4, KIND>(pass, grid, st, tab, q, k, g, p, c_log2, part, lse, imp, tickets);
}

template <class TAB>
static void launch_score(int pass, ScoreGrid grid, hipStream_t st, const TAB& tab, const void* q, const void* k,
                         const Geometry& g, const Plan& p, float c_log2, float* part, float* lse, float* imp,
                         uint32_t* tickets) {
  if (g.dtype == SLKV_BF16) {
    if (g.d == 128) launch_bf16_rows<128, 0>(pass, grid, st, tab, q, k, g, p, c_log2, part, lse, imp, tickets);
    else launch_bf16_rows<64, 0>(pass, grid, st, tab, q, k, g, p, c_log2, part, lse, imp, tickets);
  } else if (g.dtype == SLKV_F16) {
    if (g.d == 128) launch_bf16_rows<128, 1>(pass, grid, st, tab, q, k, g, p, c_log2, part, lse, imp, tickets);
    else launch_bf16_rows<64, 1>(pass, grid, st, tab, q, k, g, p, c_log2, part, lse, imp, tickets);
  } else if (g.dtype == SLKV_BF16_KV_FP8) {
    if (g.d == 128) launch_bf16_rows<128, 2>(pass, grid, st, tab, q, k, g, p, c_log2, part, lse, imp, tickets);
    else launch_bf16_rows<64, 2>(pass, grid, st, tab, q, k, g, p, c_log2, part, lse, imp, tickets);
  } else {
#define SLKV_F32_LAUNCH(DKV, PS)                                                                                     \
  SLKV_LAUNCH((score_f32_kernel<DKV, PS, TAB>), dim3(grid.chunks), dim3(256), 0, st, tab, (const float*)q, (const float*)k, \
                     g.k_stride_tok, g.k_stride_head, p.R, p.Rpad, g.w, p.CH, c_log2, part, lse, imp, lse, tickets)
    if (g.d == 128) { if (pass == 1) SLKV_F32_LAUNCH(128, 1); else SLKV_F32_LAUNCH(128, 2); }
    else { if (pass == 1) SLKV_F32_LAUNCH(64, 1); else SLKV_F32_LAUNCH(64, 2); }
#undef SLKV_F32_LAUNCH
  }
}

template <class TAB>
static void launch_select(int nseg, int blocks, hipStream_t st, const TAB& tab, const Geometry& g, const float* imp,
                          float* pooled, uint32_t* blockhist, uint32_t* lists, int32_t* kept_idx, int64_t* d_out_offsets,
                          const GatherArgs& ga) {
  const int radius = g.pool == SLKV_POOL_NONE ? 0 : g.pool_kernel / 2;
  const int pool_kernel = g.pool == SLKV_POOL_NONE ? 1 : g.pool_kernel;
#define SLKV_POOL_LAUNCH(RAD)                                                                                          \
  SLKV_LAUNCH((select_pool_kernel<RAD, TAB>), dim3(blocks), dim3(kSelThreads), 0, st, tab, g.w, pool_kernel, g.pool, imp, \
              pooled, blockhist)
  if (blocks > 0) {
    switch (radius) {
      case 0: SLKV_POOL_LAUNCH(0); break;
      case 1: SLKV_POOL_LAUNCH(1); break;
      case 2: SLKV_POOL_LAUNCH(2); break;
      case 3: SLKV_POOL_LAUNCH(3); break;
      default: SLKV_POOL_LAUNCH(-1); break;
    }
  }
#undef SLKV_POOL_LAUNCH
  // with blocks, the ordered compaction runs per block (two short launches over the whole chip)
  // instead of per segment inside the ranking workgroup
  const int split = blocks > 0 ? 1 : 0;
  int64_t longest = 0;
  for (const Seg& sg : g.segs) longest = std::max<int64_t>(longest, seg_blocks(sg, g.w));
  // block-wise launches: a grid row per segment unless that would launch mostly empty workgroups
  // (one long history among many short ones) or more rows than a grid has
  const bool rows = nseg <= 65535 && longest * nseg <= 4 * (int64_t)blocks;
  const dim3 grid = rows ? dim3((unsigned)std::max<int64_t>(longest, 1), (unsigned)nseg) : dim3((unsigned)std::max(blocks, 1));
  if (split) {
    // first-level digit per segment, then the blocks list the scores of that digit
    SLKV_LAUNCH(select_rank_kernel<TAB>, dim3(nseg), dim3(kSelThreads), 0, st, tab, g.w, (const float*)pooled,
                blockhist, kept_idx, d_out_offsets, ga, split, (const uint32_t*)lists, 0);
    SLKV_LAUNCH(select_collect_kernel<TAB>, grid, dim3(kSelEmitThreads), 0, st, tab, g.w, (const float*)pooled, blockhist,
                lists, rows ? 0 : -1);
  }
  SLKV_LAUNCH(select_rank_kernel<TAB>, dim3(nseg), dim3(kSelThreads), 0, st, tab, g.w, (const float*)pooled,
              blockhist, kept_idx, d_out_offsets, ga, split, (const uint32_t*)lists, 1);
  if (split) {
    SLKV_LAUNCH(select_count_kernel<TAB>, grid, dim3(kSelEmitThreads), 0, st, tab, g.w, (const float*)pooled, blockhist,
                rows ? 0 : -1);
    SLKV_LAUNCH(select_emit_kernel<TAB>, grid, dim3(kSelEmitThreads), 0, st, tab, g.w, (const float*)pooled,
                (const uint32_t*)blockhist, kept_idx, rows ? 0 : -1);
  }
}

// select_resident_kernel needs more LDS than a kernel gets by default: the limit is raised for all
// of its instances once per device, by slkv_init() or by the first call that selects on that
// device (setting it is not a stream operation, but the first call on a device should still not
// be the one a graph capture records).
template <int RADIUS, int EPT>
static hipError_t raise_lds_limit() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&select_resident_kernel<RADIUS, EPT, SegTable>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)kResLdsBytes);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&select_resident_kernel<RADIUS, EPT, SegTableDev>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)kResLdsBytes);
}

template <int EPT>
static hipError_t raise_lds_limits() {
  hipError_t e;
  if ((e = raise_lds_limit<0, EPT>()) != hipSuccess) return e;
  if ((e = raise_lds_limit<1, EPT>()) != hipSuccess) return e;
  if ((e = raise_lds_limit<2, EPT>()) != hipSuccess) return e;
  if ((e = raise_lds_limit<3, EPT>()) != hipSuccess) return e;
  return raise_lds_limit<-1, EPT>();
}

static hipError_t ensure_device_init() {
  static std::mutex mu;
  static uint64_t done = 0;                      // bit per device
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  std::lock_guard<std::mutex> lk(mu);
  const uint64_t bit = dev >= 0 && dev < 64 ? (uint64_t(1) << dev) : 0;
  if (done & bit) return hipSuccess;
  if ((e = raise_lds_limits<kSelEPT>()) != hipSuccess) return e;
  if ((e = raise_lds_limits<kSelEPTMid>()) != hipSuccess) return e;
  if ((e = raise_lds_limits<kSelEPTSmall>()) != hipSuccess) return e;
  done |= bit;
  return hipSuccess;
}

template <int RADIUS, int EPT, class TAB>
static hipError_t launch_select_resident_e(int ns, hipStream_t st, const TAB& tab, const Geometry& g, bool write_pooled,
                                           const float* imp, float* pooled, int32_t* kept_idx, int64_t* d_out_offsets,
                                           const GatherArgs& ga) {
  const hipError_t e = ensure_device_init();
  if (e != hipSuccess) return e;
  const int pool_kernel = g.pool == SLKV_POOL_NONE ? 1 : g.pool_kernel;
  SLKV_LAUNCH((select_resident_kernel<RADIUS, EPT, TAB>), dim3(ns), dim3(kSelThreads), kResLdsBytes, st, tab, g.w,
                     pool_kernel, g.pool, (int)write_pooled, imp, pooled, kept_idx, d_out_offsets, ga);
  return hipSuccess;
}

// Positions per thread: the fewest of 2, 8, 32 whose round holds the longest ranked history (every
// wave runs through all of a thread's positions, whether or not the history reaches them).
template <int RADIUS, class TAB>
static hipError_t launch_select_resident_r(int ns, hipStream_t st, const TAB& tab, const Geometry& g, bool write_pooled,
                                           const float* imp, float* pooled, int32_t* kept_idx, int64_t* d_out_offsets,
                                           const GatherArgs& ga) {
  int64_t longest = 0;
  for (const Seg& sg : g.segs)
    if (seg_ranked(sg.n, g.w, sg.cap)) longest = std::max<int64_t>(longest, sg.n - g.w);
  if (longest <= kSelThreads * kSelEPTSmall)
    return launch_select_resident_e<RADIUS, kSelEPTSmall>(ns, st, tab, g, write_pooled, imp, pooled, kept_idx, d_out_offsets, ga);
  if (longest <= kSelThreads * kSelEPTMid)
    return launch_select_resident_e<RADIUS, kSelEPTMid>(ns, st, tab, g, write_pooled, imp, pooled, kept_idx, d_out_offsets, ga);
  return launch_select_resident_e<RADIUS, kSelEPT>(ns, st, tab, g, write_pooled, imp, pooled, kept_idx, d_out_offsets, ga);
}

template <class TAB>
static hipError_t launch_select_resident(int ns, hipStream_t st, const TAB& tab, const Geometry& g, bool write_pooled,
                                         const float* imp, float* pooled, int32_t* kept_idx, int64_t* d_out_offsets,
                                         const GatherArgs& ga) {
  const int radius = g.pool == SLKV_POOL_NONE ? 0 : g.pool_kernel / 2;
  switch (radius) {
    case 0: return launch_select_resident_r<0>(ns, st, tab, g, write_pooled, imp, pooled, kept_idx, d_out_offsets, ga);
    case 1: return launch_select_resident_r<1>(ns, st, tab, g, write_pooled, imp, pooled, kept_idx, d_out_offsets, ga);
    case 2: return launch_select_resident_r<2>(ns, st, tab, g, write_pooled, imp, pooled, kept_idx, d_out_offsets, ga);
    case 3: return launch_select_resident_r<3>(ns, st, tab, g, write_pooled, imp, pooled, kept_idx, d_out_offsets, ga);
    default: return launch_select_resident_r<-1>(ns, st, tab, g, write_pooled, imp, pooled, kept_idx, d_out_offsets, ga);
  }
}

// SLKV_SELECT=resident|blocks in the environment forces one selection kernel (tests run both on
// every shape the resident one covers); default: chosen per call.  0 auto, 1 resident, 2 blocks.
static int select_mode() {
  const char* e = std::getenv("SLKV_SELECT");
  if (!e) return 0;
  if (!std::strcmp(e, "resident")) return 1;
  if (!std::strcmp(e, "blocks")) return 2;
  return 0;
}

// Checks and launches shared by the two entry points.
static slkv_status run_geometry(const Geometry& g, const void* d_qwin, const void* d_k, const void* d_v,
                                const int32_t* d_pos_in, void* d_k_out, void* d_v_out, int32_t* d_kept_idx,
                                int32_t* d_pos_out, int64_t* d_out_offsets, float* d_importance, float* d_pooled,
                                int64_t out_capacity_rows, void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  // an input without rows, or an output without kept rows, may come with NULL buffers
  int64_t rows_in = 0, rows_kept = 0;
  for (const Seg& sg : g.segs) {
    rows_in += sg.n;
    rows_kept += kept_rows(sg.n, g.w, sg.cap);
  }
  if (!d_qwin || !d_workspace || (rows_in > 0 && (!d_k || !d_v)) ||
      (rows_kept > 0 && (!d_k_out || !d_v_out || !d_kept_idx)))
    return fail(SLKV_ERR_NULL, "a required device pointer is NULL");
  if (rows_kept > 0 && (d_pos_in == nullptr) != (d_pos_out == nullptr))
    return fail(SLKV_ERR_NULL, "d_pos_in and d_pos_out must be given together");
  if (!d_pos_in || !d_pos_out) d_pos_in = nullptr, d_pos_out = nullptr;   // nothing kept: nothing to carry

  const void* ptrs[] = {d_qwin, d_k, d_v, d_pos_in, d_k_out, d_v_out, d_kept_idx, d_pos_out, d_out_offsets,
                        d_importance, d_pooled, d_workspace};
  for (const void* ptr : ptrs)
    if (reinterpret_cast<uintptr_t>(ptr) % 16) return fail(SLKV_ERR_BAD_ARG, "device pointer %p not 16-byte aligned", ptr);
  const int elt = g.dtype == SLKV_F32 ? 4 : (g.dtype == SLKV_BF16_KV_FP8 ? 1 : 2);   // bytes per element of K and V
  const int64_t S = (int64_t)g.segs.size();
  if (S / g.Hkv * g.Hq * g.w >= (int64_t(1) << 31)) return fail(SLKV_ERR_BAD_ARG, "B*Hq*w >= 2^31");
  int64_t total_kept = 0;
  for (int64_t i = 0; i < S; ++i) {   // the kernels address a segment's keys with 32-bit byte offsets
    const Seg& s = g.segs[(size_t)i];
    if (s.n * g.k_stride_tok * elt >= (int64_t(1) << 31))
      return fail(SLKV_ERR_UNSUPPORTED, "segment %lld spans 2 GiB or more of K", (long long)i);
    total_kept += kept_rows(s.n, g.w, s.cap);
  }
  if (total_kept >= (int64_t(1) << 31)) return fail(SLKV_ERR_BAD_ARG, "kept rows >= 2^31");
  Plan p;
  make_plan(g, p);
  if (p.ticketed > kTicketSlots)
    return fail(SLKV_ERR_UNSUPPORTED, "%lld segments span several key chunks (limit %d)",
                (long long)p.ticketed, kTicketSlots);
  if (workspace_bytes < p.total_bytes)
    return fail(SLKV_ERR_WORKSPACE, "workspace %zu < %zu bytes", workspace_bytes, p.total_bytes);
  if (out_capacity_rows < total_kept)
    return fail(SLKV_ERR_CAPACITY, "out_capacity_rows %lld < %lld", (long long)out_capacity_rows, (long long)total_kept);

  hipStream_t st = (hipStream_t)hip_stream;
  unsigned char* ws = (unsigned char*)d_workspace;
  float* part = (float*)(ws + p.off_part);
  float* lse = (float*)(ws + p.off_lse);
  float* imp = d_importance ? d_importance : (float*)(ws + p.off_imp);
  float* pooled = d_pooled ? d_pooled : (float*)(ws + p.off_pooled);
  const float c_log2 = (float)(1.4426950408889634 / std::sqrt((double)g.d));
  const int lanes_per_row = g.d * elt / 16;

  GatherArgs ga;
  ga.k = (const unsigned char*)d_k;
  ga.v = (const unsigned char*)d_v;
  ga.k_out = (unsigned char*)d_k_out;
  ga.v_out = (unsigned char*)d_v_out;
  ga.k_stride_tok = g.k_stride_tok;
  ga.k_stride_head = g.k_stride_head;
  ga.v_stride_tok = g.v_stride_tok;
  ga.v_stride_head = g.v_stride_head;
  ga.lanes_per_row = lanes_per_row;
  ga.elt_bytes = elt;
  ga.pos_in = d_pos_in;
  ga.pos_out = d_pos_out;

  uint32_t* tickets = (uint32_t*)ws;
  uint32_t* blockhist = (uint32_t*)(ws + p.off_hist);
  // candidate lists of the block-wise selection: the workspace's importance area, which is either
  // unused (the caller asked for the importance scores in an array of its own) or dead by then
  // (pooling has consumed the scores)
  uint32_t* lists = (uint32_t*)(ws + p.off_imp);

  // The kernels of the pass over the segments one table describes.
  // Selection kernel: if every history fits one round, the one-workgroup-per-segment kernel;
  // otherwise the histories are cut into blocks.
  bool resident_select = select_mode() != 2;
  for (const Seg& sg : g.segs)
    if (seg_ranked(sg.n, g.w, sg.cap) && sg.n - g.w > kSelRound) resident_select = false;
  const int nseg = (int)S;
  auto launch_group = [&](const auto& tab, int chunks, int max_chunks, int blocks, bool any_large, int64_t rows) -> slkv_status {
    using TAB = std::decay_t<decltype(tab)>;
    // one grid row per segment where that leaves at most a seventh of the grid empty (a segment with
    // fewer chunks than the longest leaves the surplus of its row empty; with more empty workgroups
    // the full ones no longer spread evenly over the CUs: a ragged batch ran 22 % slower), else one
    // row over all chunks
    ScoreGrid sgrid{chunks, 0, 0};
    if (tab.nseg <= 65535 && (int64_t)max_chunks * tab.nseg * 6 <= (int64_t)chunks * 7) {
      sgrid.per_row = max_chunks;
      sgrid.rows = tab.nseg;
    }
    if (chunks > 0) {
      {
        ScopedKernelTimer tm(SLKV_K_SCORE_STATS, st);
        launch_score(1, sgrid, st, tab, d_qwin, d_k, g, p, c_log2, part, lse, imp, tickets);
      }
      {
        ScopedKernelTimer tm(SLKV_K_SCORE_ACCUM, st);
        launch_score(2, sgrid, st, tab, d_qwin, d_k, g, p, c_log2, part, lse, imp, tickets);
      }
    }
    {
      ScopedKernelTimer tm(SLKV_K_SELECT, st);
      if (resident_select) {
        hipError_t se = launch_select_resident(nseg, st, tab, g, d_pooled != nullptr, imp, pooled, d_kept_idx, d_out_offsets, ga);
        if (se != hipSuccess) return fail(SLKV_ERR_HIP, "select launch setup failed: %s", hipGetErrorString(se));
      } else {
        launch_select(nseg, blocks, st, tab, g, imp, pooled, blockhist, lists, d_kept_idx, d_out_offsets, ga);
      }
    }
    const bool gather_all = !resident_select && blocks > 0;   // the block-wise selection copies no rows itself
    if ((any_large || gather_all) && rows > 0) {
      ScopedKernelTimer tm(SLKV_K_GATHER, st);
      const int64_t threads = rows * lanes_per_row;
      SLKV_LAUNCH(gather_kernel<TAB>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, tab, ga, d_kept_idx,
                  gather_all ? 1 : 0);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(SLKV_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(e));
    return SLKV_OK;
  };

  // Few segments: the table travels as a kernel argument.  More: the per-64 tables are written
  // to a device-resident table by a small kernel each, and one group of launches covers all segments.
  const bool dev_table = S > kMaxSegPerLaunch;
  SegTableDev dev;
  std::memset(&dev, 0, sizeof(dev));
  if (dev_table) {
    int32_t* t = (int32_t*)(ws + p.off_table);
    dev.tok_begin = t; t += S;
    dev.n = t; t += S;
    dev.kkeep = t; t += S;
    dev.head = t; t += S;
    dev.qrow_off = t; t += S;
    dev.score_off = t; t += S;
    dev.seg_global = t; t += S;
    dev.hblk = t; t += S;
    dev.tick = t; t += S;
    dev.out_off = t; t += S + 1;
    dev.chunk_begin = t; t += S + 1;
    dev.blk_begin = t;
    dev.nseg = (int32_t)S;
  }
  // running totals over the call: output rows, key chunks, selection blocks, block histograms, tickets
  int64_t out_run = 0, chunks = 0, max_chunks = 0, blocks = 0, hist_run = 0, tick_run = 0;
  bool any_large = false;
  for (int64_t s0 = 0; s0 < S; s0 += kMaxSegPerLaunch) {
    SegTable tab;
    std::memset(&tab, 0, sizeof(tab));
    const int ns = (int)std::min<int64_t>(kMaxSegPerLaunch, S - s0);
    tab.nseg = ns;
    for (int i = 0; i < ns; ++i) {
      const Seg& sg = g.segs[(size_t)(s0 + i)];
      tab.tok_begin[i] = (int32_t)sg.row_begin;
      tab.n[i] = (int32_t)sg.n;
      const bool all = sg.n <= g.w || sg.n <= sg.cap;
      tab.kkeep[i] = all ? -1 : (int32_t)std::min<int64_t>(std::max<int64_t>(sg.cap - g.w, 0), sg.n - g.w);
      tab.out_off[i] = (int32_t)out_run;
      const int64_t kept = kept_rows(sg.n, g.w, sg.cap);
      any_large |= kept > kInlineGatherRows;
      out_run += kept;
      tab.head[i] = sg.head;
      tab.qrow_off[i] = (int32_t)sg.qrow_off;
      tab.score_off[i] = (int32_t)sg.score_off;
      tab.seg_global[i] = (int32_t)(s0 + i);
      const int64_t nc = seg_chunks(sg, g.w, p.CH), nb = seg_blocks(sg, g.w);
      tab.chunk_begin[i] = (int32_t)chunks;
      tab.blk_begin[i] = (int32_t)blocks;
      tab.hblk[i] = (int32_t)hist_run;
      tab.tick[i] = (int32_t)tick_run;
      chunks += nc;
      max_chunks = std::max(max_chunks, nc);
      blocks += nb;
      hist_run += nb;
      if (nc > 1) tick_run += 1;
    }
    if (chunks >= (int64_t(1) << 31) || blocks >= (int64_t(1) << 31)) return fail(SLKV_ERR_BAD_ARG, "too many key chunks");
    // the remaining entries repeat the end values so that searches stay inside the table
    for (int i = ns; i <= kMaxSegPerLaunch; ++i) {
      tab.out_off[i] = (int32_t)out_run;
      tab.chunk_begin[i] = (int32_t)chunks;
      tab.blk_begin[i] = (int32_t)blocks;
    }
    tab.total_chunks = (int32_t)chunks;
    if (dev_table) SLKV_LAUNCH(table_write_kernel, dim3(1), dim3(kMaxSegPerLaunch + 64), 0, st, tab, (int)s0, dev);
    else return launch_group(tab, (int)chunks, (int)max_chunks, (int)blocks, any_large, out_run);
  }
  if (dev_table) {
    dev.total_chunks = (int32_t)chunks;
    return launch_group(dev, (int)chunks, (int)max_chunks, (int)blocks, any_large, out_run);
  }
  return SLKV_OK;
}

}  // namespace slkv

using namespace slkv;

// Scratch of slkv_compress_layer_static: one copy per GPU, held until the process ends.
static __device__ __align__(256) unsigned char scratch[SLKV_STATIC_SCRATCH_BYTES];

// Device address of `scratch` on the current device (looked up once per device).
static slkv_status static_scratch(void** out) {
  constexpr int kMaxDev = 64;
  static std::mutex mu;
  static void* ptrs[kMaxDev] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(SLKV_ERR_HIP, "hipGetDevice failed: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDev) return fail(SLKV_ERR_UNSUPPORTED, "device index %d outside 0..%d", dev, kMaxDev - 1);
  std::lock_guard<std::mutex> lk(mu);
  if (!ptrs[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) return fail(SLKV_ERR_HIP, "hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e));
    e = hipMemset(ptr, 0, kTicketBytes);      // the counters at its start begin at zero (once; not under capture)
    if (e != hipSuccess) return fail(SLKV_ERR_HIP, "clearing the static scratch failed: %s", hipGetErrorString(e));
    ptrs[dev] = ptr;
  }
  *out = ptrs[dev];
  return SLKV_OK;
}

extern "C" slkv_status slkv_init(void) {
  clear_error();
  const hipError_t e = ensure_device_init();
  if (e != hipSuccess) return fail(SLKV_ERR_HIP, "device set-up failed: %s", hipGetErrorString(e));
  void* ptr = nullptr;
  return static_scratch(&ptr);
}

extern "C" slkv_status slkv_workspace_bytes(const slkv_layer_desc* desc, size_t* bytes) {
  clear_error();
  if (!bytes) return fail(SLKV_ERR_NULL, "bytes is NULL");
  slkv_status st = validate_desc(desc);
  if (st != SLKV_OK) return st;
  Geometry g;
  layer_geometry(desc, g);
  Plan p;
  make_plan(g, p);
  *bytes = p.total_bytes;
  return SLKV_OK;
}

extern "C" slkv_status slkv_compress_layer(const slkv_layer_desc* desc, const void* d_qwin, const void* d_k,
                                           const void* d_v, void* d_k_out, void* d_v_out, int32_t* d_kept_idx,
                                           int64_t* d_out_offsets, float* d_importance, float* d_pooled,
                                           int64_t out_capacity_rows, void* d_workspace, size_t workspace_bytes,
                                           void* hip_stream) {
  clear_error();
  slkv_status vs = validate_desc(desc);
  if (vs != SLKV_OK) return vs;
  Geometry g;
  layer_geometry(desc, g);
  return run_geometry(g, d_qwin, d_k, d_v, nullptr, d_k_out, d_v_out, d_kept_idx, nullptr, d_out_offsets, d_importance,
                      d_pooled, out_capacity_rows, d_workspace, workspace_bytes, hip_stream);
}

extern "C" slkv_status slkv_compress_layer_static(const slkv_layer_desc* desc, const void* d_qwin, const void* d_k,
                                                  const void* d_v, void* d_k_out, void* d_v_out, int32_t* d_kept_idx,
                                                  int64_t* d_out_offsets, float* d_importance, float* d_pooled,
                                                  int64_t out_capacity_rows, void* hip_stream) {
  clear_error();
  slkv_status vs = validate_desc(desc);
  if (vs != SLKV_OK) return vs;
  Geometry g;
  layer_geometry(desc, g);
  Plan p;
  make_plan(g, p);
  if (p.total_bytes > (size_t)SLKV_STATIC_SCRATCH_BYTES)
    return fail(SLKV_ERR_WORKSPACE, "this call needs %zu bytes of scratch, the static buffer holds %zu: use slkv_compress_layer",
                p.total_bytes, (size_t)SLKV_STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  vs = static_scratch(&ws);
  if (vs != SLKV_OK) return vs;
  return run_geometry(g, d_qwin, d_k, d_v, nullptr, d_k_out, d_v_out, d_kept_idx, nullptr, d_out_offsets, d_importance,
                      d_pooled, out_capacity_rows, ws, (size_t)SLKV_STATIC_SCRATCH_BYTES, hip_stream);
}

extern "C" slkv_status slkv_recompress_workspace_bytes(const slkv_ragged_desc* desc, size_t* bytes) {
  clear_error();
  if (!bytes) return fail(SLKV_ERR_NULL, "bytes is NULL");
  slkv_status st = validate_ragged_desc(desc);
  if (st != SLKV_OK) return st;
  Geometry g;
  ragged_geometry(desc, g);
  Plan p;
  make_plan(g, p);
  *bytes = p.total_bytes;
  return SLKV_OK;
}

extern "C" slkv_status slkv_recompress_layer(const slkv_ragged_desc* desc, const void* d_qwin, const void* d_k_in,
                                             const void* d_v_in, const int32_t* d_pos_in, void* d_k_out, void* d_v_out,
                                             int32_t* d_kept_idx, int32_t* d_pos_out, int64_t* d_out_offsets,
                                             float* d_importance, float* d_pooled, int64_t out_capacity_rows,
                                             void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  clear_error();
  slkv_status vs = validate_ragged_desc(desc);
  if (vs != SLKV_OK) return vs;
  Geometry g;
  ragged_geometry(desc, g);
  return run_geometry(g, d_qwin, d_k_in, d_v_in, d_pos_in, d_k_out, d_v_out, d_kept_idx, d_pos_out,
                      d_out_offsets, d_importance, d_pooled, out_capacity_rows, d_workspace, workspace_bytes, hip_stream);
}
