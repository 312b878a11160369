// Top-K block selection (Algorithm 1 step 5) with forced sink / local blocks (Sec. 4.1).
//
// One workgroup per instance.  Scores are mapped to order-preserving 32-bit keys; a 4-pass
// radix select (8 bits per pass, histogram in LDS) finds the key T of the k_mid-th largest score
// and how many scores equal to T are still needed.  A final ordered sweep keeps every block with
// key > T and the first `need` blocks with key == T, compacting in index order, so the output is
// ascending and equal scores go to the lower index.  Integer work only: the result is exact.
// When the candidates fit (up to 32 per thread) their keys are fetched once into registers, so the five
// passes do not each wait on memory; longer rows are re-read from cache in every pass.
#pragma once

#include "ap_internal.h"

namespace ap {
namespace {

constexpr int kSelThreads = 256;           // workgroup size of the common variant
constexpr int kSelThreadsWide = 1024;      // few instances, long rows: more threads per instance
constexpr int kSelBins = 256;              // radix of one pass; the first kSelBins threads own one bin each
template <int NT> constexpr int sel_scratch_words() { return kSelBins + 3 * (NT / kWave) + 8; }

__device__ __forceinline__ uint32_t score_key(float x) {
  uint32_t u = __float_as_uint(x);
  if (u == 0x80000000u) u = 0u;                         // -0 ranks with +0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);    // larger score <=> larger key
}

// Adds one to hist[bin] for every lane with `active`.  Predicted scores of neighbouring blocks are close,
// so most lanes of a wave share a bin and per-lane LDS atomics would serialise on it: the two most common
// leading bins are counted with a ballot and added once per wave, the rest fall back to single adds.
__device__ __forceinline__ void hist_add(uint32_t* hist, uint32_t bin, bool active) {
#pragma unroll
  for (int round = 0; round < 2; ++round) {
    if (active) {                                       // (the lanes still to be counted are the ones executing here)
      const uint32_t b0 = __builtin_amdgcn_readfirstlane(bin);          // bin of the first of them
      const bool same = bin == b0;
      const unsigned long long m = __ballot(same);
      const uint32_t before = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
      if (same && before == 0) atomicAdd(&hist[b0], (uint32_t)__popcll(m));
      if (same) active = false;
    }
  }
  if (active) atomicAdd(&hist[bin], 1u);
}

// Inclusive prefix sum over the 64 lanes with DPP moves (shifts within the rows of 16 lanes, then the last lane of
// row 0 / 2 added to row 1 / 3 and the last lane of row 1 to rows 2 and 3): register moves, no trip through the LDS
// permute path.  Every lane must be active.
template <int CTRL, int ROW_MASK> __device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, true);
}
__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
  v += dpp_u32<0x111, 0xF>(v);                          // row_shr:1 (zero shifted in at the start of a row)
  v += dpp_u32<0x112, 0xF>(v);                          // row_shr:2
  v += dpp_u32<0x114, 0xF>(v);                          // row_shr:4
  v += dpp_u32<0x118, 0xF>(v);                          // row_shr:8
  v += dpp_u32<0x142, 0xA>(v);                          // row_bcast:15 into rows 1 and 3
  v += dpp_u32<0x143, 0xC>(v);                          // row_bcast:31 into rows 2 and 3
  return v;
}

// Selection for one instance by one workgroup of NT threads (a multiple of kSelBins).
//   p        the instance's scores (nb_cur valid entries)
//   out      the instance's k index slots, cnt_out its count
//   s_mem    sel_scratch_words<NT>() words of LDS, free for this call (the caller synchronises before)
template <int KPT, int NT>   // KPT: keys per thread held in registers; 0 = re-read the scores in every pass
__device__ __forceinline__ void select_topk_body(const float* __restrict__ p, int nb_cur, int k, int n_sink, int n_local,
                                        int32_t* __restrict__ out, int32_t* __restrict__ cnt_out, uint32_t* s_mem) {
  constexpr int kSelThreads = NT, kSelWaves = NT / kWave;
  uint32_t* s_hist = s_mem;                     // [kSelBins]
  uint32_t* s_wsum = s_mem + kSelBins;          // [kSelWaves]
  uint32_t* s_wgt = s_wsum + kSelWaves;         // [kSelWaves]
  uint32_t* s_weq = s_wgt + kSelWaves;          // [kSelWaves]
  uint32_t* s_found = s_mem + kSelBins + 3 * kSelWaves; // [4 passes][bin, keys above it]: a slot per pass, so no
                                                        // barrier is needed before the next pass may write
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;

  if (nb_cur <= k) {                                    // everything fits the budget
    for (int j = tid; j < nb_cur; j += kSelThreads) out[j] = j;
    if (tid == 0) *cnt_out = nb_cur;
    return;
  }
  const int lo = n_sink, hi = nb_cur - n_local;         // candidates [lo, hi), hi - lo > k_mid
  const int k_mid = k - n_sink - n_local;

  // Candidate i of thread tid is block lo + i * kSelThreads + tid; past the end the key is a sentinel that
  // no pass counts (valid is false).
  constexpr int NK = KPT > 0 ? KPT : 1;
  uint32_t keys[NK];
  if constexpr (KPT > 0) {
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
      const int j = lo + i * kSelThreads + tid;
      keys[i] = score_key(p[min(j, hi - 1)]);
    }
  }
  auto key_at = [&](int i, int j) __attribute__((always_inline)) -> uint32_t {
    if constexpr (KPT > 0) return keys[i]; else return score_key(p[min(j, hi - 1)]);
  };
  const int n_iter = KPT > 0 ? KPT : (hi - lo + kSelThreads - 1) / kSelThreads;

  uint32_t prefix = 0;                                  // high bits of T found so far
  uint32_t need = (uint32_t)k_mid;                      // still to take among keys matching prefix
  if (k_mid > 0) {
    if (tid < kSelBins) s_hist[tid] = 0;
    __syncthreads();
    for (int shift = 24, pass = 0; shift >= 0; shift -= 8, ++pass) {
#pragma unroll NK
      for (int i = 0; i < n_iter; ++i) {                   // uniform trip count: ballots need every lane
        const int j = lo + i * kSelThreads + tid;
        const uint32_t key = key_at(i, j);
        const bool match = j < hi && ((shift == 24) || ((key >> (shift + 8)) == prefix));
        hist_add(s_hist, (key >> shift) & 255u, match);
      }
      __syncthreads();
      // Suffix sums over bins: thread r < kSelBins handles bin 255 - r, inclusive scan in that order
      // (whole waves take or skip these branches).
      uint32_t c = 0, incl = 0;
      if (tid < kSelBins) {
        c = s_hist[kSelBins - 1 - tid];
        s_hist[kSelBins - 1 - tid] = 0;                 // for the next pass, whose adds come two barriers later
        incl = wave_incl_scan(c);
        if (lane == kWave - 1) s_wsum[wave] = incl;
      }
      __syncthreads();
      if (tid < kSelBins) {
        uint32_t base = 0;
        for (int w = 0; w < wave; ++w) base += s_wsum[w];
        incl += base;                                   // keys in bins >= 255 - tid
        const uint32_t excl = incl - c;                 // keys in bins >  255 - tid
        if (excl < need && need <= incl) { s_found[2 * pass] = kSelBins - 1 - tid; s_found[2 * pass + 1] = excl; }
      }
      __syncthreads();
      prefix = (prefix << 8) | s_found[2 * pass];
      need -= s_found[2 * pass + 1];
    }
  }
  const uint32_t T = prefix;

  // Ordered sweep in chunks of one workgroup width.
  uint32_t taken = 0;                                   // selected so far (all threads agree)
  uint32_t eq_seen = 0;                                 // keys == T seen so far
#pragma unroll NK
  for (int i = 0; i < n_iter; ++i) {
    if (k_mid <= 0) break;
    const int j = lo + i * kSelThreads + tid;
    bool gt = false, eq = false;
    if (j < hi) {
      const uint32_t key = key_at(i, j);
      gt = key > T;
      eq = key == T;
    }
    const unsigned long long bgt = __ballot(gt), beq = __ballot(eq);
    const unsigned long long below = (lane == 0) ? 0ull : (~0ull >> (kWave - lane));
    if (lane == 0) { s_wgt[wave] = __popcll(bgt); s_weq[wave] = __popcll(beq); }
    __syncthreads();
    uint32_t gt_before = __popcll(bgt & below), eq_before = __popcll(beq & below);
    uint32_t gt_total = 0, eq_total = 0;
    for (int w = 0; w < kSelWaves; ++w) {
      if (w < wave) { gt_before += s_wgt[w]; eq_before += s_weq[w]; }
      gt_total += s_wgt[w];
      eq_total += s_weq[w];
    }
    // equal keys taken before this lane within the chunk: those whose global rank < need
    const uint32_t eq_rank = eq_seen + eq_before;
    const uint32_t eq_taken_before = min(eq_rank, need) - min(eq_seen, need);
    const bool take = gt || (eq && eq_rank < need);
    if (take) out[n_sink + taken + gt_before + eq_taken_before] = j;
    taken += gt_total + (min(eq_seen + eq_total, need) - min(eq_seen, need));
    eq_seen += eq_total;
    __syncthreads();
  }
  for (int j = tid; j < n_sink; j += kSelThreads) out[j] = j;
  for (int j = tid; j < n_local; j += kSelThreads) out[k - n_local + j] = nb_cur - n_local + j;
  if (tid == 0) *cnt_out = k;
}


}  // namespace
}  // namespace ap
