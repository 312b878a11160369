// Top-K block selection (Algorithm 1 step 5) with forced sink / local blocks (Sec. 4.1).
//
// One workgroup per instance.  Scores are mapped to order-preserving 32-bit keys; a 4-pass
// radix select (8 bits per pass, histogram in LDS) finds the key T of the k_mid-th largest score
// and how many scores equal to T are still needed.  A final ordered sweep keeps every block with
// key > T and the first `need` blocks with key == T, compacting in index order, so the output is
// ascending and equal scores go to the lower index.  Integer work only: the result is exact.
#include "ap_internal.h"

namespace ap {
namespace {

constexpr int kSelThreads = 256;
constexpr int kSelWaves = kSelThreads / kWave;

__device__ inline uint32_t score_key(float x) {
  uint32_t u = __float_as_uint(x);
  if (u == 0x80000000u) u = 0u;                         // -0 ranks with +0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);    // larger score <=> larger key
}

// Adds one to hist[bin] for every lane with `active`.  Predicted scores of neighbouring blocks are close,
// so most lanes of a wave share a bin and per-lane LDS atomics would serialise on it: the two most common
// leading bins are counted with a ballot and added once per wave, the rest fall back to single adds.
__device__ inline void hist_add(uint32_t* hist, uint32_t bin, bool active) {
  const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
  for (int round = 0; round < 2; ++round) {
    const unsigned long long live = __ballot(active);
    if (live == 0) return;
    const int leader = __ffsll((long long)live) - 1;
    const uint32_t b0 = (uint32_t)__shfl((int)bin, leader, kWave);
    const unsigned long long same = __ballot(active && bin == b0);
    if (lane == leader) atomicAdd(&hist[b0], (uint32_t)__popcll(same));
    if (bin == b0) active = false;
  }
  if (active) atomicAdd(&hist[bin], 1u);
}

__global__ __launch_bounds__(kSelThreads) void select_topk_kernel(const float* __restrict__ pred, int nb_cap,
                                                                  int nb_cur, int k, int n_sink, int n_local,
                                                                  int inst0, int32_t* __restrict__ idx,
                                                                  int32_t* __restrict__ cnt) {
  __shared__ uint32_t s_hist[256];
  __shared__ uint32_t s_wsum[kSelWaves];
  __shared__ uint32_t s_bin, s_above;
  __shared__ uint32_t s_wgt[kSelWaves], s_weq[kSelWaves];

  const int inst = inst0 + blockIdx.x;
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const float* p = pred + (size_t)inst * nb_cap;
  int32_t* out = idx + (size_t)inst * k;

  if (nb_cur <= k) {                                    // everything fits the budget
    for (int j = tid; j < nb_cur; j += kSelThreads) out[j] = j;
    if (tid == 0) cnt[inst] = nb_cur;
    return;
  }
  const int lo = n_sink, hi = nb_cur - n_local;         // candidates [lo, hi), hi - lo > k_mid
  const int k_mid = k - n_sink - n_local;

  uint32_t prefix = 0;                                  // high bits of T found so far
  uint32_t need = (uint32_t)k_mid;                      // still to take among keys matching prefix
  if (k_mid > 0) {
    for (int shift = 24; shift >= 0; shift -= 8) {
      s_hist[tid] = 0;
      __syncthreads();
      for (int jb = lo; jb < hi; jb += kSelThreads) {        // uniform trip count: ballots need every lane
        const int j = jb + tid;
        uint32_t key = 0;
        bool match = false;
        if (j < hi) {
          key = score_key(p[j]);
          match = (shift == 24) || ((key >> (shift + 8)) == prefix);
        }
        hist_add(s_hist, (key >> shift) & 255u, match);
      }
      __syncthreads();
      // Suffix sums over bins: thread r handles bin 255 - r, inclusive scan in that order.
      const uint32_t c = s_hist[255 - tid];
      uint32_t incl = c;
#pragma unroll
      for (int o = 1; o < kWave; o <<= 1) {
        const uint32_t up = __shfl_up(incl, o, kWave);
        if (lane >= o) incl += up;
      }
      if (lane == kWave - 1) s_wsum[wave] = incl;
      __syncthreads();
      uint32_t base = 0;
      for (int w = 0; w < wave; ++w) base += s_wsum[w];
      incl += base;                                     // keys in bins >= 255 - tid
      const uint32_t excl = incl - c;                   // keys in bins >  255 - tid
      if (excl < need && need <= incl) { s_bin = 255 - tid; s_above = excl; }
      __syncthreads();
      prefix = (prefix << 8) | s_bin;
      need -= s_above;
      __syncthreads();
    }
  }
  const uint32_t T = prefix;

  // Ordered sweep in chunks of one workgroup width.
  uint32_t taken = 0;                                   // selected so far (all threads agree)
  uint32_t eq_seen = 0;                                 // keys == T seen so far
  for (int base = lo; base < hi && k_mid > 0; base += kSelThreads) {
    const int j = base + tid;
    bool gt = false, eq = false;
    if (j < hi) {
      const uint32_t key = score_key(p[j]);
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
  if (tid == 0) cnt[inst] = k;
}

}  // namespace

hipError_t launch_select(const Shape& s, int inst0, int ninst, const float* pred, int nb_cur, int32_t* idx,
                         int32_t* cnt, hipStream_t st) {
  select_topk_kernel<<<dim3(ninst), kSelThreads, 0, st>>>(pred, s.nb_cap, nb_cur, s.k, s.n_sink, s.n_local, inst0,
                                                          idx, cnt);
  return hipGetLastError();
}

}  // namespace ap
