// Top-K block selection kernel: one workgroup per instance around select_topk_body (select_body.h).
#include "select_body.h"

namespace ap {
namespace {

template <int KPT, int NT>
__global__ __launch_bounds__(NT) void select_topk_kernel(const float* __restrict__ pred, int nb_cap, int nb_cur, int k,
                                                         int n_sink, int n_local, int inst0,
                                                         int32_t* __restrict__ idx, int32_t* __restrict__ cnt) {
  __shared__ uint32_t s_mem[sel_scratch_words<NT>()];
  const int inst = inst0 + blockIdx.x;
  select_topk_body<KPT, NT>(pred + (size_t)inst * nb_cap, nb_cur, k, n_sink, n_local, idx + (size_t)inst * k,
                            cnt + inst, s_mem);
}

// A selection made for nb_prev blocks, carried over to nb_cur >= nb_prev blocks without new scores: the picks
// below the local window stay (ascending order is kept by an ordered compaction), the blocks of the old local
// window are dropped unless they are sink blocks, at most k - n_local entries survive, and the last n_local
// blocks of the current context are appended.  One workgroup per instance; smem: k ints.
__global__ __launch_bounds__(kSelThreads) void refresh_selection_kernel(int nb_prev, int nb_cur, int k, int n_sink,
                                                                        int n_local, int32_t* __restrict__ idx,
                                                                        int32_t* __restrict__ cnt) {
  extern __shared__ int s_in[];
  constexpr int kSelWaves = kSelThreads / kWave;
  __shared__ int s_wsum[kSelWaves];
  const int inst = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  int32_t* out = idx + (size_t)inst * k;
  if (nb_cur <= k) {
    for (int j = tid; j < nb_cur; j += kSelThreads) out[j] = j;
    if (tid == 0) cnt[inst] = nb_cur;
    return;
  }
  const int c = min(max(cnt[inst], 0), k);
  for (int p = tid; p < c; p += kSelThreads) s_in[p] = out[p];
  __syncthreads();
  const int hi = nb_cur - n_local, cap = k - n_local;
  const int old_lo = nb_prev > k ? nb_prev - n_local : nb_prev;      // old local window [old_lo, nb_prev)
  int taken = 0;
  for (int p0 = 0; p0 < c; p0 += kSelThreads) {
    const int p = p0 + tid;
    bool keep = false;
    int j = 0;
    if (p < c) {
      j = s_in[p];
      keep = j >= 0 && j < hi && (j < n_sink || j < old_lo || j >= nb_prev);
    }
    const unsigned long long m = __ballot(keep);
    const int before = __popcll(m & ((1ull << lane) - 1ull));
    if (lane == 0) s_wsum[wave] = __popcll(m);
    __syncthreads();
    int base = 0, total = 0;
    for (int w = 0; w < kSelWaves; ++w) {
      if (w < wave) base += s_wsum[w];
      total += s_wsum[w];
    }
    const int pos = taken + base + before;
    if (keep && pos < cap) out[pos] = j;
    taken += total;
    __syncthreads();
  }
  const int m = min(taken, cap);
  for (int j = tid; j < n_local; j += kSelThreads) out[m + j] = hi + j;
  if (tid == 0) cnt[inst] = m + n_local;
}

}  // namespace

hipError_t launch_refresh_selection(const Shape& s, int nb_prev, int nb_cur, int32_t* idx, int32_t* cnt,
                                    hipStream_t st) {
  refresh_selection_kernel<<<dim3(s.n_inst), kSelThreads, sizeof(int) * s.k, st>>>(nb_prev, nb_cur, s.k, s.n_sink,
                                                                                 s.n_local, idx, cnt);
  return hipGetLastError();
}

hipError_t launch_select(const Shape& s, int inst0, int ninst, const float* pred, int nb_cur, int32_t* idx,
                         int32_t* cnt, hipStream_t st) {
  const int n_mid = nb_cur - s.n_sink - s.n_local;
  const dim3 grid(ninst);
#define AP_SELECT_NT(KPT, NT) \
  select_topk_kernel<KPT, NT><<<grid, NT, 0, st>>>(pred, s.nb_cap, nb_cur, s.k, s.n_sink, s.n_local, inst0, idx, cnt)
#define AP_SELECT(KPT) AP_SELECT_NT(KPT, kSelThreads)
  // Few instances with long rows: 1024 threads per instance cut the serial chain of every pass (a 256-thread
  // workgroup walks 32 keys per thread at 128K context while half of the chip has no workgroup at all).
  if (ninst <= 512 && n_mid > 4 * kSelThreads) {
    if (n_mid <= 4 * kSelThreadsWide) AP_SELECT_NT(4, kSelThreadsWide);
    else if (n_mid <= 8 * kSelThreadsWide) AP_SELECT_NT(8, kSelThreadsWide);
    else if (n_mid <= 9 * kSelThreadsWide) AP_SELECT_NT(9, kSelThreadsWide);     // (a 128K context that has grown a little)
    else if (n_mid <= 12 * kSelThreadsWide) AP_SELECT_NT(12, kSelThreadsWide);
    else if (n_mid <= 16 * kSelThreadsWide) AP_SELECT_NT(16, kSelThreadsWide);
    else AP_SELECT_NT(0, kSelThreadsWide);
  }
  else if (n_mid <= 8 * kSelThreads) AP_SELECT(8);       // the variants differ only in unrolled trip count
  else if (n_mid <= 9 * kSelThreads) AP_SELECT(9);
  else if (n_mid <= 10 * kSelThreads) AP_SELECT(10);
  else if (n_mid <= 12 * kSelThreads) AP_SELECT(12);
  else if (n_mid <= 16 * kSelThreads) AP_SELECT(16);
  else if (n_mid <= 24 * kSelThreads) AP_SELECT(24);
  else if (n_mid <= 32 * kSelThreads) AP_SELECT(32);
  else AP_SELECT(0);
#undef AP_SELECT
#undef AP_SELECT_NT
  return hipGetLastError();
}

}  // namespace ap
