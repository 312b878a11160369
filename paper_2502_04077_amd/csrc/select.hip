// Top-K block selection kernel: one workgroup per instance around select_topk_body (select_body.h).
#include "select_body.h"

namespace ap {
namespace {

template <int KPT>
__global__ __launch_bounds__(kSelThreads) void select_topk_kernel(const float* __restrict__ pred, int nb_cap,
                                                                  int nb_cur, int k, int n_sink, int n_local,
                                                                  int inst0, int32_t* __restrict__ idx,
                                                                  int32_t* __restrict__ cnt) {
  __shared__ uint32_t s_mem[kSelScratchWords];
  const int inst = inst0 + blockIdx.x;
  select_topk_body<KPT>(pred + (size_t)inst * nb_cap, nb_cur, k, n_sink, n_local, idx + (size_t)inst * k, cnt + inst,
                        s_mem);
}

}  // namespace

hipError_t launch_select(const Shape& s, int inst0, int ninst, const float* pred, int nb_cur, int32_t* idx,
                         int32_t* cnt, hipStream_t st) {
  const int n_mid = nb_cur - s.n_sink - s.n_local;
  const dim3 grid(ninst);
#define AP_SELECT(KPT) \
  select_topk_kernel<KPT><<<grid, kSelThreads, 0, st>>>(pred, s.nb_cap, nb_cur, s.k, s.n_sink, s.n_local, inst0, idx, cnt)
  if (n_mid <= 8 * kSelThreads) AP_SELECT(8);            // the variants differ only in unrolled trip count
  else if (n_mid <= 9 * kSelThreads) AP_SELECT(9);
  else if (n_mid <= 10 * kSelThreads) AP_SELECT(10);
  else if (n_mid <= 12 * kSelThreads) AP_SELECT(12);
  else if (n_mid <= 16 * kSelThreads) AP_SELECT(16);
  else if (n_mid <= 24 * kSelThreads) AP_SELECT(24);
  else if (n_mid <= 32 * kSelThreads) AP_SELECT(32);
  else AP_SELECT(0);
#undef AP_SELECT
  return hipGetLastError();
}

}  // namespace ap
