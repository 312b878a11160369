// History ring (Algorithm 1 step 3): row number n lives in slot n % R of hist[n_inst][R][nb_cap];
// writing a slot drops the row that was R pushes older, so the newest H rows are always present.
#include "ap_internal.h"

namespace ap {
namespace {

__global__ __launch_bounds__(256) void push_row_kernel(float* __restrict__ hist, const float* __restrict__ row,
                                                       int R, int nb_cap, int slot) {
  const int inst = blockIdx.y;
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < nb_cap) hist[((size_t)inst * R + slot) * nb_cap + j] = row[(size_t)inst * nb_cap + j];
}

}  // namespace

hipError_t launch_push_row(const Shape& s, float* hist, int slot, const float* row, hipStream_t st) {
  push_row_kernel<<<dim3((s.nb_cap + 255) / 256, s.n_inst), 256, 0, st>>>(hist, row, s.R, s.nb_cap, slot);
  return hipGetLastError();
}

}  // namespace ap
