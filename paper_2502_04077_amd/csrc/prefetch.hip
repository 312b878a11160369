// Staging of the selected blocks for a K/V cache that lives outside the device ("KV Cache Cross-token
// Prefetching", Sec. 3.4): the blocks one selection names are gathered from the full cache - pinned host
// memory read by the kernel over PCIe, or device memory - into a compact device pool of k slots per
// instance, and a block table is filled so that the paged form of the attention kernels reads the pool.
// The token that is generated in the step the selection is for does not exist yet when its blocks are
// fetched; its K/V row is appended to the staged copy of the newest block afterwards.
#include "ap_internal.h"

namespace ap {
namespace {

constexpr int kGatherThreads = 256;

// Workgroup (p, inst) copies list position p of instance inst: block idx[p] of K and V into pool slot
// inst * k + p, 16 bytes per lane and load.  Rows of tokens >= t_avail are written as zeros.
__global__ __launch_bounds__(kGatherThreads) void gather_blocks_kernel(
    const uint4* __restrict__ K_src, const uint4* __restrict__ V_src, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ cnt, uint4* __restrict__ pool_K, uint4* __restrict__ pool_V,
    int32_t* __restrict__ table, int k, int nb_cap, int nb_cur, int b, int row_units, size_t inst_units,
    int t_avail) {
  const int inst = blockIdx.y, p = blockIdx.x;
  if (p >= min(max(cnt[inst], 0), k)) return;
  const int blk = min(max(idx[(size_t)inst * k + p], 0), nb_cur - 1);
  const int slot = inst * k + p;
  const int block_units = b * row_units;
  const uint4* ks = K_src + (size_t)inst * inst_units + (size_t)blk * block_units;
  const uint4* vs = V_src + (size_t)inst * inst_units + (size_t)blk * block_units;
  uint4* kd = pool_K + (size_t)slot * block_units;
  uint4* vd = pool_V + (size_t)slot * block_units;
  const int rows_avail = min(max(t_avail - blk * b, 0), b);
  const int units_avail = rows_avail * row_units;
  for (int u = threadIdx.x; u < block_units; u += kGatherThreads) {
    uint4 kv = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
    if (u < units_avail) { kv = ks[u]; vv = vs[u]; }
    kd[u] = kv;
    vd[u] = vv;
  }
  if (threadIdx.x == 0) table[(size_t)inst * nb_cap + blk] = slot;
}

// One new token row per instance, written into the staged copy of block t_pos / b - always the last list
// entry when it is selected at all (the list is ascending and no block lies beyond the newest).
__global__ __launch_bounds__(kWave) void append_row_kernel(const uint4* __restrict__ k_new,
                                                           const uint4* __restrict__ v_new,
                                                           const int32_t* __restrict__ idx,
                                                           const int32_t* __restrict__ cnt,
                                                           uint4* __restrict__ pool_K, uint4* __restrict__ pool_V,
                                                           int k, int nb_cur, int b, int row_units, int t_pos) {
  const int inst = blockIdx.x;
  const int c = min(max(cnt[inst], 0), k);
  if (c == 0) return;
  const int blk = min(max(idx[(size_t)inst * k + c - 1], 0), nb_cur - 1);
  if (blk != t_pos / b) return;
  const size_t dst = ((size_t)(inst * k + c - 1) * b + (t_pos % b)) * row_units;
  for (int u = threadIdx.x; u < row_units; u += kWave) {
    pool_K[dst + u] = k_new[(size_t)inst * row_units + u];
    pool_V[dst + u] = v_new[(size_t)inst * row_units + u];
  }
}

}  // namespace

hipError_t launch_gather_blocks(const Shape& s, const void* K_src, const void* V_src, int t_avail, int nb_cur,
                                const int32_t* idx, const int32_t* cnt, void* pool_K, void* pool_V, int32_t* table,
                                hipStream_t st) {
  const int row_units = s.d * (s.kv_dtype == AP_BF16 ? 2 : 4) / 16;
  gather_blocks_kernel<<<dim3(s.k, s.n_inst), kGatherThreads, 0, st>>>(
      static_cast<const uint4*>(K_src), static_cast<const uint4*>(V_src), idx, cnt, static_cast<uint4*>(pool_K),
      static_cast<uint4*>(pool_V), table, s.k, s.nb_cap, nb_cur, s.b, row_units, (size_t)s.t_cap * row_units, t_avail);
  return hipGetLastError();
}

hipError_t launch_append_row(const Shape& s, const void* k_new, const void* v_new, int t_pos, const int32_t* idx,
                             const int32_t* cnt, void* pool_K, void* pool_V, hipStream_t st) {
  const int row_units = s.d * (s.kv_dtype == AP_BF16 ? 2 : 4) / 16;
  append_row_kernel<<<dim3(s.n_inst), kWave, 0, st>>>(static_cast<const uint4*>(k_new), static_cast<const uint4*>(v_new),
                                                     idx, cnt, static_cast<uint4*>(pool_K), static_cast<uint4*>(pool_V),
                                                     s.k, t_pos / s.b + 1, s.b, row_units, t_pos);
  return hipGetLastError();
}

}  // namespace ap
