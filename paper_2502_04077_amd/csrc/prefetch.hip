// Staging of the selected blocks for a K/V cache that lives outside the device ("KV Cache Cross-token
// Prefetching", Sec. 3.4): the blocks one selection names are gathered from the full cache - pinned host
// memory read by the kernel over PCIe, or device memory - into a compact device pool of k slots per
// instance, and a block table is filled so that the paged form of the attention kernels reads the pool.
//
// Consecutive selections share many of their blocks (the re-access pattern and the slow change of the attention
// ranking between decode steps, Sec. 3.1 "Attention Temporal Patterns"), so the pool is kept as a cache: a block that
// is already staged keeps its slot and only the blocks that are new to the selection cross the link, into
// the slots of blocks that dropped out.  Per instance the state is
//   state[0 .. k)        1 + logical block held by each slot (0 = empty)
//   state[k .. 3k)       (block, slot) pairs of the last plan's fetch list
//   state[3k]            length of that list;  state[3k + 1]  blocks fetched since the state was zeroed
// The token that is generated in the step the selection is for does not exist yet when its blocks are
// fetched; its K/V row is appended to the staged copy of the newest block afterwards.
#include "ap_internal.h"

namespace ap {
namespace {

constexpr int kGatherThreads = 256;
constexpr int kGatherGrid = 48;      // workgroups of the gather kernel
constexpr int kPlanThreads = 256;    // >= k

// Exclusive prefix sum of one flag per thread over the workgroup; *total gets the sum.  s_tmp: kPlanThreads / 64 ints.
__device__ __forceinline__ int block_excl_scan(bool flag, int* s_tmp, int* total) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const unsigned long long m = __ballot(flag);
  const int before = __popcll(m & ((1ull << lane) - 1ull));
  __syncthreads();                                 // s_tmp may still be read from the previous scan
  if (lane == 0) s_tmp[wave] = __popcll(m);
  __syncthreads();
  int base = 0, sum = 0;
#pragma unroll
  for (int w = 0; w < kPlanThreads / kWave; ++w) {
    const int c = s_tmp[w];
    if (w < wave) base += c;
    sum += c;
  }
  *total = sum;
  return base + before;
}

// One workgroup per instance: which blocks of the new selection are already staged, which slots fall free,
// and the fetch list that pairs the missing blocks with the free slots.
__global__ __launch_bounds__(kPlanThreads) void plan_fetch_kernel(const int32_t* __restrict__ idx,
                                                                  const int32_t* __restrict__ cnt,
                                                                  int32_t* __restrict__ table,
                                                                  int32_t* __restrict__ state, int k, int nb_cap,
                                                                  int nb_cur, int state_stride) {
  __shared__ int s_keep[kPlanThreads], s_free[kPlanThreads], s_tmp[kPlanThreads / kWave];
  const int inst = blockIdx.x, tid = threadIdx.x;
  int32_t* slot_blk = state + (size_t)inst * state_stride;
  int32_t* fetch = slot_blk + k;
  const int c = min(max(cnt[inst], 0), k);
  s_keep[tid] = 0;
  __syncthreads();
  int blk = -1;
  bool miss = false;
  if (tid < c) {
    blk = min(max(idx[(size_t)inst * k + tid], 0), nb_cur - 1);
    const int sl = table[(size_t)inst * nb_cap + blk] - inst * k;      // may be stale: checked against the slot
    const bool hit = sl >= 0 && sl < k && slot_blk[sl] == blk + 1;
    if (hit) s_keep[sl] = 1;
    miss = !hit;
  }
  __syncthreads();
  int n_miss, n_free;
  const int miss_rank = block_excl_scan(miss, s_tmp, &n_miss);
  const bool is_free = tid < k && !s_keep[tid];
  const int free_rank = block_excl_scan(is_free, s_tmp, &n_free);
  if (is_free) s_free[free_rank] = tid;
  __syncthreads();
  if (miss) {                                      // n_miss <= n_free: every kept slot holds one of the c blocks
    const int sl = s_free[miss_rank];
    slot_blk[sl] = blk + 1;
    table[(size_t)inst * nb_cap + blk] = inst * k + sl;
    fetch[2 * miss_rank] = blk;
    fetch[2 * miss_rank + 1] = sl;
  }
  if (tid == 0) {
    slot_blk[3 * k] = n_miss;
    slot_blk[3 * k + 1] += n_miss;
  }
}

// Each workgroup walks (instance, fetch-list entry) pairs: 16 bytes per lane and load, K and V of one block per
// pass.  Rows of tokens >= t_avail are written as zeros.  The grid is kept small on purpose: a few dozen
// workgroups keep enough reads in flight to fill a PCIe link, while waves parked on host reads all over the
// chip slow down the attention kernels they run beside.
__global__ __launch_bounds__(kGatherThreads) void gather_blocks_kernel(
    const uint4* __restrict__ K_src, const uint4* __restrict__ V_src, const int32_t* __restrict__ state,
    uint4* __restrict__ pool_K, uint4* __restrict__ pool_V, int n_inst, int k, int state_stride, int b, int row_units,
    size_t inst_units, int t_avail) {
  const int block_units = b * row_units;
  for (int pair = blockIdx.x; pair < n_inst * k; pair += gridDim.x) {
    const int inst = pair / k, m = pair - inst * k;
    const int32_t* st = state + (size_t)inst * state_stride;
    if (m >= min(max(st[3 * k], 0), k)) continue;
    const int blk = st[k + 2 * m], sl = st[k + 2 * m + 1];
    const uint4* ks = K_src + (size_t)inst * inst_units + (size_t)blk * block_units;
    const uint4* vs = V_src + (size_t)inst * inst_units + (size_t)blk * block_units;
    uint4* kd = pool_K + ((size_t)inst * k + sl) * block_units;
    uint4* vd = pool_V + ((size_t)inst * k + sl) * block_units;
    const int units_avail = min(max(t_avail - blk * b, 0), b) * row_units;
    for (int u = threadIdx.x; u < block_units; u += kGatherThreads) {
      uint4 kv = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
      if (u < units_avail) { kv = ks[u]; vv = vs[u]; }
      kd[u] = kv;
      vd[u] = vv;
    }
  }
}

// One new token row per instance, written into the staged copy of block t_pos / b if that block is staged.
__global__ __launch_bounds__(kWave) void append_row_kernel(const uint4* __restrict__ k_new,
                                                           const uint4* __restrict__ v_new,
                                                           const int32_t* __restrict__ table,
                                                           const int32_t* __restrict__ state,
                                                           uint4* __restrict__ pool_K, uint4* __restrict__ pool_V,
                                                           int k, int nb_cap, int state_stride, int b, int row_units,
                                                           int t_pos) {
  const int inst = blockIdx.x;
  const int blk = t_pos / b;
  const int sl = table[(size_t)inst * nb_cap + blk] - inst * k;
  if (sl < 0 || sl >= k || state[(size_t)inst * state_stride + sl] != blk + 1) return;
  const size_t dst = (((size_t)inst * k + sl) * b + (t_pos % b)) * row_units;
  for (int u = threadIdx.x; u < row_units; u += kWave) {
    pool_K[dst + u] = k_new[(size_t)inst * row_units + u];
    pool_V[dst + u] = v_new[(size_t)inst * row_units + u];
  }
}

}  // namespace

int prefetch_state_stride(const Shape& s) { return 3 * s.k + 4; }

hipError_t launch_gather_blocks(const Shape& s, const void* K_src, const void* V_src, int t_avail, int nb_cur,
                                const int32_t* idx, const int32_t* cnt, void* pool_K, void* pool_V, int32_t* table,
                                int32_t* state, hipStream_t st) {
  const int row_units = s.d * (s.kv_dtype == AP_BF16 ? 2 : 4) / 16;
  const int stride = prefetch_state_stride(s);
  plan_fetch_kernel<<<dim3(s.n_inst), kPlanThreads, 0, st>>>(idx, cnt, table, state, s.k, s.nb_cap, nb_cur, stride);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int pairs = s.n_inst * s.k;
  gather_blocks_kernel<<<dim3(pairs < kGatherGrid ? pairs : kGatherGrid), kGatherThreads, 0, st>>>(
      static_cast<const uint4*>(K_src), static_cast<const uint4*>(V_src), state, static_cast<uint4*>(pool_K),
      static_cast<uint4*>(pool_V), s.n_inst, s.k, stride, s.b, row_units, (size_t)s.t_cap * row_units, t_avail);
  return hipGetLastError();
}

hipError_t launch_append_row(const Shape& s, const void* k_new, const void* v_new, int t_pos, const int32_t* table,
                             const int32_t* state, void* pool_K, void* pool_V, hipStream_t st) {
  const int row_units = s.d * (s.kv_dtype == AP_BF16 ? 2 : 4) / 16;
  append_row_kernel<<<dim3(s.n_inst), kWave, 0, st>>>(static_cast<const uint4*>(k_new), static_cast<const uint4*>(v_new),
                                                     table, state, static_cast<uint4*>(pool_K),
                                                     static_cast<uint4*>(pool_V), s.k, s.nb_cap,
                                                     prefetch_state_stride(s), s.b, row_units, t_pos);
  return hipGetLastError();
}

}  // namespace ap
