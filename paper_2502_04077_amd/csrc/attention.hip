// Kernels around attention_body.h: block-sparse decode (+ combine of splits) and dense calibration.
#include <mutex>

#include "attention_body.h"

// Scratch for the entry point that must not allocate (ap_sparse_decode_noalloc): the split partials of one
// sparse-decode call.  Every device the library runs on holds its own copy until the process ends.  In host code
// this name is only a handle for hipGetSymbolAddress; kernels get the address that call returned.
constexpr size_t kStaticScratchBytes = AP_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace ap {
namespace {

// (the narrow forms are only worth launching if many of their workgroups fit a CU: four waves per SIMD, 128 VGPRs)
template <typename T, int D, int G, int NW, bool PIECED>
__global__ __launch_bounds__(NW * kWave) __attribute__((amdgpu_waves_per_eu(NW < kAttnWaves ? 4 : 1)))
void sparse_decode_kernel(SparseArgs a) {
  extern __shared__ __align__(16) float smem[];
  sparse_decode_body<T, D, G, NW, PIECED>(a, a.inst0 + blockIdx.y, blockIdx.x, smem);
}

// Merges the splits of one instance: global (M, L) per head, normalised output, pooled row.  The row is nb_cap
// columns long (8K at a 128K context) and all but `cnt` of them are zero, so it is cut into chunks of
// kCombineCols columns, one workgroup each (blockIdx.x = chunk, blockIdx.y = instance): the chunk is put together
// in LDS - zeros, then the values of the listed blocks that fall into it - and written out whole and coalesced.
// Every workgroup works out the split scales for itself (n_split x G values); chunk 0 also writes the output.
constexpr int kCombineCols = 1024;

template <int D, int G>
__global__ __launch_bounds__(kAttnThreads) void sparse_combine_kernel(SparseArgs a) {
  extern __shared__ __align__(16) float smem[];
  const int inst = a.inst0 + blockIdx.y, chunk = blockIdx.x;
  const int cnt = min(max(a.cnt[inst], 0), a.k);
  float* s_scale = smem;                               // [n_split][G]  exp(m_s - M) / L
  float* s_row = s_scale + a.n_split * G;              // [kCombineCols]
  const int c0 = chunk * kCombineCols, c1 = min(a.nb_cap, c0 + kCombineCols);

  for (int j = threadIdx.x; j < c1 - c0; j += kAttnThreads) s_row[j] = 0.f;
  if (threadIdx.x < G) {
    const int h = threadIdx.x;
    const float* ml = a.part_ml + ((size_t)inst * a.n_split * G + h) * 2;
    float M = -INFINITY;
    for (int s = 0; s < a.n_split; ++s) M = fmaxf(M, ml[(size_t)s * G * 2]);
    float L = 0.f;
    for (int s = 0; s < a.n_split; ++s) {
      const float m = ml[(size_t)s * G * 2];
      const float sc = (m == -INFINITY) ? 0.f : __expf(m - M);
      s_scale[s * G + h] = sc;
      L += ml[(size_t)s * G * 2 + 1] * sc;
    }
    const float invL = L > 0.f ? 1.f / L : 0.f;          // an empty list gives a zero output
    for (int s = 0; s < a.n_split; ++s) s_scale[s * G + h] *= invL;
  }
  __syncthreads();
  if (chunk == 0) {
    for (int o = threadIdx.x; o < G * D; o += kAttnThreads) {
      const int h = o / D;
      float v = 0.f;
      for (int s = 0; s < a.n_split; ++s)
        v = fmaf(a.part_acc[((size_t)inst * a.n_split + s) * G * D + o], s_scale[s * G + h], v);
      a.out[(size_t)inst * G * D + o] = v;
    }
  }
  // pooled probability of list position jb: max over heads of (block max relative to its split) * split scale
  for (int jb = threadIdx.x; jb < cnt; jb += kAttnThreads) {
    const int blk = min(max(a.idx[(size_t)inst * a.k + jb], 0), a.nb_cur - 1);
    if (blk >= c0 && blk < c1) {
      const int s = jb / a.blk_per_split;
      float mx = 0.f;
#pragma unroll
      for (int h = 0; h < G; ++h)
        mx = fmaxf(mx, a.part_bmp[((size_t)inst * G + h) * a.k + jb] * s_scale[s * G + h]);
      s_row[blk - c0] = mx;                            // (a block listed twice: either of two equal values)
    }
  }
  __syncthreads();
  float* row = a.row + (size_t)inst * a.row_stride;
  for (int j = threadIdx.x; j < c1 - c0; j += kAttnThreads) row[c0 + j] = s_row[j];
}

struct CalibArgs {
  const void* q; const void* K;
  float* row; float* cal_ml; float* cal_bmp;
  int* counter;                   // next (instance, chunk) unit to hand out; zero at launch
  int n_units;                    // n_inst * n_chunks
  int t_cap, nb_cap, b, log2b, t_cur, nb_cur, chunk_blocks, n_chunks, chunk_slots;
  const int32_t* table;
  int n_phys;
};

__global__ void zero_counter_kernel(int* counter) { *counter = 0; }

// Workgroups are dealt to the XCDs in turn, and the XCDs do not stream equally fast (in the sparse-decode kernel the
// slowest ends 12 % after the mean): a launch of one workgroup per chunk ends with its slowest XCD.  So the
// grid is what the chip holds at once, and every workgroup takes (instance, chunk) units off a counter until
// none is left; a unit is 1024 tokens, 30-40 us of streaming.
template <typename T, int D, int G>
__global__ __launch_bounds__(kAttnThreads) void calibrate_kernel(CalibArgs a) {
  extern __shared__ __align__(16) float smem[];
  __shared__ int s_unit;
  for (;;) {
    if (threadIdx.x == 0) s_unit = atomicAdd(a.counter, 1);
    __syncthreads();
    const int unit = s_unit;
    if (unit >= a.n_units) break;                        // (the same for every thread; every workgroup gets here)
    const int inst = unit / a.n_chunks, chunk = unit - inst * a.n_chunks;
    const int c0 = chunk * a.chunk_blocks;
    const int nblk = min(a.chunk_blocks, a.nb_cur - c0);
    const int ld = a.chunk_blocks * a.b;
    const int ntok = nblk * a.b;
    float* s_p = smem;                    // [G][ld]
    float* s_bmp = s_p + G * ld;          // [G][chunk_blocks]
    float* s_m = s_bmp + G * a.chunk_blocks;
    float* s_l = s_m + G;
    int* s_phys = reinterpret_cast<int*>(s_l + G);   // [chunk_blocks] place of each block of the chunk in K
    float* s_stage = smem + (((reinterpret_cast<float*>(s_phys + a.chunk_blocks) - smem) + 3) & ~3);

    for (int j = threadIdx.x; j < nblk; j += kAttnThreads)
      s_phys[j] = a.table ? min(max(a.table[(size_t)inst * a.nb_cap + c0 + j], 0), a.n_phys - 1) : c0 + j;
    __syncthreads();
    const T* q_inst = static_cast<const T*>(a.q) + (size_t)inst * G * D;
    const T* K_inst = static_cast<const T*>(a.K) + (a.table ? 0 : (size_t)inst * a.t_cap * D);
    constexpr int kStage = std::is_same<T, bf16_t>::value ? kGroupTokens : 0;
    qk_logits<T, D, G, kStage>(q_inst, K_inst, a.b, a.log2b, a.t_cur, ntok, [&](int jb) { return c0 + jb; },
                       [&](int jb) { return s_phys[jb]; }, s_p, ld, s_stage);
    __syncthreads();
    softmax_stats<G>(s_p, ld, ntok, a.b, nblk, s_m, s_l, s_bmp);
    for (int pair = threadIdx.x; pair < G * nblk; pair += kAttnThreads) {
      const int h = pair / nblk, jb = pair - h * nblk;
      a.cal_bmp[((size_t)inst * G + h) * a.nb_cap + c0 + jb] = s_bmp[pair];
    }
    if (threadIdx.x < G) {
      float* ml = a.cal_ml + (((size_t)inst * a.chunk_slots + chunk) * G + threadIdx.x) * 2;
      ml[0] = s_m[threadIdx.x];
      ml[1] = s_l[threadIdx.x];
    }
    __syncthreads();                                     // the next unit overwrites s_unit and the tiles
  }
}

template <int G>
__global__ __launch_bounds__(kAttnThreads) void calibrate_finish_kernel(CalibArgs a) {
  extern __shared__ __align__(16) float smem[];
  const int inst = blockIdx.x;
  float* s_scale = smem;                // [n_chunks][G]
  if (threadIdx.x < G) {
    const int h = threadIdx.x;
    const float* ml = a.cal_ml + ((size_t)inst * a.chunk_slots * G + h) * 2;
    float M = -INFINITY;
    for (int c = 0; c < a.n_chunks; ++c) M = fmaxf(M, ml[(size_t)c * G * 2]);
    float L = 0.f;
    for (int c = 0; c < a.n_chunks; ++c) {
      const float sc = __expf(ml[(size_t)c * G * 2] - M);
      s_scale[c * G + h] = sc;
      L += ml[(size_t)c * G * 2 + 1] * sc;
    }
    const float invL = 1.f / L;
    for (int c = 0; c < a.n_chunks; ++c) s_scale[c * G + h] *= invL;
  }
  __syncthreads();
  float* row = a.row + (size_t)inst * a.nb_cap;
  for (int j = threadIdx.x; j < a.nb_cap; j += kAttnThreads) {
    float mx = 0.f;
    if (j < a.nb_cur) {
      const int c = j / a.chunk_blocks;
#pragma unroll
      for (int h = 0; h < G; ++h)
        mx = fmaxf(mx, a.cal_bmp[((size_t)inst * G + h) * a.nb_cap + j] * s_scale[c * G + h]);
    }
    row[j] = mx;
  }
}

int ilog2(int x) { int l = 0; while ((1 << l) < x) ++l; return l; }

// Workgroups of kernel `fn` (NT threads, lds bytes of LDS) the device holds at once; 0 if it cannot be asked.
template <class Fn> int resident_workgroups(Fn fn, int nt, size_t lds) {
  int per_cu = 0, dev = 0;
  hipDeviceProp_t prop;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, nt, lds) != hipSuccess ||
      hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess)
    return 0;
  return per_cu * prop.multiProcessorCount;
}

template <typename T, int D, int G>
hipError_t run_sparse(const Shape& s, int ninst, SparseArgs a, hipStream_t st) {
  const int nblk_cap = (a.n_split == 1) ? a.k : a.blk_per_split;
  a.piece_blocks = nblk_cap;
  const size_t lds = sizeof(float) * sparse_lds_floats<D, G, kAttnWaves>(nblk_cap, nblk_cap, a.b, a.nb_cap);
  // More instances than the chip holds four-wave workgroups: the launch runs in rounds, the last one part
  // empty, and every round pays its start-up and drain.  Workgroups of two waves or one that keep the
  // probabilities of kNarrowPieceTokens tokens at a time are small enough for more of them to be resident; the
  // widest form with the fewest rounds is used.
  if constexpr (G <= 4) if (a.n_split == 1 && nblk_cap * a.b > kNarrowPieceTokens) {   // (g = 8 would spill in those forms)
    const int pb_n = kNarrowPieceTokens / a.b;
    const size_t lds_2 = sizeof(float) * sparse_lds_floats<D, G, 2>(nblk_cap, pb_n, a.b, a.nb_cap);
    const size_t lds_1 = sizeof(float) * sparse_lds_floats<D, G, 1>(nblk_cap, pb_n, a.b, a.nb_cap);
    if (s.occ->sparse_slots[0] < 0) {
      s.occ->sparse_slots[0] = resident_workgroups(sparse_decode_kernel<T, D, G, kAttnWaves, false>, kAttnThreads, lds);
      s.occ->sparse_slots[1] = resident_workgroups(sparse_decode_kernel<T, D, G, 2, true>, 2 * kWave, lds_2);
      s.occ->sparse_slots[2] = resident_workgroups(sparse_decode_kernel<T, D, G, 1, true>, kWave, lds_1);
    }
    int form = 0, best_rounds = 0;
    for (int f = 0; f < 3; ++f) {
      if (s.occ->sparse_slots[f] <= 0) { form = 0; break; }     // occupancy unknown: stay with the four-wave form
      const int rounds = (ninst + s.occ->sparse_slots[f] - 1) / s.occ->sparse_slots[f];
      if (f == 0 || rounds < best_rounds) { form = f; best_rounds = rounds; }
    }
    if (form != 0) {
      a.piece_blocks = pb_n;
      if (form == 1) sparse_decode_kernel<T, D, G, 2, true><<<dim3(1, ninst), 2 * kWave, lds_2, st>>>(a);
      else sparse_decode_kernel<T, D, G, 1, true><<<dim3(1, ninst), kWave, lds_1, st>>>(a);
      return hipGetLastError();
    }
  }
  sparse_decode_kernel<T, D, G, kAttnWaves, false><<<dim3(a.n_split, ninst), kAttnThreads, lds, st>>>(a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || a.n_split == 1) return e;
  const size_t lds2 = sizeof(float) * ((size_t)a.n_split * G + kCombineCols);
  sparse_combine_kernel<D, G><<<dim3((a.nb_cap + kCombineCols - 1) / kCombineCols, ninst), kAttnThreads, lds2, st>>>(a);
  return hipGetLastError();
}

template <typename T, int D, int G>
hipError_t run_calib(const Shape& s, CalibArgs a, hipStream_t st) {
  const size_t stage = std::is_same<T, bf16_t>::value ? 4 + k_stage_floats<D>() : 0;     // + alignment slack
  const size_t lds = sizeof(float) * ((size_t)G * a.chunk_blocks * a.b + G * a.chunk_blocks + 2 * G + a.chunk_blocks + stage);
  if (s.occ->calib_slots < 0) s.occ->calib_slots = resident_workgroups(calibrate_kernel<T, D, G>, kAttnThreads, lds);
  a.n_units = a.n_chunks * s.n_inst;
  const int slots = s.occ->calib_slots > 0 ? s.occ->calib_slots : 2048;
  zero_counter_kernel<<<1, 1, 0, st>>>(a.counter);
  calibrate_kernel<T, D, G><<<dim3(a.n_units < slots ? a.n_units : slots), kAttnThreads, lds, st>>>(a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  calibrate_finish_kernel<G><<<dim3(s.n_inst), kAttnThreads, sizeof(float) * a.n_chunks * G, st>>>(a);
  return hipGetLastError();
}

#define AP_DISPATCH_G(FN, T, D, ...)                              \
  switch (s.g) {                                                  \
    case 1: return FN<T, D, 1>(__VA_ARGS__);                      \
    case 2: return FN<T, D, 2>(__VA_ARGS__);                      \
    case 4: return FN<T, D, 4>(__VA_ARGS__);                      \
    case 8: return FN<T, D, 8>(__VA_ARGS__);                      \
    default: return hipErrorInvalidValue;                         \
  }
#define AP_DISPATCH(FN, ...)                                                      \
  if (s.kv_dtype == AP_BF16) {                                                    \
    if (s.d == 128) { AP_DISPATCH_G(FN, bf16_t, 128, __VA_ARGS__) }               \
    if (s.d == 64) { AP_DISPATCH_G(FN, bf16_t, 64, __VA_ARGS__) }                 \
  } else {                                                                        \
    if (s.d == 128) { AP_DISPATCH_G(FN, float, 128, __VA_ARGS__) }                \
    if (s.d == 64) { AP_DISPATCH_G(FN, float, 64, __VA_ARGS__) }                  \
  }                                                                               \
  return hipErrorInvalidValue;

}  // namespace

hipError_t launch_sparse_decode(const Shape& s, int inst0, int ninst, const void* q, const void* K, const void* V,
                                int t_cur, const int32_t* idx, const int32_t* cnt, float* out, float* row,
                                size_t row_stride, float* ws, hipStream_t st) {
  const WsLayout wl = ws_layout(s);
  SparseArgs a;
  a.q = q; a.K = K; a.V = V; a.idx = idx; a.cnt = cnt; a.out = out; a.row = row; a.row_stride = row_stride;
  a.part_ml = ws + wl.part_ml; a.part_acc = ws + wl.part_acc; a.part_bmp = ws + wl.part_bmp;
  a.t_cap = s.t_cap; a.nb_cap = s.nb_cap; a.k = s.k; a.b = s.b; a.log2b = ilog2(s.b); a.t_cur = t_cur;
  a.nb_cur = (t_cur + s.b - 1) / s.b;
  a.n_split = s.n_split;
  a.blk_per_split = (s.k + s.n_split - 1) / s.n_split;
  a.inst0 = inst0;
  a.piece_blocks = s.k;
  a.table = s.table; a.n_phys = s.n_phys;
  AP_DISPATCH(run_sparse, s, ninst, a, st)
}

hipError_t static_scratch(float** ptr, size_t* bytes) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* addr[kMaxDevices] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (addr[dev] == nullptr) {                            // once per device, with that device current
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    addr[dev] = p;
  }
  *ptr = static_cast<float*>(addr[dev]);
  *bytes = kStaticScratchBytes;
  return hipSuccess;
}

hipError_t launch_calibrate(const Shape& s, const void* q, const void* K, int t_cur, float* row, float* ws,
                            hipStream_t st) {
  const WsLayout wl = ws_layout(s);
  CalibArgs a;
  a.q = q; a.K = K; a.row = row; a.cal_ml = ws + wl.cal_ml; a.cal_bmp = ws + wl.cal_bmp;
  a.counter = reinterpret_cast<int*>(ws + wl.counters);
  a.t_cap = s.t_cap; a.nb_cap = s.nb_cap; a.b = s.b; a.log2b = ilog2(s.b); a.t_cur = t_cur;
  a.nb_cur = (t_cur + s.b - 1) / s.b;
  a.chunk_blocks = kCalibChunkTokens / s.b;
  a.n_chunks = (a.nb_cur + a.chunk_blocks - 1) / a.chunk_blocks;
  a.chunk_slots = s.calib_chunks;
  a.table = s.table; a.n_phys = s.n_phys;
  AP_DISPATCH(run_calib, s, a, st)
}

}  // namespace ap
