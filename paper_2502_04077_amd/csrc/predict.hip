// The CNN predictor F (Algorithm 1 step 4; architecture table in the appendix "Implement Details"):
//   y1 = relu(conv3x3(x; w1) + b1)      1  -> C1 channels, zero padding 1 on both axes
//   y2 = relu(conv3x3(y1; w2) + b2)     C1 -> C2 channels, zero padding 1 on both axes
//   z  = mean over the H time rows of y2
//   pred = b3 + sum_c w3[c] * z[c]
// evaluated on the H x nb_cur history tile of every instance (axis 0 of the 3x3 kernels is time,
// axis 1 is the block axis; cross-correlation; padding is relative to the current tile at each layer).
//
// Full-tile kernel: a workgroup owns kTW output columns of one instance and walks the time axis in
// strips of kTS rows.  Per strip it stages the x rows (with halo) in LDS, computes the y1 strip
// (kTS + 2 rows, kTW + 2 columns, C1 channels) into LDS, then each thread evaluates y2 for two
// vertically adjacent pixels of its column for all C2 channels from LDS and adds relu(y2) to its
// running time sums.  Weights are read with wave-uniform addresses (scalar loads).
#include "ap_internal.h"

namespace ap {
namespace {

constexpr int kPredThreads = 256;
constexpr int kTW = 64;                 // output columns per workgroup
constexpr int kTS = 8;                  // time rows per strip (4 row pairs, one per wave)
constexpr int kXW = kTW + 4;            // x columns staged (halo 2 per side)
constexpr int kXR = kTS + 4;            // x rows staged per strip
constexpr int kYW = kTW + 2;            // y1 columns staged (halo 1 per side)
constexpr int kYR = kTS + 2;            // y1 rows staged per strip

typedef const float __attribute__((address_space(4))) * const_f32_ptr;

__device__ inline const_f32_ptr as_constant(const float* p) {
  return (const_f32_ptr)(uintptr_t)p;   // weights never change during a launch: read through the scalar cache
}

template <int C1, int C2>
__global__ __launch_bounds__(kPredThreads) void predict_full_kernel(const float* __restrict__ hist,
                                                                    const float* __restrict__ wts_global, int R,
                                                                    int H, int newest_slot, int nb_cur, int nb_cap,
                                                                    float* __restrict__ pred) {
  extern __shared__ __align__(16) float smem[];
  float* s_x = smem;                        // [kXR][kXW]
  float* s_y1 = s_x + kXR * kXW;            // [C1][kYR][kYW]
  float* s_z = s_y1;                        // [4][C2][kTW] after the last strip

  const_f32_ptr W = as_constant(wts_global);
  const_f32_ptr w1r = W;                    // [kh][kw][C1]
  const_f32_ptr b1 = W + 9 * C1;
  const_f32_ptr w2r = W + 10 * C1;          // [ci][kh][kw][C2]
  const_f32_ptr b2 = w2r + 9 * C1 * C2;
  const_f32_ptr w3 = b2 + C2;
  const_f32_ptr b3 = w3 + C2;

  const int inst = blockIdx.y;
  const int c0 = blockIdx.x * kTW;          // first output column of this tile
  const int tid = threadIdx.x;
  const int col = tid & (kTW - 1);
  const int rg = tid / kTW;                 // row pair within the strip
  const float* hist_inst = hist + (size_t)inst * R * nb_cap;

  float zsum[C2];
#pragma unroll
  for (int c = 0; c < C2; ++c) zsum[c] = 0.f;

  for (int r0 = 0; r0 < H; r0 += kTS) {
    // 1. x rows r0-2 .. r0+kTS+1, columns c0-2 .. c0+kTW+1, zero outside the tile.
    for (int e = tid; e < kXR * kXW; e += kPredThreads) {
      const int xr = e / kXW, xc = e - xr * kXW;
      const int r = r0 - 2 + xr, j = c0 - 2 + xc;
      float v = 0.f;
      if (r >= 0 && r < H && j >= 0 && j < nb_cur) {
        int slot = newest_slot - (H - 1 - r);
        slot %= R;
        if (slot < 0) slot += R;
        v = hist_inst[(size_t)slot * nb_cap + j];
      }
      s_x[e] = v;
    }
    __syncthreads();
    // 2. y1 rows r0-1 .. r0+kTS, columns c0-1 .. c0+kTW; zero outside the tile (layer-2 padding).
    for (int e = tid; e < kYR * kYW; e += kPredThreads) {
      const int yr = e / kYW, yc = e - yr * kYW;
      const int r = r0 - 1 + yr, j = c0 - 1 + yc;
      const bool inside = r >= 0 && r < H && j >= 0 && j < nb_cur;
      float x[3][3];
#pragma unroll
      for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) x[kh][kw] = s_x[(yr + kh) * kXW + yc + kw];
#pragma unroll
      for (int c = 0; c < C1; ++c) {
        float a = b1[c];
#pragma unroll
        for (int kh = 0; kh < 3; ++kh)
#pragma unroll
          for (int kw = 0; kw < 3; ++kw) a = fmaf(w1r[(kh * 3 + kw) * C1 + c], x[kh][kw], a);
        s_y1[(c * kYR + yr) * kYW + yc] = inside ? fmaxf(a, 0.f) : 0.f;
      }
    }
    __syncthreads();
    // 3. y2 for rows r0+2rg, r0+2rg+1 of column c0+col, all C2 channels.
    float acc0[C2], acc1[C2];
#pragma unroll
    for (int c = 0; c < C2; ++c) { acc0[c] = b2[c]; acc1[c] = acc0[c]; }
#pragma unroll 1
    for (int ci = 0; ci < C1; ++ci) {
      const float* yb = s_y1 + (ci * kYR + 2 * rg) * kYW + col;
      const_f32_ptr wc = w2r + ci * 9 * C2;
#pragma unroll
      for (int yr = 0; yr < 4; ++yr) {
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
          const float y = yb[yr * kYW + kw];
          if (yr < 3) {
#pragma unroll
            for (int c = 0; c < C2; ++c) acc0[c] = fmaf(wc[(yr * 3 + kw) * C2 + c], y, acc0[c]);
          }
          if (yr > 0) {
#pragma unroll
            for (int c = 0; c < C2; ++c) acc1[c] = fmaf(wc[((yr - 1) * 3 + kw) * C2 + c], y, acc1[c]);
          }
        }
      }
    }
    const int ra = r0 + 2 * rg;
    if (c0 + col < nb_cur) {
      if (ra < H) {
#pragma unroll
        for (int c = 0; c < C2; ++c) zsum[c] += fmaxf(acc0[c], 0.f);
      }
      if (ra + 1 < H) {
#pragma unroll
        for (int c = 0; c < C2; ++c) zsum[c] += fmaxf(acc1[c], 0.f);
      }
    }
    __syncthreads();
  }

  // Sum the four row groups, average over time, apply the 1x1 head.
#pragma unroll
  for (int c = 0; c < C2; ++c) s_z[(rg * C2 + c) * kTW + col] = zsum[c];
  __syncthreads();
  if (tid < kTW && c0 + tid < nb_cur) {
    const float invH = 1.f / (float)H;
    float out = b3[0];
#pragma unroll
    for (int c = 0; c < C2; ++c) {
      const float z = (s_z[(0 * C2 + c) * kTW + tid] + s_z[(1 * C2 + c) * kTW + tid]) +
                      (s_z[(2 * C2 + c) * kTW + tid] + s_z[(3 * C2 + c) * kTW + tid]);
      out = fmaf(w3[c], z * invH, out);
    }
    pred[(size_t)inst * nb_cap + c0 + tid] = out;
  }
}

template <int C1, int C2>
hipError_t run_full(const Shape& s, const float* dweights, const float* hist, int newest_slot, int nb_cur,
                    float* pred, hipStream_t st) {
  static_assert(C1 * kYR * kYW >= 4 * C2 * kTW, "s_z aliases s_y1");
  const size_t lds = sizeof(float) * (kXR * kXW + (size_t)C1 * kYR * kYW);
  const dim3 grid((nb_cur + kTW - 1) / kTW, s.n_inst);
  predict_full_kernel<C1, C2><<<grid, kPredThreads, lds, st>>>(hist, dweights, s.R, s.H, newest_slot, nb_cur,
                                                              s.nb_cap, pred);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_predict(const Shape& s, const float* dweights, const float* hist, int newest_slot,
                          int nb_cur, float* pred, hipStream_t st) {
  if (s.c1 == 4 && s.c2 == 4) return run_full<4, 4>(s, dweights, hist, newest_slot, nb_cur, pred, st);
  if (s.c1 == 8 && s.c2 == 8) return run_full<8, 8>(s, dweights, hist, newest_slot, nb_cur, pred, st);
  if (s.c1 == 16 && s.c2 == 32) return run_full<16, 32>(s, dweights, hist, newest_slot, nb_cur, pred, st);
  return hipErrorInvalidValue;
}

}  // namespace ap
