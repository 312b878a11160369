// The CNN predictor F (Algorithm 1 step 4; architecture table in the appendix "Implement Details"):
//   y1 = relu(conv3x3(x; w1) + b1)      1  -> C1 channels, zero padding 1 on both axes
//   y2 = relu(conv3x3(y1; w2) + b2)     C1 -> C2 channels, zero padding 1 on both axes
//   z  = mean over the H time rows of y2
//   pred = b3 + sum_c w3[c] * z[c]
// evaluated on the H x nb_cur history tile of every instance (axis 0 of the 3x3 kernels is time,
// axis 1 is the block axis; cross-correlation; padding is relative to the current tile at each layer).
//
// Two kernels compute it.
//
// Full-tile kernel: a workgroup owns kTW output columns of one instance and walks the time axis in
// strips of kTS rows.  Per strip it stages the x rows (with halo) in LDS, computes the y1 strip
// (kTS + 2 rows, kTW + 2 columns, C1 channels) into LDS, then each thread evaluates y2 for two
// vertically adjacent pixels of its column for all C2 channels from LDS.  Weights are read with
// wave-uniform addresses (scalar loads).
//
// Incremental kernel: the history only shifts by one row per decode step, and both convolutions
// commute with a time shift away from the zero-padded first/last rows.  y2 row r depends on x rows
// r-2..r+2, so rows 2..H-3 ("interior") of one step are rows 1..H-4 of the next.  Because the head is
// linear, one float per column carries everything the interior contributes:
//   state[j] = sum_{r=2}^{H-3} sum_c w3[c] * y2[c][r][j]
// and one step is  state += (row entering the interior) - (row leaving it), plus a fresh evaluation
// of the four border rows 0, 1, H-2, H-1.  That is 6 y2 rows and 8 y1 rows per column instead of H,
// from 10 history rows instead of H; the ring's spare slot still holds the row that left the window,
// which the leaving term needs.  Exact in real arithmetic; in fp32 each step adds two roundings to
// the state, so callers re-base with the full-tile kernel now and then.
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

template <int C1, int C2> struct Weights {
  const_f32_ptr w1r, b1, w2r, b2, w3, b3;
  __device__ explicit Weights(const float* g) {
    const_f32_ptr W = as_constant(g);
    w1r = W;                              // [kh][kw][C1]
    b1 = W + 9 * C1;
    w2r = W + 10 * C1;                    // [ci][kh][kw][C2]
    b2 = w2r + 9 * C1 * C2;
    w3 = b2 + C2;
    b3 = w3 + C2;
  }
};

__device__ inline int ring_slot(int newest_slot, int H, int R, int r) {
  int slot = (newest_slot - (H - 1 - r)) % R;   // logical row r (H-1 = newest, -1 = the row that just left)
  return slot < 0 ? slot + R : slot;
}

// One y1 pixel, all C1 channels, from a 3x3 x neighbourhood.
template <int C1, int C2>
__device__ inline void y1_pixel(const Weights<C1, C2>& W, const float (&x)[3][3], bool inside, float* dst,
                                int chan_stride) {
#pragma unroll
  for (int c = 0; c < C1; ++c) {
    float a = W.b1[c];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
      for (int kw = 0; kw < 3; ++kw) a = fmaf(W.w1r[(kh * 3 + kw) * C1 + c], x[kh][kw], a);
    dst[c * chan_stride] = inside ? fmaxf(a, 0.f) : 0.f;
  }
}

template <int C1, int C2>
__global__ __launch_bounds__(kPredThreads) void predict_full_kernel(const float* __restrict__ hist,
                                                                    const float* __restrict__ wts_global, int R,
                                                                    int H, int newest_slot, int nb_cur, int nb_cap,
                                                                    int col_begin, float* __restrict__ pstate,
                                                                    float* __restrict__ pred) {
  extern __shared__ __align__(16) float smem[];
  float* s_x = smem;                        // [kXR][kXW]
  float* s_y1 = s_x + kXR * kXW;            // [C1][kYR][kYW]
  float* s_z = s_y1;                        // [4][2][kTW] after the last strip
  const Weights<C1, C2> W(wts_global);

  const int inst = blockIdx.y;
  const int c0 = col_begin + blockIdx.x * kTW;   // first output column of this tile
  const int tid = threadIdx.x;
  const int col = tid & (kTW - 1);
  const int rg = tid / kTW;                 // row pair within the strip
  const float* hist_inst = hist + (size_t)inst * R * nb_cap;

  float w_int = 0.f, w_bor = 0.f;           // head-weighted time sums: interior rows 2..H-3, border rows

  for (int r0 = 0; r0 < H; r0 += kTS) {
    // 1. x rows r0-2 .. r0+kTS+1, columns c0-2 .. c0+kTW+1, zero outside the tile.
    for (int e = tid; e < kXR * kXW; e += kPredThreads) {
      const int xr = e / kXW, xc = e - xr * kXW;
      const int r = r0 - 2 + xr, j = c0 - 2 + xc;
      float v = 0.f;
      if (r >= 0 && r < H && j >= 0 && j < nb_cur) v = hist_inst[(size_t)ring_slot(newest_slot, H, R, r) * nb_cap + j];
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
      y1_pixel<C1, C2>(W, x, inside, s_y1 + yr * kYW + yc, kYR * kYW);
    }
    __syncthreads();
    // 3. y2 for rows r0+2rg, r0+2rg+1 of column c0+col, all C2 channels.
    float acc0[C2], acc1[C2];
#pragma unroll
    for (int c = 0; c < C2; ++c) { acc0[c] = W.b2[c]; acc1[c] = acc0[c]; }
#pragma unroll 1
    for (int ci = 0; ci < C1; ++ci) {
      const float* yb = s_y1 + (ci * kYR + 2 * rg) * kYW + col;
      const_f32_ptr wc = W.w2r + ci * 9 * C2;
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
    float h0 = 0.f, h1 = 0.f;
#pragma unroll
    for (int c = 0; c < C2; ++c) {
      h0 = fmaf(W.w3[c], fmaxf(acc0[c], 0.f), h0);
      h1 = fmaf(W.w3[c], fmaxf(acc1[c], 0.f), h1);
    }
    if (ra < H) { if (ra >= 2 && ra <= H - 3) w_int += h0; else w_bor += h0; }
    if (ra + 1 < H) { if (ra + 1 >= 2 && ra + 1 <= H - 3) w_int += h1; else w_bor += h1; }
    __syncthreads();
  }

  // Sum the four row groups, average over time, add the head bias.
  s_z[(rg * 2 + 0) * kTW + col] = w_int;
  s_z[(rg * 2 + 1) * kTW + col] = w_bor;
  __syncthreads();
  if (tid < kTW && c0 + tid < nb_cur) {
    const float si = (s_z[0 * kTW + tid] + s_z[2 * kTW + tid]) + (s_z[4 * kTW + tid] + s_z[6 * kTW + tid]);
    const float sb = (s_z[1 * kTW + tid] + s_z[3 * kTW + tid]) + (s_z[5 * kTW + tid] + s_z[7 * kTW + tid]);
    const size_t o = (size_t)inst * nb_cap + c0 + tid;
    if (pstate != nullptr) pstate[o] = si;
    pred[o] = W.b3[0] + (si + sb) / (float)H;
  }
}

// ---------------------------------------------------------------------------------------------------
// Incremental kernel.  IW output columns per workgroup, 2 * IW threads: threads [0, IW) ("top") evaluate
// the row leaving the interior and border rows 0, 1; threads [IW, 2 IW) ("bottom") the row entering the
// interior and border rows H-2, H-1.  Each half stages 5 x rows and 4 y1 rows:
//   top    x rows -1..3     y1: q0 = interior formula on x[-1..1]   (row 1 of the previous step's window)
//                               q1 = y1[0] (nothing above the window), q2 = y1[1], q3 = y1[2]
//          y2: leaving = (q0,q2,q3)   row0 = (-,q1,q2)   row1 = (q1,q2,q3)            [taps kh = 0,1,2]
//   bottom x rows H-5..H-1  y1: q0 = y1[H-4], q1 = y1[H-3], q2 = y1[H-2], q3 = y1[H-1] (nothing below)
//          y2: entering = row H-3 = (q0,q1,q2)   row H-2 = (q1,q2,q3)   row H-1 = (q2,q3,-)
// The leaving row is evaluated by the same instruction sequence, on the same x values, as when it
// entered, so the two cancel exactly and only the additions into `state` round.
template <int C1, int C2, int IW>
__global__ __launch_bounds__(2 * IW) void predict_inc_kernel(const float* __restrict__ hist,
                                                             const float* __restrict__ wts_global, int R, int H,
                                                             int newest_slot, int nb_cur, int nb_cap, int advance,
                                                             float* __restrict__ pstate, float* __restrict__ pred) {
  constexpr int XW = IW + 4, YW = IW + 2, NT = 2 * IW;
  extern __shared__ __align__(16) float smem[];
  float* s_x = smem;                        // [2][5][XW]
  float* s_y1 = s_x + 2 * 5 * XW;           // [2][4][C1][YW]
  float* s_red = s_y1 + 2 * 4 * C1 * YW;    // [2][2][IW]
  const Weights<C1, C2> W(wts_global);

  const int inst = blockIdx.y;
  const int c0 = blockIdx.x * IW;
  const int tid = threadIdx.x;
  const float* hist_inst = hist + (size_t)inst * R * nb_cap;

  for (int e = tid; e < 2 * 5 * XW; e += NT) {
    const int hf = e / (5 * XW), rem = e - hf * 5 * XW;
    const int xr = rem / XW, xc = rem - xr * XW;
    const int r = hf == 0 ? xr - 1 : H - 5 + xr;
    const int j = c0 - 2 + xc;
    float v = 0.f;
    if (j >= 0 && j < nb_cur) v = hist_inst[(size_t)ring_slot(newest_slot, H, R, r) * nb_cap + j];
    s_x[e] = v;
  }
  __syncthreads();
  for (int e = tid; e < 2 * 4 * YW; e += NT) {
    const int hf = e / (4 * YW), rem = e - hf * 4 * YW;
    const int q = rem / YW, yc = rem - q * YW;
    const int j = c0 - 1 + yc;
    // first x row of the 3-row window, and which tap row lies outside the history window
    const int base = hf == 0 ? (q <= 1 ? 0 : q - 1) : q;
    const int zero_kh = hf == 0 ? (q == 1 ? 0 : -1) : (q == 3 ? 2 : -1);
    const float* xs = s_x + hf * 5 * XW;
    float x[3][3];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
      for (int kw = 0; kw < 3; ++kw) x[kh][kw] = (kh == zero_kh) ? 0.f : xs[(base + kh) * XW + yc + kw];
    y1_pixel<C1, C2>(W, x, j >= 0 && j < nb_cur, s_y1 + ((hf * 4 + q) * C1) * YW + yc, YW);
  }
  __syncthreads();

  const int hf = tid / IW, col = tid - hf * IW;
  float o0[C2], o1[C2], o2[C2];
#pragma unroll
  for (int c = 0; c < C2; ++c) { o0[c] = W.b2[c]; o1[c] = o0[c]; o2[c] = o0[c]; }
#pragma unroll 1
  for (int ci = 0; ci < C1; ++ci) {
    const float* yb = s_y1 + ((hf * 4) * C1 + ci) * YW + col;
    const_f32_ptr wc = W.w2r + ci * 9 * C2;
    float y[4][3];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int kw = 0; kw < 3; ++kw) y[q][kw] = yb[q * C1 * YW + kw];
    // tap tables (y1 row q feeding tap kh of each output), -1 = outside the window
    if (hf == 0) {
#pragma unroll
      for (int kw = 0; kw < 3; ++kw)
#pragma unroll
        for (int c = 0; c < C2; ++c) {
          o0[c] = fmaf(wc[(0 * 3 + kw) * C2 + c], y[0][kw], o0[c]);
          o2[c] = fmaf(wc[(0 * 3 + kw) * C2 + c], y[1][kw], o2[c]);
        }
#pragma unroll
      for (int kw = 0; kw < 3; ++kw)
#pragma unroll
        for (int c = 0; c < C2; ++c) {
          o0[c] = fmaf(wc[(1 * 3 + kw) * C2 + c], y[2][kw], o0[c]);
          o1[c] = fmaf(wc[(1 * 3 + kw) * C2 + c], y[1][kw], o1[c]);
          o2[c] = fmaf(wc[(1 * 3 + kw) * C2 + c], y[2][kw], o2[c]);
        }
#pragma unroll
      for (int kw = 0; kw < 3; ++kw)
#pragma unroll
        for (int c = 0; c < C2; ++c) {
          o0[c] = fmaf(wc[(2 * 3 + kw) * C2 + c], y[3][kw], o0[c]);
          o1[c] = fmaf(wc[(2 * 3 + kw) * C2 + c], y[2][kw], o1[c]);
          o2[c] = fmaf(wc[(2 * 3 + kw) * C2 + c], y[3][kw], o2[c]);
        }
    } else {
#pragma unroll
      for (int kw = 0; kw < 3; ++kw)
#pragma unroll
        for (int c = 0; c < C2; ++c) {
          o0[c] = fmaf(wc[(0 * 3 + kw) * C2 + c], y[0][kw], o0[c]);
          o1[c] = fmaf(wc[(0 * 3 + kw) * C2 + c], y[1][kw], o1[c]);
          o2[c] = fmaf(wc[(0 * 3 + kw) * C2 + c], y[2][kw], o2[c]);
        }
#pragma unroll
      for (int kw = 0; kw < 3; ++kw)
#pragma unroll
        for (int c = 0; c < C2; ++c) {
          o0[c] = fmaf(wc[(1 * 3 + kw) * C2 + c], y[1][kw], o0[c]);
          o1[c] = fmaf(wc[(1 * 3 + kw) * C2 + c], y[2][kw], o1[c]);
          o2[c] = fmaf(wc[(1 * 3 + kw) * C2 + c], y[3][kw], o2[c]);
        }
#pragma unroll
      for (int kw = 0; kw < 3; ++kw)
#pragma unroll
        for (int c = 0; c < C2; ++c) {
          o0[c] = fmaf(wc[(2 * 3 + kw) * C2 + c], y[2][kw], o0[c]);
          o1[c] = fmaf(wc[(2 * 3 + kw) * C2 + c], y[3][kw], o1[c]);
        }
    }
  }
  float moving = 0.f, border = 0.f;         // head-weighted: the row leaving/entering, the two border rows
#pragma unroll
  for (int c = 0; c < C2; ++c) {
    moving = fmaf(W.w3[c], fmaxf(o0[c], 0.f), moving);
    border = fmaf(W.w3[c], fmaxf(o1[c], 0.f), border);
  }
#pragma unroll
  for (int c = 0; c < C2; ++c) border = fmaf(W.w3[c], fmaxf(o2[c], 0.f), border);
  s_red[(hf * 2 + 0) * IW + col] = moving;
  s_red[(hf * 2 + 1) * IW + col] = border;
  __syncthreads();
  if (tid < IW && c0 + tid < nb_cur) {
    const size_t o = (size_t)inst * nb_cap + c0 + tid;
    float st = pstate[o];
    if (advance) {
      st = (st - s_red[0 * IW + tid]) + s_red[2 * IW + tid];
      pstate[o] = st;
    }
    pred[o] = W.b3[0] + (st + (s_red[1 * IW + tid] + s_red[3 * IW + tid])) / (float)H;
  }
}

template <int C1, int C2>
hipError_t run_full(const Shape& s, const float* dweights, const float* hist, int newest_slot, int nb_cur,
                    int col_begin, float* pstate, float* pred, hipStream_t st) {
  static_assert(C1 * kYR * kYW >= 8 * kTW, "s_z aliases s_y1");
  const size_t lds = sizeof(float) * (kXR * kXW + (size_t)C1 * kYR * kYW);
  const dim3 grid((nb_cur - col_begin + kTW - 1) / kTW, s.n_inst);
  predict_full_kernel<C1, C2><<<grid, kPredThreads, lds, st>>>(hist, dweights, s.R, s.H, newest_slot, nb_cur,
                                                              s.nb_cap, col_begin, pstate, pred);
  return hipGetLastError();
}

template <int C1, int C2>
hipError_t run_inc(const Shape& s, const float* dweights, const float* hist, int newest_slot, int nb_cur,
                   int advance, float* pstate, float* pred, hipStream_t st) {
  constexpr int IW = C1 <= 8 ? 128 : 64;
  const size_t lds = sizeof(float) * (2 * 5 * (IW + 4) + 2 * 4 * (size_t)C1 * (IW + 2) + 4 * IW);
  const dim3 grid((nb_cur + IW - 1) / IW, s.n_inst);
  predict_inc_kernel<C1, C2, IW><<<grid, 2 * IW, lds, st>>>(hist, dweights, s.R, s.H, newest_slot, nb_cur,
                                                           s.nb_cap, advance, pstate, pred);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_predict(const Shape& s, const float* dweights, const float* hist, int newest_slot,
                          int nb_cur, int col_begin, float* pstate, float* pred, hipStream_t st) {
  if (s.c1 == 4 && s.c2 == 4) return run_full<4, 4>(s, dweights, hist, newest_slot, nb_cur, col_begin, pstate, pred, st);
  if (s.c1 == 8 && s.c2 == 8) return run_full<8, 8>(s, dweights, hist, newest_slot, nb_cur, col_begin, pstate, pred, st);
  if (s.c1 == 16 && s.c2 == 32)
    return run_full<16, 32>(s, dweights, hist, newest_slot, nb_cur, col_begin, pstate, pred, st);
  return hipErrorInvalidValue;
}

hipError_t launch_predict_inc(const Shape& s, const float* dweights, const float* hist, int newest_slot,
                              int nb_cur, int advance, float* pstate, float* pred, hipStream_t st) {
  if (s.c1 == 4 && s.c2 == 4) return run_inc<4, 4>(s, dweights, hist, newest_slot, nb_cur, advance, pstate, pred, st);
  if (s.c1 == 8 && s.c2 == 8) return run_inc<8, 8>(s, dweights, hist, newest_slot, nb_cur, advance, pstate, pred, st);
  if (s.c1 == 16 && s.c2 == 32)
    return run_inc<16, 32>(s, dweights, hist, newest_slot, nb_cur, advance, pstate, pred, st);
  return hipErrorInvalidValue;
}

}  // namespace ap
