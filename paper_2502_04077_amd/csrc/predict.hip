// The CNN predictor F (Algorithm 1 step 4; architecture table in the appendix "Implement Details"):
//   y1 = relu(conv3x3(x; w1) + b1)      1  -> C1 channels, zero padding 1 on both axes
//   y2 = relu(conv3x3(y1; w2) + b2)     C1 -> C2 channels, zero padding 1 on both axes
//   z  = mean over the H time rows of y2
//   F  = b3 + sum_c w3[c] * z[c]
// evaluated on the H x nb_cur history tile of every instance (axis 0 of the 3x3 kernels is time,
// axis 1 is the block axis; cross-correlation; padding is relative to the current tile at each layer).
// All kernels work in the difference form described in ap_internal.h and write pred = F - P0, the score relative
// to the network's response P0 to an all-zero history, which every block shares (the selection only ranks).
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
//   state[j] = sum_{r=2}^{H-3} sum_c w3[c] * (y2[c][r][j] - its value for an all-zero history)
// and one step is  state += (row entering the interior) - (row leaving it), plus a fresh evaluation
// of the four border rows 0, 1, H-2, H-1.  That is 6 y2 rows and 8 y1 rows per column instead of H,
// from 10 history rows instead of H; the ring's spare slot still holds the row that left the window,
// which the leaving term needs.  Exact in real arithmetic; in fp32 each step adds two roundings to
// the state, so callers re-base with the full-tile kernel now and then.
#include "predict_body.h"
#include "predict_body16.h"
#include "predict_inc8.h"
#include "predict_interior.h"

namespace ap {
namespace {

template <int C1, int C2>
__global__ __launch_bounds__(kPredThreads) void predict_full_kernel(const float* __restrict__ hist,
                                                                    const float* __restrict__ wts_global, int R,
                                                                    int H, int newest_slot, int nb_cur, int nb_cap,
                                                                    int inst0, int col_begin,
                                                                    float* __restrict__ pstate,
                                                                    float* __restrict__ pred) {
  extern __shared__ __align__(16) float smem[];
  float* s_x = smem;                        // [kXR][kXW]
  float* s_y1 = s_x + kXR * kXW;            // [C1][kYR][kYW]
  float* s_z = s_y1;                        // [4][2][kTW] after the last strip
  const Weights<C1, C2> W(wts_global);

  const int inst = inst0 + blockIdx.y;
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
      float x[3][3];
#pragma unroll
      for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) x[kh][kw] = s_x[(yr + kh) * kXW + yc + kw];
      y1_pixel<C1, C2>(W, x, r >= 0 && r < H, j >= 0 && j < nb_cur, s_y1 + yr * kYW + yc, kYR * kYW);
    }
    __syncthreads();
    // 3. y2 for rows r0+2rg, r0+2rg+1 of column c0+col, all C2 channels.
    const int ra = r0 + 2 * rg;               // (the same for the whole wave: scalar loads of the constants)
    const int ty0 = __builtin_amdgcn_readfirstlane(row_type(ra, H)), ty1 = __builtin_amdgcn_readfirstlane(row_type(ra + 1, H));
    float acc0[C2], acc1[C2];
#pragma unroll
    for (int c = 0; c < C2; ++c) { acc0[c] = W.init2[ty0 * C2 + c]; acc1[c] = W.init2[ty1 * C2 + c]; }
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
    float h0 = 0.f, h1 = 0.f;
#pragma unroll
    for (int c = 0; c < C2; ++c) {
      h0 = fmaf(W.w3[c], fmaxf(acc0[c], W.lo2[ty0 * C2 + c]), h0);
      h1 = fmaf(W.w3[c], fmaxf(acc1[c], W.lo2[ty1 * C2 + c]), h1);
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
    pred[o] = (si + sb) / (float)H;
  }
}

// ---------------------------------------------------------------------------------------------------
// Incremental kernel.  IW output columns per workgroup, 2 * IW threads; the first half of the waves
// ("top") evaluates the row leaving the interior and border rows 0, 1, the second half ("bottom") the
// row entering the interior and border rows H-2, H-1.  Each half stages 5 x rows and 4 y1 rows q0..q3:
//   top    x rows -1..3     q0 = y1 formula on x[-1..1] (row 1 of the previous step's window),
//                           q1 = y1[1], q2 = y1[2], q3 = y1[0] (nothing above the window)
//   bottom x rows H-5..H-1  q0 = y1[H-4], q1 = y1[H-3], q2 = y1[H-2], q3 = y1[H-1] (nothing below)
// and three y2 outputs o0..o2, each the sum over kernel rows kh of (w2 row kh) applied to one q:
//   top    o0 = leaving  row: kh 0,1,2 <- q0,q1,q2    o1 = row 0:   kh 1,2 <- q3,q1     o2 = row 1:   kh 0,1,2 <- q3,q1,q2
//   bottom o0 = entering row: kh 0,1,2 <- q0,q1,q2    o1 = row H-2: kh 0,1,2 <- q1,q2,q3  o2 = row H-1: kh 0,1 <- q2,q3
// o0 has the same operand positions in both halves, so the leaving row is evaluated by the same
// instruction sequence on the same values as when it entered: the two cancel exactly and only the
// two additions into `state` round (VALU and 8/8 MFMA variants; the 16/32 MFMA variant sums the taps of
// the two halves in different orders and cancels up to fp32 rounding).
//
// Variants:
//   VALU  fp32 FMAs, weights through scalar loads (any compiled channel pair; AP_FLAG_PREDICTOR_FP32);
//   MFMA  both layers as 32x32x16 f16 MFMA chains with fp32 accumulation, 32 columns at a time:
//         predict_inc_reg_body (C1 = C2 = 8, predict_inc8.h: both layers in registers) and
//         predict_inc_mfma16_body (C1 = 16, C2 = 32, predict_body16.h: y1 through LDS).

template <int C1, int C2, int HF>
__device__ __forceinline__ void y2_valu(const Weights<C1, C2>& W, const float* yb, int YW, float (&o)[3][C2]) {
#pragma unroll
  for (int k = 0; k < 3; ++k)
#pragma unroll
    for (int c = 0; c < C2; ++c) o[k][c] = W.init2[inc_row_type(HF, k) * C2 + c];
#pragma unroll 1
  for (int ci = 0; ci < C1; ++ci) {
    const_f32_ptr wc = W.w2r + ci * 9 * C2;
    float y[4][3];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int kw = 0; kw < 3; ++kw) y[q][kw] = yb[(q * C1 + ci) * YW + kw];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
      for (int k = 0; k < 3; ++k)
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (predictor_tap(HF, k, q) == kh) {
#pragma unroll
            for (int kw = 0; kw < 3; ++kw)
#pragma unroll
              for (int c = 0; c < C2; ++c) o[k][c] = fmaf(wc[(kh * 3 + kw) * C2 + c], y[q][kw], o[k][c]);
          }
  }
}

// Stages x rows -1..3 (half 0) and H-5..H-1 (half 1), columns c0-2 .. c0-2+XW-1, zero outside the tile.
template <int XW, int NW>
__device__ __forceinline__ void stage_x_rows(float* s_x, const float* hist_inst, int newest_slot, int H, int R, int nb_cap,
                                    int nb_cur, int c0) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  for (int rr = wave; rr < 10; rr += NW) {
    const int hf = rr / 5, xr = rr - hf * 5;
    const int r = hf == 0 ? xr - 1 : H - 5 + xr;
    const float* src = hist_inst + (size_t)ring_slot(newest_slot, H, R, r) * nb_cap;
    for (int xc = lane; xc < XW; xc += kWave) {
      const int j = c0 - 2 + xc;
      s_x[rr * XW + xc] = (j >= 0 && j < nb_cur) ? src[j] : 0.f;
    }
  }
}

// Writes state and pred for column c0 + tid from the four head-weighted partial sums in s_red[2][2][LD].
template <int LD>
__device__ __forceinline__ void finish_column(const float* s_red, int tid, size_t o, int advance, int H, float* pstate,
                                     float* pred) {
  float st = pstate[o];
  if (advance) {
    st = (st - s_red[0 * LD + tid]) + s_red[2 * LD + tid];
    pstate[o] = st;
  }
  pred[o] = (st + (s_red[1 * LD + tid] + s_red[3 * LD + tid])) / (float)H;
}

template <int C1, int C2, int IW>
__global__ __launch_bounds__(2 * IW) void predict_inc_kernel(const float* __restrict__ hist,
                                                             const float* __restrict__ wts_global, int R, int H,
                                                             int newest_slot, int nb_cur, int nb_cap, int inst0,
                                                             int advance, float* __restrict__ pstate,
                                                             float* __restrict__ pred) {
  constexpr int XW = IW + 4, YW = IW + 2, NT = 2 * IW;
  extern __shared__ __align__(16) float smem[];
  float* s_y1 = smem;                       // [2][4][C1][YW]
  float* s_x = s_y1 + 2 * 4 * C1 * YW;      // [2][5][XW]
  float* s_red = s_x + 2 * 5 * XW;          // [2][2][IW]
  const Weights<C1, C2> W(wts_global);

  const int inst = inst0 + blockIdx.y;
  const int c0 = blockIdx.x * IW;
  const int tid = threadIdx.x;
  stage_x_rows<XW, NT / kWave>(s_x, hist + (size_t)inst * R * nb_cap, newest_slot, H, R, nb_cap, nb_cur, c0);
  __syncthreads();
  // y1: thread (half, column) evaluates its four rows q0..q3; the two halo columns of each (half, q) are
  // done by 16 threads in a second pass.
  auto y1_at = [&](int hf, int q, int yc) __attribute__((always_inline)) {
    const int j = c0 - 1 + yc;
    // first staged x row of the 3-row window, and the tap row that lies outside the history window
    const int base = (hf == 0 && q == 3) ? 0 : q;
    const int zero_kh = q == 3 ? (hf == 0 ? 0 : 2) : -1;
    const float* xs = s_x + hf * 5 * XW;
    float x[3][3];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
      for (int kw = 0; kw < 3; ++kw) x[kh][kw] = (kh == zero_kh) ? 0.f : xs[(base + kh) * XW + yc + kw];
    y1_pixel<C1, C2>(W, x, true, j >= 0 && j < nb_cur, s_y1 + ((hf * 4 + q) * C1) * YW + yc, YW);
  };
  {
    const int hf = tid / IW, yc = tid - hf * IW;
#pragma unroll
    for (int q = 0; q < 4; ++q) y1_at(hf, q, yc);
    if (tid < 16) y1_at(tid >> 3, (tid >> 1) & 3, IW + (tid & 1));
  }
  __syncthreads();
  {
    const int hf = tid / IW, col = tid - hf * IW;
    float o[3][C2];
    const float* yb = s_y1 + (size_t)(hf * 4 * C1) * YW + col;
    if (hf == 0) y2_valu<C1, C2, 0>(W, yb, YW, o); else y2_valu<C1, C2, 1>(W, yb, YW, o);
    float moving = 0.f, b1sum = 0.f, b2sum = 0.f;   // head-weighted: the moving row, the two border rows
#pragma unroll
    for (int c = 0; c < C2; ++c) {
      moving = fmaf(W.w3[c], fmaxf(o[0][c], W.lo2[kRowAll * C2 + c]), moving);
      b1sum = fmaf(W.w3[c], fmaxf(o[1][c], W.lo2[(hf == 0 ? kRowTop : kRowAll) * C2 + c]), b1sum);
      b2sum = fmaf(W.w3[c], fmaxf(o[2][c], W.lo2[(hf == 0 ? kRowAll : kRowBot) * C2 + c]), b2sum);
    }
    s_red[(hf * 2 + 0) * IW + col] = moving;
    s_red[(hf * 2 + 1) * IW + col] = b1sum + b2sum;
  }
  __syncthreads();
  if (tid < IW && c0 + tid < nb_cur)
    finish_column<IW>(s_red, tid, (size_t)inst * nb_cap + c0 + tid, advance, H, pstate, pred);
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4)))   // four workgroups per CU: 128 VGPRs
void predict_inc_mfma_kernel(const float* __restrict__ hist, const float* __restrict__ wts_global, int R, int H,
                             int newest_slot, int nb_cur, int nb_cap, int inst0, int advance,
                             float* __restrict__ pstate, float* __restrict__ pred) {
  extern __shared__ __align__(16) float smem[];
  predict_inc_reg_body(hist, wts_global, R, H, newest_slot, nb_cur, nb_cap, inst0 + blockIdx.y, blockIdx.x, gridDim.x,
                       advance, pstate, pred, smem);
}

__global__ __launch_bounds__(256) void predict_inc_mfma16_kernel(const float* __restrict__ hist,
                                                                 const float* __restrict__ wts_global, int R, int H,
                                                                 int newest_slot, int nb_cur, int nb_cap, int inst0,
                                                                 int advance, float* __restrict__ pstate,
                                                                 float* __restrict__ pred) {
  extern __shared__ __align__(16) float smem[];
  predict_inc_mfma16_body(hist, wts_global, R, H, newest_slot, nb_cur, nb_cap, inst0 + blockIdx.y, blockIdx.x,
                          gridDim.x, advance, pstate, pred, smem);
}

__global__ __launch_bounds__(256) void predict_interior_mfma_kernel(const float* __restrict__ hist,
                                                                    const float* __restrict__ wts_global, int R, int H,
                                                                    int newest_slot, int nb_cur, int nb_cap, int inst0,
                                                                    float* __restrict__ pstate) {
  extern __shared__ __align__(16) float smem[];
  predict_interior_mfma_body(hist, wts_global, R, H, newest_slot, nb_cur, nb_cap, inst0 + blockIdx.y, blockIdx.x,
                             gridDim.x, pstate, smem);
}

__global__ __launch_bounds__(256) void predict_interior_mfma16_kernel(const float* __restrict__ hist,
                                                                      const float* __restrict__ wts_global, int R,
                                                                      int H, int newest_slot, int nb_cur, int nb_cap,
                                                                      int inst0, float* __restrict__ pstate) {
  extern __shared__ __align__(16) float smem[];
  predict_interior_mfma16_body(hist, wts_global, R, H, newest_slot, nb_cur, nb_cap, inst0 + blockIdx.y, blockIdx.x,
                               gridDim.x, pstate, smem);
}

// Full evaluation of a few columns (the ones whose state is void after the tile has grown by a block):
// one wave per (instance, column), lanes are time rows.  A lane fetches the five x values of its own row (one
// 32-byte sector of the ring) into LDS, takes the 5 x 5 neighbourhood of its pixel from there (the rows above
// and below were fetched by the neighbouring lanes) and evaluates y1 on the 3 x 3 pixels around it channel by
// channel, feeding y2.
template <int C1, int C2>
__global__ __launch_bounds__(kWave) void predict_columns_kernel(const float* __restrict__ hist,
                                                                const float* __restrict__ wts_global, int R, int H,
                                                                int newest_slot, int nb_cur, int nb_cap, int inst0,
                                                                int col_begin, float* __restrict__ pstate,
                                                                float* __restrict__ pred) {
  const Weights<C1, C2> W(wts_global);
  const int inst = inst0 + blockIdx.y;
  const int j = col_begin + blockIdx.x;
  const int lane = threadIdx.x;
  const float* hist_inst = hist + (size_t)inst * R * nb_cap;
  __shared__ float s_x[(kMaxHist + 4) * 5];              // rows -2 .. H + 1 of columns j - 2 .. j + 2, zero outside the tile
  for (int r = lane; r < H + 4; r += kWave) {
    const int rr = r - 2;
    const bool row_ok = rr >= 0 && rr < H;
    const float* src = hist_inst + (size_t)ring_slot(newest_slot, H, R, row_ok ? rr : 0) * nb_cap;
#pragma unroll
    for (int dc = 0; dc < 5; ++dc) {
      const int jj = j - 2 + dc;
      const float v = src[min(max(jj, 0), nb_cur - 1)];
      s_x[r * 5 + dc] = (row_ok && jj >= 0 && jj < nb_cur) ? v : 0.f;
    }
  }
  __syncthreads();
  float w_int = 0.f, w_bor = 0.f;
  for (int r = lane; r < H; r += kWave) {
    float x[5][5];
#pragma unroll
    for (int dr = 0; dr < 5; ++dr)
#pragma unroll
      for (int dc = 0; dc < 5; ++dc) x[dr][dc] = s_x[(r + dr) * 5 + dc];
    const float* init2 = wts_global + delta_const_offset(C1, C2) + 2 * C1 + row_type(r, H) * C2;   // (per lane)
    float acc[C2];
#pragma unroll
    for (int c = 0; c < C2; ++c) acc[c] = init2[c];
#pragma unroll 1
    for (int ci = 0; ci < C1; ++ci) {
      const_f32_ptr wc = W.w2r + ci * 9 * C2;
      const float lo = W.lo1[ci];
#pragma unroll
      for (int kh = 0; kh < 3; ++kh)
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
          // d1[ci] at (r + kh - 1, j + kw - 1): lo1 beside the tile, left out above and below the window
          const int rr = r + kh - 1, jj = j + kw - 1;
          float a = W.init1[ci];
#pragma unroll
          for (int a_kh = 0; a_kh < 3; ++a_kh)
#pragma unroll
            for (int a_kw = 0; a_kw < 3; ++a_kw)
              a = fmaf(W.w1r[(a_kh * 3 + a_kw) * C1 + ci], x[kh + a_kh][kw + a_kw], a);
          const float y = (rr >= 0 && rr < H) ? ((jj >= 0 && jj < nb_cur) ? fmaxf(a, lo) : lo) : 0.f;
#pragma unroll
          for (int c = 0; c < C2; ++c) acc[c] = fmaf(wc[(kh * 3 + kw) * C2 + c], y, acc[c]);
        }
    }
    float hsum = 0.f;
#pragma unroll
    for (int c = 0; c < C2; ++c) hsum = fmaf(W.w3[c], fmaxf(acc[c], init2[4 * C2 + c]), hsum);
    if (r >= 2 && r <= H - 3) w_int += hsum; else w_bor += hsum;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    w_int += __shfl_xor(w_int, o, kWave);
    w_bor += __shfl_xor(w_bor, o, kWave);
  }
  if (lane == 0) {
    const size_t o = (size_t)inst * nb_cap + j;
    if (pstate != nullptr) pstate[o] = w_int;
    pred[o] = (w_int + w_bor) / (float)H;
  }
}

template <int C1, int C2>
hipError_t run_columns(const Shape& s, int inst0, int ninst, const float* dweights, const float* hist, int newest_slot,
                       int nb_cur, int col_begin, float* pstate, float* pred, hipStream_t st) {
  predict_columns_kernel<C1, C2><<<dim3(nb_cur - col_begin, ninst), kWave, 0, st>>>(
      hist, dweights, s.R, s.H, newest_slot, nb_cur, s.nb_cap, inst0, col_begin, pstate, pred);
  return hipGetLastError();
}

template <int C1, int C2>
hipError_t run_full(const Shape& s, int inst0, int ninst, const float* dweights, const float* hist, int newest_slot,
                    int nb_cur, int col_begin, float* pstate, float* pred, hipStream_t st) {
  static_assert(C1 * kYR * kYW >= 8 * kTW, "s_z aliases s_y1");
  const size_t lds = sizeof(float) * (kXR * kXW + (size_t)C1 * kYR * kYW);
  const dim3 grid((nb_cur - col_begin + kTW - 1) / kTW, ninst);
  predict_full_kernel<C1, C2><<<grid, kPredThreads, lds, st>>>(hist, dweights, s.R, s.H, newest_slot, nb_cur,
                                                              s.nb_cap, inst0, col_begin, pstate, pred);
  return hipGetLastError();
}

template <int C1, int C2>
hipError_t run_inc(const Shape& s, int inst0, int ninst, const float* dweights, const float* hist, int newest_slot,
                   int nb_cur, int advance, float* pstate, float* pred, hipStream_t st) {
  if (C1 == 8 && C2 == 8 && s.predictor_mfma) {
    const size_t lds = sizeof(float) * kPredRegLdsFloats;
    const int blocks = (nb_cur + kRiOut - 1) / kRiOut;
    int chunks = (2048 + s.n_inst - 1) / s.n_inst;       // about eight workgroups per CU when instances are few
    if (chunks > (blocks + 3) / 4) chunks = (blocks + 3) / 4;   // at least a block per wave
    predict_inc_mfma_kernel<<<dim3(chunks, ninst), 256, lds, st>>>(
        hist, dweights, s.R, s.H, newest_slot, nb_cur, s.nb_cap, inst0, advance, pstate, pred);
    return hipGetLastError();
  }
  if (C1 == 16 && C2 == 32 && s.predictor_mfma) {
    const size_t lds = sizeof(float) * kPred16LdsFloats;
    const int tiles = (nb_cur + kP16IW - 1) / kP16IW;
    int chunks = (1024 + s.n_inst - 1) / s.n_inst;       // two workgroups fit a CU
    if (chunks > tiles) chunks = tiles;
    predict_inc_mfma16_kernel<<<dim3(chunks, ninst), 256, lds, st>>>(
        hist, dweights, s.R, s.H, newest_slot, nb_cur, s.nb_cap, inst0, advance, pstate, pred);
    return hipGetLastError();
  }
  constexpr int IW = C1 <= 8 ? 128 : 64;
  const size_t lds = sizeof(float) * (2 * 4 * (size_t)C1 * (IW + 2) + 2 * 5 * (IW + 4) + 4 * IW);
  predict_inc_kernel<C1, C2, IW><<<dim3((nb_cur + IW - 1) / IW, ninst), 2 * IW, lds, st>>>(
      hist, dweights, s.R, s.H, newest_slot, nb_cur, s.nb_cap, inst0, advance, pstate, pred);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_predict(const Shape& s, int inst0, int ninst, const float* dweights, const float* hist,
                          int newest_slot, int nb_cur, int col_begin, float* pstate, float* pred, hipStream_t st) {
  if (s.c1 == 4 && s.c2 == 4)
    return run_full<4, 4>(s, inst0, ninst, dweights, hist, newest_slot, nb_cur, col_begin, pstate, pred, st);
  if (s.c1 == 8 && s.c2 == 8)
    return run_full<8, 8>(s, inst0, ninst, dweights, hist, newest_slot, nb_cur, col_begin, pstate, pred, st);
  if (s.c1 == 16 && s.c2 == 32)
    return run_full<16, 32>(s, inst0, ninst, dweights, hist, newest_slot, nb_cur, col_begin, pstate, pred, st);
  return hipErrorInvalidValue;
}

hipError_t launch_predict_interior(const Shape& s, int inst0, int ninst, const float* dweights, const float* hist,
                                   int newest_slot, int nb_cur, float* pstate, hipStream_t st) {
  const bool c8 = s.c1 == 8 && s.c2 == 8, c16 = s.c1 == 16 && s.c2 == 32;
  if (!(c8 || c16) || s.H < 6) return hipErrorInvalidValue;
  const int groups = (nb_cur + 4 * kPiOut - 1) / (4 * kPiOut);
  int chunks = (2048 + s.n_inst - 1) / s.n_inst;         // about eight workgroups per CU when instances are few
  if (chunks > groups) chunks = groups;
  if (c8)
    predict_interior_mfma_kernel<<<dim3(chunks, ninst), 256, sizeof(float) * kPredInteriorLdsFloats, st>>>(
        hist, dweights, s.R, s.H, newest_slot, nb_cur, s.nb_cap, inst0, pstate);
  else
    predict_interior_mfma16_kernel<<<dim3(chunks, ninst), 256, sizeof(float) * kPredInterior16LdsFloats, st>>>(
        hist, dweights, s.R, s.H, newest_slot, nb_cur, s.nb_cap, inst0, pstate);
  return hipGetLastError();
}

hipError_t launch_predict_columns(const Shape& s, int inst0, int ninst, const float* dweights, const float* hist,
                                  int newest_slot, int nb_cur, int col_begin, float* pstate, float* pred,
                                  hipStream_t st) {
  if (s.c1 == 4 && s.c2 == 4)
    return run_columns<4, 4>(s, inst0, ninst, dweights, hist, newest_slot, nb_cur, col_begin, pstate, pred, st);
  if (s.c1 == 8 && s.c2 == 8)
    return run_columns<8, 8>(s, inst0, ninst, dweights, hist, newest_slot, nb_cur, col_begin, pstate, pred, st);
  if (s.c1 == 16 && s.c2 == 32)
    return run_columns<16, 32>(s, inst0, ninst, dweights, hist, newest_slot, nb_cur, col_begin, pstate, pred, st);
  return hipErrorInvalidValue;
}

hipError_t launch_predict_inc(const Shape& s, int inst0, int ninst, const float* dweights, const float* hist,
                              int newest_slot, int nb_cur, int advance, float* pstate, float* pred, hipStream_t st) {
  if (s.c1 == 4 && s.c2 == 4)
    return run_inc<4, 4>(s, inst0, ninst, dweights, hist, newest_slot, nb_cur, advance, pstate, pred, st);
  if (s.c1 == 8 && s.c2 == 8)
    return run_inc<8, 8>(s, inst0, ninst, dweights, hist, newest_slot, nb_cur, advance, pstate, pred, st);
  if (s.c1 == 16 && s.c2 == 32)
    return run_inc<16, 32>(s, inst0, ninst, dweights, hist, newest_slot, nb_cur, advance, pstate, pred, st);
  return hipErrorInvalidValue;
}

}  // namespace ap
