// Shared device code of the predictor kernels: weight access, ring addressing, operand types and the tile
// geometry of the LDS-staged MFMA kernels (see predict.hip for the method).
#pragma once

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

__device__ __forceinline__ const_f32_ptr as_constant(const float* p) {
  return (const_f32_ptr)(uintptr_t)p;   // weights never change during a launch: read through the scalar cache
}

template <int C1, int C2> struct Weights {
  const_f32_ptr w1r, w2r, w3;
  const_f32_ptr init1, lo1, init2, lo2;       // constants of the difference form (ap_internal.h)
  __device__ explicit Weights(const float* g) {
    const_f32_ptr W = as_constant(g);
    w1r = W;                              // [kh][kw][C1]
    w2r = W + 10 * C1;                    // [ci][kh][kw][C2]
    w3 = w2r + 9 * C1 * C2 + C2;
    init1 = W + delta_const_offset(C1, C2);
    lo1 = init1 + C1;
    init2 = lo1 + C1;                     // [type][C2]
    lo2 = init2 + 4 * C2;                 // [type][C2]
  }
};

// Row type of history row r (which kernel rows of the second layer fall inside the window).
__device__ __forceinline__ int row_type(int r, int H) { return (r == 0 ? 1 : 0) + (r == H - 1 ? 2 : 0); }

__device__ __forceinline__ int ring_slot(int newest_slot, int H, int R, int r) {
  int slot = (newest_slot - (H - 1 - r)) % R;   // logical row r (H-1 = newest, -1 = the row that just left)
  return slot < 0 ? slot + R : slot;
}

// One first-layer pixel, all C1 channels, from a 3x3 x neighbourhood, as the difference d1 = y1 - relu(b1).
// A pixel beside the tile in its own row stands for y1 = 0 (layer-2 padding), i.e. d1 = -relu(b1) = lo1; a pixel
// of a row outside the window is left out of the second layer's sums altogether (its constant is not part of
// that row type's B2), i.e. 0.
template <int C1, int C2>
__device__ __forceinline__ void y1_pixel(const Weights<C1, C2>& W, const float (&x)[3][3], bool row_inside,
                                bool col_inside, float* dst, int chan_stride) {
#pragma unroll
  for (int c = 0; c < C1; ++c) {
    float a = W.init1[c];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
      for (int kw = 0; kw < 3; ++kw) a = fmaf(W.w1r[(kh * 3 + kw) * C1 + c], x[kh][kw], a);
    const float lo = W.lo1[c];
    dst[c * chan_stride] = row_inside ? (col_inside ? fmaxf(a, lo) : lo) : 0.f;
  }
}

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

// Row type of output k of a half of the incremental kernels (0 = top: leaving row, row 0, row 1; 1 = bottom:
// entering row, row H-2, row H-1): the moving row and rows 1, H-2 meet all three kernel rows, rows 0 and H-1 two.
__host__ __device__ constexpr int inc_row_type(int half, int k) {
  return half == 0 ? (k == 1 ? kRowTop : kRowAll) : (k == 2 ? kRowBot : kRowAll);
}

// One staged x value of the MFMA variants: 2^12 x as f16 hi (low half of the word) + f16 lo (high half);
// hi + lo carry 22 significant bits, so tiny probabilities keep their precision.
__device__ __forceinline__ uint32_t split_hi_lo(float xv) {
  typedef _Float16 half2v __attribute__((ext_vector_type(2)));
  const _Float16 hi = (_Float16)xv;
  const half2v pr = {hi, (_Float16)(xv - (float)hi)};
  return __builtin_bit_cast(uint32_t, pr);
}

// Tile geometry of the incremental MFMA kernel for 16/32 channels: 124 output columns per tile; x columns c0-2 .. c0+125 (128) and y1
// columns c0-1 .. c0+126 (128) are staged, of which outputs 0..123 use x columns 0..127 and y1 columns 0..125.
// The two surplus columns of each MFMA block read past their row into finite values and feed only outputs
// that are dropped.
constexpr int kPmIW = 124;
constexpr int kPmXW = 128;
constexpr int kPmYW = 130;                        // y1 columns per plane (layer-2 reads run 2 past the 128 written)
constexpr int kPmLD = 128;
constexpr int kPmXBuf = 10 * kPmXW + 4;           // words per x buffer (layer-1 reads run 2 past the last row)

}  // namespace
}  // namespace ap
