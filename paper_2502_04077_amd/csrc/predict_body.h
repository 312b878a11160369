// Shared device code of the predictor kernels: weight access, ring addressing and the MFMA form of the
// incremental predictor (see predict.hip for the method).
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

// Geometry shared by the MFMA variants: 124 output columns per tile; x columns c0-2 .. c0+125 (128) and y1
// columns c0-1 .. c0+126 (128) are staged, of which outputs 0..123 use x columns 0..127 and y1 columns 0..125.
// The two surplus columns of each MFMA block read past their row into finite values and feed only outputs
// that are dropped.
constexpr int kPmIW = 124;
constexpr int kPmXW = 128;
constexpr int kPmYW = 130;                        // y1 columns per plane (layer-2 reads run 2 past the 128 written)
constexpr int kPmLD = 128;
constexpr int kPmXBuf = 10 * kPmXW + 4;           // words per x buffer (layer-1 reads run 2 past the last row)

// MFMA variant for 8/8 channels.  4 waves: waves 0,1 are the top half, waves 2,3 the bottom half; each wave owns
// two 32-column blocks.  v_mfma_f32_32x32x16_f16 computes D[32 x 32] += A[32 x 16] * B[16 x 32]; lane l
// supplies row/column l % 32 and K entries 8 (l / 32) .. + 7, and receives D rows 8 (v / 4) + 4 (l / 32) + v % 4
// (v = 0..15) of column l % 32.
//   layer 1: rows = (q, c1) (all 32 used), K = 16 = (x row 0..4, kw 0..2) + one unused slot, columns = 32
//            y1 columns.  x arrives as hi + lo f16 halves of 2^12 x (two MFMAs); the weights are f16 scaled
//            by 2^-4 (A table built on the host, zero where a tap row falls outside the history window) and
//            the accumulator starts at 2^8 b1, so the result is 2^8 y1 before the ReLU.  It is rounded to
//            f16 (the scale keeps y1 up to 255 inside the f16 range), clamped at 0, zeroed outside the tile
//            and stored as [q][column][8 channels].
//   layer 2: rows = (output o, c2) (24 used), K = 96 = (q, kw, c1) in six steps, columns = 32 output columns;
//            the B operand of a step is one 16-byte LDS read.  Accumulators start at 2^8 b2; the head weights
//            carry the 2^-8.
// The contractions are dense (layer 2 is 84 % of the predictor's arithmetic), which is what MFMA is for;
// f16 operands with fp32 accumulation move pred by about 1e-4 of its magnitude at worst (eleven
// significant bits per operand, exact products).
//
// Workgroups are dispatched at a finite rate, and one tile is only a few microseconds of work, so a
// workgroup walks a contiguous range of tiles of its instance: the x rows and the state of tile t + 1 are
// fetched into registers while tile t is computed, and the operand tables are loaded once.
constexpr int kPredMfmaLdsFloats = 2 * 4 * kPmYW * 4 + 2 * kPmXBuf + 8 * kPmLD;

// Workgroup `chunk` of `n_chunks` of instance `inst` (256 threads); smem: kPredMfmaLdsFloats floats, 16-byte aligned.
__device__ __forceinline__ void predict_inc_mfma_body(const float* __restrict__ hist, const float* __restrict__ wts_global,
                                             int R, int H, int newest_slot, int nb_cur, int nb_cap, int inst,
                                             int chunk, int n_chunks, int advance, float* __restrict__ pstate,
                                             float* __restrict__ pred, float* smem) {
  constexpr int C = 8, IW = kPmIW, XW = kPmXW, YW = kPmYW, LD = kPmLD, XBUF = kPmXBuf;
  constexpr float kXScale = 4096.f, kAccScale = 256.f;
  half8* s_y1 = reinterpret_cast<half8*>(smem);          // [half 2][q 4][YW] x 8 f16
  uint32_t* s_xb = reinterpret_cast<uint32_t*>(smem + 2 * 4 * YW * 4);   // 2 buffers of [10][XW] (+4) hi|lo words
  float* s_red = reinterpret_cast<float*>(s_xb + 2 * XBUF);              // [half 2][moving | border][lane half 2][LD]

  const int tiles = (nb_cur + IW - 1) / IW;
  const int per_wg = (tiles + n_chunks - 1) / n_chunks;
  const int t_begin = chunk * per_wg;
  const int t_end = min(tiles, t_begin + per_wg);
  if (t_begin >= t_end) return;

  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int hf = wave >> 1;
  const int n = lane & 31, hsel = lane >> 5;
  const float* hist_inst = hist + (size_t)inst * R * nb_cap;
  float* pstate_inst = pstate + (size_t)inst * nb_cap;
  float* pred_inst = pred + (size_t)inst * nb_cap;

  // Operand tables and per-lane constants.
  const half8* tab2 = reinterpret_cast<const half8*>(wts_global + kMfmaTableFloatOffset) + (size_t)hf * 6 * kWave;
  const half8* tab1 = reinterpret_cast<const half8*>(wts_global + kMfmaTableFloatOffset) + 2 * 6 * kWave + hf * kWave;
  half8 A2[6];
#pragma unroll
  for (int s = 0; s < 6; ++s) A2[s] = tab2[s * kWave + lane];
  const half8 A1 = tab1[lane];
  // Difference form (ap_internal.h): accumulators start at 2^8 init, the ReLU is a clamp at 2^8 lo.
  const float* dc = wts_global + delta_const_offset(C, C);
  float16v b1acc, b2acc;                                 // entry v is D row 8 (v / 4) + c, c = 4 hsel + v % 4
  float w3v[4], lo2v[12];
  half4 lo1h;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    b1acc[v] = kAccScale * dc[4 * hsel + v % 4];
    b2acc[v] = v < 12 ? kAccScale * dc[2 * C + inc_row_type(0, v / 4) * C + 4 * hsel + v % 4] : 0.f;
    if (hf && v < 12) b2acc[v] = kAccScale * dc[2 * C + inc_row_type(1, v / 4) * C + 4 * hsel + v % 4];
  }
#pragma unroll
  for (int v = 0; v < 12; ++v) {
    const int ty = hf ? inc_row_type(1, v / 4) : inc_row_type(0, v / 4);
    lo2v[v] = kAccScale * dc[2 * C + (4 + ty) * C + 4 * hsel + v % 4];
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    w3v[j] = wts_global[10 * C + 9 * C * C + C + 4 * hsel + j] * (1.f / kAccScale);
    lo1h[j] = (_Float16)(kAccScale * dc[C + 4 * hsel + j]);
  }
  const float inv_H = 1.f / (float)H;                     // the time mean as a multiplication
  // layer-1 K slot e of this lane is (x row, kw) = divmod(8 hsel + e, 3); slot 15 has zero weights
  int xoff[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int ka = e, kb = 8 + e;
    const int oa = (ka / 3) * XW + ka % 3, ob = kb < 15 ? (kb / 3) * XW + kb % 3 : 0;
    xoff[e] = hsel ? ob : oa;
  }
  if (tid < 4) s_xb[XBUF - 4 + tid] = s_xb[2 * XBUF - 4 + tid] = 0u;
  // x staging: thread tid fetches column tid % 128 of staged rows hf, hf + 2, .., hf + 8; staged rows 0..4 are
  // history rows -1..3, staged rows 5..9 are rows H-5..H-1.
  const int xcol = (tid & (XW - 1)) - 2;
  int xrow_off[5];
#pragma unroll
  for (int i = 0; i < 5; ++i) {
    const int rr = hf + 2 * i;
    // (the same for the whole wave: kept scalar, so that the loads take a scalar base and a 32-bit lane offset)
    xrow_off[i] = __builtin_amdgcn_readfirstlane(ring_slot(newest_slot, H, R, rr < 5 ? rr - 1 : H - 10 + rr) * nb_cap);
  }
  float xpre[5], pst_cur = 0.f, pst_next = 0.f;
  // Loads are unconditional on clamped addresses (no divergent branches); the raw values stay untouched in
  // registers until `stash` masks them, so nothing waits on them while the current tile is computed.
  auto fetch = [&](int tile, float& pst) __attribute__((always_inline)) {
    const int c0 = tile * IW;
    const int j = min(max(c0 + xcol, 0), nb_cur - 1);
    const unsigned jb = (unsigned)j * 4u;               // byte offsets of 32 bits off scalar bases
#pragma unroll
    for (int i = 0; i < 5; ++i)
      xpre[i] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(hist_inst + xrow_off[i]) + jb);
    pst = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(pstate_inst) +
                                          (unsigned)min(c0 + tid, nb_cur - 1) * 4u);
  };
  auto stash = [&](int tile, uint32_t* s_x) __attribute__((always_inline)) {
    const int j = tile * IW + xcol;
    const float scale = (j >= 0 && j < nb_cur) ? kXScale : 0.f;
#pragma unroll
    for (int i = 0; i < 5; ++i) s_x[(hf + 2 * i) * XW + (tid & (XW - 1))] = split_hi_lo(xpre[i] * scale);
  };
  float inf = INFINITY;                 // opaque, so that med3(a, 0, inf) stays one instruction
  asm volatile("" : "+v"(inf));
  fetch(t_begin, pst_cur);
  stash(t_begin, s_xb);
  __syncthreads();

#pragma unroll 1
  for (int tile = t_begin; tile < t_end; ++tile) {
    const int c0 = tile * IW;
    const uint32_t* s_x = s_xb + ((tile - t_begin) & 1) * XBUF;
    const bool more = tile + 1 < t_end;
    if (more) fetch(tile + 1, pst_next);

    // Layer 1.
    const uint32_t* xs = s_x + hf * 5 * XW;
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      const int yc = ((wave & 1) * 2 + blk) * 32 + n;    // y1 column 0..127  <->  tile column c0 - 1 + yc
      uint4v whi, wlo;
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        const uint32_t wa = xs[yc + xoff[e]], wb = xs[yc + xoff[e + 1]];
        whi[e / 2] = __builtin_amdgcn_perm(wb, wa, 0x05040100u);
        wlo[e / 2] = __builtin_amdgcn_perm(wb, wa, 0x07060302u);
      }
      float16v acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(A1, __builtin_bit_cast(half8, whi), b1acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(A1, __builtin_bit_cast(half8, wlo), acc, 0, 0, 0);
      const int j = c0 - 1 + yc;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        half4 h;
#pragma unroll
        for (int c = 0; c < 4; ++c) h[c] = (_Float16)acc[4 * q + c];
        h = __builtin_elementwise_max(h, lo1h);
        reinterpret_cast<half4*>(s_y1 + (hf * 4 + q) * YW + yc)[hsel] = h;
      }
      if (j < 0 || j >= nb_cur) {                        // layer-2 padding: y1 = 0 beside the tile, d1 = lo1
#pragma unroll
        for (int q = 0; q < 4; ++q) reinterpret_cast<half4*>(s_y1 + (hf * 4 + q) * YW + yc)[hsel] = lo1h;
      }
    }
    __syncthreads();

    // Layer 2 and the head.
    const half8* yh = s_y1 + (size_t)hf * 4 * YW;
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      const int cb = ((wave & 1) * 2 + blk) * 32;
      float16v acc;
#pragma unroll
      for (int s = 0; s < 6; ++s) {
        const int cc = 2 * s + hsel;                     // K chunk = one (q, kw) pair, 8 channels
        const int q = cc / 3, kw = cc - 3 * q;
        const half8 B = yh[q * YW + cb + n + kw];
        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(A2[s], B, s == 0 ? b2acc : acc, 0, 0, 0);
      }
      float p[3];
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        float t = 0.f;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) t = fmaf(w3v[jj], __builtin_amdgcn_fmed3f(acc[4 * k + jj], lo2v[4 * k + jj], inf), t);
        p[k] = t;
      }
      s_red[((hf * 2 + 0) * 2 + hsel) * LD + cb + n] = p[0];
      s_red[((hf * 2 + 1) * 2 + hsel) * LD + cb + n] = p[1] + p[2];
    }
    __syncthreads();
    if (tid < IW && c0 + tid < nb_cur) {
      auto part = [&](int half, int kind) __attribute__((always_inline)) {
        return s_red[((half * 2 + kind) * 2 + 0) * LD + tid] + s_red[((half * 2 + kind) * 2 + 1) * LD + tid];
      };
      float st = pst_cur;
      if (advance) {
        st = (st - part(0, 0)) + part(1, 0);
        pstate_inst[(unsigned)(c0 + tid)] = st;
      }
      pred_inst[(unsigned)(c0 + tid)] = (st + (part(0, 1) + part(1, 1))) * inv_H;
    }
    if (more) stash(tile + 1, s_xb + (((tile - t_begin) & 1) ^ 1) * XBUF);
    pst_cur = pst_next;
    __syncthreads();
  }
}

}  // namespace
}  // namespace ap
