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

__device__ __forceinline__ int ring_slot(int newest_slot, int H, int R, int r) {
  int slot = (newest_slot - (H - 1 - r)) % R;   // logical row r (H-1 = newest, -1 = the row that just left)
  return slot < 0 ? slot + R : slot;
}

// One y1 pixel, all C1 channels, from a 3x3 x neighbourhood.
template <int C1, int C2>
__device__ __forceinline__ void y1_pixel(const Weights<C1, C2>& W, const float (&x)[3][3], bool inside, float* dst,
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

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));

// MFMA variant for 8/8 channels.  126 output columns per workgroup, 4 waves: waves 0,1 are the top half,
// waves 2,3 the bottom half; each wave owns two 32-column blocks.  v_mfma_f32_32x32x16_f16 computes
// D[32 x 32] += A[32 x 16] * B[16 x 32]; lane l supplies row/column l % 32 and K entries 8 (l / 32) .. + 7, and
// receives D rows 8 (v / 4) + 4 (l / 32) + v % 4 (v = 0..15) of column l % 32.
//   layer 1: rows = (q, c1) (all 32 used), K = 16 = (x row 0..4, kw 0..2) + one unused slot, columns = 32
//            y1 columns.  x is scaled by 2^12 and split into f16 hi + lo (two MFMAs), so tiny probabilities
//            keep full precision; the weights are f16 (A table built on the host, zero where a tap row falls
//            outside the history window).  y1 = relu(acc * 2^-12 + b1), zeroed outside the tile, is rounded
//            to f16 and stored as [q][column][8 channels].
//   layer 2: rows = (output o, c2) (24 used), K = 96 = (q, kw, c1) in six steps, columns = 32 output columns;
//            the B operand of a step is one 16-byte LDS read.  Accumulators start at b2.
// The contractions are dense (layer 2 is 84 % of the predictor's arithmetic), which is what MFMA is for;
// f16 operands with fp32 accumulation move pred by about 1e-4 of its magnitude at worst (eleven
// significant bits per operand, exact products).
//
// Workgroups are dispatched at a finite rate, and one 126-column tile is only a few microseconds of
// work, so a workgroup walks a contiguous range of tiles of its instance: the x rows and the state of
// tile t + 1 are fetched into registers while tile t is computed, and the operand tables are loaded once.
constexpr int kPredMfmaLdsFloats = 2 * 4 * 128 * 4 + 2 * (2 * 5 * 130 + 12) + 4 * 128;

// Workgroup `chunk` of `n_chunks` of instance `inst` (256 threads); smem: kPredMfmaLdsFloats floats, 16-byte aligned.
__device__ __forceinline__ void predict_inc_mfma_body(const float* __restrict__ hist, const float* __restrict__ wts_global,
                                             int R, int H, int newest_slot, int nb_cur, int nb_cap, int inst,
                                             int chunk, int n_chunks, int advance, float* __restrict__ pstate,
                                             float* __restrict__ pred, float* smem) {
  constexpr int C = 8, IW = 126, XW = 130, YW = 128, LD = 128, XBUF = 2 * 5 * XW + 12;
  constexpr float kScale = 4096.f, kInvScale = 1.f / 4096.f;
  half8* s_y1 = reinterpret_cast<half8*>(smem);          // [2][4][YW] x 8 f16 (reads may run 2 entries past a row)
  float* s_xb = smem + 2 * 4 * YW * 4;                   // 2 buffers of [2][5][XW]
  float* s_red = s_xb + 2 * XBUF;                        // [2][2][LD]

  const int tiles = (nb_cur + IW - 1) / IW;
  const int per_wg = (tiles + n_chunks - 1) / n_chunks;
  const int t_begin = chunk * per_wg;
  const int t_end = min(tiles, t_begin + per_wg);
  if (t_begin >= t_end) return;

  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
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
  float b1v[4], b2v[4], w3v[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    b1v[j] = wts_global[9 * C + 4 * hsel + j];
    b2v[j] = wts_global[10 * C + 9 * C * C + 4 * hsel + j];
    w3v[j] = wts_global[10 * C + 9 * C * C + C + 4 * hsel + j];
  }
  const float b3 = wts_global[10 * C + 9 * C * C + 2 * C];
  // layer-1 K slot e of this lane is (x row, kw) = divmod(8 hsel + e, 3); slot 15 is unused
  int xoff[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int ka = e, kb = 8 + e;
    const int oa = (ka / 3) * XW + ka % 3, ob = kb < 15 ? (kb / 3) * XW + kb % 3 : 0;
    xoff[e] = hsel ? ob : oa;
  }
  // x staging: wave w fetches staged rows w, w + 4, w + 8 (of 10: five per half), three column chunks each.
  const float* xsrc[3];
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    const int rr = min(wave + 4 * i, 9);
    const int r = rr < 5 ? rr - 1 : H - 10 + rr;          // rows -1..3, then H-5..H-1
    xsrc[i] = hist_inst + (size_t)ring_slot(newest_slot, H, R, r) * nb_cap;
  }
  float xpre[9], pst_cur = 0.f, pst_next = 0.f;
  // Loads are unconditional on clamped addresses (no divergent branches); the raw values stay untouched in
  // registers until `stash` masks them, so nothing waits on them while the current tile is computed.
  auto fetch = [&](int tile, float& pst) __attribute__((always_inline)) {
    const int c0 = tile * IW;
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
      for (int c = 0; c < 3; ++c) xpre[i * 3 + c] = xsrc[i][min(max(c0 - 2 + lane + kWave * c, 0), nb_cur - 1)];
    pst = pstate_inst[min(c0 + tid, nb_cur - 1)];
  };
  auto stash = [&](int tile, float* s_x) __attribute__((always_inline)) {
    const int c0 = tile * IW;
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
      for (int c = 0; c < 3; ++c) {
        const int rr = wave + 4 * i, xc = lane + kWave * c, j = c0 - 2 + xc;
        if (rr < 10 && xc < XW) s_x[rr * XW + xc] = (j >= 0 && j < nb_cur) ? xpre[i * 3 + c] : 0.f;
      }
  };
  fetch(t_begin, pst_cur);
  stash(t_begin, s_xb);
  __syncthreads();

#pragma unroll 1
  for (int tile = t_begin; tile < t_end; ++tile) {
    const int c0 = tile * IW;
    const float* s_x = s_xb + ((tile - t_begin) & 1) * XBUF;
    const bool more = tile + 1 < t_end;
    if (more) fetch(tile + 1, pst_next);

    // Layer 1.
    const float* xs = s_x + hf * 5 * XW;
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      const int yc = ((wave & 1) * 2 + blk) * 32 + n;    // y1 column 0..127  <->  tile column c0 - 1 + yc
      half8 Bhi, Blo;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float xv = xs[yc + xoff[e]] * kScale;
        if (e == 7 && hsel) xv = 0.f;
        const _Float16 hi = (_Float16)xv;
        Bhi[e] = hi;
        Blo[e] = (_Float16)(xv - (float)hi);
      }
      float16v acc;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = 0.f;
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(A1, Bhi, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(A1, Blo, acc, 0, 0, 0);
      const int j = c0 - 1 + yc;
      const float hi_clamp = (j >= 0 && j < nb_cur) ? INFINITY : 0.f;   // med3(a, 0, inf) = relu(a); med3(a, 0, 0) = 0
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        half4 h;
#pragma unroll
        for (int c = 0; c < 4; ++c)
          h[c] = (_Float16)__builtin_amdgcn_fmed3f(fmaf(acc[4 * q + c], kInvScale, b1v[c]), 0.f, hi_clamp);
        reinterpret_cast<half4*>(s_y1 + (hf * 4 + q) * YW + yc)[hsel] = h;
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
      for (int v = 0; v < 16; ++v) acc[v] = (v < 12) ? b2v[v & 3] : 0.f;
#pragma unroll
      for (int s = 0; s < 6; ++s) {
        const int cc = 2 * s + hsel;                     // K chunk = one (q, kw) pair, 8 channels
        const int q = cc / 3, kw = cc - 3 * q;
        const half8 B = yh[q * YW + cb + n + kw];
        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(A2[s], B, acc, 0, 0, 0);
      }
      float p[3];
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        float t = 0.f;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) t = fmaf(w3v[jj], fmaxf(acc[4 * k + jj], 0.f), t);
        p[k] = t + __shfl_xor(t, 32, kWave);
      }
      if (hsel == 0) {
        s_red[(hf * 2 + 0) * LD + cb + n] = p[0];
        s_red[(hf * 2 + 1) * LD + cb + n] = p[1] + p[2];
      }
    }
    __syncthreads();
    if (tid < IW && c0 + tid < nb_cur) {
      float st = pst_cur;
      if (advance) {
        st = (st - s_red[0 * LD + tid]) + s_red[2 * LD + tid];
        pstate_inst[c0 + tid] = st;
      }
      pred_inst[c0 + tid] = b3 + (st + (s_red[1 * LD + tid] + s_red[3 * LD + tid])) / (float)H;
    }
    if (more) stash(tile + 1, s_xb + (((tile - t_begin) & 1) ^ 1) * XBUF);
    pst_cur = pst_next;
    __syncthreads();
  }
}

}  // namespace
}  // namespace ap
