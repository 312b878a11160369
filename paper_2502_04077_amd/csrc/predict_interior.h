// MFMA evaluation of the interior state of the incremental predictor from scratch (8/8 channels):
//   state[j] = sum_{r=2}^{H-3} sum_c w3[c] * (relu(y2[c][r][j]) - relu(B2[c]))      (difference form, ap_internal.h)
// i.e. what a re-base needs; the border rows 0, 1, H-2, H-1 and the head are then added by the incremental
// kernel run without an advance.  Same arithmetic as the incremental kernels (f16 operands - x as one f16 of
// 2^12 x for 8/8 channels, as hi + lo for 16/32 -, fp32 accumulation, y1 kept as f16 of 2^8 d1), so a re-based
// state continues the advanced one without a step.
//
// Rows 2..H-3 have no zero padding in time, so every row is the same contraction and the time axis is walked in
// strips of three output rows:
//   pass p    layer 1 for y1 rows 1+3p .. 3+3p from x rows 3p .. 3p+4: one 32-row MFMA block (3 rows x 8 channels,
//             8 rows idle), K = 5 x rows x 3 taps (+1 unused)
//   strip s   layer 2 for output rows 2+3s .. 4+3s from y1 rows 1+3s .. 5+3s, i.e. the rows of passes s and s+1:
//             rows = (3 outputs x 8 channels), K = 5 y1 rows x 3 taps x 8 channels = 15 chunks in 8 steps
// A ring row beyond the newest one is some other finite row of the ring; it only reaches outputs beyond row H-3,
// which are dropped.  Each wave owns 32 y1 columns and the 30 outputs inside them and keeps its x rows and y1
// rows in its own piece of LDS, so the four waves of a workgroup never wait for each other; the running sum of a
// column stays in a register over all strips.
#pragma once

#include "predict_body.h"

namespace ap {
namespace {

constexpr int kPiOut = 30;                          // output columns per wave
constexpr int kPiXW = 36;                           // staged x columns per row (34 used)
constexpr int kPiYW = 34;                           // y1 columns per row (32 written, reads run 2 further)
constexpr int kPiWaveWords = 5 * kPiXW + 4 + 6 * kPiYW * 4;   // x rows (hi|lo words) + six y1 rows of half8
constexpr int kPredInteriorLdsFloats = 4 * kPiWaveWords;

// Operand tables (f16), appended to the 8/8 MFMA tables of the weight buffer:
//   layer 2  [step 8][lane 64][8]: lane (m, h): row m = 8 o + c2 (o = 0..2), chunk 2 step + h = (q, kw) = divmod(., 3),
//            kernel row kh = q - o (zero outside 0..2 and for chunk 15)
//   layer 1  [lane 64][8]: row m = 8 q + c1 (q = 0..2), K slot k = 3 xrow + kw, kernel row kh = xrow - q, scaled 2^-4

// Workgroup `chunk` of `n_chunks` of instance `inst` walks the 120-column groups chunk, chunk + n_chunks, ..;
// wave `wave` of it takes outputs [c0, c0 + 30), c0 = (4 group + wave) * 30, of each group (the operand tables
// and constants are loaded once per wave, which would otherwise cost as much as a group's arithmetic).
__device__ __forceinline__ void predict_interior_mfma_body(const float* __restrict__ hist,
                                                           const float* __restrict__ wts_global, int R, int H,
                                                           int newest_slot, int nb_cur, int nb_cap, int inst,
                                                           int chunk, int n_chunks, float* __restrict__ pstate,
                                                           float* smem) {
  constexpr int C = 8, XW = kPiXW, YW = kPiYW;
  constexpr float kXScale = 4096.f, kAccScale = 256.f;
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int n = lane & 31, hsel = lane >> 5;
  uint32_t* s_x = reinterpret_cast<uint32_t*>(smem) + wave * kPiWaveWords;     // [5][XW] (+4)
  half8* s_y1 = reinterpret_cast<half8*>(s_x + 5 * XW + 4);                    // [6][YW]
  const float* hist_inst = hist + (size_t)inst * R * nb_cap;

  const half8* tab = reinterpret_cast<const half8*>(wts_global + kMfmaTableFloatOffset) + kMfmaTableHalfs / 8;
  half8 A2[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) A2[s] = tab[s * kWave + lane];
  const half8 A1 = tab[8 * kWave + lane];
  // Difference form (ap_internal.h): accumulators start at 2^8 init, the ReLU is a clamp at 2^8 lo; every row
  // here meets all three kernel rows.
  const float* dc = wts_global + delta_const_offset(C, C);
  float16v b1acc, b2acc;                                 // entry v is D row 8 (v / 4) + c, c = 4 hsel + v % 4
  float w3v[4], lo2v[4];
  half4 lo1h;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    b1acc[v] = v < 12 ? kAccScale * dc[4 * hsel + v % 4] : 0.f;
    b2acc[v] = v < 12 ? kAccScale * dc[2 * C + kRowAll * C + 4 * hsel + v % 4] : 0.f;
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    w3v[j] = wts_global[10 * C + 9 * C * C + C + 4 * hsel + j] * (1.f / kAccScale);
    lo2v[j] = kAccScale * dc[2 * C + (4 + kRowAll) * C + 4 * hsel + j];
    lo1h[j] = (_Float16)(kAccScale * dc[C + 4 * hsel + j]);
  }
  int xoff[8];                                           // layer-1 K slot e of this lane -> offset in s_x
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int ka = e, kb = 8 + e;
    const int oa = (ka / 3) * XW + ka % 3, ob = kb < 15 ? (kb / 3) * XW + kb % 3 : 0;
    xoff[e] = hsel ? ob : oa;
  }
  if (lane < 4) s_x[5 * XW + lane] = 0u;
  // x staging: element lane + 64 i of the [5][34] window (x columns c0-2 .. c0+31 of five consecutive rows).
  int xslot0[3], xwcol[3], xdst[3];
  bool xuse[3];
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    const int e = lane + kWave * i, row = min(e / 34, 4);
    xwcol[i] = e - (e / 34) * 34;
    xuse[i] = e < 5 * 34;
    xdst[i] = row * XW + xwcol[i];
    xslot0[i] = ring_slot(newest_slot, H, R, row);       // logical row `row` of pass 0; + 3 per pass
  }
  float inf = INFINITY;                                  // opaque, so that med3(a, 0, inf) stays one instruction
  asm volatile("" : "+v"(inf));
  const int n_groups = (nb_cur + 4 * kPiOut - 1) / (4 * kPiOut);

#pragma unroll 1
  for (int group = chunk; group < n_groups; group += n_chunks) {
  const int c0 = (4 * group + wave) * kPiOut;
  if (c0 >= nb_cur) break;
  int xslot[3], xcol[3];
  bool xin[3];
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    const int j = c0 - 2 + xwcol[i];
    xin[i] = j >= 0 && j < nb_cur;
    xcol[i] = min(max(j, 0), nb_cur - 1);
    xslot[i] = xslot0[i];
  }
  const int j_y1 = c0 - 1 + n;                           // tile column of this lane's y1 column
  const bool y1_outside = j_y1 < 0 || j_y1 >= nb_cur;

  // x rows of the next pass are fetched while the current pass and strip compute.
  float xv[3];
  auto fetch = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      xv[i] = hist_inst[(size_t)xslot[i] * nb_cap + xcol[i]];
      xslot[i] += 3;
      if (xslot[i] >= R) xslot[i] -= R;
    }
  };
  // Layer 1 of pass p into y1 slots 3 (p & 1) .. + 2.
  auto pass = [&](int p) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 3; ++i)
      if (xuse[i]) s_x[xdst[i]] = split_hi_lo(xin[i] ? xv[i] * kXScale : 0.f);
    fetch();
    // One wave reads what it has just written: the LDS keeps a wave's accesses in order, the compiler has to as well.
    asm volatile("" ::: "memory");
    uint4v whi;                                          // (the low halves of the staged words: x as one f16)
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      const uint32_t wa = s_x[n + xoff[e]], wb = s_x[n + xoff[e + 1]];
      whi[e / 2] = __builtin_amdgcn_perm(wb, wa, 0x05040100u);
    }
    float16v acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(A1, __builtin_bit_cast(half8, whi), b1acc, 0, 0, 0);
    half8* dst = s_y1 + 3 * (p & 1) * YW + n;
#pragma unroll
    for (int q = 0; q < 3; ++q) {
      half4 h;
#pragma unroll
      for (int c = 0; c < 4; ++c) h[c] = (_Float16)acc[4 * q + c];
      h = __builtin_elementwise_max(h, lo1h);
      if (y1_outside) h = lo1h;                          // layer-2 padding: y1 = 0 beside the tile, d1 = lo1
      reinterpret_cast<half4*>(dst + q * YW)[hsel] = h;
    }
    asm volatile("" ::: "memory");
  };

  const int n_rows = H - 4;                              // interior rows 2 .. H-3
  const int n_strips = (n_rows + 2) / 3;
  float sum = 0.f;
  fetch();
  pass(0);
#pragma unroll 1
  for (int s = 0; s < n_strips; ++s) {
    pass(s + 1);
    // y1 row q of this strip: q < 3 from pass s, else from pass s + 1
    const int lo_base = 3 * (s & 1) * YW, hi_base = 3 * ((s + 1) & 1) * YW;
    float16v acc;
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      const int cc = min(2 * st + hsel, 14);             // chunk 15 has zero weights: any valid address
      const int q = cc / 3, kw = cc - 3 * q;
      const int row_off = q < 3 ? lo_base + q * YW : hi_base + (q - 3) * YW;
      const half8 B = s_y1[row_off + n + kw];
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(A2[st], B, st == 0 ? b2acc : acc, 0, 0, 0);
    }
    asm volatile("" ::: "memory");                       // the next pass overwrites rows read above
    const int left = n_rows - 3 * s;                     // output rows of this strip that exist
#pragma unroll
    for (int o = 0; o < 3; ++o) {
      float t = 0.f;
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) t = fmaf(w3v[jj], __builtin_amdgcn_fmed3f(acc[4 * o + jj], lo2v[jj], inf), t);
      if (o < left) sum += t;
    }
  }
  sum += __shfl_xor(sum, 32, kWave);
  const int j = c0 + n;
  if (hsel == 0 && n < kPiOut && j < nb_cur) pstate[(size_t)inst * nb_cap + j] = sum;
  asm volatile("" ::: "memory");                         // the next group re-uses this wave's LDS rows
  }
}

// ---------------------------------------------------------------------------------------------------------
// The same for 16 and 32 channels.  Strips of two output rows:
//   pass p    y1 rows 1+2p, 2+2p from x rows 2p .. 2p+3: one 32-row MFMA block (2 rows x 16 channels), K = 12
//   strip s   output rows 2+2s, 3+2s, one 32-row block each (32 output channels), from y1 rows 1+2s .. 4+2s.
//             Output o meets y1 row o + kh through kernel row kh, so both outputs share one set of nine
//             (kh, kw) operands: 18 MFMAs per strip, each B operand read once for the outputs that use it.
// y1 is kept as [slot 4][channel half 2][column] x 8 f16.  Operand tables (f16) follow the 16/32 tables of the
// weight buffer: layer 2 [kh 3][kw 3][lane 64][8] (lane (c2, h): input channels 8h..8h+7), layer 1 [lane 64][8]
// (row m = 16 q + c1, K slot k = 3 xrow + kw, kernel row xrow - q, scaled 2^-4).
constexpr int kPi16WaveWords = 4 * kPiXW + 4 + 4 * 2 * kPiYW * 4;
constexpr int kPredInterior16LdsFloats = 4 * kPi16WaveWords;

__device__ __forceinline__ void predict_interior_mfma16_body(const float* __restrict__ hist,
                                                             const float* __restrict__ wts_global, int R, int H,
                                                             int newest_slot, int nb_cur, int nb_cap, int inst,
                                                             int chunk, int n_chunks, float* __restrict__ pstate,
                                                             float* smem) {
  constexpr int C1 = 16, C2 = 32, XW = kPiXW, YW = kPiYW;
  constexpr float kXScale = 4096.f, kAccScale = 256.f;
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int n = lane & 31, hsel = lane >> 5;
  uint32_t* s_x = reinterpret_cast<uint32_t*>(smem) + wave * kPi16WaveWords;   // [4][XW] (+4)
  half8* s_y1 = reinterpret_cast<half8*>(s_x + 4 * XW + 4);                    // [slot 4][channel half 2][YW]
  const float* hist_inst = hist + (size_t)inst * R * nb_cap;

  const half8* tab = reinterpret_cast<const half8*>(wts_global + kMfma16TableFloatOffset) + kMfma16TableHalfs / 8;
  half8 A2[9];
#pragma unroll
  for (int i = 0; i < 9; ++i) A2[i] = tab[i * kWave + lane];
  const half8 A1 = tab[9 * kWave + lane];
  // Difference form (ap_internal.h): accumulators start at 2^8 init, the ReLU is a clamp at 2^8 lo; every row
  // here meets all three kernel rows.
  const float* dc = wts_global + delta_const_offset(C1, C2);
  const float* b2 = wts_global + 10 * C1 + 9 * C1 * C2;
  float16v b1acc, b2acc;
  float w3v[16], lo2v[16];
  half4 lo1h[2];                                         // channels 8 pl + 4 hsel .. + 3
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int row = 8 * (v / 4) + 4 * hsel + v % 4;      // D row of accumulator entry v
    b1acc[v] = kAccScale * dc[row % C1];
    b2acc[v] = kAccScale * dc[2 * C1 + kRowAll * C2 + row];
    lo2v[v] = kAccScale * dc[2 * C1 + (4 + kRowAll) * C2 + row];
    w3v[v] = b2[C2 + row] * (1.f / kAccScale);
  }
#pragma unroll
  for (int pl = 0; pl < 2; ++pl)
#pragma unroll
    for (int c = 0; c < 4; ++c) lo1h[pl][c] = (_Float16)(kAccScale * dc[C1 + 8 * pl + 4 * hsel + c]);
  int xoff[8];                                           // layer-1 K slot e of this lane -> offset in s_x
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int ka = e, kb = 8 + e;
    const int oa = (ka / 3) * XW + ka % 3, ob = kb < 12 ? (kb / 3) * XW + kb % 3 : 0;
    xoff[e] = hsel ? ob : oa;
  }
  if (lane < 4) s_x[4 * XW + lane] = 0u;
  // x staging: element lane + 64 i of the [4][34] window (x columns c0-2 .. c0+31 of four consecutive rows).
  int xslot0[3], xwcol[3], xdst[3];
  bool xuse[3];
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    const int e = lane + kWave * i, row = min(e / 34, 3);
    xwcol[i] = e - (e / 34) * 34;
    xuse[i] = e < 4 * 34;
    xdst[i] = row * XW + xwcol[i];
    xslot0[i] = ring_slot(newest_slot, H, R, row);       // logical row `row` of pass 0; + 2 per pass
  }
  float inf = INFINITY;                                  // opaque, so that med3(a, 0, inf) stays one instruction
  asm volatile("" : "+v"(inf));
  const int n_groups = (nb_cur + 4 * kPiOut - 1) / (4 * kPiOut);

#pragma unroll 1
  for (int group = chunk; group < n_groups; group += n_chunks) {
    const int c0 = (4 * group + wave) * kPiOut;
    if (c0 >= nb_cur) break;
    int xslot[3], xcol[3];
    bool xin[3];
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      const int j = c0 - 2 + xwcol[i];
      xin[i] = j >= 0 && j < nb_cur;
      xcol[i] = min(max(j, 0), nb_cur - 1);
      xslot[i] = xslot0[i];
    }
    const int j_y1 = c0 - 1 + n;                         // tile column of this lane's y1 column
    const bool y1_outside = j_y1 < 0 || j_y1 >= nb_cur;

    float xv[3];
    auto fetch = [&]() __attribute__((always_inline)) {
#pragma unroll
      for (int i = 0; i < 3; ++i) {
        xv[i] = hist_inst[(size_t)xslot[i] * nb_cap + xcol[i]];
        xslot[i] += 2;
        if (xslot[i] >= R) xslot[i] -= R;
      }
    };
    // Layer 1 of pass p into y1 slots 2 (p & 1), 2 (p & 1) + 1.
    auto pass = [&](int p) __attribute__((always_inline)) {
#pragma unroll
      for (int i = 0; i < 3; ++i)
        if (xuse[i]) s_x[xdst[i]] = split_hi_lo(xin[i] ? xv[i] * kXScale : 0.f);
      fetch();
      asm volatile("" ::: "memory");                     // a wave reads what it has just written, in order
      uint4v whi, wlo;
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        const uint32_t wa = s_x[n + xoff[e]], wb = s_x[n + xoff[e + 1]];
        whi[e / 2] = __builtin_amdgcn_perm(wb, wa, 0x05040100u);
        wlo[e / 2] = __builtin_amdgcn_perm(wb, wa, 0x07060302u);
      }
      float16v acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(A1, __builtin_bit_cast(half8, whi), b1acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(A1, __builtin_bit_cast(half8, wlo), acc, 0, 0, 0);
      // entry v: y1 row q = v / 8 of the pass, channel 8 (v / 4 % 2) + 4 hsel + v % 4
#pragma unroll
      for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int pl = 0; pl < 2; ++pl) {
          half4 h;
#pragma unroll
          for (int c = 0; c < 4; ++c) h[c] = (_Float16)acc[8 * q + 4 * pl + c];
          h = __builtin_elementwise_max(h, lo1h[pl]);
          if (y1_outside) h = lo1h[pl];                  // layer-2 padding: y1 = 0 beside the tile, d1 = lo1
          reinterpret_cast<half4*>(s_y1 + ((2 * (p & 1) + q) * 2 + pl) * YW + n)[hsel] = h;
        }
      asm volatile("" ::: "memory");
    };

    const int n_rows = H - 4;                            // interior rows 2 .. H-3
    const int n_strips = (n_rows + 1) / 2;
    float sum = 0.f;
    fetch();
    pass(0);
#pragma unroll 1
    for (int s = 0; s < n_strips; ++s) {
      pass(s + 1);
      // y1 row q of this strip (0..3): q < 2 from pass s, else from pass s + 1
      const int slot_lo = 2 * (s & 1), slot_hi = 2 * ((s + 1) & 1);
      float16v acc0, acc1;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int slot = q < 2 ? slot_lo + q : slot_hi + q - 2;
        const half8* yrow = s_y1 + (slot * 2 + hsel) * YW + n;
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
          const half8 B = yrow[kw];
          if (q <= 2) acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(A2[q * 3 + kw], B, (q == 0 && kw == 0) ? b2acc : acc0, 0, 0, 0);
          if (q >= 1) acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(A2[(q - 1) * 3 + kw], B, (q == 1 && kw == 0) ? b2acc : acc1, 0, 0, 0);
        }
      }
      asm volatile("" ::: "memory");                     // the next pass overwrites rows read above
      float t0 = 0.f, t1 = 0.f;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        t0 = fmaf(w3v[v], __builtin_amdgcn_fmed3f(acc0[v], lo2v[v], inf), t0);
        t1 = fmaf(w3v[v], __builtin_amdgcn_fmed3f(acc1[v], lo2v[v], inf), t1);
      }
      sum += t0;
      if (2 * s + 1 < n_rows) sum += t1;
    }
    sum += __shfl_xor(sum, 32, kWave);
    const int j = c0 + n;
    if (hsel == 0 && n < kPiOut && j < nb_cur) pstate[(size_t)inst * nb_cap + j] = sum;
    asm volatile("" ::: "memory");                       // the next group re-uses this wave's LDS rows
  }
}

}  // namespace
}  // namespace ap
