// Incremental predictor for 8/8 channels on MFMA with both layers held in registers (see predict.hip for the
// method: the interior state moves by (row entering) - (row leaving), the four border rows are evaluated afresh).
//
// A wave owns 32 consecutive history columns at a time (lane l: column n = l % 32, channel half h = l / 32) and
// works one half of the method on them: waves 0,1 the top half (leaving row, rows 0, 1), waves 2,3 the bottom half
// (entering row, rows H-2, H-1).  v_mfma_f32_32x32x16_f16 computes D[32 x 32] += A[32 x 16] * B[16 x 32]; lane l
// supplies row / column l % 32 and K entries 8 (l / 32) .. + 7 and receives D rows 8 (v / 4) + 4 (l / 32) + v % 4
// (v = 0..15) of column l % 32.  What makes the registers enough:
//   layer 1  rows = (staged y1 row q, channel c1), K = 16 = 15 (x row, tap) pairs + a constant 1 that carries the
//            accumulator start.  The ten history rows of a pass of columns go from global memory straight to LDS
//            (global_load_lds, no registers), asked for a whole pass ahead; at the start of the pass they are
//            converted once - scaled by 2^12, rounded to f16 - into the words a lane's K slots are made of, so
//            that an operand is four 4-byte LDS reads and no arithmetic.
//   layer 2  the result of layer 1 is, per lane, channels 4h .. 4h+3 of the four y1 rows of its own column: exactly
//            half of the K entries of a layer-2 step whose 16 entries are two (y1 row, tap) pairs of 8 channels.
//            The centre tap takes those registers as they are, the outer taps the same registers moved by one
//            lane with DPP wave shifts (16 moves): K = 96 in six steps, no LDS and no barrier.
//   head     fp32: clamp (the ReLU in difference form), weight, sum the four channels of the lane, and one
//            half-wave swap adds the two channel halves.
// Columns next to the ends of the 32 get wrong neighbours, so a block yields 28 outputs (lanes 2..29) and blocks
// overlap by four columns.  All arithmetic is in the difference form of ap_internal.h: accumulators start at
// 2^8 init, the ReLUs are clamps at 2^8 lo, y1 is kept as f16 of 2^8 d1.  f16 operands, fp32 accumulation.
// Measured alternatives that came out within 3 % of their baseline at cfg2's shape: the outer taps through a
// wave-private piece of LDS instead of DPP moves, the head as a third MFMA on the clamped f16 result, a load or
// two per block instead of a staged pass, five waves per SIMD instead of four, staggered first passes.  What did
// pay: no 64-bit address arithmetic or predication on the pass's loads, and the loads a pass ahead.
// The two halves of a column meet once per pass of up to kRiPassCols columns, through LDS: the state and pred
// are written by a short epilogue after the pass's last barrier.  The leaving row is evaluated by the same instruction
// sequence on the same values as when it entered (both halves run this code, and a block always covers the same
// columns), so it cancels exactly.
#pragma once

#include <type_traits>

#include "predict_body.h"

namespace ap {
namespace {

constexpr int kRiOut = 28;                              // outputs per 32-column block
constexpr int kRiPassBlocks = 15;                       // most blocks whose halves meet in one pass
constexpr int kRiPassCols = kRiOut * kRiPassBlocks;     // 420 output columns per pass
constexpr int kRiStageCols = kRiPassCols + 8;           // staged history columns: four more on either side (428)
constexpr int kRiRawSegs = (kRiStageCols + kWave - 1) / kWave;   // a raw history row arrives in wave-wide pieces (7)
constexpr int kRiRawStride = kRiRawSegs * kWave;        // floats per raw row in LDS (448)
// LDS words: the ten raw history rows of the next pass [row][kRiRawStride]; staged x operands
// [x01 | x2][half 2][lane half 2][kRiStageCols]; the partial sums [half][column of the pass][moving | border]
constexpr int kRiRawWords = 10 * kRiRawStride;
constexpr int kRiStageWords = 2 * 2 * 2 * kRiStageCols;
constexpr int kRiPartWords = 2 * kRiPassCols * 2;
constexpr int kPredRegLdsFloats = kRiRawWords + kRiStageWords + kRiPartWords;

// Every lane is written (a lane without a source lane gets 0), so no previous value has to be set up.
template <int CTRL> __device__ __forceinline__ uint32_t dpp_all(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, CTRL, 0xF, 0xF, true);
}
constexpr int kWaveShr1 = 0x138, kWaveShl1 = 0x130;     // lane l reads lane l - 1 / l + 1 of the whole wave

// 64 consecutive floats of LDS starting at `dst` (wave-uniform) are filled from global memory, lane l from
// row[byte_off / 4] of its own choosing, without passing through registers; completion is counted by vmcnt.
__device__ __forceinline__ void load_to_lds(const float* row, uint32_t byte_off, float* dst) {
  typedef const __attribute__((address_space(1))) void* gptr_t;
  typedef __attribute__((address_space(3))) void* lptr_t;
  __builtin_amdgcn_global_load_lds((gptr_t)(reinterpret_cast<const char*>(row) + byte_off), (lptr_t)dst, 4, 0, 0);
}

// One float at a 32-bit byte offset from a wave-uniform row pointer (scalar base + vector offset addressing).
__device__ __forceinline__ float ld_row(const float* row, uint32_t byte_off) {
  return *reinterpret_cast<const float*>(reinterpret_cast<const char*>(row) + byte_off);
}

// Workgroup `chunk` of `n_chunks` of instance `inst` (256 threads); smem: kPredRegLdsFloats floats.
__device__ __forceinline__ void predict_inc_reg_body(const float* __restrict__ hist, const float* __restrict__ wts_global,
                                                     int R, int H, int newest_slot, int nb_cur, int nb_cap, int inst,
                                                     int chunk, int n_chunks, int advance, float* __restrict__ pstate,
                                                     float* __restrict__ pred, float* smem) {
  constexpr int C = 8;
  constexpr float kXScale = 4096.f, kAccScale = 256.f;
  typedef _Float16 half2v __attribute__((ext_vector_type(2)));

  const int n_blocks = (nb_cur + kRiOut - 1) / kRiOut;
  const int per_wg = (n_blocks + n_chunks - 1) / n_chunks;
  const int b_begin = chunk * per_wg;
  const int b_end = min(n_blocks, b_begin + per_wg);
  if (b_begin >= b_end) return;                          // (the whole workgroup: no barrier is skipped by part of it)

  const int tid = threadIdx.x, lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
  const int hf = wave >> 1, wsub = wave & 1;
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
  const float* dc = wts_global + delta_const_offset(C, C);
  float16v b2init;                                       // entry v is D row 8 (v / 4) + c, c = 4 hsel + v % 4
  half4 lo1h;
  float lo2v[12], w3v[4];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int ty = hf ? inc_row_type(1, v / 4) : inc_row_type(0, v / 4);
    b2init[v] = v < 12 ? kAccScale * dc[2 * C + ty * C + 4 * hsel + v % 4] : 0.f;
    if (v < 12) lo2v[v] = kAccScale * dc[2 * C + (4 + ty) * C + 4 * hsel + v % 4];
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    lo1h[j] = (_Float16)(kAccScale * dc[C + 4 * hsel + j]);
    w3v[j] = wts_global[10 * C + 9 * C * C + C + 4 * hsel + j];
  }
  float inf = INFINITY;                                  // opaque, so that med3(a, lo, inf) stays one instruction
  asm volatile("" : "+v"(inf));
  const float inv_H = 1.f / (float)H;                    // the time mean as a multiplication
  constexpr float kUnscale = 1.f / kAccScale;            // the head sums come out times 2^8 (exact to undo)
  // Ring rows of the ten staged x rows: staged rows 0..4 of the top half are history rows -1..3, of the bottom
  // half H-5..H-1.  (Wave-uniform pointers: they live in scalar registers.)
  const float* row_base[2][5];
#pragma unroll
  for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
    for (int r = 0; r < 5; ++r)
      row_base[h2][r] = hist_inst + (size_t)__builtin_amdgcn_readfirstlane(ring_slot(newest_slot, H, R, h2 ? H - 5 + r : r - 1)) * nb_cap;
  float* s_raw = smem;                                   // [staged row of top half 0..4 | of bottom half 0..4][kRiRawStride]
  uint32_t* s_x01 = reinterpret_cast<uint32_t*>(smem + kRiRawWords);   // [half][lane half][column]: (row 0 | row 1) or (row 3 | row 4)
  uint32_t* s_x2 = s_x01 + 2 * 2 * kRiStageCols;         // [half][lane half][column]: row 2 (col - 1 | col) or (col + 1 | 1)
  float2* s_part = reinterpret_cast<float2*>(smem + kRiRawWords + kRiStageWords);   // [half][column]: (moving, border)
  const uint32_t* my_x01 = s_x01 + (hf * 2 + hsel) * kRiStageCols + n;
  const uint32_t* my_x2 = s_x2 + (hf * 2 + hsel) * kRiStageCols + n;

  // Passes of equal length, as few as the LDS allows.
  const int n_pass = (b_end - b_begin + kRiPassBlocks - 1) / kRiPassBlocks;
  const int pass_blocks = (b_end - b_begin + n_pass - 1) / n_pass;
  // The raw rows of a pass are asked for a whole pass ahead and go straight to LDS: wave w brings pieces w and
  // w + 4 of each of the ten rows (every address is clamped into the tile; what lies outside is masked when the
  // rows are converted).
  auto fetch_pass = [&](int pb) __attribute__((always_inline)) {
    const int col0 = pb * kRiOut;
    const int n_cols = (min(b_end, pb + pass_blocks) - pb) * kRiOut + 8;   // staged columns of that pass
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      const int k = wave + 4 * kk;
      if (k < kRiRawSegs && k * kWave <= n_cols) {         // (wave-uniform; the conversion reads one column past the staged ones)
        const uint32_t off = (uint32_t)min(max(col0 - 4 + k * kWave + lane, 0), nb_cur - 1) * 4u;
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
          for (int r = 0; r < 5; ++r) load_to_lds(row_base[h2][r], off, s_raw + (h2 * 5 + r) * kRiRawStride + k * kWave);
      }
    }
  };
  fetch_pass(b_begin);
  __builtin_amdgcn_s_waitcnt(0x0F70);                    // vmcnt(0): this wave's pieces of the first pass are in LDS
#pragma unroll 1
  for (int pb = b_begin; pb < b_end; pb += pass_blocks) {
    const int pe = min(b_end, pb + pass_blocks);
    const int col0 = pb * kRiOut;                        // first output column of the pass
    const int col_end = min(nb_cur, pe * kRiOut);
    // Every wave has seen its own pieces of this pass's raw rows arrive (before the loop, or before the last
    // barrier of the pass before).
    __syncthreads();
    // Raw rows -> the words a lane's K slots are made of: x scaled by 2^12 and rounded to f16, zero outside the
    // tile.  Thread tid takes staged columns tid and tid + 256.
    {
      constexpr int kChunks = (kRiStageCols + 255) / 256;
#pragma unroll
      for (int ch = 0; ch < kChunks; ++ch) {
        const int i = ch * 256 + tid;
        if (i < (pe - pb) * kRiOut + 8) {                  // the staged columns of this pass
          const int c = col0 - 4 + i;
          const float sc = (uint32_t)c < (uint32_t)nb_cur ? kXScale : 0.f;
          const float sm = (uint32_t)(c - 1) < (uint32_t)nb_cur ? kXScale : 0.f;
          const float sp = (uint32_t)(c + 1) < (uint32_t)nb_cur ? kXScale : 0.f;
          const int im = max(i - 1, 0);
#pragma unroll
          for (int h2 = 0; h2 < 2; ++h2) {
            const float* x = s_raw + h2 * 5 * kRiRawStride;
            const half2v a01 = {(_Float16)(x[i] * sc), (_Float16)(x[kRiRawStride + i] * sc)};
            const half2v a34 = {(_Float16)(x[3 * kRiRawStride + i] * sc), (_Float16)(x[4 * kRiRawStride + i] * sc)};
            const half2v a2l = {(_Float16)(x[2 * kRiRawStride + im] * sm), (_Float16)(x[2 * kRiRawStride + i] * sc)};
            const half2v a2r = {(_Float16)(x[2 * kRiRawStride + i + 1] * sp), (_Float16)1};
            s_x01[(h2 * 2 + 0) * kRiStageCols + i] = __builtin_bit_cast(uint32_t, a01);
            s_x01[(h2 * 2 + 1) * kRiStageCols + i] = __builtin_bit_cast(uint32_t, a34);
            s_x2[(h2 * 2 + 0) * kRiStageCols + i] = __builtin_bit_cast(uint32_t, a2l);
            s_x2[(h2 * 2 + 1) * kRiStageCols + i] = __builtin_bit_cast(uint32_t, a2r);
          }
        }
      }
    }
    __syncthreads();
    // The raw rows are free again: the next pass's loads, and the state of this thread's columns, are asked for
    // now and have the block loop to arrive in.
    if (pb + pass_blocks < b_end) fetch_pass(pb + pass_blocks);
    constexpr int kPerThread = (kRiPassCols + 255) / 256;
    float pst[kPerThread];
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) pst[i] = pstate_inst[min(col0 + tid + 256 * i, nb_cur - 1)];

    // One block.  BORDER: the block reaches beyond the tile, where x is zero and y1 = 0 (d1 = lo1); the other
    // blocks skip those selects.
    auto block = [&](int b, auto border_tag) __attribute__((always_inline)) {
      constexpr bool BORDER = decltype(border_tag)::value;
      const int X0 = b * kRiOut - 2;                     // history column of lane n = 0
      const int col = X0 + n;
      const bool inside = !BORDER || (col >= 0 && col < nb_cur);
      // Layer 1 operand: the K slots of this lane half (ri_slot_row / ri_slot_kw), as staged.
      const int at = (b - pb) * kRiOut + 2;              // staged index of column X0
      uint4v b1;
      b1[0] = my_x01[at - 1];
      b1[1] = my_x01[at];
      b1[2] = my_x01[at + 1];
      b1[3] = my_x2[at];
      float16v acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(A1, __builtin_bit_cast(half8, b1), acc, 0, 0, 0);
      // y1 row q, channels 4 hsel .. + 3 of this lane's column: f16 of 2^8 d1
      half4 y[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        half4 h;
#pragma unroll
        for (int c = 0; c < 4; ++c) h[c] = (_Float16)acc[4 * q + c];
        y[q] = __builtin_elementwise_max(h, lo1h);
        if (BORDER) y[q] = inside ? y[q] : lo1h;         // layer-2 padding: y1 = 0 beside the tile
      }

      // Layer 2: centre taps from the registers as they are, outer taps moved by a lane.
      typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
      uint4v bc[2], bm[2], bp[2];                        // steps (q0, q1) and (q2, q3) of tap 1, 0, 2
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const u32x2 w = __builtin_bit_cast(u32x2, y[q]);
#pragma unroll
        for (int r = 0; r < 2; ++r) {
          bc[q >> 1][2 * (q & 1) + r] = w[r];
          bm[q >> 1][2 * (q & 1) + r] = dpp_all<kWaveShr1>(w[r]);
          bp[q >> 1][2 * (q & 1) + r] = dpp_all<kWaveShl1>(w[r]);
        }
      }
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(A2[0], __builtin_bit_cast(half8, bc[0]), b2init, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(A2[1], __builtin_bit_cast(half8, bc[1]), acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(A2[2], __builtin_bit_cast(half8, bm[0]), acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(A2[3], __builtin_bit_cast(half8, bm[1]), acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(A2[4], __builtin_bit_cast(half8, bp[0]), acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(A2[5], __builtin_bit_cast(half8, bp[1]), acc, 0, 0, 0);
      float p[3];                                        // 2^8 x the head-weighted sums of this lane's four channels
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        float t = 0.f;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) t = fmaf(w3v[jj], __builtin_amdgcn_fmed3f(acc[4 * k + jj], lo2v[4 * k + jj], inf), t);
        p[k] = t;
      }
      // Sum the two channel halves: afterwards lanes 0..31 hold the moving row, lanes 32..63 the two border rows.
      const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(p[0]), __float_as_uint(p[1] + p[2]), false, false);
      const float total = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
      if (n >= 2 && n < 2 + kRiOut)
        reinterpret_cast<float*>(s_part)[(hf * kRiPassCols + (b - pb) * kRiOut + n - 2) * 2 + hsel] = total;
    };
#pragma unroll 1
    for (int b = pb + wsub; b < pe; b += 2) {
      if (b == 0 || b * kRiOut + 30 > nb_cur) block(b, std::true_type{});   // (the same for the whole wave)
      else block(b, std::false_type{});
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0): this wave's pieces of the next pass are in LDS
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const int rel = tid + 256 * i, c = col0 + rel;
      if (rel < kRiPassCols && c < col_end) {
        const float2 top = s_part[rel], bot = s_part[kRiPassCols + rel];
        float st = pst[i];
        if (advance) {
          st = (st - top.x * kUnscale) + bot.x * kUnscale;
          pstate_inst[c] = st;
        }
        pred_inst[c] = (st + (top.y + bot.y) * kUnscale) * inv_H;
      }
    }
    // (the next pass writes its partials after its own first barrier, which every thread reaches after this loop)
  }
}

}  // namespace
}  // namespace ap
