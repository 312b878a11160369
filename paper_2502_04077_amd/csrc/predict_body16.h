// MFMA form of the incremental predictor for the paper's own network (16 and 32 hidden channels; architecture
// table of the appendix "Implement Details").  Same method as predict_inc_mfma_body (see predict.hip): per
// column, the state of the interior rows moves by (row entering) - (row leaving) and the four border rows are
// evaluated afresh; 124 output columns per tile, waves 0,1 = top half, waves 2,3 = bottom half, each wave
// owning two 32-column blocks.
//
// v_mfma_f32_32x32x16_f16: D[32 x 32] += A[32 x 16] * B[16 x 32]; lane l supplies row/column l % 32 and K
// entries 8 (l / 32) .. + 7, and receives D rows 8 (v / 4) + 4 (l / 32) + v % 4 (v = 0..15) of column l % 32.
//   layer 1: rows = (y1 row q, c1): two row blocks (q = 0,1 and q = 2,3); K = 16 = (x row 0..4, kw 0..2) + one
//            unused slot; columns = 32 y1 columns.  x is scaled by 2^12 and split into f16 hi + lo (two MFMAs; the
//            split is done once, when a tile's rows are staged),
//            the weights are f16 scaled by 2^-4, the accumulator starts at 2^8 b1: the result is 2^8 y1 before
//            the ReLU.  It is rounded to f16 (the scale keeps y1 up to 255 inside the f16 range), clamped at 0
//            and stored as [half][q][channel half][column] x 8 channels, so a layer-2 operand is one 16-byte read.
//   layer 2: one row block (32 output channels) per output o; K-step = (q, kw) with its 16 input channels.
//            Each output only meets the y1 rows it taps (3 + 3 + 2), 24 MFMAs per column block instead of 36.
//            The staged rows and outputs of the bottom half are numbered so that both halves have the same
//            (q, o) structure; which kernel row a pair stands for is in the operand table built on the host:
//              q0 -> o0     q1 -> o0, o1, o2     q2 -> o0, o2     q3 -> o1, o2        (o0 = the moving row)
//              top:    q0..q3 = x[-1..1] formula, y1[1], y1[2], y1[0]      o1, o2 = rows 0, 1
//              bottom: q0..q3 = y1[H-4], y1[H-2], y1[H-3], y1[H-1]         o1, o2 = rows H-1, H-2
//            Accumulators start at 2^8 b2; the head weights carry the 2^-8.
// The moving row of the bottom half and that of the top half sum their taps in different orders, so the value
// that leaves the state is the one that entered only up to fp32 rounding; callers re-base now and then anyway.
#pragma once

#include "predict_body.h"

namespace ap {
namespace {

constexpr int kP16IW = kPmIW, kP16XW = kPmXW, kP16YW = kPmYW, kP16LD = kPmLD, kP16XBuf = kPmXBuf;   // same tile geometry
constexpr int kP16Y1Floats = 2 * 4 * 2 * kP16YW * 4;
// A1 | 2^8 init1 | 2^-8 w3 | x offsets | 2^8 init2 of (half, row type all / border) | 2^8 lo2 of the same | 2^8 lo1 (f16)
constexpr int kP16ConstFloats = 2 * 2 * kWave * 4 + 2 * 16 + 2 * 16 + 2 * 8 + 2 * 2 * 2 * 16 + 2 * 2 * 2 * 16 + 2 * 4;
constexpr int kPred16LdsFloats = kP16Y1Floats + 2 * kP16XBuf + 8 * kP16LD + kP16ConstFloats;

// Workgroup `chunk` of `n_chunks` of instance `inst` (256 threads); smem: kPred16LdsFloats floats, 16-byte aligned.
__device__ __forceinline__ void predict_inc_mfma16_body(const float* __restrict__ hist,
                                                        const float* __restrict__ wts_global, int R, int H,
                                                        int newest_slot, int nb_cur, int nb_cap, int inst, int chunk,
                                                        int n_chunks, int advance, float* __restrict__ pstate,
                                                        float* __restrict__ pred, float* smem) {
  constexpr int C1 = 16, C2 = 32, IW = kP16IW, XW = kP16XW, YW = kP16YW, LD = kP16LD, XBUF = kP16XBuf;
  constexpr float kXScale = 4096.f, kAccScale = 256.f;
  half8* s_y1 = reinterpret_cast<half8*>(smem);          // [half 2][q 4][channel half 2][YW] x 8 f16
  uint32_t* s_xb = reinterpret_cast<uint32_t*>(smem + kP16Y1Floats);   // 2 buffers of [10][XW] (+4) hi|lo words
  float* s_red = reinterpret_cast<float*>(s_xb + 2 * XBUF);                        // [half 2][moving | border][lane half 2][LD]
  // Per-lane operands that only one phase of a tile needs live here and are re-read in that phase, which
  // keeps the kernel at two waves per SIMD next to the 96 registers of layer-2 weights:
  half8* s_a1 = reinterpret_cast<half8*>(s_red + 8 * LD);   // [half 2][row block 2][lane 64]
  float* s_b1 = reinterpret_cast<float*>(s_a1 + 2 * 2 * kWave);   // [lane half 2][16] accumulator start of layer 1
  float* s_w3 = s_b1 + 2 * 16;                           // [lane half 2][16] head weight of accumulator entry v
  int* s_xoff = reinterpret_cast<int*>(s_w3 + 2 * 16);   // [lane half 2][8]  x offset of layer-1 K slot e
  // Difference form (ap_internal.h): where the accumulators of the second layer start and where they are clamped,
  // for the outputs that meet all three kernel rows (o0, o2) and for the half's border row (o1: row 0 or row H-1).
  float* s_i2 = reinterpret_cast<float*>(s_xoff + 2 * 8);   // [half 2][all | border][lane half 2][16]
  float* s_l2 = s_i2 + 2 * 2 * 2 * 16;                      // the same layout
  half4* s_l1 = reinterpret_cast<half4*>(s_l2 + 2 * 2 * 2 * 16);   // [channel half pl 2][lane half 2] clamp of the first layer

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

  // Operand tables and constants.
  const half8* tab = reinterpret_cast<const half8*>(wts_global + kMfma16TableFloatOffset);
  const half8* tab2 = tab + (size_t)hf * 24 * kWave;     // [pair 8][kw 3][lane]
  half8 A2[24];
#pragma unroll
  for (int i = 0; i < 24; ++i) A2[i] = tab2[i * kWave + lane];
  const float* b2 = wts_global + 10 * C1 + 9 * C1 * C2;
  const float* dc = wts_global + delta_const_offset(C1, C2);
  s_a1[tid] = tab[2 * 24 * kWave + tid];
  if (tid < 32) {
    const int h = tid >> 4, v = tid & 15, row = 8 * (v / 4) + 4 * h + v % 4;   // D row of accumulator entry v
    s_b1[tid] = kAccScale * dc[row % C1];
    s_w3[tid] = b2[C2 + row] * (1.f / kAccScale);
  }
  if (tid < 128) {
    const int half = tid >> 6, border = (tid >> 5) & 1, h = (tid >> 4) & 1, v = tid & 15;
    const int row = 8 * (v / 4) + 4 * h + v % 4;
    const int type = border ? (half == 0 ? kRowTop : kRowBot) : kRowAll;
    s_i2[tid] = kAccScale * dc[2 * C1 + type * C2 + row];
    s_l2[tid] = kAccScale * dc[2 * C1 + (4 + type) * C2 + row];
  }
  if (tid < 4) {
    const int pl = tid >> 1, h = tid & 1;
    half4 l;
#pragma unroll
    for (int c = 0; c < 4; ++c) l[c] = (_Float16)(kAccScale * dc[C1 + 8 * pl + 4 * h + c]);
    s_l1[tid] = l;
  }
  if (tid < 16) {   // layer-1 K slot 8 h + e is (x row, kw) = divmod(8 h + e, 3); slot 15 has zero weights
    const int k = tid;
    s_xoff[tid] = k < 15 ? (k / 3) * XW + k % 3 : 0;
  }
  if (tid < 4) s_xb[XBUF - 4 + tid] = s_xb[2 * XBUF - 4 + tid] = 0u;

  // x staging: thread tid fetches column tid % 128 of staged rows hf, hf + 2, .., hf + 8; staged rows 0..4 are
  // history rows -1..3, staged rows 5..9 are rows H-5..H-1.
  const int xcol = (tid & (XW - 1)) - 2;
  int xrow_off[5];
#pragma unroll
  for (int i = 0; i < 5; ++i) {
    const int rr = hf + 2 * i;
    xrow_off[i] = ring_slot(newest_slot, H, R, rr < 5 ? rr - 1 : H - 10 + rr) * nb_cap;
  }
  float xpre[5], pst_cur = 0.f, pst_next = 0.f;
  // Loads are unconditional on clamped addresses; the raw values stay untouched in registers until `stash`
  // masks them, so nothing waits on them while the current tile is computed.
  auto fetch = [&](int tile, float& pst) __attribute__((always_inline)) {
    const int c0 = tile * IW;
    const int j = min(max(c0 + xcol, 0), nb_cur - 1);
#pragma unroll
    for (int i = 0; i < 5; ++i) xpre[i] = hist_inst[xrow_off[i] + j];
    pst = pstate_inst[min(c0 + tid, nb_cur - 1)];
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
    int fresh = 0;                      // opaque zero: the phase operands are read again in every tile
    asm volatile("" : "+v"(fresh));

    // Layer 1.
    {
      const uint32_t* xs = s_x + hf * 5 * XW;
      const half8 A1a = s_a1[fresh + (hf * 2 + 0) * kWave + lane], A1b = s_a1[fresh + (hf * 2 + 1) * kWave + lane];
      float16v b1acc;
      int xoff[8];
#pragma unroll
      for (int v = 0; v < 16; ++v) b1acc[v] = s_b1[fresh + hsel * 16 + v];
#pragma unroll
      for (int e = 0; e < 8; ++e) xoff[e] = s_xoff[fresh + hsel * 8 + e];
      const half4 lo1a = s_l1[fresh + 0 * 2 + hsel], lo1b = s_l1[fresh + 1 * 2 + hsel];
#pragma unroll
      for (int blk = 0; blk < 2; ++blk) {
        const int yc = ((wave & 1) * 2 + blk) * 32 + n;  // y1 column 0..127  <->  tile column c0 - 1 + yc
        uint4v whi, wlo;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          const uint32_t wa = xs[yc + xoff[e]], wb = xs[yc + xoff[e + 1]];
          whi[e / 2] = __builtin_amdgcn_perm(wb, wa, 0x05040100u);
          wlo[e / 2] = __builtin_amdgcn_perm(wb, wa, 0x07060302u);
        }
        const half8 Bhi = __builtin_bit_cast(half8, whi), Blo = __builtin_bit_cast(half8, wlo);
        const int j = c0 - 1 + yc;
        const bool outside = j < 0 || j >= nb_cur;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
          float16v acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(rb ? A1b : A1a, Bhi, b1acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(rb ? A1b : A1a, Blo, acc, 0, 0, 0);
          // entry v: y1 row q = 2 rb + v / 8, channel 8 (v / 4 % 2) + 4 hsel + v % 4
#pragma unroll
          for (int ql = 0; ql < 2; ++ql)
#pragma unroll
            for (int p = 0; p < 2; ++p) {
              half4 h;
#pragma unroll
              for (int c = 0; c < 4; ++c) h[c] = (_Float16)acc[8 * ql + 4 * p + c];
              h = __builtin_elementwise_max(h, p ? lo1b : lo1a);
              reinterpret_cast<half4*>(s_y1 + ((hf * 4 + 2 * rb + ql) * 2 + p) * YW + yc)[hsel] = h;
            }
        }
        if (outside) {                                   // layer-2 padding: y1 = 0 beside the tile, d1 = lo1
#pragma unroll
          for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int p = 0; p < 2; ++p)
              reinterpret_cast<half4*>(s_y1 + ((hf * 4 + q) * 2 + p) * YW + yc)[hsel] = p ? lo1b : lo1a;
        }
      }
    }
    __syncthreads();

    // Layer 2 and the head.
    float16v b2acc, b2bor;                // accumulator starts: rows with all kernel rows (o0, o2), the border row (o1)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      b2acc[v] = s_i2[fresh + ((hf * 2 + 0) * 2 + hsel) * 16 + v];
      b2bor[v] = s_i2[fresh + ((hf * 2 + 1) * 2 + hsel) * 16 + v];
    }
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      const int cb = ((wave & 1) * 2 + blk) * 32;
      const half8* yq = s_y1 + ((size_t)hf * 4 * 2 + hsel) * YW + cb + n;   // + q * 2 * YW + kw
      float16v acc0, acc1, acc2;
#pragma unroll
      for (int kw = 0; kw < 3; ++kw) {
        const half8 B = yq[0 * 2 * YW + kw];
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(A2[0 * 3 + kw], B, kw == 0 ? b2acc : acc0, 0, 0, 0);
      }
#pragma unroll
      for (int kw = 0; kw < 3; ++kw) {
        const half8 B = yq[1 * 2 * YW + kw];
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(A2[1 * 3 + kw], B, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(A2[2 * 3 + kw], B, kw == 0 ? b2bor : acc1, 0, 0, 0);
        acc2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(A2[3 * 3 + kw], B, kw == 0 ? b2acc : acc2, 0, 0, 0);
      }
#pragma unroll
      for (int kw = 0; kw < 3; ++kw) {
        const half8 B = yq[2 * 2 * YW + kw];
        acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(A2[4 * 3 + kw], B, acc0, 0, 0, 0);
        acc2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(A2[5 * 3 + kw], B, acc2, 0, 0, 0);
      }
#pragma unroll
      for (int kw = 0; kw < 3; ++kw) {
        const half8 B = yq[3 * 2 * YW + kw];
        acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(A2[6 * 3 + kw], B, acc1, 0, 0, 0);
        acc2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(A2[7 * 3 + kw], B, acc2, 0, 0, 0);
      }
      float t0 = 0.f, t1 = 0.f, t2 = 0.f;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float w = s_w3[fresh + hsel * 16 + v];
        const float la = s_l2[fresh + ((hf * 2 + 0) * 2 + hsel) * 16 + v], lb = s_l2[fresh + ((hf * 2 + 1) * 2 + hsel) * 16 + v];
        t0 = fmaf(w, __builtin_amdgcn_fmed3f(acc0[v], la, inf), t0);
        t1 = fmaf(w, __builtin_amdgcn_fmed3f(acc1[v], lb, inf), t1);
        t2 = fmaf(w, __builtin_amdgcn_fmed3f(acc2[v], la, inf), t2);
      }
      s_red[((hf * 2 + 0) * 2 + hsel) * LD + cb + n] = t0;
      s_red[((hf * 2 + 1) * 2 + hsel) * LD + cb + n] = t1 + t2;
    }
    __syncthreads();
    if (tid < IW && c0 + tid < nb_cur) {
      auto part = [&](int half, int kind) __attribute__((always_inline)) {
        return s_red[((half * 2 + kind) * 2 + 0) * LD + tid] + s_red[((half * 2 + kind) * 2 + 1) * LD + tid];
      };
      float st = pst_cur;
      if (advance) {
        st = (st - part(0, 0)) + part(1, 0);
        pstate_inst[c0 + tid] = st;
      }
      pred_inst[c0 + tid] = (st + (part(0, 1) + part(1, 1))) / (float)H;
    }
    if (more) stash(tile + 1, s_xb + (((tile - t_begin) & 1) ^ 1) * XBUF);
    pst_cur = pst_next;
    __syncthreads();
  }
}

}  // namespace
}  // namespace ap
