// Internal declarations shared by the kernel files and the C-ABI layer.  Not installed.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "attnpred.h"

namespace ap {

constexpr int kWave = 64;
constexpr int kAttnThreads = 256;             // 4 waves per attention workgroup
constexpr int kAttnWaves = kAttnThreads / kWave;
constexpr int kNarrowPieceTokens = 512;       // tokens whose probabilities a two- or one-wave sparse-decode workgroup holds in LDS at a time
constexpr int kMaxHist = 256;                 // longest history ap_create accepts
constexpr int kGroupTokens = 16;              // tokens one wave covers per load group (4 x dwordx4 loads)
constexpr int kCalibChunkTokens = 1024;       // tokens per calibration workgroup

// Device-side layout of the predictor weights (all fp32), re-packed by ap_set_weights so that the
// weights one inner loop iteration needs are contiguous:
//   w1r[kh][kw][c1]            at 0
//   b1[c1]                     at 9*c1
//   w2r[ci][kh][kw][c2]        at 10*c1
//   b2[c2]                     at 10*c1 + 9*c1*c2
//   w3[c2]                     at 10*c1 + 9*c1*c2 + c2
//   b3                         at 10*c1 + 9*c1*c2 + 2*c2
// What the runtime says the device holds at once (asked at the first launch that needs it).  Lives in the
// context; a Shape points at it, so that copies of a Shape (the offload calls make two) share the answers.
struct Occupancy {
  int sparse_slots[3] = {-1, -1, -1};   // sparse-decode workgroups in the four-, two- and one-wave form
  int calib_slots = -1;                 // calibration workgroups
};

struct Shape {
  int n_inst, g, d, b, H, R, t_cap, nb_cap, k, n_sink, n_local, c1, c2, kv_dtype;
  int predictor_mfma; // incremental predictor on f16 MFMA (8/8 and 16/32 channels)
  int n_split;        // workgroups per instance in sparse decode
  Occupancy* occ;     // owned by the context, never null
  int calib_chunks;   // max workgroups per instance in calibrate
  const int32_t* table;  // device block table of a paged K/V cache [n_inst][nb_cap], or null (caller-owned)
  int n_phys;            // physical blocks in the pool
};

// Difference form of the predictor.  With an all-zero history the first layer gives c[ci] = relu(b1[ci]) at every
// pixel of the tile and the second layer a constant per channel and row type (which of the three kernel rows fall
// into the window).  Every kernel carries only the difference from that response - d1 = y1 - c (and -c where
// layer 2 is padded with y1 = 0 beside the tile), d2 = relu(y2) - relu(B2) - so that fp32 sums and f16 operands
// resolve the part of pred that differs between blocks instead of the constant all blocks share, and adds the
// constant part P0 = b3 + (1/H) sum_r sum_c w3[c] relu(B2[type(r)][c]) is never added on the device: pred is
// the score relative to P0 (fp32 would spend its mantissa on it), and ap_score_offset hands P0 to whoever wants
// the raw head output.  The constants are worked out in float64 by ap_set_weights and appended to the weight
// buffer at delta_const_offset floats:
//   init1[c1] = min(b1, 0) | lo1[c1] = -max(b1, 0) |
//   init2[type 4][c2] = min(B2, 0) | lo2[type 4][c2] = -max(B2, 0),   B2[type][co] = b2 + sum over the type's taps of w2 c
// so that d1 = max(init1 + sum w1 x, lo1) and d2 = max(init2 + sum w2 d1, lo2) are one clamp each.
// The interior state of the incremental form is the sum of the head-weighted d2 over rows 2..H-3 (type kRowAll).
constexpr int kRowAll = 0, kRowTop = 1, kRowBot = 2, kRowOnly = 3;   // = (row == 0) + 2 * (row == H-1)
__host__ __device__ constexpr int delta_const_offset(int c1, int c2);
__host__ __device__ constexpr int delta_const_floats(int c1, int c2) { return 2 * c1 + 8 * c2; }

// Workspace carve-up (float offsets from ws).
struct WsLayout {
  size_t part_ml;     // [n_inst][n_split][g][2]        split max / sum
  size_t part_acc;    // [n_inst][n_split][g][d]        split un-normalised output
  size_t part_bmp;    // [n_inst][g][k]                 per selected block: max prob relative to split max
  size_t cal_ml;      // [n_inst][calib_chunks][g][2]
  size_t cal_bmp;     // [n_inst][g][nb_cap]
  size_t pred_state;  // [n_inst][nb_cap]               interior state of a full-tile prediction without a caller state
  size_t counters;    // [4] ints                       work counters of persistent kernels (zeroed by the launch that uses them)
  size_t total;       // floats
};

WsLayout ws_layout(const Shape& s);

// Incremental predictor: kernel row kh through which staged y1 row q feeds output `out` of half `half`
// (0 = top: leaving row, row 0, row 1; 1 = bottom: entering row, row H-2, row H-1), or -1 if unused.
__host__ __device__ constexpr int predictor_tap(int half, int out, int q) {
  constexpr int T[2][3][4] = {{{0, 1, 2, -1}, {-1, 2, -1, 1}, {-1, 1, 2, 0}},
                              {{0, 1, 2, -1}, {-1, 0, 1, 2}, {-1, -1, 0, 1}}};
  return T[half][out][q];
}

// f16 operand tables of the MFMA incremental kernel for 8/8 channels, built on the host by ap_set_weights and
// placed kMfmaTableFloatOffset floats into the weight buffer (the fp32 section is 10*8 + 9*64 + 2*8 + 1 = 673
// floats; 676 keeps 16-byte alignment): layer 2 [half 2][K-step 6][lane 64][8 f16], then layer 1
// [half 2][lane 64][8 f16]; what a lane's entries stand for is said in predict_inc8.h.
//   layer 2  lane (m = 8 o + c2, h) of K-step s: entries e = 0..3 belong to the step's first (y1 row q, tap kw)
//            pair, 4..7 to its second, input channel 4 h + e % 4; the pairs of step s are (ri_pair_q(s, 0), kw) and
//            (ri_pair_q(s, 1), kw) with kw = ri_pair_kw(s): centre taps first (their operands are registers as
//            they come out of layer 1), then the two outer taps
//   layer 1  lane (m = 8 q + c1, h): entry e is K slot (h, e) = (staged x row ri_slot_row, tap ri_slot_kw); row -1
//            is the constant 1, whose weight 2^8 min(b1, 0) is the accumulator start; weights scaled by 2^-4
__host__ __device__ constexpr int ri_pair_q(int step, int second) { return 2 * (step & 1) + second; }
__host__ __device__ constexpr int ri_pair_kw(int step) { return step < 2 ? 1 : (step < 4 ? 0 : 2); }
__host__ __device__ constexpr int ri_slot_row(int h, int e) { return e < 6 ? (h ? 3 : 0) + (e & 1) : ((h && e == 7) ? -1 : 2); }
__host__ __device__ constexpr int ri_slot_kw(int h, int e) { return e < 6 ? e / 2 : (h ? 2 : e - 6); }
constexpr int kMfmaTableFloatOffset = 676;
constexpr int kMfmaTableHalfs = 2 * 6 * 64 * 8 + 2 * 64 * 8;
// ... and by the tables of the interior-state kernel (predict_interior.h): layer 2 [step 8][lane 64][8 f16],
// layer 1 [lane 64][8 f16].
constexpr int kMfmaInteriorTableHalfs = 8 * 64 * 8 + 64 * 8;
// The same for 16/32 channels (fp32 section: 10*16 + 9*16*32 + 2*32 + 1 = 4833 floats):
// layer 2 [half 2][pair 8][kw 3][lane 64][8 f16], lane (m = lane % 32, h = lane / 32) holding input channels
// 8h..8h+7 of output channel m for the kernel row that pair (q, o) stands for; then layer 1
// [half 2][row block 2][lane 64][8 f16], row m = 16 (q % 2) + c1 of row block q / 2, K slot k = 3 * xrow + kw,
// scaled by 2^-4.  Pairs in table order, with staged rows q and outputs o numbered as the kernel does:
constexpr int kMfma16TableFloatOffset = 4836;
constexpr int kMfma16TableHalfs = 2 * 24 * 64 * 8 + 2 * 2 * 64 * 8;
constexpr int kMfma16InteriorTableHalfs = 9 * 64 * 8 + 64 * 8;   // interior-state kernel (predict_interior.h)
constexpr int kMfma16PairQ[8] = {0, 1, 1, 1, 2, 2, 3, 3};
constexpr int kMfma16PairO[8] = {0, 0, 1, 2, 0, 2, 1, 2};
// Kernel numbering -> the numbering predictor_tap uses (rows and outputs 1, 2 swap in the bottom half).
__host__ __device__ constexpr int mfma16_phys(int half, int i) { return (half == 1 && (i == 1 || i == 2)) ? 3 - i : i; }

__host__ __device__ constexpr int delta_const_offset(int c1, int c2) {
  return (c1 == 8 && c2 == 8)     ? kMfmaTableFloatOffset + (kMfmaTableHalfs + kMfmaInteriorTableHalfs) / 2
         : (c1 == 16 && c2 == 32) ? kMfma16TableFloatOffset + (kMfma16TableHalfs + kMfma16InteriorTableHalfs) / 2
                                  : (10 * c1 + 9 * c1 * c2 + 2 * c2 + 1 + 3) / 4 * 4;
}

// Launchers.  Each returns hipSuccess or the launch error.
// Full-tile predictor over columns [col_begin, nb_cur); also writes the interior state if pstate != null.
// Launchers that take (inst0, ninst) work on instances [inst0, inst0 + ninst) of the same buffers.
hipError_t launch_predict(const Shape& s, int inst0, int ninst, const float* dweights, const float* hist,
                          int newest_slot, int nb_cur, int col_begin, float* pstate, float* pred, hipStream_t st);
// Interior state (rows 2..H-3) of every column from scratch on MFMA (8/8 or 16/32 channels, H >= 6); the incremental
// kernel without an advance then adds the border rows and writes pred.
hipError_t launch_predict_interior(const Shape& s, int inst0, int ninst, const float* dweights, const float* hist,
                                   int newest_slot, int nb_cur, float* pstate, hipStream_t st);
// The same evaluation for a handful of columns [col_begin, nb_cur): one wave per (instance, column).
hipError_t launch_predict_columns(const Shape& s, int inst0, int ninst, const float* dweights, const float* hist,
                                  int newest_slot, int nb_cur, int col_begin, float* pstate, float* pred,
                                  hipStream_t st);
// Incremental predictor over all columns; advance != 0 moves the state forward by one pushed row first.
hipError_t launch_predict_inc(const Shape& s, int inst0, int ninst, const float* dweights, const float* hist,
                              int newest_slot, int nb_cur, int advance, float* pstate, float* pred, hipStream_t st);
hipError_t launch_select(const Shape& s, int inst0, int ninst, const float* pred, int nb_cur, int32_t* idx,
                         int32_t* cnt, hipStream_t st);
// row_stride: floats between consecutive instances' rows (nb_cap for a plain row buffer,
// R * nb_cap when writing straight into a ring slot).
hipError_t launch_sparse_decode(const Shape& s, int inst0, int ninst, const void* q, const void* K, const void* V,
                                int t_cur, const int32_t* idx, const int32_t* cnt, float* out, float* row,
                                size_t row_stride, float* ws, hipStream_t st);
hipError_t launch_calibrate(const Shape& s, const void* q, const void* K, int t_cur, float* row,
                            float* ws, hipStream_t st);
// Carries a selection made for nb_prev blocks over to nb_cur blocks without new scores (in place).
hipError_t launch_refresh_selection(const Shape& s, int nb_prev, int nb_cur, int32_t* idx, int32_t* cnt,
                                    hipStream_t st);
// Stages the selected blocks of the full cache (pinned host or device memory) that the pool does not hold yet,
// into slots freed by blocks that left the selection; records slots in `table` and in `state`
// (int32 [n_inst][prefetch_state_stride]); rows of tokens >= t_avail are zero-filled.
int prefetch_state_stride(const Shape& s);
hipError_t launch_gather_blocks(const Shape& s, const void* K_src, const void* V_src, int t_avail, int nb_cur,
                                const int32_t* idx, const int32_t* cnt, void* pool_K, void* pool_V, int32_t* table,
                                int32_t* state, hipStream_t st);
// Writes the K/V row of token t_pos into the staged copy of its block (if that block is staged).
hipError_t launch_append_row(const Shape& s, const void* k_new, const void* v_new, int t_pos, const int32_t* table,
                             const int32_t* state, void* pool_K, void* pool_V, hipStream_t st);
hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, int n_wg, hipStream_t st);
hipError_t launch_stream_copy(const void* src, size_t bytes, void* dst, int n_wg, hipStream_t st);
hipError_t launch_push_row(const Shape& s, float* hist, int slot, const float* row, hipStream_t st);

// Floats of workspace that launch_sparse_decode touches (the split partials, which lead the layout).
size_t sparse_ws_floats(const Shape& s);
// The current device's copy of the library's static scratch array (for callers that may not allocate) and its
// size in bytes; looked up once per device.  Returns hipSuccess or the lookup error.
hipError_t static_scratch(float** ptr, size_t* bytes);

}  // namespace ap
