// C ABI of the library: argument validation, context, workspace layout, launch sequencing.
#include <new>
#include <vector>

#include "ap_internal.h"

struct ap_ctx {
  ap::Shape s;
  float* dweights;      // device copy of the re-packed predictor weights, owned
  bool have_weights;
  double score_offset;  // P0: what the predictor answers to an all-zero history (pred is relative to it)
  // ap_offload_*: "selection for the next token is written" / "its blocks are staged"; created on first use, owned
  hipEvent_t ev_selected, ev_staged;
  bool have_events;
  ap::Occupancy occ;         // what the device holds at once; s.occ points here
};

namespace ap {

static size_t align4(size_t x) { return (x + 3) & ~(size_t)3; }

WsLayout ws_layout(const Shape& s) {
  WsLayout w;
  size_t o = 0;
  w.part_ml = o;  o = align4(o + (size_t)s.n_inst * s.n_split * s.g * 2);
  w.part_acc = o; o = align4(o + (size_t)s.n_inst * s.n_split * s.g * s.d);
  w.part_bmp = o; o = align4(o + (size_t)s.n_inst * s.g * s.k);
  w.cal_ml = o;   o = align4(o + (size_t)s.n_inst * s.calib_chunks * s.g * 2);
  w.cal_bmp = o;  o = align4(o + (size_t)s.n_inst * s.g * s.nb_cap);
  w.pred_state = o; o = align4(o + (size_t)s.n_inst * s.nb_cap);
  w.counters = o; o = align4(o + 4);
  w.total = o;
  return w;
}

// The split partials lead the layout; a context with one workgroup per instance has none.
size_t sparse_ws_floats(const Shape& s) { return s.n_split > 1 ? ws_layout(s).cal_ml : 0; }

static bool pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

// Workgroups per instance for sparse decode: enough to give the chip work when there are few
// instances, at least one 16-token group per wave, and a logits tile that fits in 32 KiB of LDS.
static int choose_split(const Shape& s) {
  const int groups = (s.k * s.b + kGroupTokens - 1) / kGroupTokens;
  const int by_work = groups / kAttnWaves > 1 ? groups / kAttnWaves : 1;
  int want = (1024 + s.n_inst - 1) / s.n_inst;
  if (want > by_work) want = by_work;
  const int by_lds = (int)(((size_t)s.g * s.k * s.b * sizeof(float) + 32767) / 32768);
  if (want < by_lds) want = by_lds;
  if (want > s.k) want = s.k;
  if (want < 1) want = 1;
  const int per = (s.k + want - 1) / want;
  return (s.k + per - 1) / per;
}

}  // namespace ap

using ap::Shape;

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#define AP_REQUIRE_PTR(p)                 \
  do {                                    \
    if ((p) == nullptr) return AP_ERR_ARG; \
    if (!aligned16(p)) return AP_ERR_ALIGN; \
  } while (0)

extern "C" {

int ap_create(const ap_config* c, ap_ctx** out) {
  if (c == nullptr || out == nullptr) return AP_ERR_ARG;
  if (c->n_inst <= 0 || c->t_cap <= 0 || c->hist_len <= 0 || c->k_blocks <= 0) return AP_ERR_ARG;
  if (c->n_sink < 0 || c->n_local < 0 || c->n_sink + c->n_local > c->k_blocks) return AP_ERR_ARG;
  if (!ap::pow2(c->block) || c->block < 8 || c->block > 64) return AP_ERR_UNSUPPORTED;
  if (c->t_cap % c->block != 0) return AP_ERR_ARG;
  if (c->g != 1 && c->g != 2 && c->g != 4 && c->g != 8) return AP_ERR_UNSUPPORTED;
  if (c->head_dim != 64 && c->head_dim != 128) return AP_ERR_UNSUPPORTED;
  if (c->kv_dtype != AP_F32 && c->kv_dtype != AP_BF16) return AP_ERR_UNSUPPORTED;
  if (c->hist_len > ap::kMaxHist) return AP_ERR_UNSUPPORTED;
  if (c->k_blocks > 16384) return AP_ERR_UNSUPPORTED;
  const bool chan_ok = (c->c1 == 4 && c->c2 == 4) || (c->c1 == 8 && c->c2 == 8) || (c->c1 == 16 && c->c2 == 32);
  if (!chan_ok) return AP_ERR_UNSUPPORTED;
  if (c->n_inst > 65535) return AP_ERR_UNSUPPORTED;     // instances ride on gridDim.y

  ap_ctx* ctx = new (std::nothrow) ap_ctx;
  if (ctx == nullptr) return AP_ERR_ARG;
  Shape& s = ctx->s;
  s.occ = &ctx->occ;
  s.n_inst = c->n_inst; s.g = c->g; s.d = c->head_dim; s.b = c->block; s.H = c->hist_len;
  s.R = c->hist_len + 1; s.t_cap = c->t_cap; s.nb_cap = c->t_cap / c->block; s.k = c->k_blocks;
  s.n_sink = c->n_sink; s.n_local = c->n_local; s.c1 = c->c1; s.c2 = c->c2; s.kv_dtype = c->kv_dtype;
  s.predictor_mfma = (((c->c1 == 8 && c->c2 == 8) || (c->c1 == 16 && c->c2 == 32)) &&
                      !(c->flags & AP_FLAG_PREDICTOR_FP32)) ? 1 : 0;
  s.n_split = ap::choose_split(s);
  {
    // Dynamic LDS of the attention workgroup (sparse_lds_floats) and of the combine kernel must fit 64 KiB.
    const size_t nblk = s.n_split == 1 ? s.k : (s.k + s.n_split - 1) / s.n_split;
    const size_t partials = (size_t)ap::kAttnWaves * s.g * s.d, tile = (size_t)ap::kAttnWaves * 8 * (2 * s.d + 16) / 4;
    const size_t attn = (size_t)s.g * nblk * s.b + (partials > tile ? partials : tile) + (size_t)s.g * nblk + 2 * nblk + 4 * s.g + 2 * (size_t)((s.nb_cap + 31) / 32);
    const size_t comb = (size_t)s.n_split * s.g + 1024;     // (sparse_combine_kernel: scales + a chunk of the row)
    if (attn * sizeof(float) > 65536 || comb * sizeof(float) > 65536) { delete ctx; return AP_ERR_UNSUPPORTED; }
  }
  const int chunk_blocks = ap::kCalibChunkTokens / s.b;
  s.calib_chunks = (s.nb_cap + chunk_blocks - 1) / chunk_blocks;
  if ((size_t)s.calib_chunks * s.g * sizeof(float) > 60000) { delete ctx; return AP_ERR_UNSUPPORTED; }
  s.table = nullptr;
  s.n_phys = 0;
  ctx->dweights = nullptr;
  ctx->have_weights = false;
  ctx->score_offset = 0.0;
  ctx->have_events = false;
  *out = ctx;
  return AP_OK;
}

int ap_destroy(ap_ctx* ctx) {
  if (ctx == nullptr) return AP_ERR_ARG;
  int rc = AP_OK;
  if (ctx->dweights != nullptr && hipFree(ctx->dweights) != hipSuccess) rc = AP_ERR_HIP;
  if (ctx->have_events) {
    if (hipEventDestroy(ctx->ev_selected) != hipSuccess) rc = AP_ERR_HIP;
    if (hipEventDestroy(ctx->ev_staged) != hipSuccess) rc = AP_ERR_HIP;
  }
  delete ctx;
  return rc;
}

size_t ap_workspace_bytes(const ap_ctx* ctx) {
  if (ctx == nullptr) return 0;
  return ap::ws_layout(ctx->s).total * sizeof(float);
}

int32_t ap_hist_slots(const ap_ctx* ctx) { return ctx ? ctx->s.R : 0; }
int32_t ap_nb_cap(const ap_ctx* ctx) { return ctx ? ctx->s.nb_cap : 0; }

int ap_set_block_table(ap_ctx* ctx, const int32_t* block_table, int32_t n_phys_blocks) {
  if (ctx == nullptr) return AP_ERR_ARG;
  if (block_table == nullptr) {
    ctx->s.table = nullptr;
    ctx->s.n_phys = 0;
    return AP_OK;
  }
  if (!aligned16(block_table)) return AP_ERR_ALIGN;
  if (n_phys_blocks < 1) return AP_ERR_ARG;
  ctx->s.table = block_table;
  ctx->s.n_phys = n_phys_blocks;
  return AP_OK;
}

int ap_set_weights(ap_ctx* ctx, const float* blob, size_t n_floats, void* stream) {
  if (ctx == nullptr || blob == nullptr) return AP_ERR_ARG;
  const int c1 = ctx->s.c1, c2 = ctx->s.c2;
  const size_t expect = 9 * (size_t)c1 + c1 + 9 * (size_t)c1 * c2 + c2 + c2 + 1;
  if (n_floats != expect) return AP_ERR_ARG;
  const float* w1 = blob;                 // [c1][3][3]
  const float* b1 = w1 + 9 * c1;
  const float* w2 = b1 + c1;              // [c2][c1][3][3]
  const float* b2 = w2 + 9 * (size_t)c1 * c2;
  const float* w3 = b2 + c2;
  const float* b3 = w3 + c2;
  const bool mfma_table = (c1 == 8 && c2 == 8), mfma16_table = (c1 == 16 && c2 == 32);
  const size_t dc_off = ap::delta_const_offset(c1, c2);
  const size_t total = dc_off + ap::delta_const_floats(c1, c2);
  std::vector<float> packed(total, 0.f);
  float* p = packed.data();
  for (int t = 0; t < 9; ++t)
    for (int c = 0; c < c1; ++c) p[t * c1 + c] = w1[c * 9 + t];
  p += 9 * c1;
  for (int c = 0; c < c1; ++c) p[c] = b1[c];
  p += c1;
  for (int ci = 0; ci < c1; ++ci)
    for (int t = 0; t < 9; ++t)
      for (int co = 0; co < c2; ++co) p[(ci * 9 + t) * c2 + co] = w2[((size_t)co * c1 + ci) * 9 + t];
  p += 9 * (size_t)c1 * c2;
  for (int c = 0; c < c2; ++c) p[c] = b2[c];
  p += c2;
  for (int c = 0; c < c2; ++c) p[c] = w3[c];
  p += c2;
  p[0] = b3[0];
  if (mfma_table) {
    // Operands of the register-resident incremental kernel (layout and K-slot maps: predict_inc8.h).
    _Float16* t = reinterpret_cast<_Float16*>(packed.data() + ap::kMfmaTableFloatOffset);
    for (int half = 0; half < 2; ++half)
      for (int s = 0; s < 6; ++s)
        for (int lane = 0; lane < 64; ++lane) {
          const int m = lane % 32, h = lane / 32, kw = ap::ri_pair_kw(s);
          for (int e = 0; e < 8; ++e) {
            const int q = ap::ri_pair_q(s, e / 4), ci = 4 * h + e % 4;
            float v = 0.f;
            if (m < 24) {
              const int kh = ap::predictor_tap(half, m / 8, q);
              if (kh >= 0) v = w2[(((size_t)(m % 8) * c1 + ci) * 3 + kh) * 3 + kw];
            }
            t[((half * 6 + s) * 64 + lane) * 8 + e] = (_Float16)v;
          }
        }
    // Layer 1: y1 row q of a half reads staged x rows base .. base + 2; a tap row outside the history window is
    // dropped; the constant slot carries the accumulator start 2^8 min(b1, 0).
    _Float16* t1 = t + 2 * 6 * 64 * 8;
    for (int half = 0; half < 2; ++half)
      for (int lane = 0; lane < 64; ++lane)
        for (int e = 0; e < 8; ++e) {
          const int m = lane % 32, h = lane / 32, q = m / 8, c = m % 8;
          const int xrow = ap::ri_slot_row(h, e), kw = ap::ri_slot_kw(h, e);
          const int base = (half == 0 && q == 3) ? 0 : q;
          const int zero_kh = q == 3 ? (half == 0 ? 0 : 2) : -1;
          float v = 0.f;
          if (xrow < 0) {
            v = 256.f * (b1[c] < 0.f ? b1[c] : 0.f);
          } else {
            const int kh = xrow - base;
            if (kh >= 0 && kh < 3 && kh != zero_kh) v = w1[(c * 3 + kh) * 3 + kw] * (1.f / 16.f);
          }
          t1[(half * 64 + lane) * 8 + e] = (_Float16)v;
        }
  }
  if (mfma_table) {
    // Interior-state kernel: strips of three output rows o from five y1 rows q (kernel row q - o), and three y1
    // rows q from five x rows (kernel row xrow - q); no row of it touches the zero padding in time.
    _Float16* t = reinterpret_cast<_Float16*>(packed.data() + ap::kMfmaTableFloatOffset) + ap::kMfmaTableHalfs;
    for (int step = 0; step < 8; ++step)
      for (int lane = 0; lane < 64; ++lane) {
        const int m = lane % 32, chunk = 2 * step + lane / 32, q = chunk / 3, kw = chunk % 3;
        const int kh = q - m / 8;
        for (int ci = 0; ci < 8; ++ci) {
          float v = 0.f;
          if (m < 24 && chunk < 15 && kh >= 0 && kh < 3) v = w2[(((size_t)(m % 8) * c1 + ci) * 3 + kh) * 3 + kw];
          t[(step * 64 + lane) * 8 + ci] = (_Float16)v;
        }
      }
    _Float16* t1 = t + 8 * 64 * 8;
    for (int lane = 0; lane < 64; ++lane)
      for (int e = 0; e < 8; ++e) {
        const int m = lane % 32, k = 8 * (lane / 32) + e;
        float v = 0.f;
        if (m < 24 && k < 15) {
          const int kh = k / 3 - m / 8, kw = k % 3;
          if (kh >= 0 && kh < 3) v = w1[((m % 8) * 3 + kh) * 3 + kw] * (1.f / 16.f);
        }
        t1[lane * 8 + e] = (_Float16)v;
      }
  }
  if (mfma16_table) {
    // A operands of the 16/32-channel kernel (layout and numbering: ap_internal.h).
    _Float16* t = reinterpret_cast<_Float16*>(packed.data() + ap::kMfma16TableFloatOffset);
    for (int half = 0; half < 2; ++half)
      for (int pair = 0; pair < 8; ++pair) {
        const int kh = ap::predictor_tap(half, ap::mfma16_phys(half, ap::kMfma16PairO[pair]),
                                         ap::mfma16_phys(half, ap::kMfma16PairQ[pair]));
        for (int kw = 0; kw < 3; ++kw)
          for (int lane = 0; lane < 64; ++lane)
            for (int e = 0; e < 8; ++e) {
              const int co = lane % 32, ci = 8 * (lane / 32) + e;
              const float v = kh < 0 ? 0.f : w2[(((size_t)co * c1 + ci) * 3 + kh) * 3 + kw];
              t[(((half * 8 + pair) * 3 + kw) * 64 + lane) * 8 + e] = (_Float16)v;
            }
      }
    _Float16* t1 = t + 2 * 24 * 64 * 8;
    for (int half = 0; half < 2; ++half)
      for (int rb = 0; rb < 2; ++rb)
        for (int lane = 0; lane < 64; ++lane)
          for (int e = 0; e < 8; ++e) {
            const int m = lane % 32, k = 8 * (lane / 32) + e, c = m % 16;
            const int q = ap::mfma16_phys(half, 2 * rb + m / 16);
            const int base = (half == 0 && q == 3) ? 0 : q;
            const int zero_kh = q == 3 ? (half == 0 ? 0 : 2) : -1;
            float v = 0.f;
            if (k < 15) {
              const int kh = k / 3 - base, kw = k % 3;
              if (kh >= 0 && kh < 3 && kh != zero_kh) v = w1[(c * 3 + kh) * 3 + kw] * (1.f / 16.f);
            }
            t1[((half * 2 + rb) * 64 + lane) * 8 + e] = (_Float16)v;
          }
  }
  if (mfma16_table) {
    // Interior-state kernel for 16/32 channels: one operand per (kernel row, tap) for layer 2, two y1 rows from four
    // x rows for layer 1.
    _Float16* t = reinterpret_cast<_Float16*>(packed.data() + ap::kMfma16TableFloatOffset) + ap::kMfma16TableHalfs;
    for (int kh = 0; kh < 3; ++kh)
      for (int kw = 0; kw < 3; ++kw)
        for (int lane = 0; lane < 64; ++lane)
          for (int e = 0; e < 8; ++e) {
            const int co = lane % 32, ci = 8 * (lane / 32) + e;
            t[(((kh * 3 + kw) * 64) + lane) * 8 + e] = (_Float16)w2[(((size_t)co * c1 + ci) * 3 + kh) * 3 + kw];
          }
    _Float16* t1 = t + 9 * 64 * 8;
    for (int lane = 0; lane < 64; ++lane)
      for (int e = 0; e < 8; ++e) {
        const int m = lane % 32, k = 8 * (lane / 32) + e;
        float v = 0.f;
        if (k < 12) {
          const int kh = k / 3 - m / 16, kw = k % 3;
          if (kh >= 0 && kh < 3) v = w1[((m % 16) * 3 + kh) * 3 + kw] * (1.f / 16.f);
        }
        t1[lane * 8 + e] = (_Float16)v;
      }
  }
  double score_offset = 0.0;
  {
    // Constants of the difference form (layout: ap_internal.h), in float64.
    const int H = ctx->s.H;
    float* dc = packed.data() + dc_off;
    std::vector<double> c(c1);
    for (int ci = 0; ci < c1; ++ci) {
      c[ci] = b1[ci] > 0.f ? (double)b1[ci] : 0.0;
      dc[ci] = b1[ci] < 0.f ? b1[ci] : 0.f;
      dc[c1 + ci] = (float)-c[ci];
    }
    double hc[4];
    for (int type = 0; type < 4; ++type) {
      // kernel rows inside the window: all three, not the first (row 0), not the last (row H-1), the middle one only
      const int kh0 = (type & 1) ? 1 : 0, kh1 = (type & 2) ? 1 : 2;
      hc[type] = 0.0;
      for (int co = 0; co < c2; ++co) {
        double B = b2[co];
        for (int ci = 0; ci < c1; ++ci)
          for (int kh = kh0; kh <= kh1; ++kh)
            for (int kw = 0; kw < 3; ++kw) B += (double)w2[(((size_t)co * c1 + ci) * 3 + kh) * 3 + kw] * c[ci];
        dc[2 * c1 + type * c2 + co] = (float)(B < 0.0 ? B : 0.0);
        dc[2 * c1 + (4 + type) * c2 + co] = (float)(B > 0.0 ? -B : 0.0);
        hc[type] += (double)w3[co] * (B > 0.0 ? B : 0.0);
      }
    }
    double sum = 0.0;
    for (int r = 0; r < H; ++r) sum += hc[(r == 0 ? 1 : 0) + (r == H - 1 ? 2 : 0)];
    score_offset = (double)b3[0] + sum / H;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (ctx->dweights == nullptr &&
      hipMalloc(reinterpret_cast<void**>(&ctx->dweights), total * sizeof(float)) != hipSuccess) {
    ctx->dweights = nullptr;
    return AP_ERR_HIP;
  }
  if (hipMemcpyAsync(ctx->dweights, packed.data(), total * sizeof(float), hipMemcpyHostToDevice, st) != hipSuccess)
    return AP_ERR_HIP;
  if (hipStreamSynchronize(st) != hipSuccess) return AP_ERR_HIP;   // `packed` dies on return
  ctx->have_weights = true;
  ctx->score_offset = score_offset;
  return AP_OK;
}

double ap_score_offset(const ap_ctx* ctx) { return (ctx != nullptr && ctx->have_weights) ? ctx->score_offset : 0.0; }

static int newest_slot_of(const Shape& s, int64_t n_pushed) {
  return n_pushed <= 0 ? s.R - 1 : (int)((n_pushed - 1) % s.R);
}

// Runs the predictor in the requested mode; shared by ap_predict_incremental and ap_step.
static int run_predictor(const ap_ctx* ctx, const float* hist, int64_t n_pushed, int nb_cur, int nb_prev, int mode,
                         float* pstate, float* pred, float* ws, hipStream_t st) {
  const Shape& s = ctx->s;
  const int newest = newest_slot_of(s, n_pushed);
  if (pstate == nullptr || mode == AP_PRED_REBASE || s.H < 6) {
    if (s.H >= 6 && s.predictor_mfma) {
      // Full tile on MFMA: the interior state from scratch (into the caller's pstate, or into the workspace when
      // the caller keeps none), then the borders and the head as in a HOLD call.
      float* state = pstate != nullptr ? pstate : ws + ap::ws_layout(s).pred_state;
      if (ap::launch_predict_interior(s, 0, s.n_inst, ctx->dweights, hist, newest, nb_cur, state, st) != hipSuccess ||
          ap::launch_predict_inc(s, 0, s.n_inst, ctx->dweights, hist, newest, nb_cur, 0, state, pred, st) != hipSuccess)
        return AP_ERR_HIP;
      return AP_OK;
    }
    return ap::launch_predict(s, 0, s.n_inst, ctx->dweights, hist, newest, nb_cur, 0, pstate, pred, st) == hipSuccess
               ? AP_OK : AP_ERR_HIP;
  }
  if (ap::launch_predict_inc(s, 0, s.n_inst, ctx->dweights, hist, newest, nb_cur, mode == AP_PRED_ADVANCE, pstate,
                             pred, st) != hipSuccess)
    return AP_ERR_HIP;
  if (nb_cur > nb_prev) {
    // The tile grew: column nb_prev - 1 gained a right neighbour inside the tile and the new columns
    // have no state yet; evaluate those columns in full.
    const int col_begin = nb_prev > 1 ? nb_prev - 1 : 0;
    const hipError_t e =
        nb_cur - col_begin <= 8
            ? ap::launch_predict_columns(s, 0, s.n_inst, ctx->dweights, hist, newest, nb_cur, col_begin, pstate, pred, st)
            : ap::launch_predict(s, 0, s.n_inst, ctx->dweights, hist, newest, nb_cur, col_begin, pstate, pred, st);
    if (e != hipSuccess) return AP_ERR_HIP;
  }
  return AP_OK;
}

int ap_predict(ap_ctx* ctx, const float* hist, int64_t n_pushed, int32_t nb_cur, float* pred, void* ws,
               void* stream) {
  if (ctx == nullptr) return AP_ERR_ARG;
  AP_REQUIRE_PTR(hist); AP_REQUIRE_PTR(pred); AP_REQUIRE_PTR(ws);
  const Shape& s = ctx->s;
  if (!ctx->have_weights) return AP_ERR_STATE;
  if (n_pushed < 0 || nb_cur < 1 || nb_cur > s.nb_cap) return AP_ERR_RANGE;
  return run_predictor(ctx, hist, n_pushed, nb_cur, nb_cur, AP_PRED_REBASE, nullptr, pred, static_cast<float*>(ws),
                       static_cast<hipStream_t>(stream));
}

int ap_predict_incremental(ap_ctx* ctx, const float* hist, int64_t n_pushed, int32_t nb_cur, int32_t nb_prev,
                           int32_t mode, float* pstate, float* pred, void* ws, void* stream) {
  if (ctx == nullptr) return AP_ERR_ARG;
  AP_REQUIRE_PTR(hist); AP_REQUIRE_PTR(pstate); AP_REQUIRE_PTR(pred); AP_REQUIRE_PTR(ws);
  const Shape& s = ctx->s;
  if (!ctx->have_weights) return AP_ERR_STATE;
  if (mode != AP_PRED_REBASE && mode != AP_PRED_ADVANCE && mode != AP_PRED_HOLD) return AP_ERR_ARG;
  if (n_pushed < 0 || nb_cur < 1 || nb_cur > s.nb_cap) return AP_ERR_RANGE;
  if (mode != AP_PRED_REBASE && (nb_prev < 1 || nb_prev > nb_cur)) return AP_ERR_RANGE;
  return run_predictor(ctx, hist, n_pushed, nb_cur, nb_prev, mode, pstate, pred, static_cast<float*>(ws),
                       static_cast<hipStream_t>(stream));
}

int ap_select_topk(ap_ctx* ctx, const float* pred, int32_t nb_cur, int32_t* idx, int32_t* cnt, void* ws,
                   void* stream) {
  if (ctx == nullptr) return AP_ERR_ARG;
  AP_REQUIRE_PTR(pred); AP_REQUIRE_PTR(idx); AP_REQUIRE_PTR(cnt); AP_REQUIRE_PTR(ws);
  const Shape& s = ctx->s;
  if (nb_cur < 1 || nb_cur > s.nb_cap) return AP_ERR_RANGE;
  hipError_t e = ap::launch_select(s, 0, s.n_inst, pred, nb_cur, idx, cnt, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? AP_OK : AP_ERR_HIP;
}

int ap_refresh_selection(ap_ctx* ctx, int32_t nb_prev, int32_t nb_cur, int32_t* idx, int32_t* cnt, void* stream) {
  if (ctx == nullptr) return AP_ERR_ARG;
  AP_REQUIRE_PTR(idx); AP_REQUIRE_PTR(cnt);
  const Shape& s = ctx->s;
  if (nb_prev < 1 || nb_prev > nb_cur || nb_cur > s.nb_cap) return AP_ERR_RANGE;
  hipError_t e = ap::launch_refresh_selection(s, nb_prev, nb_cur, idx, cnt, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? AP_OK : AP_ERR_HIP;
}

int ap_sparse_decode(ap_ctx* ctx, const void* q, const void* K, const void* V, int32_t t_cur,
                     const int32_t* idx, const int32_t* cnt, float* out, float* row, void* ws, void* stream) {
  if (ctx == nullptr) return AP_ERR_ARG;
  AP_REQUIRE_PTR(q); AP_REQUIRE_PTR(K); AP_REQUIRE_PTR(V); AP_REQUIRE_PTR(idx); AP_REQUIRE_PTR(cnt);
  AP_REQUIRE_PTR(out); AP_REQUIRE_PTR(row); AP_REQUIRE_PTR(ws);
  const Shape& s = ctx->s;
  if (t_cur < 1 || t_cur > s.t_cap) return AP_ERR_RANGE;
  hipError_t e = ap::launch_sparse_decode(s, 0, s.n_inst, q, K, V, t_cur, idx, cnt, out, row, (size_t)s.nb_cap,
                                          static_cast<float*>(ws), static_cast<hipStream_t>(stream));
  return e == hipSuccess ? AP_OK : AP_ERR_HIP;
}

int ap_sparse_decode_noalloc(ap_ctx* ctx, const void* q, const void* K, const void* V, int32_t t_cur,
                             const int32_t* idx, const int32_t* cnt, float* out, float* row, void* stream) {
  if (ctx == nullptr) return AP_ERR_ARG;
  AP_REQUIRE_PTR(q); AP_REQUIRE_PTR(K); AP_REQUIRE_PTR(V); AP_REQUIRE_PTR(idx); AP_REQUIRE_PTR(cnt);
  AP_REQUIRE_PTR(out); AP_REQUIRE_PTR(row);
  const Shape& s = ctx->s;
  if (t_cur < 1 || t_cur > s.t_cap) return AP_ERR_RANGE;
  if (ap::sparse_ws_floats(s) * sizeof(float) > AP_NOALLOC_SCRATCH_BYTES) return AP_ERR_RANGE;
  float* ws = nullptr;
  size_t bytes = 0;
  if (ap::static_scratch(&ws, &bytes) != hipSuccess) {
    (void)hipGetLastError();
    return AP_ERR_HIP;
  }
  hipError_t e = ap::launch_sparse_decode(s, 0, s.n_inst, q, K, V, t_cur, idx, cnt, out, row, (size_t)s.nb_cap, ws,
                                          static_cast<hipStream_t>(stream));
  return e == hipSuccess ? AP_OK : AP_ERR_HIP;
}

// A pointer a kernel may read: device memory, or host memory that is pinned and mapped.  Pageable host memory
// would fault the GPU, so it is refused here.  The runtime is asked on every call: an answer remembered from an
// earlier call could outlive the buffer it was given for.
static int check_device_readable(const void* p) {
  hipPointerAttribute_t a;
  if (hipPointerGetAttributes(&a, p) != hipSuccess) {
    (void)hipGetLastError();
    return AP_ERR_ARG;
  }
  const bool ok = a.type == hipMemoryTypeHost || a.type == hipMemoryTypeDevice || a.type == hipMemoryTypeManaged;
  return ok ? AP_OK : AP_ERR_ARG;
}

int ap_calibrate(ap_ctx* ctx, const void* q, const void* K, int32_t t_cur, float* row, void* ws, void* stream) {
  if (ctx == nullptr) return AP_ERR_ARG;
  AP_REQUIRE_PTR(q); AP_REQUIRE_PTR(K); AP_REQUIRE_PTR(row); AP_REQUIRE_PTR(ws);
  const Shape& s = ctx->s;
  if (t_cur < 1 || t_cur > s.t_cap) return AP_ERR_RANGE;
  if (check_device_readable(K) != AP_OK) return AP_ERR_ARG;
  hipError_t e = ap::launch_calibrate(s, q, K, t_cur, row, static_cast<float*>(ws), static_cast<hipStream_t>(stream));
  return e == hipSuccess ? AP_OK : AP_ERR_HIP;
}

int ap_update_history(ap_ctx* ctx, float* hist, int64_t n_pushed, const float* row, void* stream) {
  if (ctx == nullptr) return AP_ERR_ARG;
  AP_REQUIRE_PTR(hist); AP_REQUIRE_PTR(row);
  const Shape& s = ctx->s;
  if (n_pushed < 0) return AP_ERR_RANGE;
  hipError_t e = ap::launch_push_row(s, hist, (int)(n_pushed % s.R), row, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? AP_OK : AP_ERR_HIP;
}

int ap_step(ap_ctx* ctx, float* hist, int64_t n_pushed, const void* q, const void* K, const void* V,
            int32_t t_cur, float* out, int32_t* idx, int32_t* cnt, float* pred, float* pstate, int32_t pred_mode,
            void* ws, void* stream) {
  if (ctx == nullptr) return AP_ERR_ARG;
  AP_REQUIRE_PTR(hist); AP_REQUIRE_PTR(q); AP_REQUIRE_PTR(K); AP_REQUIRE_PTR(V); AP_REQUIRE_PTR(out);
  AP_REQUIRE_PTR(idx); AP_REQUIRE_PTR(cnt); AP_REQUIRE_PTR(pred); AP_REQUIRE_PTR(ws);
  if (pstate != nullptr && !aligned16(pstate)) return AP_ERR_ALIGN;
  const Shape& s = ctx->s;
  if (!ctx->have_weights) return AP_ERR_STATE;
  const bool reuse = (pred_mode & AP_STEP_REUSE_SELECTION) != 0;
  pred_mode &= ~AP_STEP_REUSE_SELECTION;
  if (pred_mode != AP_PRED_REBASE && pred_mode != AP_PRED_ADVANCE && pred_mode != AP_PRED_HOLD &&
      !(reuse && pred_mode == AP_PRED_SKIP))
    return AP_ERR_ARG;
  if (n_pushed < 0 || t_cur < 1 || t_cur > s.t_cap) return AP_ERR_RANGE;
  const int nb_cur = (t_cur + s.b - 1) / s.b;
  const int nb_prev = t_cur > 1 ? (t_cur - 1 + s.b - 1) / s.b : 1;   // one token is appended per step
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (pred_mode != AP_PRED_SKIP) {
    int rc = run_predictor(ctx, hist, n_pushed, nb_cur, nb_prev, pred_mode, pstate, pred, static_cast<float*>(ws), st);
    if (rc != AP_OK) return rc;
  }
  if (reuse) {
    if (nb_cur != nb_prev && ap::launch_refresh_selection(s, nb_prev, nb_cur, idx, cnt, st) != hipSuccess)
      return AP_ERR_HIP;
  } else if (ap::launch_select(s, 0, s.n_inst, pred, nb_cur, idx, cnt, st) != hipSuccess) {
    return AP_ERR_HIP;
  }
  const int slot = (int)(n_pushed % s.R);
  float* slot_row = hist + (size_t)slot * s.nb_cap;
  if (ap::launch_sparse_decode(s, 0, s.n_inst, q, K, V, t_cur, idx, cnt, out, slot_row, (size_t)s.R * s.nb_cap,
                               static_cast<float*>(ws), st) != hipSuccess)
    return AP_ERR_HIP;
  return AP_OK;
}

size_t ap_prefetch_state_bytes(const ap_ctx* ctx) {
  if (ctx == nullptr) return 0;
  return (size_t)ctx->s.n_inst * ap::prefetch_state_stride(ctx->s) * sizeof(int32_t);
}

int ap_prefetch_blocks(ap_ctx* ctx, const void* K_src, const void* V_src, int32_t t_avail, int32_t nb_cur,
                       const int32_t* idx, const int32_t* cnt, void* pool_K, void* pool_V, int32_t* block_table,
                       int32_t* state, void* stream) {
  if (ctx == nullptr) return AP_ERR_ARG;
  AP_REQUIRE_PTR(K_src); AP_REQUIRE_PTR(V_src); AP_REQUIRE_PTR(idx); AP_REQUIRE_PTR(cnt);
  AP_REQUIRE_PTR(pool_K); AP_REQUIRE_PTR(pool_V); AP_REQUIRE_PTR(block_table); AP_REQUIRE_PTR(state);
  const Shape& s = ctx->s;
  if (s.k > 256) return AP_ERR_UNSUPPORTED;
  if (nb_cur < 1 || nb_cur > s.nb_cap || t_avail < 0 || t_avail > s.t_cap) return AP_ERR_RANGE;
  if (check_device_readable(K_src) != AP_OK || check_device_readable(V_src) != AP_OK) return AP_ERR_ARG;
  hipError_t e = ap::launch_gather_blocks(s, K_src, V_src, t_avail, nb_cur, idx, cnt, pool_K, pool_V, block_table,
                                          state, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? AP_OK : AP_ERR_HIP;
}

int ap_append_kv(ap_ctx* ctx, const void* k_new, const void* v_new, int32_t t_pos, const int32_t* block_table,
                 const int32_t* state, void* pool_K, void* pool_V, void* stream) {
  if (ctx == nullptr) return AP_ERR_ARG;
  AP_REQUIRE_PTR(k_new); AP_REQUIRE_PTR(v_new); AP_REQUIRE_PTR(block_table); AP_REQUIRE_PTR(state);
  AP_REQUIRE_PTR(pool_K); AP_REQUIRE_PTR(pool_V);
  const Shape& s = ctx->s;
  if (t_pos < 0 || t_pos >= s.t_cap) return AP_ERR_RANGE;
  hipError_t e = ap::launch_append_row(s, k_new, v_new, t_pos, block_table, state, pool_K, pool_V,
                                       static_cast<hipStream_t>(stream));
  return e == hipSuccess ? AP_OK : AP_ERR_HIP;
}

static int offload_events(ap_ctx* ctx) {
  if (ctx->have_events) return AP_OK;
  if (hipEventCreateWithFlags(&ctx->ev_selected, hipEventDisableTiming) != hipSuccess) return AP_ERR_HIP;
  if (hipEventCreateWithFlags(&ctx->ev_staged, hipEventDisableTiming) != hipSuccess) {
    (void)hipEventDestroy(ctx->ev_selected);
    return AP_ERR_HIP;
  }
  ctx->have_events = true;
  return AP_OK;
}

// Predict + select for context length t_next on `cs`, then the gather of that selection on `ps`.
static int offload_select_and_fetch(ap_ctx* ctx, const float* hist, int64_t n_pushed, const void* K_src,
                                    const void* V_src, int t_next, int t_avail, int mode, int32_t* idx, int32_t* cnt,
                                    float* pred, float* pstate, void* pool_K, void* pool_V, int32_t* table,
                                    int32_t* state, float* ws, hipStream_t cs, hipStream_t ps) {
  const Shape& s = ctx->s;
  const int nb_next = (t_next + s.b - 1) / s.b;
  const int nb_prev = t_next > 1 ? (t_next - 1 + s.b - 1) / s.b : 1;
  int rc = run_predictor(ctx, hist, n_pushed, nb_next, nb_prev, mode, pstate, pred, ws, cs);
  if (rc != AP_OK) return rc;
  if (ap::launch_select(s, 0, s.n_inst, pred, nb_next, idx, cnt, cs) != hipSuccess) return AP_ERR_HIP;
  if (hipEventRecord(ctx->ev_selected, cs) != hipSuccess) return AP_ERR_HIP;
  if (hipStreamWaitEvent(ps, ctx->ev_selected, 0) != hipSuccess) return AP_ERR_HIP;
  if (ap::launch_gather_blocks(s, K_src, V_src, t_avail, nb_next, idx, cnt, pool_K, pool_V, table, state, ps) !=
      hipSuccess)
    return AP_ERR_HIP;
  if (hipEventRecord(ctx->ev_staged, ps) != hipSuccess) return AP_ERR_HIP;
  return AP_OK;
}

int ap_offload_begin(ap_ctx* ctx, const float* hist, int64_t n_pushed, const void* K_src, const void* V_src,
                     int32_t t_first, int32_t* idx, int32_t* cnt, float* pred, float* pstate, void* pool_K,
                     void* pool_V, int32_t* block_table, int32_t* state, void* ws, void* compute_stream,
                     void* copy_stream) {
  if (ctx == nullptr) return AP_ERR_ARG;
  AP_REQUIRE_PTR(hist); AP_REQUIRE_PTR(K_src); AP_REQUIRE_PTR(V_src); AP_REQUIRE_PTR(idx); AP_REQUIRE_PTR(cnt);
  AP_REQUIRE_PTR(pred); AP_REQUIRE_PTR(pstate); AP_REQUIRE_PTR(pool_K); AP_REQUIRE_PTR(pool_V);
  AP_REQUIRE_PTR(block_table); AP_REQUIRE_PTR(state); AP_REQUIRE_PTR(ws);
  const Shape& s = ctx->s;
  if (!ctx->have_weights) return AP_ERR_STATE;
  if (s.n_local < 1 || s.k > 256) return AP_ERR_UNSUPPORTED;
  if (n_pushed < 0 || t_first < 1 || t_first > s.t_cap) return AP_ERR_RANGE;
  if (check_device_readable(K_src) != AP_OK || check_device_readable(V_src) != AP_OK) return AP_ERR_ARG;
  int rc = offload_events(ctx);
  if (rc != AP_OK) return rc;
  return offload_select_and_fetch(ctx, hist, n_pushed, K_src, V_src, t_first, t_first - 1, AP_PRED_REBASE, idx, cnt, pred,
                                  pstate, pool_K, pool_V, block_table, state, static_cast<float*>(ws),
                                  static_cast<hipStream_t>(compute_stream), static_cast<hipStream_t>(copy_stream));
}

int ap_offload_step(ap_ctx* ctx, float* hist, int64_t n_pushed, const void* q, const void* k_new, const void* v_new,
                    const void* K_src, const void* V_src, int32_t t_cur, int32_t calibrate, float* out, int32_t* idx,
                    int32_t* cnt, float* pred, float* pstate, int32_t pred_mode, void* pool_K, void* pool_V,
                    int32_t* block_table, int32_t* state, float* row, void* ws, void* compute_stream,
                    void* copy_stream) {
  if (ctx == nullptr) return AP_ERR_ARG;
  AP_REQUIRE_PTR(hist); AP_REQUIRE_PTR(q); AP_REQUIRE_PTR(k_new); AP_REQUIRE_PTR(v_new); AP_REQUIRE_PTR(K_src);
  AP_REQUIRE_PTR(V_src); AP_REQUIRE_PTR(out); AP_REQUIRE_PTR(idx); AP_REQUIRE_PTR(cnt); AP_REQUIRE_PTR(pred);
  AP_REQUIRE_PTR(pstate); AP_REQUIRE_PTR(pool_K); AP_REQUIRE_PTR(pool_V); AP_REQUIRE_PTR(block_table);
  AP_REQUIRE_PTR(state); AP_REQUIRE_PTR(row); AP_REQUIRE_PTR(ws);
  const Shape& s = ctx->s;
  if (!ctx->have_weights || !ctx->have_events) return AP_ERR_STATE;      // ap_offload_begin comes first
  if (pred_mode != AP_PRED_REBASE && pred_mode != AP_PRED_ADVANCE) return AP_ERR_ARG;
  if (n_pushed < 0 || t_cur < 1 || t_cur > s.t_cap) return AP_ERR_RANGE;
  if (check_device_readable(K_src) != AP_OK || check_device_readable(V_src) != AP_OK) return AP_ERR_ARG;
  hipStream_t cs = static_cast<hipStream_t>(compute_stream), ps = static_cast<hipStream_t>(copy_stream);
  if (hipStreamWaitEvent(cs, ctx->ev_staged, 0) != hipSuccess) return AP_ERR_HIP;
  if (ap::launch_append_row(s, k_new, v_new, t_cur - 1, block_table, state, pool_K, pool_V, cs) != hipSuccess)
    return AP_ERR_HIP;
  Shape paged = s;                       // the staged pools are a paged cache of n_inst * k blocks
  paged.table = block_table;
  paged.n_phys = s.n_inst * s.k;
  float* slot_row = hist + (size_t)(n_pushed % s.R) * s.nb_cap;
  if (ap::launch_sparse_decode(paged, 0, s.n_inst, q, pool_K, pool_V, t_cur, idx, cnt, out, slot_row,
                               (size_t)s.R * s.nb_cap, static_cast<float*>(ws), cs) != hipSuccess)
    return AP_ERR_HIP;
  if (calibrate) {
    Shape flat = s;                      // the dense pass reads the full cache where it lives
    flat.table = nullptr;
    if (ap::launch_calibrate(flat, q, K_src, t_cur, row, static_cast<float*>(ws), cs) != hipSuccess) return AP_ERR_HIP;
    if (ap::launch_push_row(s, hist, (int)(n_pushed % s.R), row, cs) != hipSuccess) return AP_ERR_HIP;
  }
  if (t_cur + 1 > s.t_cap) return AP_OK; // the cache is full: no next token to prepare
  return offload_select_and_fetch(ctx, hist, n_pushed + 1, K_src, V_src, t_cur + 1, t_cur, pred_mode, idx, cnt, pred,
                                  pstate, pool_K, pool_V, block_table, state, static_cast<float*>(ws), cs, ps);
}

int ap_stream_read(const void* src, size_t bytes, void* sink, int32_t n_workgroups, void* stream) {
  AP_REQUIRE_PTR(src); AP_REQUIRE_PTR(sink);
  if (bytes < 16 || n_workgroups < 1 || n_workgroups > 65535) return AP_ERR_ARG;
  return ap::launch_stream_read(src, bytes, sink, n_workgroups, static_cast<hipStream_t>(stream)) == hipSuccess
             ? AP_OK : AP_ERR_HIP;
}

int ap_stream_copy(const void* src, size_t bytes, void* dst, int32_t n_workgroups, void* stream) {
  AP_REQUIRE_PTR(src); AP_REQUIRE_PTR(dst);
  if (bytes < 16 || n_workgroups < 1 || n_workgroups > 65535) return AP_ERR_ARG;
  return ap::launch_stream_copy(src, bytes, dst, n_workgroups, static_cast<hipStream_t>(stream)) == hipSuccess
             ? AP_OK : AP_ERR_HIP;
}

const char* ap_strerror(int code) {
  switch (code) {
    case AP_OK: return "ok";
    case AP_ERR_ARG: return "invalid argument (null pointer, bad size or inconsistent configuration)";
    case AP_ERR_ALIGN: return "device pointer is not 16-byte aligned";
    case AP_ERR_RANGE: return "t_cur, nb_cur or n_pushed outside the range the context was created for, or a "
                              "context too large for the static scratch of a no-allocation call";
    case AP_ERR_HIP: return "a HIP runtime call failed";
    case AP_ERR_UNSUPPORTED: return "shape outside the compiled kernel set";
    case AP_ERR_STATE: return "predictor weights have not been set";
    default: return "unknown error code";
  }
}

}  // extern "C"
