// Block-sparse GQA decode attention and dense calibration for gfx950.
//
// Both kernels share the same first two phases:
//   1. logits  l[h][tok] = (q_h . K_tok) / sqrt(d) for the tokens of a list of blocks, fp32
//      accumulate, written to LDS (tokens at or beyond t_cur get -inf);
//   2. per head: M = max l, p = exp(l - M) in place, L = sum p; per (head, block) the max p.
// The sparse kernel continues with  3. acc[h][:] = sum_tok p[h][tok] * V_tok  and either finishes
// (one workgroup per instance) or leaves (M, L, acc, block maxima) for the combine kernel.
// Softmax definition: Sec. 3.1; block max-pooling of the probabilities: Algorithm 1 steps 1-2
// (softmax is monotone, so the pooled probability of a block is exp(max logit - M) / L).
//
// Memory access: a K or V row is d * sizeof(T) bytes (256 B for bf16, d = 128).  LPT = row bytes / 16
// adjacent lanes read one row with one 16-byte load each, so every load instruction of a wave covers
// 64 / LPT whole rows = 1 KiB of contiguous memory inside a block.
#pragma once

#include <type_traits>

#include "ap_internal.h"

namespace ap {
namespace {


struct bf16_t { uint16_t bits; };
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));

template <typename T> struct KvT;
template <> struct KvT<float> { static constexpr int E = 4; };
template <> struct KvT<bf16_t> { static constexpr int E = 8; };

__device__ __forceinline__ void unpack16(const uint4& w, float (&f)[4], float) {
  f[0] = __uint_as_float(w.x); f[1] = __uint_as_float(w.y);
  f[2] = __uint_as_float(w.z); f[3] = __uint_as_float(w.w);
}
__device__ __forceinline__ void unpack16(const uint4& w, float (&f)[8], bf16_t) {
  f[0] = __uint_as_float(w.x << 16); f[1] = __uint_as_float(w.x & 0xffff0000u);
  f[2] = __uint_as_float(w.y << 16); f[3] = __uint_as_float(w.y & 0xffff0000u);
  f[4] = __uint_as_float(w.z << 16); f[5] = __uint_as_float(w.z & 0xffff0000u);
  f[6] = __uint_as_float(w.w << 16); f[7] = __uint_as_float(w.w & 0xffff0000u);
}

// V rows and bf16 K rows are read once per call, a whole row per load instruction (the K rows through a staged
// tile, see qk_logits): 16-byte non-temporal loads, which stream faster than plain ones and keep the rows
// from displacing data that is re-used from cache.
template <typename T> __device__ __forceinline__ uint4 ld_stream(const T* p) {
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

template <int CTRL> __device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

// Sum over the LPT adjacent lanes that share one token; every lane of the group gets the total.
template <int LPT> __device__ __forceinline__ float lane_group_sum(float v) {
  v += dpp_move<0xB1>(v);                       // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);                       // quad_perm [2,3,0,1]
  if (LPT >= 8) v += dpp_move<0x141>(v);        // row_half_mirror: pairs the two quads of 8 lanes
  if (LPT >= 16) v += dpp_move<0x140>(v);       // row_mirror: pairs the two halves of 16 lanes
  if (LPT >= 32) v += __shfl_xor(v, 16, 64);
  return v;
}

// Reductions over the 64 lanes on DPP moves - shifts within the rows of 16 lanes, then the last lane of row 0 / 2
// combined into row 1 / 3 and the last lane of row 1 into rows 2 and 3 - so that lane 63 holds the result, which a
// scalar read hands to every lane: register moves instead of six trips through the LDS permute path.  Every lane
// must be active.  FILL is the value shifted in at a row's start and kept by rows a step does not address.
template <int CTRL, int ROW_MASK> __device__ __forceinline__ float dpp_fill(float fill, float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(fill), __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_fill<0x111, 0xF>(-INFINITY, v));     // row_shr:1
  v = fmaxf(v, dpp_fill<0x112, 0xF>(-INFINITY, v));     // row_shr:2
  v = fmaxf(v, dpp_fill<0x114, 0xF>(-INFINITY, v));     // row_shr:4
  v = fmaxf(v, dpp_fill<0x118, 0xF>(-INFINITY, v));     // row_shr:8
  v = fmaxf(v, dpp_fill<0x142, 0xA>(-INFINITY, v));     // row_bcast:15 into rows 1 and 3
  v = fmaxf(v, dpp_fill<0x143, 0xC>(-INFINITY, v));     // row_bcast:31 into rows 2 and 3
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), kWave - 1));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_fill<0x111, 0xF>(0.f, v);
  v += dpp_fill<0x112, 0xF>(0.f, v);
  v += dpp_fill<0x114, 0xF>(0.f, v);
  v += dpp_fill<0x118, 0xF>(0.f, v);
  v += dpp_fill<0x142, 0xA>(0.f, v);
  v += dpp_fill<0x143, 0xC>(0.f, v);
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), kWave - 1));
}

template <typename T, int D, int G> struct Geom {
  static constexpr int E = KvT<T>::E;           // elements per 16-byte load
  static constexpr int LPT = D / E;             // lanes per token row
  static constexpr int TPI = kWave / LPT;       // token rows per load instruction
  static constexpr int NL = kGroupTokens / TPI; // load instructions per 16-token group
  static_assert(LPT >= 8 && LPT <= 32 && G <= LPT, "unsupported geometry");
};

// Phase 1.  `block_of(jb)` gives the logical block index of list position jb (its token positions decide the
// causal mask), `phys_of(jb)` the block's place in K (the same unless a block table is in use).  s_p is [G][ld].
//
// bf16: the g x d by d x 16-token contraction runs on v_mfma_f32_16x16x32_bf16 (A = 16 K rows, B = q^T
// padded to 16 columns, fp32 accumulate); with VALU dot products plus cross-lane sums the kernel spends
// two thirds of its issue slots on arithmetic and cannot keep HBM busy.  In the operand layout lane l supplies
// token l % 16 and, the order of the contraction index being free as long as A and B agree, dims
// (l / 16) d/4 .. + d/4 - 1, eight per K-step.  D comes back as lane (head = l % 16, 4 (l / 16) + v = token), so
// lanes with head < G hold the logits.
// The K rows do not come from global memory in that layout (a row would get 64 bytes per load instruction):
// they are fetched whole - LPT adjacent lanes read one row with non-temporal loads, as V rows are - and pass
// through a wave-private LDS tile of STAGE rows from which the operand layout is read.  A plain streaming read
// of this machine is 14 % faster with non-temporal loads, but only if an instruction covers whole 128-byte lines;
// a non-temporal load of part of a line fetches the line again for the other part.
//   STAGE = 16  one tile per 16-token group (calibration, which has the LDS to spare)
//   STAGE = 8   an 8-row tile, two passes per 16 tokens through an MFMA whose other eight rows repeat the tile:
//               it fits into the region that holds the output partials later (sparse decode)
// fp32 K/V keeps the VALU form: LPT adjacent lanes share one row, 16 bytes each.
constexpr int kStageRowPad = 16;   // bytes added to a staged K row so that 16 rows spread over the LDS banks
template <int D, int ROWS = kGroupTokens, int NW = kAttnWaves> constexpr int k_stage_floats() {
  return NW * ROWS * (D * 2 + kStageRowPad) / 4;
}

template <typename T, int D, int G, int STAGE, int NW = kAttnWaves, class BlockOf, class PhysOf>
__device__ __forceinline__ void qk_logits(const T* __restrict__ q_inst, const T* __restrict__ K_inst, int b, int log2b,
                                          int t_cur, int ntok, BlockOf block_of, PhysOf phys_of, float* s_p, int ld,
                                          float* s_stage) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const float scale = rsqrtf((float)D);
  const int ngroups = (ntok + kGroupTokens - 1) / kGroupTokens;
  if constexpr (std::is_same<T, bf16_t>::value) {
    constexpr int KS = D / 32;
    const int row = lane & 15, g = lane >> 4;
    bf16x8 qb[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      uint4 w = make_uint4(0, 0, 0, 0);
      if (row < G) w = *reinterpret_cast<const uint4*>(q_inst + (size_t)row * D + g * (D / 4) + s * 8);
      qb[s] = __builtin_bit_cast(bf16x8, w);
    }
    {
      static_assert(STAGE == 8 || STAGE == 16, "bf16 K rows go through a staged tile of 8 or 16 rows");
      constexpr int ROWS = STAGE;                        // tokens per pass
      constexpr int NPRE = 2;                            // passes of a wave in flight (3, 4 and 6 measured the same)
      constexpr int LPT = D / 8, TPI = kWave / LPT, NLK = ROWS / TPI, RS = D * 2 + kStageRowPad;
      static_assert(NLK >= 1, "a pass is at least one load instruction");
      char* stage = reinterpret_cast<char*>(s_stage) + wave * ROWS * RS;
      const int npass = (ntok + ROWS - 1) / ROWS;
      auto load_pass = [&](int ps, uint4 (&v)[NLK]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NLK; ++i) {
          const int tau = ps * ROWS + i * TPI + lane / LPT;
          v[i] = make_uint4(0, 0, 0, 0);
          if (tau < ntok) {
            const int ptok = phys_of(tau >> log2b) * b + (tau & (b - 1));
            v[i] = ld_stream(K_inst + (size_t)ptok * D + (lane % LPT) * 8);
          }
        }
      };
      // One pass: stage the fetched rows, refill the registers with pass `refill` (NPRE passes of this wave ahead),
      // contract, store the logits.
      auto do_pass = [&](int ps, uint4 (&v)[NLK], int refill) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NLK; ++i)
          *reinterpret_cast<uint4*>(stage + (i * TPI + lane / LPT) * RS + (lane % LPT) * 16) = v[i];
        asm volatile("" ::: "memory");                   // a wave's LDS accesses stay in order; so must the compiler
        if (refill < npass) load_pass(refill, v);
        float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KS; ++s) {
          const uint4 kw = *reinterpret_cast<const uint4*>(stage + (row & (ROWS - 1)) * RS + (g * (D / 4) + s * 8) * 2);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kw), qb[s], acc, 0, 0, 0);
        }
        asm volatile("" ::: "memory");                   // the next pass overwrites the tile read above
        // lane (head = row, tokens 4 g .. 4 g + 3 of the pass); with 8 rows only g < 2 holds tokens
        const int tau0 = ps * ROWS + 4 * g;
        if (row < G && 4 * g < ROWS && tau0 < ntok) {
          const int gtok0 = block_of(tau0 >> log2b) * b + (tau0 & (b - 1));
          float4 o;
          o.x = gtok0 + 0 < t_cur ? acc[0] * scale : -INFINITY;
          o.y = gtok0 + 1 < t_cur ? acc[1] * scale : -INFINITY;
          o.z = gtok0 + 2 < t_cur ? acc[2] * scale : -INFINITY;
          o.w = gtok0 + 3 < t_cur ? acc[3] * scale : -INFINITY;
          *reinterpret_cast<float4*>(s_p + row * ld + tau0) = o;
        }
      };
      // Rows of this wave's next NPRE passes wait in registers.
      uint4 v[NPRE][NLK];
#pragma unroll
      for (int i = 0; i < NPRE; ++i)
        if (wave + i * NW < npass) load_pass(wave + i * NW, v[i]);
      for (int ps = wave; ps < npass; ps += NPRE * NW) {
#pragma unroll
        for (int i = 0; i < NPRE; ++i)
          if (ps + i * NW < npass) do_pass(ps + i * NW, v[i], ps + (i + NPRE) * NW);
      }
    }
  } else {
    using Ge = Geom<T, D, G>;
    constexpr int E = Ge::E, LPT = Ge::LPT, TPI = Ge::TPI, NL = Ge::NL;
    const int dpart = lane % LPT;
    const int tslot = lane / LPT;
    float qr[G][E];
#pragma unroll
    for (int h = 0; h < G; ++h) {
      static_assert(E * sizeof(T) == 16, "one 16-byte load per lane");
      uint4 w = *reinterpret_cast<const uint4*>(q_inst + (size_t)h * D + dpart * E);
      float f[E];
      unpack16(w, f, T{});
#pragma unroll
      for (int e = 0; e < E; ++e) qr[h][e] = f[e] * scale;
    }
    for (int grp = wave; grp < ngroups; grp += NW) {
      uint4 kw[NL];
      int gtok[NL];
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        const int tau = grp * kGroupTokens + i * TPI + tslot;
        kw[i] = make_uint4(0, 0, 0, 0);
        gtok[i] = -1;
        if (tau < ntok) {
          gtok[i] = block_of(tau >> log2b) * b + (tau & (b - 1));
          const int ptok = phys_of(tau >> log2b) * b + (tau & (b - 1));
          kw[i] = *reinterpret_cast<const uint4*>(K_inst + (size_t)ptok * D + dpart * E);
        }
      }
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        const int tau = grp * kGroupTokens + i * TPI + tslot;
        float kf[E];
        unpack16(kw[i], kf, T{});
        float mine = 0.f;
#pragma unroll
        for (int h = 0; h < G; ++h) {
          float sdot = 0.f;
#pragma unroll
          for (int e = 0; e < E; ++e) sdot = fmaf(qr[h][e], kf[e], sdot);
          sdot = lane_group_sum<LPT>(sdot);
          if (dpart == h) mine = sdot;
        }
        if (dpart < G && tau < ntok) s_p[dpart * ld + tau] = (gtok[i] < t_cur) ? mine : -INFINITY;
      }
    }
  }
}

// Phase 2.  Leaves p in s_p, (M, L) in s_m / s_l, per (head, block) max p in s_bmp[h * bmp_ld + jb].
// One wave per head; a lane handles four consecutive tokens per 16-byte LDS access (ntok and ld are multiples
// of the block size, hence of 4), so the b / 4 adjacent lanes of a block find its maximum with DPP moves.
// With s_alpha the statistics run on over several calls (pieces of one list): M is the maximum so far, p is
// relative to it, L is carried over as L * alpha + sum with alpha = exp(M_before - M), which s_alpha[h]
// receives for the caller to rescale what it has accumulated (0 on the first piece, M_before = -inf).
template <int G, int NW = kAttnWaves>
__device__ __forceinline__ void softmax_stats(float* s_p, int ld, int ntok, int b, int bmp_ld, float* s_m, float* s_l,
                                     float* s_bmp, float* s_alpha = nullptr) {
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x / kWave;
  const int nquad = ntok >> 2;
  const int lanes_per_blk = b >> 2;                      // 2, 4, 8 or 16
  const int blk_shift = __ffs(lanes_per_blk) - 1;
  // Heads wave, wave + NW, ... of this wave are worked on together: their loads, reductions and exponentials
  // are independent chains that hide each other's latency.
  constexpr int HPW = (G + NW - 1) / NW;
  float m[HPW], m_old[HPW], l_old[HPW], sum[HPW];
#pragma unroll
  for (int j = 0; j < HPW; ++j) { m[j] = -INFINITY; m_old[j] = -INFINITY; l_old[j] = 0.f; sum[j] = 0.f; }
  for (int qd = lane; qd < nquad; qd += kWave) {
#pragma unroll
    for (int j = 0; j < HPW; ++j) {
      const int h = wave + j * NW;
      if (h < G) {
        const float4 v = reinterpret_cast<const float4*>(s_p + (size_t)h * ld)[qd];
        m[j] = fmaxf(m[j], fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w)));
      }
    }
  }
#pragma unroll
  for (int j = 0; j < HPW; ++j) m[j] = wave_max(m[j]);   // (independent chains: the compiler interleaves them)
  if (s_alpha != nullptr) {
#pragma unroll
    for (int j = 0; j < HPW; ++j) {
      const int h = wave + j * NW;
      if (h < G) {
        m_old[j] = s_m[h];
        l_old[j] = s_l[h];
        m[j] = fmaxf(m[j], m_old[j]);
      }
    }
  }
  for (int q0 = 0; q0 < nquad; q0 += kWave) {            // uniform trip count: the DPP moves need every lane
    const int qd = q0 + lane;
#pragma unroll
    for (int j = 0; j < HPW; ++j) {
      const int h = wave + j * NW;
      if (h >= G) continue;                              // (wave-uniform)
      float4* prow = reinterpret_cast<float4*>(s_p + (size_t)h * ld);
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (qd < nquad) {
        v = prow[qd];
        v.x = __expf(v.x - m[j]); v.y = __expf(v.y - m[j]); v.z = __expf(v.z - m[j]); v.w = __expf(v.w - m[j]);
        prow[qd] = v;
      }
      sum[j] += (v.x + v.y) + (v.z + v.w);
      float bm = fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w));
      bm = fmaxf(bm, dpp_move<0xB1>(bm));                                   // quad_perm [1,0,3,2]
      if (lanes_per_blk >= 4) bm = fmaxf(bm, dpp_move<0x4E>(bm));           // quad_perm [2,3,0,1]
      if (lanes_per_blk >= 8) bm = fmaxf(bm, dpp_move<0x141>(bm));          // row_half_mirror
      if (lanes_per_blk >= 16) bm = fmaxf(bm, dpp_move<0x140>(bm));         // row_mirror
      if (qd < nquad && (lane & (lanes_per_blk - 1)) == 0) s_bmp[h * bmp_ld + (qd >> blk_shift)] = bm;
    }
  }
#pragma unroll
  for (int j = 0; j < HPW; ++j) sum[j] = wave_sum(sum[j]);
  if (lane == 0) {
#pragma unroll
    for (int j = 0; j < HPW; ++j) {
      const int h = wave + j * NW;
      if (h < G) {
        const float alpha = (m_old[j] == -INFINITY) ? 0.f : __expf(m_old[j] - m[j]);
        s_m[h] = m[j];
        s_l[h] = l_old[j] * alpha + sum[j];
        if (s_alpha != nullptr) s_alpha[h] = alpha;
      }
    }
  }
  __syncthreads();
}

constexpr int kSparseStage = 8;
// Floats of the region shared by the staged K tile (phase 1) and the per-wave output partials (after phase 3).
template <int D, int G, int NW> constexpr int sparse_acc_floats() {
  return NW * G * D > k_stage_floats<D, kSparseStage, NW>() ? NW * G * D : k_stage_floats<D, kSparseStage, NW>();
}

struct SparseArgs {
  const void* q; const void* K; const void* V;
  const int32_t* idx; const int32_t* cnt;
  float* out; float* row; size_t row_stride;
  float* part_ml; float* part_acc; float* part_bmp;
  int t_cap, nb_cap, k, b, log2b, t_cur, nb_cur, n_split, blk_per_split, inst0;
  const int32_t* table;           // block table [n_inst][nb_cap] of a paged cache, or null
  int n_phys;                     // blocks in the pool (table entries are clamped into it)
  int piece_blocks;               // list positions whose probabilities are in LDS at a time
};

// Sparse decode of instance `inst`, split `split`, by one workgroup of NW waves.
// The list is worked off in pieces of a.piece_blocks positions - logits, softmax statistics, acc += p * V per
// piece, the statistics running on and acc rescaled when the maximum moves - so that the LDS holds the
// probabilities of one piece only.  PIECED = false: a.piece_blocks covers the list, one piece, no rescaling
// (and the accumulators are not live during phase 1).
// smem: sparse_lds_floats(...) floats of LDS, 16-byte aligned.
template <typename T, int D, int G, int NW, bool PIECED>
__device__ __forceinline__ void sparse_decode_body(const SparseArgs& a, int inst, int split, float* smem) {
  using Ge = Geom<T, D, G>;
  constexpr int E = Ge::E, LPT = Ge::LPT, NL = Ge::NL, NT = NW * kWave;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
  const int dpart = lane % LPT, tslot = lane / LPT;

  const int cnt = min(max(a.cnt[inst], 0), a.k);
  // With one workgroup per instance the whole list is local; otherwise this split's slice.
  const int j0 = (a.n_split == 1) ? 0 : min(cnt, split * a.blk_per_split);
  const int j1 = (a.n_split == 1) ? cnt : min(cnt, j0 + a.blk_per_split);
  const int nblk = j1 - j0;
  const int nblk_cap = (a.n_split == 1) ? a.k : a.blk_per_split;
  const int pb = PIECED ? min(a.piece_blocks, nblk_cap) : nblk_cap;   // positions per piece
  const int n_pieces_cap = (nblk_cap + pb - 1) / pb;
  const int ld = pb * a.b;

  float* s_p = smem;                                   // [G][ld]
  float* s_acc = s_p + G * ld;                         // [waves][G][D]
  float* s_bmp = s_acc + sparse_acc_floats<D, G, NW>();   // [G][nblk_cap]
  float* s_m = s_bmp + G * nblk_cap;                   // [G] running maximum
  float* s_l = s_m + G;                                // [G] running sum
  float* s_alpha = s_l + G;                            // [G] rescaling factor of the piece at hand
  float* s_mpiece = s_alpha + G;                       // [n_pieces_cap][G] maximum the piece's p are relative to
  int* s_idx = reinterpret_cast<int*>(s_mpiece + n_pieces_cap * G);   // [nblk_cap] logical block of each position
  int* s_phys = s_idx + nblk_cap;                      // [nblk_cap] its place in K / V
  // For the pooled row, written whole by the workgroup that has the whole list: one bit per block (is it
  // listed) and, per 32-block word, the number of listed blocks before it, so that a column finds its list
  // position without a search.
  uint32_t* s_listed = reinterpret_cast<uint32_t*>(s_phys + nblk_cap);   // [ceil(nb_cap / 32)]
  int* s_rank = reinterpret_cast<int*>(s_listed) + (a.nb_cap + 31) / 32; // [ceil(nb_cap / 32)]
  const int nwords = (a.nb_cap + 31) / 32;
  const bool whole_row = a.n_split == 1;

  if (whole_row) {
    for (int w = threadIdx.x; w < nwords; w += NT) s_listed[w] = 0u;
  }
  if (threadIdx.x < G) { s_m[threadIdx.x] = -INFINITY; s_l[threadIdx.x] = 0.f; }
  __syncthreads();
  for (int j = threadIdx.x; j < nblk; j += NT) {
    const int blk = min(max(a.idx[(size_t)inst * a.k + j0 + j], 0), a.nb_cur - 1);
    s_idx[j] = blk;
    s_phys[j] = a.table ? min(max(a.table[(size_t)inst * a.nb_cap + blk], 0), a.n_phys - 1) : blk;
    if (whole_row) atomicOr(&s_listed[blk >> 5], 1u << (blk & 31));
  }
  __syncthreads();
  if (whole_row && wave == NW - 1) {                   // exclusive prefix sum of the words' bit counts
    const int per_lane = (nwords + kWave - 1) / kWave;
    const int w0 = lane * per_lane;
    int mine = 0;
    for (int i = 0; i < per_lane; ++i)
      if (w0 + i < nwords) mine += __popc(s_listed[w0 + i]);
    int incl = mine;                                   // inclusive prefix sum over the lanes, on DPP moves
    incl += __builtin_amdgcn_update_dpp(0, incl, 0x111, 0xF, 0xF, true);   // row_shr:1
    incl += __builtin_amdgcn_update_dpp(0, incl, 0x112, 0xF, 0xF, true);   // row_shr:2
    incl += __builtin_amdgcn_update_dpp(0, incl, 0x114, 0xF, 0xF, true);   // row_shr:4
    incl += __builtin_amdgcn_update_dpp(0, incl, 0x118, 0xF, 0xF, true);   // row_shr:8
    incl += __builtin_amdgcn_update_dpp(0, incl, 0x142, 0xA, 0xF, true);   // row_bcast:15 into rows 1 and 3
    incl += __builtin_amdgcn_update_dpp(0, incl, 0x143, 0xC, 0xF, true);   // row_bcast:31 into rows 2 and 3
    int run = incl - mine;
    for (int i = 0; i < per_lane; ++i)
      if (w0 + i < nwords) { s_rank[w0 + i] = run; run += __popc(s_listed[w0 + i]); }
  }                                                    // (read after the barriers that follow)

  // Contiguous cache: [n_inst][t_cap][d].  Paged cache: one pool [n_phys][b][d] for all instances.
  const size_t kv_off = a.table ? 0 : (size_t)inst * a.t_cap * D;
  const T* q_inst = static_cast<const T*>(a.q) + (size_t)inst * G * D;
  const T* K_inst = static_cast<const T*>(a.K) + kv_off;
  const T* V_inst = static_cast<const T*>(a.V) + kv_off;

  float acc[G][E];
#pragma unroll
  for (int h = 0; h < G; ++h)
#pragma unroll
    for (int e = 0; e < E; ++e) acc[h][e] = 0.f;

  int p0 = 0, piece = 0;
  if (nblk > 0) do {
    const int nb_p = min(pb, nblk - p0);
    const int ntok = nb_p * a.b;
    // (the staged K tile lives where the waves' output partials go after the last piece)
    qk_logits<T, D, G, kSparseStage, NW>(q_inst, K_inst, a.b, a.log2b, a.t_cur, ntok,
                                         [&](int jb) { return s_idx[p0 + jb]; },
                                         [&](int jb) { return s_phys[p0 + jb]; }, s_p, ld, s_acc);
    // The V rows of this wave's first 16-token group do not depend on the probabilities: they are requested before
    // the softmax pass and arrive while it runs - where the registers allow it.  The pieced forms with g = 4 are at
    // their 128 VGPRs already and would spill (0.201 vs 0.183 ms at cfg2); with g <= 2 they gain 1.5 % at cfg4, and
    // the four-wave form, which has registers to spare, 2 % at cfg3.
    constexpr bool kEarlyV = (PIECED && G <= 2) || !PIECED;
    const int ngroups = (ntok + kGroupTokens - 1) / kGroupTokens;
    uint4 vw[NL];
    auto load_v = [&](int grp) __attribute__((always_inline)) {
      const int tau0 = grp * kGroupTokens + tslot * NL;
#pragma unroll
      for (int i = 0; i < NL; ++i) vw[i] = make_uint4(0, 0, 0, 0);
      if (tau0 < ntok) {
        // Tokens at or beyond t_cur (the tail of the newest block) carry probability 0, but their V rows may hold
        // anything, NaN included, and 0 * NaN is NaN: such a token reads the block's last real row instead.
        const int jb = p0 + (tau0 >> a.log2b), off = tau0 & (a.b - 1);
        const int last = min(a.t_cur - 1 - s_idx[jb] * a.b, a.b - 1);   // >= 0: a listed block starts before t_cur
        const int prow0 = s_phys[jb] * a.b;
#pragma unroll
        for (int i = 0; i < NL; ++i) vw[i] = ld_stream(V_inst + (size_t)(prow0 + min(off + i, last)) * D + dpart * E);
      }
    };
    if (kEarlyV && wave < ngroups) load_v(wave);
    __syncthreads();
    softmax_stats<G, NW>(s_p, ld, ntok, a.b, nblk, s_m, s_l, s_bmp + p0, s_alpha);
    if (threadIdx.x < G) s_mpiece[piece * G + threadIdx.x] = s_m[threadIdx.x];
    if (PIECED && piece > 0) {                         // the maximum may have moved: bring acc along
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const float al = s_alpha[h];
#pragma unroll
        for (int e = 0; e < E; ++e) acc[h][e] *= al;
      }
    }

    // Phase 3: acc += p * V.  A lane group takes NL consecutive tokens of a 16-token group (they lie in one
    // block, so one table lookup places them), load instruction i covers the i-th row of each of the TPI lane
    // groups - whole 256-byte rows - and the NL probabilities of a head come in one LDS access.
    static_assert(NL == 2 || NL == 4 || NL == 8, "probabilities are fetched as 8- or 16-byte vectors");
    for (int grp = wave; grp < ngroups; grp += NW) {
      const int tau0 = grp * kGroupTokens + tslot * NL;   // ntok is a multiple of 8 >= NL: all NL tokens or none
      const bool live = tau0 < ntok;
      if (!kEarlyV || grp != wave) load_v(grp);
      float pw[G][NL];
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const float* src = s_p + h * ld + tau0;
        if constexpr (NL == 2) {
          const float2 t = *reinterpret_cast<const float2*>(src);
          pw[h][0] = t.x; pw[h][1] = t.y;
        } else {
#pragma unroll
          for (int c = 0; c < NL / 4; ++c) {
            const float4 t = *reinterpret_cast<const float4*>(src + 4 * c);
            pw[h][4 * c] = t.x; pw[h][4 * c + 1] = t.y; pw[h][4 * c + 2] = t.z; pw[h][4 * c + 3] = t.w;
          }
        }
      }
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        float vf[E];
        unpack16(vw[i], vf, T{});
#pragma unroll
        for (int h = 0; h < G; ++h) {
          const float p = live ? pw[h][i] : 0.f;
#pragma unroll
          for (int e = 0; e < E; ++e) acc[h][e] = fmaf(p, vf[e], acc[h][e]);
        }
      }
    }
    __syncthreads();                                   // the next piece, or the partials, overwrite what was read
    p0 += pb;
    ++piece;
  } while (PIECED && p0 < nblk);

  // Block maxima of earlier pieces are relative to the maximum of their time: bring them to the final one.
  if (PIECED && nblk > pb) {
    for (int pair = threadIdx.x; pair < G * nblk; pair += NT) {
      const int h = pair / nblk, jb = pair - h * nblk;
      s_bmp[pair] *= __expf(s_mpiece[(jb / pb) * G + h] - s_m[h]);
    }
  }

  // Sum the token slots of a wave (lanes that hold the same dims), then the waves through LDS.
#pragma unroll
  for (int h = 0; h < G; ++h)
#pragma unroll
    for (int e = 0; e < E; ++e) {
      float v = acc[h][e];
#pragma unroll
      for (int o = LPT; o < kWave; o <<= 1) v += __shfl_xor(v, o, 64);
      acc[h][e] = v;
    }
  if (tslot == 0) {
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int e = 0; e < E; ++e) s_acc[(wave * G + h) * D + dpart * E + e] = acc[h][e];
  }
  __syncthreads();

  if (a.n_split == 1) {
    for (int o = threadIdx.x; o < G * D; o += NT) {
      float v = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) v += s_acc[w * G * D + o];
      const float L = s_l[o / D];
      a.out[(size_t)inst * G * D + o] = L > 0.f ? v / L : 0.f;      // an empty list gives a zero output
    }
    // Pooled row: column j of a listed block gets the largest block maximum over the heads, the rest zero.
    float* row = a.row + (size_t)inst * a.row_stride;
    for (int j = threadIdx.x; j < a.nb_cap; j += NT) {
      const uint32_t word = s_listed[j >> 5];
      float mx = 0.f;
      if ((word >> (j & 31)) & 1u) {
        const int pos = min(s_rank[j >> 5] + __popc(word & ((1u << (j & 31)) - 1u)), nblk - 1);
#pragma unroll
        for (int h = 0; h < G; ++h) mx = fmaxf(mx, s_bmp[h * nblk + pos] / s_l[h]);
      }
      row[j] = mx;
    }
  } else {
    const size_t ps = (size_t)inst * a.n_split + split;
    for (int o = threadIdx.x; o < G * D; o += NT) {
      float v = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) v += s_acc[w * G * D + o];
      a.part_acc[ps * G * D + o] = v;
    }
    if (threadIdx.x < G) {
      a.part_ml[(ps * G + threadIdx.x) * 2 + 0] = s_m[threadIdx.x];
      a.part_ml[(ps * G + threadIdx.x) * 2 + 1] = s_l[threadIdx.x];
    }
    for (int pair = threadIdx.x; pair < G * nblk; pair += NT) {
      const int h = pair / nblk, jb = pair - h * nblk;
      a.part_bmp[((size_t)inst * G + h) * a.k + j0 + jb] = s_bmp[pair];
    }
  }
}


// LDS floats sparse_decode_body needs for a list of up to nblk_cap blocks of b tokens out of nb_cap, worked off
// in pieces of piece_blocks.
template <int D, int G, int NW> inline size_t sparse_lds_floats(int nblk_cap, int piece_blocks, int b, int nb_cap) {
  const int pb = piece_blocks < nblk_cap ? piece_blocks : nblk_cap;
  const int n_pieces = (nblk_cap + pb - 1) / pb;
  return (size_t)G * pb * b + sparse_acc_floats<D, G, NW>() + (size_t)G * nblk_cap + 3 * G + (size_t)n_pieces * G +
         2 * nblk_cap + 2 * (size_t)((nb_cap + 31) / 32);
}

}  // namespace
}  // namespace ap
