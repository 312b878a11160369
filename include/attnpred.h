/*
 * attnpred.h - C ABI of the AttentionPredictor decode hot path for AMD MI355X (gfx950).
 *
 * The calls follow the paper's problem statement (Sec. 3.2 "Problem Formulation") and Algorithm 1
 * "Identify Critical Tokens": a history of block-max-pooled attention rows per KV head is run
 * through the small CNN predictor, the top-K blocks are selected, decode attention runs over the
 * selected blocks only and yields the next pooled row, which is pushed into the history.
 *
 * Vocabulary
 *   instance  one (layer, batch, KV head) triple; instances never interact.       n_inst
 *   g         query heads sharing the KV head (GQA group)
 *   d         head_dim
 *   b         block size (tokens pooled into one history column)
 *   H         history length in rows (decode steps)
 *   nb        ceil(t / b), blocks currently in the context;  nb_cap = t_cap / b
 *   k         budget in blocks (B / b), including n_sink leading and n_local trailing forced blocks
 *   R         ring slots of the history buffer, R = H + 1 (one spare row, see ap_hist_slots)
 *
 * Conventions
 *   - Every pointer named below as "device" is a device pointer owned by the caller, contiguous
 *     in the stated row-major shape and 16-byte aligned.  The library never frees or keeps them.
 *     (Only ap_prefetch_blocks also takes pinned host memory, and says so.)
 *   - `stream` is a hipStream_t passed as void*; all work is enqueued on it, nothing synchronises.
 *   - Calls return AP_OK or a negative error code; an error found on the host leaves all outputs
 *     untouched.  No call throws.  Only ap_create / ap_set_weights / ap_destroy allocate or free
 *     (ap_offload_begin creates two events on its first call).
 *   - The first attention call of a context (ap_sparse_decode, ap_calibrate, ap_step and the offload calls)
 *     asks the runtime once how many of its workgroups the device holds at a time; it is a host query,
 *     nothing is enqueued for it, but make that first call outside a stream capture.
 *   - Calls that use one context or one workspace are issued in stream order on one stream: the workspace
 *     (partial results, the work counter of the calibration kernel) is shared by them.
 *   - All instances share one length t_cur per call.
 *   - Inputs must be finite; NaN scores give an unspecified (but in-range, duplicate-free) selection.
 */
#ifndef ATTNPRED_H
#define ATTNPRED_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AP_OK 0
#define AP_ERR_ARG (-1)         /* null pointer, non-positive size, inconsistent config            */
#define AP_ERR_ALIGN (-2)       /* a device pointer is not 16-byte aligned                          */
#define AP_ERR_RANGE (-3)       /* t_cur / nb_cur / slot outside what the context was created for  */
#define AP_ERR_HIP (-4)         /* a HIP runtime call failed (allocation, copy, launch)             */
#define AP_ERR_UNSUPPORTED (-5) /* shape outside the compiled kernel set                            */
#define AP_ERR_STATE (-6)       /* predictor weights not set                                        */

#define AP_F32 0
#define AP_BF16 1

/* ap_config.flags */
#define AP_FLAG_PREDICTOR_FP32 1 /* evaluate the incremental predictor with fp32 FMAs.  Default for 8/8
                                    and 16/32 channels: both conv layers on MFMA with f16 operands
                                    and fp32 accumulation, on differences from the response to an
                                    all-zero history (the scores move by ~1e-4 of their variable part). */

/* Predictor evaluation modes (ap_predict_incremental, ap_step). */
#define AP_PRED_REBASE 0  /* evaluate the full H x nb tile; (re)writes pstate if one is given        */
#define AP_PRED_ADVANCE 1 /* pstate is valid for n_pushed - 1 rows: move it forward by one row       */
#define AP_PRED_HOLD 2    /* pstate is already valid for n_pushed rows: use it as it is              */
#define AP_PRED_SKIP 3    /* ap_step with AP_STEP_REUSE_SELECTION only: do not run the predictor     */
#define AP_STEP_REUSE_SELECTION 16 /* OR-ed into ap_step's pred_mode: keep the previous step's selection  */

typedef struct ap_ctx ap_ctx; /* opaque host object; owns only the device copy of the weights */

typedef struct ap_config {
  int32_t n_inst;   /* instances handled per call                                                   */
  int32_t g;        /* query heads per KV head: 1, 2, 4 or 8                                        */
  int32_t head_dim; /* 64 or 128                                                                    */
  int32_t block;    /* b: power of two, 8..64                                                       */
  int32_t hist_len; /* H: 1..256                                                                    */
  int32_t t_cap;    /* token capacity of K/V, a multiple of b                                       */
  int32_t k_blocks; /* k = B / b, n_sink + n_local <= k <= 16384; k = t_cap / b gives dense attention  */
  int32_t n_sink;   /* forced leading blocks  (Sec. 4.1: prefix tokens are part of the budget)      */
  int32_t n_local;  /* forced trailing blocks (Sec. 4.1: local tokens are part of the budget)       */
  int32_t c1, c2;   /* predictor channels; compiled pairs: (4,4) (8,8) (16,32)                      */
  int32_t kv_dtype; /* AP_F32 or AP_BF16: dtype of q, K and V                                       */
  int32_t flags;    /* 0 or a combination of AP_FLAG_*                                              */
} ap_config;

/* Validates the configuration and creates a context (host object only, no device work).
 * *out is untouched on error. */
int ap_create(const ap_config* cfg, ap_ctx** out);
int ap_destroy(ap_ctx* ctx);

/* Bytes of caller-allocated device scratch that every per-step call takes as `ws` (16-B aligned).
 * Its contents carry nothing between calls. */
size_t ap_workspace_bytes(const ap_ctx* ctx);

/* R, the number of row slots in the history ring (H + 1).  The history buffer is
 * float hist[n_inst][R][nb_cap]; it must be zero-filled before the first push (missing early rows
 * are zero rows, appendix "Training Details").  Row number n (0-based count of pushes) lives in
 * slot n % R; the spare slot keeps the row that has just left the H-row window. */
int32_t ap_hist_slots(const ap_ctx* ctx);
int32_t ap_nb_cap(const ap_ctx* ctx);

/* Predictor weights (architecture table, appendix "Implement Details"): host pointer to a flat fp32
 * blob in the order w1[c1][3][3], b1[c1], w2[c2][c1][3][3], b2[c2], w3[c2], b3 - the layout of the
 * corresponding Conv2d / Conv1d parameters, kernel axis 0 = time, axis 1 = block.  The blob is
 * copied into device memory the context owns (allocated on the first call); the call waits for the
 * copy on `stream`, so the caller may free the blob on return. */
int ap_set_weights(ap_ctx* ctx, const float* host_blob, size_t n_floats, void* stream);

/* Paged K/V cache (Sec. 2.1: the block-based sparsification also applies to paged attention).
 * After this call the K and V arguments of ap_sparse_decode, ap_calibrate and ap_step are pools
 * [n_phys_blocks][b][d] shared by all instances, and block_table[inst][nb_cap] (device int32,
 * caller-owned, must stay valid; its contents may change between calls) gives the physical block of
 * logical block j of an instance.  Entries are clamped into the pool.  History, scores and selected
 * indices stay in logical block numbers.  block_table = NULL returns to the contiguous layout. */
int ap_set_block_table(ap_ctx* ctx, const int32_t* block_table, int32_t n_phys_blocks);

/* Algorithm 1 step 4: the predictor F(A_H) on the H x nb_cur tile (zero outside it at every conv layer),
 * time average over H, raw linear head.  The scores are only ever ranked (Algorithm 1 step 5), and most of F is a
 * constant every block shares: P0, what the network answers to an all-zero history.  pred holds F - P0, so that
 * fp32 resolves the part in which blocks differ; ap_score_offset returns P0 (float64, known once the weights are
 * set; its border effects are those of a tile that is more than two blocks wide) for callers that want F itself.
 *   hist      device float [n_inst][R][nb_cap]
 *   n_pushed  rows pushed so far; the newest row is in slot (n_pushed - 1) % R
 *   pred      device float [n_inst][nb_cap]; entries [0, nb_cur) are written */
double ap_score_offset(const ap_ctx* ctx);
int ap_predict(ap_ctx* ctx, const float* hist, int64_t n_pushed, int32_t nb_cur, float* pred,
               void* ws, void* stream);

/* The same prediction, evaluated incrementally.  Both convolutions commute with a one-row time
 * shift except in the first and last two rows, and the head is linear, so the contribution of
 * rows 2..H-3 is carried in one float per column (pstate) that moves forward by subtracting the row
 * that leaves those rows and adding the one that enters; only 6 of the H second-layer rows are
 * evaluated per step.  Equal to ap_predict in real arithmetic; every ADVANCE adds two fp32
 * roundings per column to pstate, so REBASE every few hundred steps.
 *   pstate   device float [n_inst][nb_cap], owned by the caller, meaningful only to this library
 *   mode     AP_PRED_REBASE | AP_PRED_ADVANCE | AP_PRED_HOLD.  ADVANCE must be called exactly once
 *            per pushed row (it needs the row that left the window, still in the ring's spare slot)
 *   nb_prev  nb_cur of the call that last wrote pstate (<= nb_cur); columns from nb_prev - 1 on are
 *            re-evaluated in full when the tile has grown.  Ignored for REBASE.
 * With hist_len < 6 every mode evaluates the full tile. */
int ap_predict_incremental(ap_ctx* ctx, const float* hist, int64_t n_pushed, int32_t nb_cur,
                           int32_t nb_prev, int32_t mode, float* pstate, float* pred, void* ws,
                           void* stream);

/* Algorithm 1 step 5 with the budget split of Sec. 4.1: blocks [0, n_sink) and
 * [nb_cur - n_local, nb_cur) are always selected; the other k - n_sink - n_local go to the
 * highest pred among the blocks in between, equal scores to the lower index (-0 == +0).
 * If nb_cur <= k every block is selected.
 *   idx  device int32 [n_inst][k]   ascending block indices; entries beyond cnt are left alone
 *   cnt  device int32 [n_inst]      number of valid entries (min(k, nb_cur)) */
int ap_select_topk(ap_ctx* ctx, const float* pred, int32_t nb_cur, int32_t* idx, int32_t* cnt,
                   void* ws, void* stream);

/* Sec. 3.3 (last sentence of "Distribution Error Calibration"): the positions S are predicted and updated only
 * every several steps.  This carries a selection made for nb_prev blocks over to a context of nb_cur >=
 * nb_prev blocks without new scores, in place: the picks below the local window stay, the local window moves
 * to the last n_local blocks of the current context, blocks of the old local window that fell out of it are
 * dropped (sink blocks always stay), and at most k entries result.  nb_cur <= k selects every block. */
int ap_refresh_selection(ap_ctx* ctx, int32_t nb_prev, int32_t nb_cur, int32_t* idx, int32_t* cnt,
                         void* stream);

/* Block-sparse decode attention (Sec. 3.1 restricted to the tokens of the selected blocks;
 * Algorithm 1 step 6 is implicit: whole blocks are read) plus Algorithm 1 steps 1-2 as a
 * by-product.  The caller has appended the new token's K/V, t_cur counts it; tokens >= t_cur of
 * the last block are masked.
 *   q    device [n_inst][g][d]      kv dtype
 *   K,V  device [n_inst][t_cap][d]  kv dtype
 *   idx  ascending, in [0, ceil(t_cur/b)); out-of-range entries are clamped into it
 *   cnt  entries of idx that count, clamped into [0, k]; any value is allowed (the selection calls
 *        write min(k, nb_cur)); with cnt = 0 the instance's out and row are all zero
 *   out  device float [n_inst][g][d]
 *   row  device float [n_inst][nb_cap]: max over the group's heads and over the block's tokens of
 *        the sparse softmax probability for selected blocks, 0 for all others (up to nb_cap) */
int ap_sparse_decode(ap_ctx* ctx, const void* q, const void* K, const void* V, int32_t t_cur,
                     const int32_t* idx, const int32_t* cnt, float* out, float* row, void* ws,
                     void* stream);

/* ap_sparse_decode for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as ap_sparse_decode
 * without `ws`: the split partials go to a static device array of AP_NOALLOC_SCRATCH_BYTES that the library keeps
 * on every GPU it runs on (looked up once per device; nothing is allocated or freed here, nor by anything this
 * calls).  A context whose partials need more (many instances with several workgroups each) is refused with
 * AP_ERR_RANGE before anything is launched; contexts with one workgroup per instance need none.  All calls on one
 * GPU share the array, whatever their context or stream: calls that overlap on one GPU race, issue them in
 * stream order on one stream.  Nothing in the array has to start at zero (every word read was written by the same
 * call). */
#define AP_NOALLOC_SCRATCH_BYTES (4u << 20)
int ap_sparse_decode_noalloc(ap_ctx* ctx, const void* q, const void* K, const void* V, int32_t t_cur,
                             const int32_t* idx, const int32_t* cnt, float* out, float* row, void* stream);

/* Distribution error calibration (Sec. 3.3): the pooled row of the dense attention of q over all
 * t_cur tokens.  Reads K only and produces no attention output.  K may also be pinned (mapped) host
 * memory, which the kernel then reads over PCIe; pageable host memory is refused with AP_ERR_ARG.
 *   row  device float [n_inst][nb_cap]; entries >= ceil(t_cur/b) are written as 0 */
int ap_calibrate(ap_ctx* ctx, const void* q, const void* K, int32_t t_cur, float* row, void* ws,
                 void* stream);

/* Algorithm 1 step 3: push `row` as row number n_pushed (slot n_pushed % R), dropping the oldest.
 * All nb_cap columns of the slot are written. */
int ap_update_history(ap_ctx* ctx, float* hist, int64_t n_pushed, const float* row, void* stream);

/* One fused decode step: predict -> select -> sparse decode -> push, with the pooled row written
 * straight into ring slot n_pushed % R.  Equivalent to ap_predict_incremental (ap_predict if pstate
 * is NULL), ap_select_topk, ap_sparse_decode and ap_update_history in that order, with
 * nb_prev = ceil((t_cur - 1) / b): decoding appends one token per step.
 * pred, idx and cnt are outputs as in the single calls.
 * pred_mode | AP_STEP_REUSE_SELECTION: idx / cnt hold the previous step's selection and are carried over with
 * ap_refresh_selection instead of being re-made; the predictor still runs in the given mode (which keeps
 * pstate current, one ADVANCE per pushed row) unless the mode is AP_PRED_SKIP, after which the next
 * predicting step has to REBASE. */
int ap_step(ap_ctx* ctx, float* hist, int64_t n_pushed, const void* q, const void* K,
            const void* V, int32_t t_cur, float* out, int32_t* idx, int32_t* cnt, float* pred,
            float* pstate, int32_t pred_mode, void* ws, void* stream);

/* K/V cache kept outside the device ("KV Cache Cross-token Prefetching", Sec. 3.4; timeline figure of the
 * appendix): stage the blocks of one selection in a device pool of k slots per instance.  The pool works as
 * a cache: a selected block that is already staged keeps its slot; a block that is new to the selection is
 * copied from K_src / V_src into a slot whose block has left the selection.  block_table[inst][block] receives
 * the slot (inst * k + slot index) of every selected block, so that after
 * ap_set_block_table(ctx, block_table, n_inst * k) the K/V arguments of ap_sparse_decode are the pools.
 * Meant to run on a stream of its own for the NEXT token's selection while other layers compute; the caller
 * orders it against the calls that produce idx and consume the pools.
 *   K_src,V_src  [n_inst][t_cap][d] in the kv dtype: device memory, or pinned (mapped) host memory, which
 *                the kernel then reads over PCIe.  Pageable host memory is refused with AP_ERR_ARG.
 *   t_avail      tokens whose K/V exist in the source now; rows of later tokens are staged as zeros
 *                (the token of the step the selection is for is generated after the fetch: ap_append_kv)
 *   nb_cur       block count the selection was made for (idx entries are clamped into [0, nb_cur))
 *   pool_K,pool_V device [n_inst * k][b][d] kv dtype; block_table device int32 [n_inst][nb_cap]
 *   state        device int32, ap_prefetch_state_bytes(ctx) bytes, zero-filled before the first call and
 *                then only touched by these calls: which block each slot holds.  Zero-filling it again
 *                empties the cache (every selected block is then fetched).  Word 3k+1 of each instance's
 *                3k+4 words counts the blocks fetched since the state was zeroed.
 * k <= 256. */
size_t ap_prefetch_state_bytes(const ap_ctx* ctx);
int ap_prefetch_blocks(ap_ctx* ctx, const void* K_src, const void* V_src, int32_t t_avail, int32_t nb_cur,
                       const int32_t* idx, const int32_t* cnt, void* pool_K, void* pool_V,
                       int32_t* block_table, int32_t* state, void* stream);

/* Appends the new token's K/V row (token index t_pos, so t_cur = t_pos + 1 in the decode call that follows) to
 * the staged copy of block t_pos / b.  Nothing is written for an instance that has not staged that block (with
 * n_local >= 1 it always has).  The full cache itself is not updated: writing the row back to it is the
 * caller's business.
 *   k_new,v_new  device [n_inst][d] kv dtype */
int ap_append_kv(ap_ctx* ctx, const void* k_new, const void* v_new, int32_t t_pos, const int32_t* block_table,
                 const int32_t* state, void* pool_K, void* pool_V, void* stream);

/* One layer's decode step in the cross-token prefetching schedule (Sec. 3.4; timeline figure of the appendix),
 * enqueued in one call so that a model with many layers is not bound by the host's launch rate:
 *   compute_stream  wait until this context's staged blocks have arrived -> ap_append_kv -> ap_sparse_decode over
 *                   the pools (pooled row written into ring slot n_pushed % R) -> if `calibrate`: ap_calibrate
 *                   from K_src and ap_update_history over that slot -> predict (with n_pushed + 1 rows, pred_mode
 *                   = AP_PRED_ADVANCE or AP_PRED_REBASE) and select for context length t_cur + 1
 *   copy_stream     after that selection: ap_prefetch_blocks with t_avail = t_cur
 * idx / cnt hold this token's selection on entry and the next token's on return; out is this token's output.
 * ap_offload_begin makes the first selection (full-tile predictor) and stages it with t_avail = t_first - 1;
 * it must precede the first ap_offload_step.  Both streams must be distinct from each other only if overlap
 * is wanted; the context owns the two events that order them.  Nothing is prepared when t_cur = t_cap.
 * Arguments as in the single calls; the context's own block-table setting is neither used nor changed.
 * Requires n_local >= 1 (the newest block is then always staged). */
int ap_offload_begin(ap_ctx* ctx, const float* hist, int64_t n_pushed, const void* K_src, const void* V_src,
                     int32_t t_first, int32_t* idx, int32_t* cnt, float* pred, float* pstate, void* pool_K,
                     void* pool_V, int32_t* block_table, int32_t* state, void* ws, void* compute_stream,
                     void* copy_stream);
int ap_offload_step(ap_ctx* ctx, float* hist, int64_t n_pushed, const void* q, const void* k_new,
                    const void* v_new, const void* K_src, const void* V_src, int32_t t_cur, int32_t calibrate,
                    float* out, int32_t* idx, int32_t* cnt, float* pred, float* pstate, int32_t pred_mode,
                    void* pool_K, void* pool_V, int32_t* block_table, int32_t* state, float* row, void* ws,
                    void* compute_stream, void* copy_stream);

/* Measurement aids (no part of Algorithm 1): a streaming read of `bytes` bytes (multiple of 16) of
 * device memory with 16-byte non-temporal loads per lane, and a plain copy.  They give the read bandwidth the
 * machine actually reaches, quoted beside the published peak, and a kernel of known traffic against
 * which hardware byte counters are scaled.
 *   sink  device, at least 16 * n_workgroups bytes (read: one checksum word per workgroup is xor-ed in)
 *   dst   device, `bytes` bytes */
int ap_stream_read(const void* src, size_t bytes, void* sink, int32_t n_workgroups, void* stream);
int ap_stream_copy(const void* src, size_t bytes, void* dst, int32_t n_workgroups, void* stream);

const char* ap_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* ATTNPRED_H */
