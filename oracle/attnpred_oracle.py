"""CPU oracle for the AttentionPredictor per-decode-step path (numpy, float64).

THIS IS TEST INFRASTRUCTURE.  It is a plain, slow statement of what the path
computes, written from the paper, and exists only so that the HIP kernels can be
checked against it.  Only the tests, the smoke check and the bench's CPU-baseline
leg may call it; the product path never does.  It shares no code, tables or
helpers with the HIP path and imports nothing from it.

Everything is float64.  Inputs that are stored as bf16/fp32 are widened exactly
by the caller before they get here.

One *instance* is one (layer, batch, KV head): `g` query heads attend one K/V
sequence.  The paper is silent on grouped-query attention; here the history, the
predictor and the selection are kept per KV head, and the block pooling window is
extended over the group (maximum over the g heads), max being the paper's pooling
operator.  With g = 1 this is exactly the paper's per-head procedure.

Pins (tests/test_oracle_*.py): brute-force loops on tiny inputs, torch's CPU
conv/softmax library routines, closed forms for zero/delta predictors, the
paper's parameter count and feature-map footprint, budget == context reproducing
dense attention, Eq. (1) special cases.
Whole multi-step trajectories have no printed values in the paper: parity unpinned
against the paper for `decode_step` chains (each of its stages is pinned).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


# --------------------------------------------------------------------------------------------
# Predictor weights
# --------------------------------------------------------------------------------------------
@dataclass
class PredictorWeights:
    """Weights of the CNN in the paper's architecture table (appendix "Implement Details"):
    Conv2d(1->c1, 3x3, pad 1) - ReLU - Conv2d(c1->c2, 3x3, pad 1) - ReLU -
    average over the time axis - Conv1d(c2->1, kernel 1).  Kernel axis 0 is time, axis 1 is block.
    """

    w1: np.ndarray   # [c1][3][3]
    b1: np.ndarray   # [c1]
    w2: np.ndarray   # [c2][c1][3][3]
    b2: np.ndarray   # [c2]
    w3: np.ndarray   # [c2]
    b3: float

    @staticmethod
    def from_blob(blob, c1: int, c2: int) -> "PredictorWeights":
        """Blob order: w1, b1, w2, b2, w3, b3 (each row-major)."""
        x = np.asarray(blob, dtype=np.float64).ravel()
        sizes = [c1 * 9, c1, c2 * c1 * 9, c2, c2, 1]
        if x.size != sum(sizes):
            raise ValueError(f"blob has {x.size} floats, expected {sum(sizes)}")
        o = np.cumsum([0] + sizes)
        return PredictorWeights(
            x[o[0]:o[1]].reshape(c1, 3, 3), x[o[1]:o[2]].copy(),
            x[o[2]:o[3]].reshape(c2, c1, 3, 3), x[o[3]:o[4]].copy(),
            x[o[4]:o[5]].copy(), float(x[o[5]]))

    def n_params(self) -> int:
        return self.w1.size + self.b1.size + self.w2.size + self.b2.size + self.w3.size + 1


# --------------------------------------------------------------------------------------------
# Algorithm 1, steps 1-3: block-wise compression and the history roll
# --------------------------------------------------------------------------------------------
def maxpool_blocks(a: np.ndarray, b: int) -> np.ndarray:
    """Algorithm 1 steps 1-2: zero-pad the score row to a multiple of b, then max over each block."""
    a = np.asarray(a, dtype=np.float64)
    nb = -(-a.size // b)
    padded = np.zeros(nb * b)
    padded[:a.size] = a
    return padded.reshape(nb, b).max(axis=1)


def history_push(hist: np.ndarray, row: np.ndarray) -> np.ndarray:
    """Algorithm 1 step 3: drop the oldest row, append the new one (index H-1 = newest).

    `hist` is [H][width]; a shorter `row` is zero-padded on the right ("Training Details":
    short rows are padded with zeros at the end).
    """
    H, width = hist.shape
    new = np.zeros(width)
    new[:row.size] = row
    return np.concatenate([hist[1:], new[None, :]], axis=0)


# --------------------------------------------------------------------------------------------
# Algorithm 1 step 4: the predictor F
# --------------------------------------------------------------------------------------------
def _conv3x3_same(x: np.ndarray, w: np.ndarray, bias: np.ndarray) -> np.ndarray:
    """Cross-correlation with zero padding 1 on both axes.
    x: [cin][R][C], w: [cout][cin][3][3] -> [cout][R][C]
    y[o][r][j] = bias[o] + sum_{i,kh,kw} w[o][i][kh][kw] * x[i][r+kh-1][j+kw-1], x = 0 outside.
    """
    cin, R, C = x.shape
    cout = w.shape[0]
    xp = np.zeros((cin, R + 2, C + 2))
    xp[:, 1:R + 1, 1:C + 1] = x
    y = np.empty((cout, R, C))
    for o in range(cout):
        acc = np.full((R, C), bias[o])
        for i in range(cin):
            for kh in range(3):
                for kw in range(3):
                    acc = acc + w[o, i, kh, kw] * xp[i, kh:kh + R, kw:kw + C]
        y[o] = acc
    return y


def predict(hist: np.ndarray, nb: int, wts: PredictorWeights) -> np.ndarray:
    """Predicted block scores for the next step from the H x nb history tile.

    Follows the architecture table layer by layer.  Zero padding is applied at each
    conv layer relative to the current tile [0,H) x [0,nb); the time average always
    divides by H (missing early rows are zero rows); the output is the raw linear
    head, no activation.
    """
    H = hist.shape[0]
    x = np.asarray(hist[:, :nb], dtype=np.float64)[None]            # [1][H][nb]
    y1 = np.maximum(_conv3x3_same(x, wts.w1[:, None], wts.b1), 0.0)   # [c1][H][nb]
    y2 = np.maximum(_conv3x3_same(y1, wts.w2, wts.b2), 0.0)           # [c2][H][nb]
    z = y2.sum(axis=1) / H                                           # [c2][nb]
    return wts.b3 + np.tensordot(wts.w3, z, axes=(0, 0))             # [nb]


# --------------------------------------------------------------------------------------------
# Algorithm 1 steps 5-6: block selection and expansion
# --------------------------------------------------------------------------------------------
def select_blocks(pred: np.ndarray, nb: int, k: int, n_sink: int, n_local: int) -> np.ndarray:
    """Top-K over block scores with the budget split of Sec. 4.1: the first n_sink and last
    n_local blocks are always kept (they are part of the budget k), the remaining k - n_sink -
    n_local go to the highest predicted scores among the blocks in between.  Equal scores go to
    the lower block index.  If the context has no more than k blocks, every block is selected.
    Returns ascending block indices.
    """
    if nb <= k:
        return np.arange(nb, dtype=np.int64)
    forced = list(range(n_sink)) + list(range(nb - n_local, nb))
    mid = list(range(n_sink, nb - n_local))
    k_mid = k - n_sink - n_local
    # full sort: score descending, then index ascending
    order = sorted(mid, key=lambda j: (-float(pred[j]), j))
    chosen = forced + order[:k_mid]
    return np.array(sorted(chosen), dtype=np.int64)


def refresh_selection(prev: np.ndarray, nb_prev: int, nb: int, k: int, n_sink: int, n_local: int) -> np.ndarray:
    """A selection made for nb_prev blocks, re-used for a context of nb >= nb_prev blocks on a step that does
    not predict (Sec. 3.3: the positions S are predicted and updated only every several steps).  The paper
    does not say what happens to the forced blocks meanwhile; the reading taken here keeps the budget split
    of Sec. 4.1 valid at every step: the predicted picks stay as they are, the local window moves with the
    context (the last n_local blocks of the current length), and a block that has dropped out of the local
    window is not kept.  If the context has no more than k blocks every block is selected; if the old
    selection was such an all-blocks one and no longer fits, its highest-numbered blocks below the local
    window are dropped.
    """
    if nb <= k:
        return np.arange(nb, dtype=np.int64)
    old_local = set(range(nb_prev - n_local, nb_prev)) if nb_prev > k else set()
    keep = sorted(int(j) for j in prev if int(j) < nb - n_local and (int(j) not in old_local or int(j) < n_sink))
    keep = keep[:k - n_local]
    return np.array(keep + list(range(nb - n_local, nb)), dtype=np.int64)


def expand_blocks(blocks: np.ndarray, b: int, t: int) -> np.ndarray:
    """Algorithm 1 step 6: block indices -> token indices {i*b .. i*b+b-1}, clipped to t tokens."""
    tok = (np.asarray(blocks, dtype=np.int64)[:, None] * b + np.arange(b)[None, :]).ravel()
    return tok[tok < t]


# --------------------------------------------------------------------------------------------
# Attention (Sec. 3.1 "Preliminary")
# --------------------------------------------------------------------------------------------
def attention_scores(q: np.ndarray, K: np.ndarray, tokens: np.ndarray) -> np.ndarray:
    """A = softmax(q K^T / sqrt(d)) restricted to `tokens`, one row per head, returned as a
    length-t vector per head with zeros at unselected positions.  q: [g][d], K: [t][d]."""
    g, d = q.shape
    t = K.shape[0]
    logits = (q @ K[tokens].T) / np.sqrt(d)                  # [g][n_sel]
    m = logits.max(axis=1, keepdims=True)
    e = np.exp(logits - m)
    p = e / e.sum(axis=1, keepdims=True)
    A = np.zeros((g, t))
    A[:, tokens] = p
    return A


def pooled_row(A: np.ndarray, b: int) -> np.ndarray:
    """Block-compressed score row of one KV head: max-pool each head's scores over blocks of b
    (Algorithm 1 steps 1-2), then max over the heads of the group."""
    return np.max(np.stack([maxpool_blocks(a, b) for a in A], axis=0), axis=0)


def sparse_attention(q, K, V, blocks, b: int, t: int):
    """Attention of the g heads over only the tokens of the selected blocks.
    Returns (out [g][d], A [g][t])."""
    tokens = expand_blocks(blocks, b, t)
    A = attention_scores(q, K[:t], tokens)
    return A @ V[:t], A


def dense_row(q, K, b: int, t: int) -> np.ndarray:
    """Distribution error calibration: the pooled row of the full (dense) attention."""
    A = attention_scores(q, K[:t], np.arange(t))
    return pooled_row(A, b)


def recovery_rate(A_dense_row: np.ndarray, tokens: np.ndarray) -> float:
    """Eq. (1): share of the dense attention mass that the selected tokens keep."""
    a = np.asarray(A_dense_row, dtype=np.float64)
    return float(a[tokens].sum() / np.abs(a).sum())


# --------------------------------------------------------------------------------------------
# One decode step of one instance
# --------------------------------------------------------------------------------------------
@dataclass
class StepResult:
    pred: np.ndarray      # [nb]   predicted block scores
    blocks: np.ndarray    # ascending selected block indices
    out: np.ndarray       # [g][d] attention output over the selected blocks
    row: np.ndarray       # [nb]   pooled score row pushed into the history
    hist: np.ndarray      # [H][width] history after the push


def decode_step(hist, q, K, V, t: int, wts: PredictorWeights, *, b: int, k: int, n_sink: int,
                n_local: int, calibrate: bool, reuse=None) -> StepResult:
    """predict -> select -> sparse attention -> pooled row (dense on a calibration step) -> push.

    `K`, `V` already hold the new token (t includes it).  On a calibration step only the row
    stored in the history comes from dense attention; the output still uses the sparse set
    ("Distribution Error Calibration").  reuse = (blocks, nb_prev) of an earlier step makes this a step
    that does not update the positions (Sec. 3.3): the selection is that one, refreshed.
    """
    nb = -(-t // b)
    pred = predict(hist, nb, wts)
    if reuse is None:
        blocks = select_blocks(pred, nb, k, n_sink, n_local)
    else:
        blocks = refresh_selection(reuse[0], reuse[1], nb, k, n_sink, n_local)
    out, A = sparse_attention(q, K, V, blocks, b, t)
    row = dense_row(q, K, b, t) if calibrate else pooled_row(A, b)
    return StepResult(pred, blocks, out, row, history_push(hist, row))
