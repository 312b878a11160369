"""Pins for the oracle's selection, attention, pooling, calibration, history and Eq. (1)."""
import math

import numpy as np
import pytest
import torch

from oracle import attnpred_oracle as orc


# ----------------------------------------------------------------------------- top-k selection
def _brute_select(pred, nb, k, n_sink, n_local):
    """Repeatedly take the largest remaining score, scanning left to right (first maximum wins)."""
    if nb <= k:
        return list(range(nb))
    chosen = set(range(n_sink)) | set(range(nb - n_local, nb))
    for _ in range(k - n_sink - n_local):
        best = None
        for j in range(n_sink, nb - n_local):
            if j in chosen:
                continue
            if best is None or pred[j] > pred[best]:
                best = j
        chosen.add(best)
    return sorted(chosen)


@pytest.mark.parametrize("seed", range(6))
def test_select_matches_brute_force_with_heavy_ties(seed):
    rng = np.random.default_rng(seed)
    nb = int(rng.integers(20, 200))
    k = int(rng.integers(8, 20))
    n_sink, n_local = int(rng.integers(0, 4)), int(rng.integers(0, 4))
    pred = rng.integers(0, 5, size=nb).astype(np.float64) * 0.25 - 0.5   # few distinct values
    got = orc.select_blocks(pred, nb, k, n_sink, n_local)
    assert got.tolist() == _brute_select(pred, nb, k, n_sink, n_local)
    assert len(got) == k and np.all(np.diff(got) > 0)
    assert set(range(n_sink)) <= set(got.tolist())
    assert set(range(nb - n_local, nb)) <= set(got.tolist())


def test_select_all_equal_takes_lowest_indices():
    got = orc.select_blocks(np.zeros(50), 50, 10, 2, 3)
    assert got.tolist() == [0, 1, 2, 3, 4, 5, 6, 47, 48, 49]


def test_select_small_context_takes_everything():
    assert orc.select_blocks(np.arange(7.0), 7, 16, 1, 2).tolist() == list(range(7))
    assert orc.select_blocks(np.arange(16.0), 16, 16, 1, 2).tolist() == list(range(16))


def test_select_agrees_with_library_sort_on_distinct_values():
    rng = np.random.default_rng(11)
    nb, k, ns, nl = 300, 32, 4, 4
    pred = rng.standard_normal(nb)
    mid = np.arange(ns, nb - nl)
    top = mid[np.argsort(-pred[mid], kind="stable")[:k - ns - nl]]
    exp = sorted(list(range(ns)) + top.tolist() + list(range(nb - nl, nb)))
    assert orc.select_blocks(pred, nb, k, ns, nl).tolist() == exp


def test_expand_blocks():
    assert orc.expand_blocks(np.array([0, 2]), 4, 100).tolist() == [0, 1, 2, 3, 8, 9, 10, 11]
    assert orc.expand_blocks(np.array([1, 2]), 4, 10).tolist() == [4, 5, 6, 7, 8, 9]    # clipped at t


# ----------------------------------------------------------------------------- attention
def _brute_softmax_attention(q, K, V, tokens):
    """Scalar loops: Sec. 3.1's definition restricted to `tokens`."""
    g, d = q.shape
    out = np.zeros((g, d))
    probs = []
    for h in range(g):
        logit = [sum(q[h][x] * K[i][x] for x in range(d)) / math.sqrt(d) for i in tokens]
        den = sum(math.exp(v) for v in logit)
        p = [math.exp(v) / den for v in logit]
        probs.append(p)
        for pi, i in zip(p, tokens):
            for x in range(d):
                out[h][x] += pi * V[i][x]
    return out, probs


def test_sparse_attention_matches_scalar_brute_force():
    rng = np.random.default_rng(0)
    g, d, t, b = 2, 8, 37, 4
    q, K, V = rng.standard_normal((g, d)), rng.standard_normal((t, d)), rng.standard_normal((t, d))
    blocks = np.array([0, 3, 9])           # block 9 is the partial last block (tokens 36)
    out, A = orc.sparse_attention(q, K, V, blocks, b, t)
    tokens = [0, 1, 2, 3, 12, 13, 14, 15, 36]
    ref_out, ref_p = _brute_softmax_attention(q, K, V, tokens)
    np.testing.assert_allclose(out, ref_out, rtol=1e-12, atol=1e-14)
    for h in range(g):
        np.testing.assert_allclose(A[h][tokens], ref_p[h], rtol=1e-12)
        assert A[h].sum() == pytest.approx(1.0, abs=1e-14)
        mask = np.ones(t, bool)
        mask[tokens] = False
        assert np.all(A[h][mask] == 0.0)


def test_full_budget_reproduces_dense_attention_library():
    """Budget equal to the context: the sparse path is dense softmax attention (torch library)."""
    rng = np.random.default_rng(1)
    g, d, t, b = 4, 16, 203, 16
    q, K, V = rng.standard_normal((g, d)), rng.standard_normal((t, d)), rng.standard_normal((t, d))
    nb = -(-t // b)
    blocks = orc.select_blocks(np.zeros(nb), nb, nb, 1, 2)
    out, A = orc.sparse_attention(q, K, V, blocks, b, t)
    p = torch.softmax(torch.from_numpy(q) @ torch.from_numpy(K).T / math.sqrt(d), dim=-1)
    np.testing.assert_allclose(A, p.numpy(), rtol=1e-12, atol=1e-16)
    np.testing.assert_allclose(out, (p @ torch.from_numpy(V)).numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(A.sum(axis=1), np.ones(g), atol=1e-14)


def test_block_order_does_not_matter_and_group_replication():
    rng = np.random.default_rng(2)
    d, t, b = 8, 64, 8
    q1 = rng.standard_normal((1, d))
    K, V = rng.standard_normal((t, d)), rng.standard_normal((t, d))
    o1, A1 = orc.sparse_attention(q1, K, V, np.array([0, 2, 5, 7]), b, t)
    o2, _ = orc.sparse_attention(q1, K, V, np.array([7, 0, 5, 2]), b, t)
    np.testing.assert_allclose(o1, o2, rtol=1e-13)
    o4, A4 = orc.sparse_attention(np.repeat(q1, 4, axis=0), K, V, np.array([0, 2, 5, 7]), b, t)
    for h in range(4):
        np.testing.assert_allclose(o4[h], o1[0], rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(orc.pooled_row(A4, b), orc.pooled_row(A1, b), rtol=1e-13)


# ----------------------------------------------------------------------------- pooling / calibration
def test_maxpool_zero_pads_the_tail():
    a = np.array([0.1, 0.4, 0.2, 0.05, 0.25])
    assert orc.maxpool_blocks(a, 2).tolist() == [0.4, 0.2, 0.25]
    assert orc.maxpool_blocks(a, 4).tolist() == [0.4, 0.25]
    # library cross-check: torch max_pool1d on the zero-padded row
    r = np.random.default_rng(3).random(45)
    pad = np.concatenate([r, np.zeros(3)])
    ref = torch.nn.functional.max_pool1d(torch.from_numpy(pad)[None, None], 16)[0, 0].numpy()
    np.testing.assert_array_equal(orc.maxpool_blocks(r, 16), ref)


def test_pooled_row_equals_exp_of_block_max_logit():
    """Softmax is monotone, so the pooled score is exp(max logit - M) / L (used by the kernels)."""
    rng = np.random.default_rng(4)
    g, d, t, b = 3, 8, 50, 4
    q, K, V = rng.standard_normal((g, d)), rng.standard_normal((t, d)), rng.standard_normal((t, d))
    blocks = np.array([0, 1, 6, 12])
    _, A = orc.sparse_attention(q, K, V, blocks, b, t)
    row = orc.pooled_row(A, b)
    logits = q @ K.T / math.sqrt(d)
    tok = orc.expand_blocks(blocks, b, t)
    exp = np.zeros(13)
    for h in range(g):
        M = logits[h][tok].max()
        L = np.exp(logits[h][tok] - M).sum()
        for j in blocks:
            sel = [i for i in range(j * b, min(t, j * b + b))]
            exp[j] = max(exp[j], math.exp(logits[h][sel].max() - M) / L)
    np.testing.assert_allclose(row, exp, rtol=1e-12)
    assert np.all(row[[2, 3, 4, 5, 7, 8, 9, 10, 11]] == 0.0)
    assert np.all((row >= 0) & (row <= 1))


def test_dense_row_bounds_and_definition():
    rng = np.random.default_rng(5)
    g, d, t, b = 4, 8, 100, 16
    q, K = rng.standard_normal((g, d)), rng.standard_normal((t, d))
    row = orc.dense_row(q, K, b, t)
    p = torch.softmax(torch.from_numpy(q) @ torch.from_numpy(K).T / math.sqrt(d), dim=-1).numpy()
    exp = np.stack([orc.maxpool_blocks(p[h], b) for h in range(g)]).max(axis=0)
    np.testing.assert_allclose(row, exp, rtol=1e-12)
    # each head's pooled values sum to between 1/b and 1; the group max is below g
    assert 1.0 / b <= row.sum() <= g
    # calibration == sparse path with every block selected
    _, A = orc.sparse_attention(q, K, np.zeros((t, d)), np.arange(7), b, t)
    np.testing.assert_allclose(orc.pooled_row(A, b), row, rtol=1e-14)


# ----------------------------------------------------------------------------- history
def test_history_push_is_a_fifo():
    H, width = 4, 6
    hist = np.zeros((H, width))
    rows = [np.full(3 + i % 3, float(i + 1)) for i in range(7)]
    for n, r in enumerate(rows, 1):
        hist = orc.history_push(hist, r)
        for i in range(min(n, H)):
            exp = np.zeros(width)
            exp[:rows[n - 1 - i].size] = rows[n - 1 - i]
            np.testing.assert_array_equal(hist[H - 1 - i], exp)
        for i in range(n, H):
            assert np.all(hist[H - 1 - i] == 0.0)


# ----------------------------------------------------------------------------- Eq. (1)
def test_recovery_rate_special_cases():
    rng = np.random.default_rng(6)
    a = rng.random(40)
    a /= a.sum()
    assert orc.recovery_rate(a, np.arange(40)) == pytest.approx(1.0, abs=1e-15)
    assert orc.recovery_rate(a, np.array([], dtype=int)) == 0.0
    assert orc.recovery_rate(a, np.array([3, 7])) == pytest.approx(a[3] + a[7], rel=1e-14)
    # the best B tokens are the B largest scores
    top = np.argsort(-a)[:5]
    for _ in range(20):
        other = rng.choice(40, 5, replace=False)
        assert orc.recovery_rate(a, top) >= orc.recovery_rate(a, other) - 1e-15


# ----------------------------------------------------------------------------- one whole step
def test_decode_step_wiring():
    """With centre-tap weights the predictor is the windowed mean, so the selected set must be
    the forced blocks plus the highest column sums of the history, and the pushed row must be the
    pooled sparse scores (dense on a calibration step) while the output stays sparse."""
    rng = np.random.default_rng(7)
    g, d, t, b, H, k = 2, 8, 130, 8, 5, 6
    nb = -(-t // b)
    q, K, V = rng.standard_normal((g, d)), rng.standard_normal((t, d)), rng.standard_normal((t, d))
    hist = rng.random((H, nb + 2))
    hist[:, nb:] = 0
    w = orc.PredictorWeights.from_blob(np.zeros(2 * 9 + 2 + 2 * 2 * 9 + 2 + 2 + 1), 2, 2)
    w.w1[0, 1, 1] = w.w2[0, 0, 1, 1] = w.w3[0] = 1.0
    colsum = hist[:, :nb].sum(axis=0)
    mid = np.arange(1, nb - 2)
    exp_blocks = sorted([0, nb - 2, nb - 1] + mid[np.argsort(-colsum[mid], kind="stable")[:k - 3]].tolist())
    for calib in (False, True):
        r = orc.decode_step(hist, q, K, V, t, w, b=b, k=k, n_sink=1, n_local=2, calibrate=calib)
        assert r.blocks.tolist() == exp_blocks
        np.testing.assert_allclose(r.pred, colsum / H, rtol=1e-13)
        ref_out, _ = orc.sparse_attention(q, K, V, np.array(exp_blocks), b, t)
        np.testing.assert_array_equal(r.out, ref_out)
        np.testing.assert_array_equal(r.hist[:-1], hist[1:])
        np.testing.assert_array_equal(r.hist[-1, :nb], r.row)
        if calib:
            np.testing.assert_allclose(r.row, orc.dense_row(q, K, b, t))
            assert np.count_nonzero(r.row) == nb
        else:
            assert np.count_nonzero(r.row) == k


def test_decode_step_reuse_branch_wiring():
    """A step that does not update the positions (Sec. 3.3): the selection comes from the earlier step's list,
    not from this step's scores.  Expectations are written out by hand for the case at hand: the context grew
    from 16 to 18 blocks (t 128 -> 137 with b = 8) since the list was made, n_sink = 1, n_local = 2, k = 6.
    Old list {0, 3, 7, 11, 14, 15}: 14 and 15 were the old local window and are dropped (neither is a sink),
    0, 3, 7, 11 stay, the new local window {16, 17} joins: {0, 3, 7, 11, 16, 17} - although the scores of this
    step (windowed mean of a history that peaks at blocks 5 and 9) would have picked 5 and 9."""
    rng = np.random.default_rng(8)
    g, d, t, b, H, k = 2, 8, 137, 8, 4, 6
    nb = -(-t // b)
    assert nb == 18
    q, K, V = rng.standard_normal((g, d)), rng.standard_normal((t, d)), rng.standard_normal((t, d))
    hist = 0.01 * rng.random((H, nb))
    hist[:, 5] += 1.0
    hist[:, 9] += 0.5
    w = orc.PredictorWeights.from_blob(np.zeros(2 * 9 + 2 + 2 * 2 * 9 + 2 + 2 + 1), 2, 2)
    w.w1[0, 1, 1] = w.w2[0, 0, 1, 1] = w.w3[0] = 1.0
    old = np.array([0, 3, 7, 11, 14, 15])
    expected = [0, 3, 7, 11, 16, 17]
    fresh = orc.decode_step(hist, q, K, V, t, w, b=b, k=k, n_sink=1, n_local=2, calibrate=False)
    assert {5, 9} <= set(fresh.blocks.tolist())                      # what predicting would have chosen
    for calib in (False, True):
        r = orc.decode_step(hist, q, K, V, t, w, b=b, k=k, n_sink=1, n_local=2, calibrate=calib, reuse=(old, 16))
        assert r.blocks.tolist() == expected
        np.testing.assert_allclose(r.pred, hist.sum(axis=0) / H, rtol=1e-13)   # the scores are still reported
        # attention over exactly the tokens of the carried-over blocks, by the definition of Sec. 3.1
        tok = np.concatenate([np.arange(j * b, min((j + 1) * b, t)) for j in expected])
        logits = q @ K[tok].T / np.sqrt(d)
        p = np.exp(logits - logits.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        np.testing.assert_allclose(r.out, p @ V[tok], rtol=1e-12, atol=1e-14)
        np.testing.assert_array_equal(r.hist[:-1], hist[1:])
        if calib:
            assert np.count_nonzero(r.row) == nb
        else:
            assert sorted(np.nonzero(r.row)[0].tolist()) == expected
            # pooled probabilities: per block the largest probability over tokens and heads
            want = np.zeros(nb)
            for j in expected:
                sel = (tok // b) == j
                want[j] = p[:, sel].max()
            np.testing.assert_allclose(r.row, want, rtol=1e-12)
    # a list made for the same width is used as it is
    same = orc.decode_step(hist, q, K, V, t, w, b=b, k=k, n_sink=1, n_local=2, calibrate=False,
                           reuse=(np.array(expected), nb))
    assert same.blocks.tolist() == expected
