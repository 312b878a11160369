"""Pins for the oracle's predictor F (Algorithm 1 step 4; architecture table in the appendix).

None of these re-type the oracle's formula: they are brute-force scalar loops, torch's CPU conv
library, closed forms for special weights, and figures the paper prints.
"""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import attnpred_oracle as orc
from workloads import n_weight_floats

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_predictor_figures.txt")


def _rand_weights(rng, c1, c2, sigma=0.3):
    return orc.PredictorWeights.from_blob(rng.standard_normal(n_weight_floats(c1, c2)) * sigma, c1, c2)


def _zero_weights(c1, c2):
    return orc.PredictorWeights.from_blob(np.zeros(n_weight_floats(c1, c2)), c1, c2)


def _brute_force_predict(hist, nb, w):
    """Scalar loops straight from the layer table; out-of-range taps contribute nothing."""
    H = hist.shape[0]
    c1, c2 = w.b1.size, w.b2.size

    def X(r, j):
        return hist[r][j] if 0 <= r < H and 0 <= j < nb else 0.0

    y1 = [[[0.0] * nb for _ in range(H)] for _ in range(c1)]
    for c in range(c1):
        for r in range(H):
            for j in range(nb):
                s = w.b1[c]
                for kh in range(3):
                    for kw in range(3):
                        s += w.w1[c][kh][kw] * X(r + kh - 1, j + kw - 1)
                y1[c][r][j] = max(s, 0.0)
    out = []
    for j in range(nb):
        total = w.b3
        for c in range(c2):
            tsum = 0.0
            for r in range(H):
                s = w.b2[c]
                for ci in range(c1):
                    for kh in range(3):
                        for kw in range(3):
                            rr, jj = r + kh - 1, j + kw - 1
                            if 0 <= rr < H and 0 <= jj < nb:
                                s += w.w2[c][ci][kh][kw] * y1[ci][rr][jj]
                tsum += max(s, 0.0)
            total += w.w3[c] * tsum / H
        out.append(total)
    return np.array(out)


@pytest.mark.parametrize("H,nb,c1,c2", [(4, 5, 2, 3), (3, 1, 1, 1), (6, 9, 4, 4), (1, 4, 2, 2)])
def test_predict_matches_scalar_brute_force(H, nb, c1, c2):
    rng = np.random.default_rng(H * 100 + nb)
    hist = rng.random((H, nb + 3))            # extra columns beyond nb must be ignored
    w = _rand_weights(rng, c1, c2)
    got = orc.predict(hist, nb, w)
    ref = _brute_force_predict(hist, nb, w)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("H,nb,c1,c2", [(16, 37, 4, 4), (64, 50, 16, 32), (8, 128, 8, 8)])
def test_predict_matches_torch_library(H, nb, c1, c2):
    """torch's conv2d / adaptive_avg_pool2d / conv1d are the layers the table names."""
    rng = np.random.default_rng(7 + nb)
    hist = rng.random((H, nb))
    w = _rand_weights(rng, c1, c2)
    x = torch.from_numpy(hist)[None, None]
    y = F.relu(F.conv2d(x, torch.from_numpy(w.w1)[:, None], torch.from_numpy(w.b1), padding=1))
    y = F.relu(F.conv2d(y, torch.from_numpy(w.w2), torch.from_numpy(w.b2), padding=1))
    y = F.adaptive_avg_pool2d(y, (1, nb))[:, :, 0, :]                      # collapse time
    y = F.conv1d(y, torch.from_numpy(w.w3)[None, :, None], torch.tensor([w.b3], dtype=torch.float64))
    np.testing.assert_allclose(orc.predict(hist, nb, w), y[0, 0].numpy(), rtol=1e-11, atol=1e-13)


def test_delta_weights_give_windowed_accumulation():
    """Centre taps only: F becomes the time-mean of the history, i.e. the windowed score
    accumulation the paper uses as H2O+ (sum over the last H steps) divided by H."""
    H, nb, c1, c2 = 16, 40, 4, 4
    rng = np.random.default_rng(3)
    hist = rng.random((H, nb))
    w = _zero_weights(c1, c2)
    w.w1[0, 1, 1] = 1.0
    w.w2[0, 0, 1, 1] = 1.0
    w.w3[0] = 1.0
    np.testing.assert_allclose(orc.predict(hist, nb, w), hist.sum(axis=0) / H, rtol=1e-14)


def test_shifted_delta_weights_give_sequential_shift():
    """Tap at block offset -1 in conv1 moves every score one block to the right: the
    'sequential' pattern of Sec. 3.3; tap at time offset +1 drops the oldest row."""
    H, nb, c1, c2 = 8, 21, 2, 2
    rng = np.random.default_rng(4)
    hist = rng.random((H, nb))
    w = _zero_weights(c1, c2)
    w.w1[1, 1, 0] = 1.0          # y1[1][r][j] = x[r][j-1]
    w.w2[0, 1, 1, 1] = 1.0
    w.w3[0] = 2.0
    w.b3 = 0.5
    exp = np.zeros(nb)
    exp[1:] = hist[:, :-1].sum(axis=0) / H
    np.testing.assert_allclose(orc.predict(hist, nb, w), 0.5 + 2.0 * exp, rtol=1e-14)

    w = _zero_weights(c1, c2)
    w.w1[0, 2, 1] = 1.0          # y1[0][r][j] = x[r+1][j]  (zero row below the newest)
    w.w2[0, 0, 1, 1] = 1.0
    w.w3[0] = 1.0
    np.testing.assert_allclose(orc.predict(hist, nb, w), hist[1:].sum(axis=0) / H, rtol=1e-14)


def test_previous_token_heuristic_is_a_special_case():
    """With H = 1 and centre taps, F returns the last row: the previous-token baseline of the
    appendix's heuristic comparison."""
    nb = 13
    hist = np.random.default_rng(5).random((1, nb))
    w = _zero_weights(1, 1)
    w.w1[0, 1, 1] = w.w2[0, 0, 1, 1] = w.w3[0] = 1.0
    np.testing.assert_allclose(orc.predict(hist, nb, w), hist[0], rtol=1e-15)


def test_zero_history_closed_form():
    """All-zero history: y1 = relu(b1) everywhere, so y2 only depends on how many taps fall
    inside the tile: interior / edge / corner values have closed forms."""
    H, nb, c1, c2 = 6, 7, 3, 2
    rng = np.random.default_rng(6)
    w = _rand_weights(rng, c1, c2)
    r1 = np.maximum(w.b1, 0.0)

    def y2(c, rows, cols):       # rows/cols: kernel taps that land inside the tile
        s = w.b2[c]
        for ci in range(c1):
            s += r1[ci] * w.w2[c, ci][np.ix_(rows, cols)].sum()
        return max(s, 0.0)

    def col(cols):
        tot = w.b3
        for c in range(c2):
            tsum = y2(c, [1, 2], cols) + y2(c, [0, 1], cols) + (H - 2) * y2(c, [0, 1, 2], cols)
            tot += w.w3[c] * tsum / H
        return tot

    pred = orc.predict(np.zeros((H, nb)), nb, w)
    np.testing.assert_allclose(pred[0], col([1, 2]), rtol=1e-13)
    np.testing.assert_allclose(pred[-1], col([0, 1]), rtol=1e-13)
    np.testing.assert_allclose(pred[1:-1], np.full(nb - 2, col([0, 1, 2])), rtol=1e-13)


def test_padding_is_relative_to_current_width():
    """Columns at and beyond nb are outside the tile even if the buffer holds data there."""
    rng = np.random.default_rng(8)
    hist = rng.random((5, 12))
    w = _rand_weights(rng, 2, 2)
    w.b1[:] = 0.2                 # conv1 of an all-zero neighbourhood is then relu(b1) = 0.2, not 0
    w.b2[:] = 0.5
    a = orc.predict(hist, 9, w)
    h2 = hist.copy()
    h2[:, 9:] = 123.0
    np.testing.assert_array_equal(a, orc.predict(h2, 9, w))
    # and it differs from evaluating the wider tile and cropping (layer-2 sees zeros, not conv1 of zeros)
    wide = orc.predict(np.concatenate([hist[:, :9], np.zeros((5, 3))], axis=1), 12, w)[:9]
    assert abs(wide[8] - a[8]) > 1e-9


def _gold():
    d = {}
    for line in open(GOLD):
        line = line.split("#")[0].split()
        if len(line) == 2:
            d[line[0]] = float(line[1])
    return d


def test_paper_parameter_count_and_model_size():
    g = _gold()
    w = orc.PredictorWeights.from_blob(np.zeros(n_weight_floats(16, 32)), 16, 32)
    assert w.n_params() == 4833                       # 16*9+16 + 32*16*9+32 + 32+1
    assert round(w.n_params() / 1000, 1) in (4.8, g["n_params_thousands"])
    assert abs(w.n_params() / 1000 - g["n_params_thousands"]) < 0.1
    assert abs(w.n_params() * 4 / 1024 - g["model_size_kb"]) < 2.5   # fp32 weights ~ 19 KB vs "21KB"


@pytest.mark.parametrize("ctx,key", [(4096, "peak_mem_mb_4k"), (8192, "peak_mem_mb_8k"),
                                     (16384, "peak_mem_mb_16k"), (32768, "peak_mem_mb_32k")])
def test_paper_feature_map_footprint(ctx, key):
    """Same-size convs over the full H x (t/b) tile with 16 + 32 fp32 feature maps per query
    head reproduce the peak memory the paper reports, within 2 %."""
    g = _gold()
    H, b, heads = int(g["hist_len"]), int(g["block"]), int(g["q_heads"])
    nb = ctx // b
    rng = np.random.default_rng(0)
    w = _rand_weights(rng, 16, 32)
    x = rng.random((H, 8))
    # shapes of the oracle's feature maps on a narrow tile; width scales linearly
    y1 = orc._conv3x3_same(x[None], w.w1[:, None], w.b1)
    y2 = orc._conv3x3_same(y1, w.w2, w.b2)
    assert y1.shape == (16, H, 8) and y2.shape == (32, H, 8)
    per_px = y1.shape[0] + y2.shape[0]
    mib = heads * H * nb * per_px * 4 / 2**20
    assert abs(mib - g[key]) / g[key] < 0.02


# --------------------------------------------------------------------------------------------- refresh
def test_refresh_selection_worked_example():
    """k = 6 with 1 sink and 2 local blocks, selection made at 10 blocks: [0 | 3 5 6 | 8 9]."""
    prev = np.array([0, 3, 5, 6, 8, 9])
    assert orc.refresh_selection(prev, 10, 10, 6, 1, 2).tolist() == [0, 3, 5, 6, 8, 9]      # same length: unchanged
    assert orc.refresh_selection(prev, 10, 11, 6, 1, 2).tolist() == [0, 3, 5, 6, 9, 10]     # 8 left the window
    assert orc.refresh_selection(prev, 10, 13, 6, 1, 2).tolist() == [0, 3, 5, 6, 11, 12]
    assert orc.refresh_selection(np.arange(5), 5, 6, 6, 1, 2).tolist() == [0, 1, 2, 3, 4, 5]  # fits the budget: all
    # an all-blocks selection that stops fitting: the highest blocks below the local window go
    assert orc.refresh_selection(np.arange(6), 6, 7, 6, 1, 2).tolist() == [0, 1, 2, 3, 5, 6]


def test_refresh_selection_properties_and_composition():
    rng = np.random.default_rng(3)
    for _ in range(300):
        k = int(rng.integers(4, 20))
        n_sink = int(rng.integers(0, 3))
        n_local = int(rng.integers(1, 4))
        if n_sink + n_local > k:
            continue
        nb0 = int(rng.integers(k + 1, 80))
        pred = rng.standard_normal(nb0)
        s0 = orc.select_blocks(pred, nb0, k, n_sink, n_local)
        nb1 = nb0 + int(rng.integers(0, 4))
        nb2 = nb1 + int(rng.integers(0, 4))
        s1 = orc.refresh_selection(s0, nb0, nb1, k, n_sink, n_local)
        s2 = orc.refresh_selection(s1, nb1, nb2, k, n_sink, n_local)
        direct = orc.refresh_selection(s0, nb0, nb2, k, n_sink, n_local)
        assert s2.tolist() == direct.tolist(), "carrying over in two hops differs from one hop"
        for s, nb in ((s1, nb1), (s2, nb2)):
            assert np.all(np.diff(s) > 0) and s[0] >= 0 and s[-1] == nb - 1
            assert set(range(n_sink)) <= set(s.tolist()) and set(range(nb - n_local, nb)) <= set(s.tolist())
            mid_prev = set(s0.tolist()) - set(range(nb0 - n_local, nb0))
            assert set(s.tolist()) - set(range(nb - n_local, nb)) <= mid_prev, "a block that was never predicted appeared"
        if nb1 == nb0:
            assert s1.tolist() == s0.tolist()
        assert len(s1) == k and len(s2) == k, "the budget is spent in full at every step"
