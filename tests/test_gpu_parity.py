"""GPU parity: every C-ABI call against the CPU oracle on the same seeded inputs.

Bars (stated by the benchmark spec): selected block indices bit-exact; attention outputs,
pooled rows and predicted scores within 1e-3 relative, taken per vector as
max|gpu - ref| <= 1e-3 * max|ref| (out per head; pred and row per instance).
Index decisions are taken on the fp32 scores the kernel produced (both sides decide in that
precision); against the oracle's own float64 scores a differing pair must be a near tie.
"""
import math

import numpy as np
import pytest
import torch

from oracle import attnpred_oracle as orc
from workloads import CONFIGS, kv_cache, predictor_weights, queries, to_f64, n_weight_floats, Workload

pytestmark = pytest.mark.gpu

REL = 1e-3


def _dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    return torch.device("cuda:0")


def _ap():
    import paper_2502_04077_amd as ap
    ap.load_library()
    return ap


def _run(w, dev, flags=0):
    from paper_2502_04077_amd.runner import DecodeRun
    r = DecodeRun(w, dev, flags=flags)
    r.set_weights(predictor_weights(w))
    return r


class ScoreStats:
    """What the selection sees of the predictor's error, gathered over the checked (step, instance) pairs.

    The selection ranks the candidate blocks [n_sink, nb - n_local) only, and only differences between their
    scores matter: the error is therefore also measured against the spread (max - min) of the oracle's scores over
    those blocks, not only against max|pred|, most of which is a constant every block shares.
    If the GPU picks x where the oracle picks y, then oracle[y] >= oracle[x] and gpu[x] >= gpu[y], hence
    oracle[y] - oracle[x] <= 2 max|gpu - oracle|: every swapped pair has to meet that bound, or the selection is
    wrong and not merely rounded differently."""

    def __init__(self):
        self.rows = 0                # (step, instance) pairs checked
        self.picks = 0               # predicted picks in them (k - n_sink - n_local each)
        self.mismatch = 0            # picks that differ from the selection on the oracle's float64 scores
        self.err_over_spread = 0.0   # max over rows of max|gpu - ref| / spread, candidates only
        self.err_over_max = 0.0      # max over rows of max|gpu - ref| / max|ref|, all blocks

    def add(self, what, gpu_pred, ref_pred, got_idx, nb, k, n_sink, n_local):
        self.rows += 1
        self.err_over_max = max(self.err_over_max, np.abs(gpu_pred - ref_pred).max() / np.abs(ref_pred).max())
        if nb <= k:
            return
        cand = slice(n_sink, nb - n_local)
        err = np.abs(gpu_pred[cand] - ref_pred[cand]).max()
        spread = ref_pred[cand].max() - ref_pred[cand].min()
        if spread > 0:
            self.err_over_spread = max(self.err_over_spread, err / spread)
        self.picks += k - n_sink - n_local
        o_idx = orc.select_blocks(ref_pred, nb, k, n_sink, n_local)
        a = sorted(set(got_idx.tolist()) - set(o_idx.tolist()))       # picked here, not by the oracle
        b = sorted(set(o_idx.tolist()) - set(got_idx.tolist()))       # picked by the oracle, not here
        assert len(a) == len(b)
        if a:
            self.mismatch += len(a)
            gap = max(ref_pred[y] - ref_pred[x] for x in a for y in b)
            assert gap <= 2 * err, f"{what}: swapped blocks differ by {gap:.3e} in the oracle's scores, " \
                                   f"more than twice the score error {err:.3e}"

    def report(self, name):
        frac = self.mismatch / self.picks if self.picks else 0.0
        print(f"{name}: {self.rows} rows, score error {self.err_over_max:.2e} of max|pred|, "
              f"{self.err_over_spread:.2e} of the candidates' spread; picks differing from the float64 selection: "
              f"{self.mismatch} of {self.picks} ({100 * frac:.2f} %)")
        return frac


def assert_close(gpu, ref, what, rel=REL):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape, f"{what}: shape {gpu.shape} vs {ref.shape}"
    scale = np.abs(ref).max()
    err = np.abs(gpu - ref).max()
    assert np.isfinite(gpu).all(), f"{what}: non-finite values"
    assert err <= rel * scale + 1e-30, f"{what}: max err {err:.3e} > {rel} * {scale:.3e}"


def small(name="t", **kw):
    base = dict(name=name, layers=1, batch=1, kv_heads=3, g=4, head_dim=128, kv_dtype="bf16", t0=1000, block=16,
                hist_len=16, budget_tokens=256, n_sink=1, n_local=2, c1=8, c2=8, steps=8, calib_every=4,
                seed=11, value_scale=1.0)
    base.update(kw)
    return Workload(**base)


# --------------------------------------------------------------------------------------------- select
@pytest.mark.parametrize("nb,k,ns,nl,mode,n_inst", [
    (128, 16, 1, 2, "ties", 5), (2048, 64, 4, 4, "normal", 5), (2051, 64, 4, 4, "ties", 5),
    (8200, 128, 4, 4, "normal", 5), (300, 64, 0, 0, "allequal", 5), (64, 64, 4, 4, "normal", 5),
    (10, 64, 4, 4, "normal", 5), (65, 64, 4, 4, "ties", 5), (500, 8, 4, 4, "normal", 5),
    (700, 33, 3, 5, "signedzero", 5), (1000, 40, 2, 2, "negative", 5),
    # many instances keep 256 threads per instance; few instances with long rows take 1024
    (2051, 64, 4, 4, "ties", 600), (2400, 64, 4, 4, "normal", 520), (8200, 128, 4, 4, "ties", 513),
    (9000, 64, 4, 4, "normal", 515), (5000, 128, 4, 4, "ties", 3), (12000, 200, 1, 1, "normal", 2),
    (20000, 64, 4, 4, "ties", 2), (4104, 64, 4, 4, "allequal", 1),
    (8210, 128, 4, 4, "normal", 5), (9100, 128, 4, 4, "ties", 7), (9224, 64, 4, 4, "allequal", 3),
    (9225, 64, 4, 4, "normal", 3),
])
def test_select_topk_bit_exact(nb, k, ns, nl, mode, n_inst):
    dev = _dev()
    ap = _ap()
    b = 16
    nb_cap = nb + 3
    ctx = ap.Context(n_inst=n_inst, g=1, head_dim=64, block=b, hist_len=4, t_cap=nb_cap * b, k_blocks=k,
                     n_sink=ns, n_local=nl, c1=4, c2=4, kv_dtype="f32")
    rng = np.random.default_rng(nb * 7 + k)
    if mode == "normal":
        p = rng.standard_normal((n_inst, nb_cap))
    elif mode == "ties":
        p = rng.integers(0, 6, size=(n_inst, nb_cap)) * 0.125 - 0.25
    elif mode == "allequal":
        p = np.full((n_inst, nb_cap), 0.375)
    elif mode == "signedzero":
        p = rng.choice(np.array([0.0, -0.0, 1e-30, -1e-30]), size=(n_inst, nb_cap))
    else:
        p = -np.abs(rng.standard_normal((n_inst, nb_cap))) - 1.0
    p = p.astype(np.float32)
    pred = torch.from_numpy(p).to(dev)
    idx = torch.full((n_inst, k), -7, dtype=torch.int32, device=dev)
    cnt = torch.zeros((n_inst,), dtype=torch.int32, device=dev)
    ws = torch.zeros((max(16, ctx.workspace_bytes()),), dtype=torch.uint8, device=dev)
    ctx.select_topk(pred, nb, idx, cnt, ws)
    torch.cuda.synchronize()
    idx, cnt = idx.cpu().numpy(), cnt.cpu().numpy()
    for i in range(n_inst):
        exp = orc.select_blocks(p[i].astype(np.float64), nb, k, ns, nl)
        assert cnt[i] == len(exp)
        assert idx[i, :cnt[i]].tolist() == exp.tolist(), f"instance {i}"
        assert np.all(idx[i, cnt[i]:] == -7)


# --------------------------------------------------------------------------------------------- predict
@pytest.mark.parametrize("H,nb,c1,c2,pushed", [
    (16, 128, 4, 4, 16), (16, 131, 4, 4, 40), (64, 200, 8, 8, 64), (64, 70, 8, 8, 7), (13, 65, 8, 8, 100),
    (64, 130, 16, 32, 64), (5, 1, 4, 4, 9), (8, 63, 8, 8, 0),
    # longest and shortest histories of the MFMA kernels
    (256, 150, 8, 8, 300), (256, 90, 16, 32, 256), (6, 200, 8, 8, 10), (7, 130, 16, 32, 3),
])
def test_predict_vs_oracle(H, nb, c1, c2, pushed):
    dev = _dev()
    ap = _ap()
    n_inst, b = 3, 16
    nb_cap = nb + 5
    ctx = ap.Context(n_inst=n_inst, g=1, head_dim=64, block=b, hist_len=H, t_cap=nb_cap * b, k_blocks=4,
                     n_sink=1, n_local=1, c1=c1, c2=c2, kv_dtype="f32")
    R = ctx.hist_slots()
    assert R == H + 1
    rng = np.random.default_rng(H * 1000 + nb)
    blob = (rng.standard_normal(n_weight_floats(c1, c2)) * 0.2).astype(np.float32)
    ctx.set_weights(blob)
    wts = orc.PredictorWeights.from_blob(blob, c1, c2)
    # ring content: rows numbered 0..pushed-1 were pushed; slots never written stay zero.
    ring = np.zeros((n_inst, R, nb_cap), dtype=np.float32)
    rows = {}
    for n in range(pushed):
        r = (rng.random((n_inst, nb_cap)) ** 4).astype(np.float32)   # probability-like, mostly small
        r[:, nb:] = 7.0                                             # junk beyond nb_cur must be ignored
        ring[:, n % R, :] = r
        rows[n] = r
    hist = torch.from_numpy(ring).to(dev)
    pred = torch.full((n_inst, nb_cap), -5.0, dtype=torch.float32, device=dev)
    ws = torch.zeros((max(16, ctx.workspace_bytes()),), dtype=torch.uint8, device=dev)
    ctx.predict(hist, pushed, nb, pred, ws)
    torch.cuda.synchronize()
    got = pred.cpu().numpy().astype(np.float64)
    got[:, :nb] += ctx.score_offset()                   # pred is relative to the all-zero-history score
    for i in range(n_inst):
        logical = np.zeros((H, nb_cap))
        for r in range(H):
            n = pushed - H + r
            if n >= 0:
                logical[r] = rows[n][i]
        ref = orc.predict(logical, nb, wts)
        assert_close(got[i, :nb], ref, f"pred inst {i}")
        assert np.all(got[i, nb:] == -5.0)


@pytest.mark.parametrize("H,c1,c2,fp32", [(64, 8, 8, 0), (64, 8, 8, 1), (16, 4, 4, 0), (64, 16, 32, 0), (6, 8, 8, 0),
                                          (5, 8, 8, 0), (1, 4, 4, 0), (2, 8, 8, 0)])
def test_score_offset_is_the_zero_history_score(H, c1, c2, fp32):
    """pred is the predictor's output minus what it answers to an all-zero history (ap_score_offset).  So the offset
    must equal the oracle's score of an all-zero tile away from the tile's edges, the kernels must return exact zeros
    there for such a tile, and at the edge blocks (where the second layer's zero padding shows) offset + pred must
    still be the oracle's score."""
    dev = _dev()
    ap = _ap()
    n_inst, b, nb = 2, 16, 40
    ctx = ap.Context(n_inst=n_inst, g=1, head_dim=64, block=b, hist_len=H, t_cap=(nb + 3) * b, k_blocks=4, n_sink=1,
                     n_local=1, c1=c1, c2=c2, kv_dtype="f32", flags=ap.AP_FLAG_PREDICTOR_FP32 if fp32 else 0)
    rng = np.random.default_rng(H + c1)
    blob = (rng.standard_normal(n_weight_floats(c1, c2)) * 0.3).astype(np.float32)
    assert ctx.score_offset() == 0.0                    # nothing to report before the weights are set
    ctx.set_weights(blob)
    wts = orc.PredictorWeights.from_blob(blob, c1, c2)
    ref = orc.predict(np.zeros((H, nb)), nb, wts)
    off = ctx.score_offset()
    assert abs(off - ref[nb // 2]) <= 1e-12 * max(1.0, abs(ref[nb // 2]))
    hist = torch.zeros((n_inst, ctx.hist_slots(), nb + 3), dtype=torch.float32, device=dev)
    pred = torch.full((n_inst, nb + 3), -5.0, dtype=torch.float32, device=dev)
    pstate = torch.full((n_inst, nb + 3), 3.0, dtype=torch.float32, device=dev)
    ws = torch.zeros((max(16, ctx.workspace_bytes()),), dtype=torch.uint8, device=dev)
    for call in ("full", "rebase", "advance"):
        if call == "full":
            ctx.predict(hist, 7, nb, pred, ws)
        else:
            ctx.predict_incremental(hist, 7 if call == "rebase" else 8, nb, nb,
                                    ap.AP_PRED_REBASE if call == "rebase" else ap.AP_PRED_ADVANCE, pstate, pred, ws)
        torch.cuda.synchronize()
        got = pred.cpu().numpy().astype(np.float64)
        assert np.all(got[:, 1:nb - 1] == 0.0), call
        assert_close(got[0, :nb] + off, ref, f"zero history, {call}")


@pytest.mark.parametrize("H,nb0,c1,c2,n_steps,grow_every,fp32", [
    (16, 130, 8, 8, 60, 5, 0), (64, 200, 8, 8, 150, 16, 0), (6, 70, 4, 4, 40, 3, 0), (64, 65, 16, 32, 70, 0, 0),
    (16, 1, 8, 8, 40, 4, 0), (5, 40, 8, 8, 12, 0, 0), (16, 130, 8, 8, 60, 5, 1), (64, 300, 8, 8, 150, 16, 1),
    (64, 2049, 8, 8, 20, 4, 0), (64, 300, 16, 32, 80, 8, 0), (16, 122, 16, 32, 40, 5, 1), (6, 123, 16, 32, 24, 2, 0),
    (64, 2049, 16, 32, 12, 4, 0),
])
def test_predict_incremental_tracks_oracle(H, nb0, c1, c2, n_steps, grow_every, fp32):
    """ADVANCE once per pushed row (no re-base in between), tile growing, ring wrapping: every
    prediction must match the oracle's full evaluation of the same history; HOLD repeats it bit for bit."""
    dev = _dev()
    ap = _ap()
    n_inst, b = 2, 16
    nb_cap = nb0 + (n_steps // grow_every if grow_every else 0) + 4
    ctx = ap.Context(n_inst=n_inst, g=1, head_dim=64, block=b, hist_len=H, t_cap=nb_cap * b, k_blocks=4,
                     n_sink=1, n_local=1, c1=c1, c2=c2, kv_dtype="f32",
                     flags=ap.AP_FLAG_PREDICTOR_FP32 if fp32 else 0)
    R = ctx.hist_slots()
    rng = np.random.default_rng(H * 31 + nb0)
    blob = (rng.standard_normal(n_weight_floats(c1, c2)) * 0.2).astype(np.float32)
    ctx.set_weights(blob)
    wts = orc.PredictorWeights.from_blob(blob, c1, c2)
    hist = torch.zeros((n_inst, R, nb_cap), dtype=torch.float32, device=dev)
    row = torch.zeros((n_inst, nb_cap), dtype=torch.float32, device=dev)
    pred = torch.zeros((n_inst, nb_cap), dtype=torch.float32, device=dev)
    pstate = torch.full((n_inst, nb_cap), 123.0, dtype=torch.float32, device=dev)
    ws = torch.zeros((max(16, ctx.workspace_bytes()),), dtype=torch.uint8, device=dev)
    logical = np.zeros((n_inst, H, nb_cap))
    nb, nb_prev, worst = nb0, nb0, 0.0
    for n in range(n_steps):
        mode = ap.AP_PRED_REBASE if n == 0 else ap.AP_PRED_ADVANCE
        ctx.predict_incremental(hist, n, nb, nb_prev, mode, pstate, pred, ws)
        torch.cuda.synchronize()
        got = pred.cpu().numpy().astype(np.float64) + ctx.score_offset()
        if n % 7 == 3:
            ctx.predict_incremental(hist, n, nb, nb, ap.AP_PRED_HOLD, pstate, pred, ws)
            torch.cuda.synchronize()
            again = pred.cpu().numpy().astype(np.float64) + ctx.score_offset()
            if nb == nb_prev:
                assert np.array_equal(again[:, :nb], got[:, :nb]), f"HOLD changed the prediction at n={n}"
            else:   # the last columns came from the full-tile kernel in the first call
                assert np.array_equal(again[:, :nb_prev - 1], got[:, :nb_prev - 1])
                assert_close(again[:, :nb], got[:, :nb], f"HOLD after growth at n={n}", rel=1e-4)
        if n < 3 * H or n % 5 == 0 or n == n_steps - 1:
            for i in range(n_inst):
                ref = orc.predict(logical[i], nb, wts)
                assert_close(got[i, :nb], ref, f"n={n} inst {i} nb={nb}")
                worst = max(worst, np.abs(got[i, :nb] - ref).max() / np.abs(ref).max())
        # push a new row of the current width, then maybe grow the tile for the next call
        r = np.zeros((n_inst, nb_cap), dtype=np.float32)
        r[:, :nb] = (rng.random((n_inst, nb)) ** 4).astype(np.float32)
        row.copy_(torch.from_numpy(r))
        ctx.update_history(hist, n, row)
        for i in range(n_inst):
            logical[i] = orc.history_push(logical[i], r[i].astype(np.float64))
        nb_prev = nb
        if grow_every and (n + 1) % grow_every == 0:
            nb += 1
    print(f"incremental predictor worst relative error over {n_steps} un-rebased steps: {worst:.2e}")


@pytest.mark.parametrize("c1,c2", [(8, 8), (16, 32)])
def test_predict_stress_large_weights(c1, c2):
    """Weights five times the workloads' (sigma 0.5) on rows with entries up to 1: the f16-operand kernels still
    have to stay within the 1e-3 bar.  Bound by the arithmetic: an f16 operand carries a relative rounding of at
    most 2^-11, the products are exact and summed in fp32, so the variable part of a score is off by about
    2^-11 x sqrt(2) per operand pair, averaged down over the 72 to 144 taps and H rows; the result here is a few
    1e-4 of max|pred| for 8/8 and for 16/32 channels."""
    dev = _dev()
    ap = _ap()
    H, nb, n_inst, b = 64, 200, 2, 16
    nb_cap = nb + 4
    ctx = ap.Context(n_inst=n_inst, g=1, head_dim=64, block=b, hist_len=H, t_cap=nb_cap * b, k_blocks=4, n_sink=1,
                     n_local=1, c1=c1, c2=c2, kv_dtype="f32")
    R = ctx.hist_slots()
    rng = np.random.default_rng(c1 * 100 + c2)
    blob = (rng.standard_normal(n_weight_floats(c1, c2)) * 0.5).astype(np.float32)
    ctx.set_weights(blob)
    wts = orc.PredictorWeights.from_blob(blob, c1, c2)
    off = ctx.score_offset()
    hist = torch.zeros((n_inst, R, nb_cap), dtype=torch.float32, device=dev)
    row = torch.zeros((n_inst, nb_cap), dtype=torch.float32, device=dev)
    pred = torch.zeros((n_inst, nb_cap), dtype=torch.float32, device=dev)
    pstate = torch.zeros((n_inst, nb_cap), dtype=torch.float32, device=dev)
    ws = torch.zeros((max(16, ctx.workspace_bytes()),), dtype=torch.uint8, device=dev)
    logical = np.zeros((n_inst, H, nb_cap))
    worst = 0.0
    for n in range(H + 24):
        r = np.zeros((n_inst, nb_cap), dtype=np.float32)
        r[:, :nb] = (rng.random((n_inst, nb)) ** 2).astype(np.float32)
        row.copy_(torch.from_numpy(r))
        ctx.update_history(hist, n, row)
        for i in range(n_inst):
            logical[i] = orc.history_push(logical[i], r[i].astype(np.float64))
        if n < H - 1:
            continue
        mode = ap.AP_PRED_REBASE if n == H - 1 else ap.AP_PRED_ADVANCE
        ctx.predict_incremental(hist, n + 1, nb, nb, mode, pstate, pred, ws)
        torch.cuda.synchronize()
        got = pred.cpu().numpy().astype(np.float64) + off
        for i in range(n_inst):
            ref = orc.predict(logical[i], nb, wts)
            assert_close(got[i, :nb], ref, f"({c1},{c2}) sigma 0.5, row {n} inst {i}")
            worst = max(worst, np.abs(got[i, :nb] - ref).max() / np.abs(ref).max())
    ctx.predict(hist, H + 24, nb, pred, ws)
    torch.cuda.synchronize()
    full = pred.cpu().numpy().astype(np.float64) + off
    for i in range(n_inst):
        assert_close(full[i, :nb], orc.predict(logical[i], nb, wts), f"({c1},{c2}) sigma 0.5, full tile inst {i}")
    print(f"({c1},{c2}) predictor, sigma 0.5 weights: worst error {worst:.2e} of max|pred|")


# --------------------------------------------------------------------------------------------- attention
ATTN_CASES = [
    # name, kwargs, t_cur, n_inst hint
    ("cfg0-shape", dict(kv_heads=1, g=4, head_dim=64, kv_dtype="f32", t0=2048, budget_tokens=256), 2048),
    ("bf16-g4", dict(kv_heads=3, g=4, head_dim=128, budget_tokens=1024, t0=5000), 4999),
    ("bf16-g4-ragged", dict(kv_heads=2, g=4, head_dim=128, budget_tokens=512, t0=3000), 2987),
    ("bf16-g1", dict(kv_heads=5, g=1, head_dim=128, budget_tokens=1024, t0=4000), 3999),
    ("bf16-g8-d64", dict(kv_heads=2, g=8, head_dim=64, budget_tokens=256, t0=1500), 1490),
    ("bf16-g2-b32", dict(kv_heads=2, g=2, head_dim=128, block=32, budget_tokens=512, t0=4000), 3990),
    ("f32-d128-b8", dict(kv_heads=2, g=2, head_dim=128, kv_dtype="f32", block=8, budget_tokens=200, t0=900), 899),
    ("many-inst", dict(kv_heads=8, batch=160, g=4, head_dim=128, budget_tokens=256, t0=600), 600),
    ("many-inst-k64", dict(kv_heads=8, batch=130, g=4, head_dim=128, budget_tokens=1024, t0=1100), 1099),
    ("big-budget", dict(kv_heads=2, g=4, head_dim=128, budget_tokens=4096, t0=9000), 8999),
    # more instances than the chip holds four-wave workgroups: the pieced two-wave form (pieces of 32 + 16 blocks)
    # and, with g = 1 and 4096 instances, the one-wave form
    ("two-wave", dict(kv_heads=8, batch=200, g=4, head_dim=128, budget_tokens=768, t0=1100), 1093),
    ("one-wave", dict(kv_heads=16, batch=256, g=1, head_dim=128, budget_tokens=640, t0=900), 899),
]


def _random_blocks(rng, nb, k, ns, nl):
    if nb <= k:
        return np.arange(nb)
    mid = rng.choice(np.arange(ns, nb - nl), size=k - ns - nl, replace=False)
    return np.sort(np.concatenate([np.arange(ns), mid, np.arange(nb - nl, nb)]))


@pytest.mark.parametrize("name,kw,t_cur", ATTN_CASES, ids=[c[0] for c in ATTN_CASES])
def test_sparse_decode_vs_oracle(name, kw, t_cur):
    dev = _dev()
    w = small(name, **kw)
    run = _run(w, dev)
    K, V = kv_cache(w, dev)
    q = queries(w, 0, dev)
    rng = np.random.default_rng(5)
    nb = run.nb(t_cur)
    blocks = np.stack([_random_blocks(rng, nb, w.k_blocks, w.n_sink, w.n_local) for _ in range(w.n_inst)])
    cnt = np.full((w.n_inst,), blocks.shape[1], dtype=np.int32)
    run.idx[:, :blocks.shape[1]] = torch.from_numpy(blocks.astype(np.int32)).to(dev)
    run.cnt[:] = torch.from_numpy(cnt).to(dev)
    run.row.fill_(9.0)
    run.ctx.sparse_decode(q, K, V, t_cur, run.idx, run.cnt, run.out, run.row, run.ws)
    torch.cuda.synchronize()
    out, row = run.out.cpu().numpy(), run.row.cpu().numpy()
    sample = range(w.n_inst) if w.n_inst <= 8 else [0, 1, w.n_inst // 2, w.n_inst - 1]
    for i in sample:
        ref_out, A = orc.sparse_attention(to_f64(q[i]), to_f64(K[i]), to_f64(V[i]), blocks[i], w.block, t_cur)
        for h in range(w.g):
            assert_close(out[i, h], ref_out[h], f"{name} out inst {i} head {h}")
        ref_row = np.zeros(run.nb_cap)
        ref_row[:nb] = orc.pooled_row(A, w.block)
        assert_close(row[i], ref_row, f"{name} row inst {i}")
        unsel = np.ones(run.nb_cap, bool)
        unsel[blocks[i]] = False
        assert np.all(row[i][unsel] == 0.0)


@pytest.mark.parametrize("kw", [dict(kv_heads=6, g=4, head_dim=128, budget_tokens=512, t0=3000),
                                dict(kv_heads=8, batch=130, g=4, head_dim=128, budget_tokens=256, t0=600),
                                dict(kv_heads=8, batch=200, g=4, head_dim=128, budget_tokens=1024, t0=1100)],
                         ids=["split", "whole", "two-wave"])
def test_sparse_decode_ragged_counts(kw):
    """Lists shorter than the budget, one of them empty; the idx entries past cnt are garbage and must be ignored.
    An empty list gives a zero output and a zero row."""
    dev = _dev()
    w = small("ragged", **kw)
    run = _run(w, dev)
    K, V = kv_cache(w, dev)
    q = queries(w, 0, dev)
    rng = np.random.default_rng(11)
    t_cur = w.t0 - 3
    nb, k = run.nb(t_cur), w.k_blocks
    cnt = rng.integers(1, k + 1, size=w.n_inst).astype(np.int32)
    cnt[0], cnt[1], cnt[2] = 0, 1, k - 1
    idx = np.full((w.n_inst, k), 2**30, dtype=np.int32)
    lists = []
    for i in range(w.n_inst):
        blk = np.sort(rng.choice(nb, size=cnt[i], replace=False))
        lists.append(blk)
        idx[i, :cnt[i]] = blk
    run.idx.copy_(torch.from_numpy(idx).to(dev))
    run.cnt.copy_(torch.from_numpy(cnt).to(dev))
    run.row.fill_(9.0)
    run.out.fill_(9.0)
    run.ctx.sparse_decode(q, K, V, t_cur, run.idx, run.cnt, run.out, run.row, run.ws)
    torch.cuda.synchronize()
    out, row = run.out.cpu().numpy(), run.row.cpu().numpy()
    assert np.all(out[0] == 0.0) and np.all(row[0] == 0.0)
    for i in [1, 2, 3, w.n_inst // 2, w.n_inst - 1]:
        ref_out, A = orc.sparse_attention(to_f64(q[i]), to_f64(K[i]), to_f64(V[i]), lists[i], w.block, t_cur)
        for h in range(w.g):
            assert_close(out[i, h], ref_out[h], f"ragged out inst {i} head {h}")
        ref_row = np.zeros(run.nb_cap)
        ref_row[:nb] = orc.pooled_row(A, w.block)
        assert_close(row[i], ref_row, f"ragged row inst {i}")
        unsel = np.ones(run.nb_cap, bool)
        unsel[lists[i]] = False
        assert np.all(row[i][unsel] == 0.0)


NAN_TAIL_CASES = [
    ("four-wave-split", dict(kv_heads=3, g=4, head_dim=128, budget_tokens=1024, t0=5000), 4987, False),
    ("four-wave-whole", dict(kv_heads=8, batch=130, g=4, head_dim=128, budget_tokens=256, t0=600), 595, False),
    ("two-wave", dict(kv_heads=8, batch=200, g=4, head_dim=128, budget_tokens=768, t0=1100), 1093, False),
    ("one-wave", dict(kv_heads=16, batch=256, g=1, head_dim=128, budget_tokens=640, t0=900), 899, False),
    ("f32", dict(kv_heads=2, g=2, head_dim=64, kv_dtype="f32", budget_tokens=256, t0=900), 890, False),
    ("paged-bf16", dict(kv_heads=3, g=4, head_dim=128, budget_tokens=1024, t0=3000), 2990, True),
    ("paged-two-wave", dict(kv_heads=8, batch=200, g=4, head_dim=128, budget_tokens=768, t0=1100), 1093, True),
]


@pytest.mark.parametrize("name,kw,t_cur,paged", NAN_TAIL_CASES, ids=[c[0] for c in NAN_TAIL_CASES])
def test_rows_beyond_the_context_may_hold_anything(name, kw, t_cur, paged):
    """K/V rows at and after t_cur are not part of the context (Algorithm 1 step 1 pads the score row with
    zeros): whatever the cache holds there - NaN here, as a recycled page might - must not reach out or row."""
    dev = _dev()
    w = small(name, **kw)
    run = _run(w, dev)
    K, V = kv_cache(w, dev)
    q = queries(w, 0, dev)
    assert t_cur % w.block != 0                         # the newest block has a masked tail
    Kc = {i: to_f64(K[i]) for i in (0, w.n_inst - 1)}
    Vc = {i: to_f64(V[i]) for i in (0, w.n_inst - 1)}
    K[:, t_cur:, :] = float("nan")
    V[:, t_cur:, :] = float("nan")
    rng = np.random.default_rng(17)
    nb = run.nb(t_cur)
    blocks = np.stack([_random_blocks(rng, nb, w.k_blocks, w.n_sink, w.n_local) for _ in range(w.n_inst)])
    run.idx[:, :blocks.shape[1]] = torch.from_numpy(blocks.astype(np.int32)).to(dev)
    run.cnt[:] = blocks.shape[1]
    Ka, Va = K, V
    if paged:
        Ka, Va, table, n_phys = _paged_copy(w, run, K, V, dev)
        run.ctx.set_block_table(table, n_phys)
    run.ctx.sparse_decode(q, Ka, Va, t_cur, run.idx, run.cnt, run.out, run.row, run.ws)
    run.pred.fill_(5.0)
    run.ctx.calibrate(q, Ka, t_cur, run.pred, run.ws)      # (pred serves as a second row buffer)
    torch.cuda.synchronize()
    out, row, dense = run.out.cpu().numpy(), run.row.cpu().numpy(), run.pred.cpu().numpy()
    assert np.isfinite(out).all() and np.isfinite(row).all() and np.isfinite(dense).all()
    for i in (0, w.n_inst - 1):
        ref_out, A = orc.sparse_attention(to_f64(q[i]), Kc[i], Vc[i], blocks[i], w.block, t_cur)
        for h in range(w.g):
            assert_close(out[i, h], ref_out[h], f"{name} out inst {i} head {h}")
        assert_close(row[i, :nb], orc.pooled_row(A, w.block), f"{name} row inst {i}")
        assert_close(dense[i, :nb], orc.dense_row(to_f64(q[i]), Kc[i], w.block, t_cur), f"{name} dense row inst {i}")


def test_full_budget_is_dense_attention():
    """Budget >= context: the sparse path must reproduce dense attention (rows of the softmax sum to 1)."""
    dev = _dev()
    w = small("dense", kv_heads=2, g=4, head_dim=128, t0=700, budget_tokens=1024)
    run = _run(w, dev)
    K, V = kv_cache(w, dev)
    q = queries(w, 0, dev)
    t = 700
    nb = run.nb(t)
    run.pred.zero_()
    run.ctx.select_topk(run.pred, nb, run.idx, run.cnt, run.ws)
    run.ctx.sparse_decode(q, K, V, t, run.idx, run.cnt, run.out, run.row, run.ws)
    torch.cuda.synchronize()
    assert run.cnt.cpu().tolist() == [nb] * w.n_inst
    for i in range(w.n_inst):
        qi, Ki, Vi = to_f64(q[i]), to_f64(K[i]), to_f64(V[i])
        p = torch.softmax(torch.from_numpy(qi @ Ki[:t].T / math.sqrt(w.head_dim)), dim=-1).numpy()
        dense = p @ Vi[:t]
        for h in range(w.g):
            assert_close(run.out[i, h].cpu().numpy(), dense[h], f"dense out {i}/{h}")
        assert_close(run.row[i, :nb].cpu().numpy(), orc.dense_row(qi, Ki, w.block, t), "dense row")


CAL_CASES = [
    ("cfg0-shape", dict(kv_heads=1, g=4, head_dim=64, kv_dtype="f32", t0=2048), 2048),
    ("bf16-g4", dict(kv_heads=3, g=4, head_dim=128, t0=5000), 4999),
    ("bf16-g4-one-chunk", dict(kv_heads=2, g=4, head_dim=128, t0=600), 555),
    ("bf16-g1", dict(kv_heads=3, g=1, head_dim=128, t0=4000), 3173),
    ("bf16-g8-d64-b32", dict(kv_heads=2, g=8, head_dim=64, block=32, t0=2500), 2490),
]


@pytest.mark.parametrize("name,kw,t_cur", CAL_CASES, ids=[c[0] for c in CAL_CASES])
def test_calibrate_vs_oracle(name, kw, t_cur):
    dev = _dev()
    w = small(name, **kw)
    run = _run(w, dev)
    K, _ = kv_cache(w, dev)
    q = queries(w, 3, dev)
    run.row.fill_(9.0)
    run.ctx.calibrate(q, K, t_cur, run.row, run.ws)
    torch.cuda.synchronize()
    row = run.row.cpu().numpy()
    nb = run.nb(t_cur)
    for i in range(w.n_inst):
        ref = np.zeros(run.nb_cap)
        ref[:nb] = orc.dense_row(to_f64(q[i]), to_f64(K[i]), w.block, t_cur)
        assert_close(row[i], ref, f"{name} dense row inst {i}")
        assert np.all(row[i, nb:] == 0.0)


# --------------------------------------------------------------------------------------------- history
def test_update_history_ring_is_a_fifo():
    dev = _dev()
    w = small("ring", kv_heads=2, hist_len=5, t0=300)
    run = _run(w, dev)
    H = w.hist_len
    logical = np.zeros((w.n_inst, H, run.nb_cap))
    rng = np.random.default_rng(1)
    for n in range(3 * H + 2):
        r = rng.random((w.n_inst, run.nb_cap)).astype(np.float32)
        run.row.copy_(torch.from_numpy(r))
        run.ctx.update_history(run.hist, run.n_pushed, run.row)
        run.n_pushed += 1
        for i in range(w.n_inst):
            logical[i] = orc.history_push(logical[i], r[i].astype(np.float64))
        got = run.logical_history().cpu().numpy()
        assert np.array_equal(got, logical.astype(np.float32))


# --------------------------------------------------------------------------------------------- whole steps
def lockstep(w, dev, steps, sample, fused_every=2, incremental=True, warm_checks=(0, -1), warm=True, flags=0,
             check=None, rebase_every=None):
    """Runs decode steps on the GPU; at each checked step (all, or those in `check`) the oracle starts from the
    GPU's own history.  Only the sampled instances are copied to the host.  Returns the ScoreStats of the run."""
    run = _run(w, dev, flags)
    run.incremental = incremental
    if rebase_every is not None:
        run.rebase_every = rebase_every
    K, V = kv_cache(w, dev)
    wts = orc.PredictorWeights.from_blob(predictor_weights(w), w.c1, w.c2)
    H, b = w.hist_len, w.block
    sample = list(sample)
    pos = {i: n for n, i in enumerate(sample)}
    Kc = {i: to_f64(K[i]) for i in sample}
    Vc = {i: to_f64(V[i]) for i in sample}
    sel = torch.as_tensor(sample, device=dev)
    # history warm-up: the last H prefill steps, dense rows (appendix "Training Details")
    for j in range(H if warm else 0):
        t = w.t0 - H + 1 + j
        q = queries(w, j - H, dev)
        run.warmup_calibrate(q, K, t)
        if j in [c % H for c in warm_checks]:
            torch.cuda.synchronize()
            for i in sample:
                ref = orc.dense_row(to_f64(q[i]), Kc[i], b, t)
                assert_close(run.row[i, :run.nb(t)].cpu().numpy(), ref, f"warm-up row {j} inst {i}")
    stats = ScoreStats()
    modes = stats.modes = []         # predictor mode of every step (0 = re-base, 1 = advance)
    off = run.ctx.score_offset()     # pred is relative to the all-zero-history score
    for s in range(steps):
        t = w.t_at(s)
        nb = run.nb(t)
        q = queries(w, s, dev)
        calib = w.is_calibration_step(s)
        checked = check is None or s in check
        if checked:
            before = run.logical_history(sample).cpu().numpy().astype(np.float64)
        if s % fused_every == 0:
            mode = run.step(q, K, V, t, calibrate=calib)
        else:
            mode = run.step_unfused(q, K, V, t, calibrate=calib)
        modes.append(mode)
        if not checked:
            continue
        torch.cuda.synchronize()
        after = run.logical_history(sample).cpu().numpy()
        pred, idx, cnt = run.pred[sel].cpu().numpy(), run.idx[sel].cpu().numpy(), run.cnt[sel].cpu().numpy()
        out = run.out[sel].cpu().numpy()
        qs = q[sel]
        for i in sample:
            n = pos[i]
            qi = to_f64(qs[n])
            ref_pred = orc.predict(before[n], nb, wts)
            assert_close(pred[n, :nb].astype(np.float64) + off, ref_pred, f"step {s} inst {i} pred")
            got_idx = idx[n, :cnt[n]]
            # decision in the kernel's precision: the oracle's selection on the kernel's fp32 scores
            exp_idx = orc.select_blocks(pred[n, :nb].astype(np.float64), nb, w.k_blocks, w.n_sink, w.n_local)
            assert got_idx.tolist() == exp_idx.tolist(), f"step {s} inst {i}: selection differs"
            # against the oracle's float64 scores: counted, and every swapped pair bounded by the score error
            stats.add(f"step {s} inst {i}", pred[n, :nb].astype(np.float64) + off, ref_pred, got_idx, nb, w.k_blocks,
                      w.n_sink, w.n_local)
            ref_out, A = orc.sparse_attention(qi, Kc[i], Vc[i], got_idx, b, t)
            for h in range(w.g):
                assert_close(out[n, h], ref_out[h], f"step {s} inst {i} head {h} out")
            ref_row = np.zeros(run.nb_cap)
            ref_row[:nb] = orc.dense_row(qi, Kc[i], b, t) if calib else orc.pooled_row(A, b)
            assert_close(after[n, H - 1], ref_row, f"step {s} inst {i} pushed row")
            assert np.array_equal(after[n, :H - 1], before[n, 1:].astype(np.float32)), "history did not shift"
    del K, V, run
    torch.cuda.empty_cache()
    return stats


# Ceilings for the share of predicted picks that may differ from the selection on the oracle's float64 scores
# (measured on the seeded workloads, with head-room; the counts are reproducible).  cfg0 and the small workloads
# have well separated scores, and the fp32 predictor resolves every configuration.  cfg1-3 draw N(0,1)/sqrt(128)
# keys, whose attention is nearly uniform: blocks that were never selected carry almost identical histories, the
# gaps at the selection boundary go down to 1e-5 of the candidates' spread, and the f16-operand predictor
# (error 2e-3 of the spread) resolves a few percent of the picks the other way.  cfg4's planted structure
# separates the blocks that matter.  Measured: cfg1 4.0 %, cfg2 2.9 %, cfg3 1.2 %, cfg4 0.04 %.
MISMATCH_CEILING = {"cfg0": 0.0, "cfg1": 0.08, "cfg1-fp32": 0.0, "cfg2": 0.06, "cfg3": 0.04, "cfg4": 0.005,
                    "small": 0.01}


def check_stats(name, st, key, rows=None):
    frac = st.report(name)
    if rows is not None:
        assert st.rows == rows
    assert frac <= MISMATCH_CEILING[key], f"{name}: {100 * frac:.2f} % of the picks differ from the float64 selection"
    return frac


def test_lockstep_cfg0_all_steps():
    dev = _dev()
    w = CONFIGS["cfg0"]
    st = lockstep(w, dev, w.steps, sample=[0], fused_every=2)
    check_stats("cfg0 lock-step", st, "cfg0", rows=w.steps)
    assert st.mismatch == 0


def test_lockstep_cfg0_full_tile_predictor():
    dev = _dev()
    w = CONFIGS["cfg0"]
    st = lockstep(w, dev, 10, sample=[0], fused_every=2, incremental=False)
    check_stats("cfg0 lock-step, full-tile predictor", st, "cfg0", rows=10)


def test_lockstep_small_bf16_block_boundary():
    """t crosses a block boundary during the run (nb grows) and calibration fires."""
    dev = _dev()
    w = small("grow", kv_heads=4, g=4, head_dim=128, t0=1020, budget_tokens=256, hist_len=16, steps=12, calib_every=4)
    st = lockstep(w, dev, w.steps, sample=[0, 3])
    check_stats("grow lock-step", st, "small")


@pytest.mark.parametrize("H,c1,c2", [(8, 8, 8), (4, 4, 4)])
def test_lockstep_from_first_token(H, c1, c2):
    """Decoding from an empty context: the first step sees one token and a history of zero rows (the rows that
    are missing early on are zero rows, appendix "Training Details"); the tile grows from one block, and the
    budget of four blocks starts to bind after 32 tokens."""
    dev = _dev()
    w = small("first", kv_heads=2, t0=0, block=8, hist_len=H, budget_tokens=32, n_sink=1, n_local=1, c1=c1, c2=c2,
              steps=60, calib_every=7)
    st = lockstep(w, dev, w.steps, sample=[0, 1], warm=False)
    check_stats("from-first-token lock-step", st, "small", rows=120)


def test_lockstep_many_instances():
    """1040 instances, one workgroup per instance in every kernel."""
    dev = _dev()
    w = small("many", kv_heads=8, batch=130, g=4, head_dim=128, t0=630, budget_tokens=256, hist_len=16, steps=8,
              calib_every=4)
    st = lockstep(w, dev, w.steps, sample=[0, 259, 260, 519, 520, 779, 780, 1039], fused_every=1)
    check_stats("many-instance lock-step", st, "small")


@pytest.mark.parametrize("fp32", [0, 1], ids=["f16-mfma", "fp32"])
def test_lockstep_cfg1_sampled_steps(fp32):
    dev = _dev()
    ap = _ap()
    w = CONFIGS["cfg1"].with_(steps=6, calib_every=3)
    st = lockstep(w, dev, w.steps, sample=[0, 5], flags=ap.AP_FLAG_PREDICTOR_FP32 if fp32 else 0)
    check_stats("cfg1 lock-step, " + ("fp32 predictor" if fp32 else "f16 MFMA predictor"), st,
                "cfg1-fp32" if fp32 else "cfg1", rows=12)


# --------------------------------------------------------------------------------------------- full-size configs
# The configurations of the task at their real sizes, in the launch configuration the bench times
# (fused ap_step, incremental predictor), checked on a sample of instances the oracle can afford.
# Sixteen instances per configuration, spread over the launch: the first and last, and those around multiples
# of the number of workgroups the chip holds at once (256 CUs x 1, 4 or 8).  The steps checked include a
# calibration step, the step on which the predictor state is re-based and the one after it, and (cfg2, cfg4) the
# step on which the context starts a new block, so that the tile grows by a column.
FULLSIZE_SAMPLES = {
    "cfg2": [0, 1, 255, 256, 511, 512, 777, 1023, 1024, 1025, 1279, 1300, 1536, 1791, 2046, 2047],
    "cfg3": [0, 1, 2, 15, 16, 31, 32, 47, 63, 64, 65, 95, 96, 111, 126, 127],
    "cfg4": [0, 1, 255, 256, 1023, 1024, 1025, 1500, 2047, 2048, 2049, 2500, 3071, 3072, 4094, 4095],
}


def _fullsize(name, steps, check, rebase_at):
    dev = _dev()
    w = CONFIGS[name].with_(steps=steps, calib_every=3)
    st = lockstep(w, dev, steps, sample=FULLSIZE_SAMPLES[name], fused_every=1, warm_checks=(-1,), check=set(check),
                  rebase_every=w.hist_len + rebase_at)
    assert st.modes[rebase_at] == 0 and st.modes[rebase_at + 1] == 1     # a re-base, then an advance from it
    check_stats(f"{name} full-size lock-step", st, name, rows=len(check) * 16)


def test_fullsize_cfg2_sampled():
    # t = 32769 + s: block 2050 starts at s = 16
    _fullsize("cfg2", 18, check=[0, 2, 3, 4, 16, 17], rebase_at=3)


def test_fullsize_cfg3_sampled():
    _fullsize("cfg3", 5, check=[0, 2, 3, 4], rebase_at=3)


def test_fullsize_cfg4_sampled():
    _fullsize("cfg4", 18, check=[0, 2, 3, 4, 16, 17], rebase_at=3)


def test_repeated_step_is_bitwise_deterministic():
    """The same call on the same inputs gives the same bytes (split partials are merged in a fixed order)."""
    dev = _dev()
    for kw in (dict(kv_heads=3, t0=3000, budget_tokens=1024), dict(kv_heads=8, batch=130, t0=700, budget_tokens=256)):
        w = small("det", g=4, head_dim=128, hist_len=16, **kw)
        run = _run(w, dev)
        K, V = kv_cache(w, dev)
        for j in range(w.hist_len):
            run.warmup_calibrate(queries(w, j - w.hist_len, dev), K, w.t0 - w.hist_len + 1 + j)
        q = queries(w, 0, dev)
        t = w.t_at(0)
        hist0, n0 = run.hist.clone(), run.n_pushed
        results = []
        for _ in range(3):
            run.hist.copy_(hist0)
            run.n_pushed, run.state_n, run.state_t = n0, None, None
            run.step(q, K, V, t)
            torch.cuda.synchronize()
            results.append((run.out.clone(), run.idx.clone(), run.pred.clone(), run.hist.clone()))
        for r in results[1:]:
            for a, b in zip(results[0], r):
                assert torch.equal(a, b)


# --------------------------------------------------------------------------------------------- paged K/V
def _paged_copy(w, run, K, V, dev, seed=3):
    """Scatters the contiguous caches into one pool of shuffled physical blocks; returns (Kp, Vp, table)."""
    b, nbc = w.block, run.nb_cap
    n_phys = w.n_inst * nbc + 5
    g = torch.Generator(device="cpu").manual_seed(seed)
    perm = torch.randperm(n_phys, generator=g)[: w.n_inst * nbc].to(dev)
    table = perm.view(w.n_inst, nbc).to(torch.int32).contiguous()
    Kp = torch.zeros((n_phys, b, w.head_dim), dtype=K.dtype, device=dev)
    Vp = torch.zeros_like(Kp)
    Kp[perm] = K.view(w.n_inst * nbc, b, w.head_dim)
    Vp[perm] = V.view(w.n_inst * nbc, b, w.head_dim)
    return Kp, Vp, table, n_phys


@pytest.mark.parametrize("kw", [dict(kv_heads=3, t0=3000, budget_tokens=1024), dict(kv_heads=8, batch=130, t0=700),
                                dict(kv_heads=2, g=1, t0=1500, kv_dtype="f32", head_dim=64),
                                # more instances than resident four-wave workgroups: the two-wave, pieced form
                                dict(kv_heads=8, batch=200, t0=1100, budget_tokens=768)],
                         ids=["split", "one-wg-per-instance", "f32", "two-wave"])
def test_paged_kv_equals_contiguous(kw):
    """A block table that scatters the cache over a pool changes addresses only: same bytes out."""
    dev = _dev()
    w = small("paged", hist_len=16, steps=6, calib_every=3, **kw)
    K, V = kv_cache(w, dev)
    ref, pag = _run(w, dev), _run(w, dev)
    Kp, Vp, table, n_phys = _paged_copy(w, pag, K, V, dev)
    pag.ctx.set_block_table(table, n_phys)
    H = w.hist_len
    for j in range(H):
        q, t = queries(w, j - H, dev), w.t0 - H + 1 + j
        ref.warmup_calibrate(q, K, t)
        pag.warmup_calibrate(q, Kp, t)
    assert torch.equal(ref.hist, pag.hist)
    for s in range(w.steps):
        q, t, cal = queries(w, s, dev), w.t_at(s), w.is_calibration_step(s)
        ref.step(q, K, V, t, calibrate=cal)
        pag.step(q, Kp, Vp, t, calibrate=cal)
        torch.cuda.synchronize()
        assert torch.equal(ref.idx, pag.idx) and torch.equal(ref.out, pag.out) and torch.equal(ref.hist, pag.hist)
    # and against the oracle, which sees the gathered contiguous cache
    i = w.n_inst - 1
    got_idx = pag.idx[i, :int(pag.cnt[i])].cpu().numpy()
    o, _ = orc.sparse_attention(to_f64(q[i]), to_f64(K[i]), to_f64(V[i]), got_idx, w.block, t)
    for h in range(w.g):
        assert_close(pag.out[i, h].cpu().numpy(), o[h], f"paged out head {h}")
    pag.ctx.set_block_table(None)
    pag.ctx.sparse_decode(q, K, V, t, pag.idx, pag.cnt, pag.out, pag.row, pag.ws)
    torch.cuda.synchronize()
    assert torch.equal(ref.out, pag.out)


# --------------------------------------------------------------------------------------------- refresh / dense
@pytest.mark.parametrize("k,n_sink,n_local,nb_prev,nb_cur", [
    (64, 4, 4, 2049, 2049), (64, 4, 4, 2049, 2050), (64, 4, 4, 2040, 2047), (16, 1, 2, 70, 71), (16, 0, 1, 16, 17),
    (16, 1, 2, 10, 12), (300, 2, 3, 400, 401), (8, 1, 7, 20, 22), (8, 3, 2, 9, 10),
])
def test_refresh_selection_bit_exact(k, n_sink, n_local, nb_prev, nb_cur):
    dev = _dev()
    ap = _ap()
    n_inst, b = 7, 16
    nb_cap = nb_cur + 3
    ctx = ap.Context(n_inst=n_inst, g=1, head_dim=64, block=b, hist_len=8, t_cap=nb_cap * b, k_blocks=k,
                     n_sink=n_sink, n_local=n_local, c1=4, c2=4, kv_dtype="f32")
    rng = np.random.default_rng(k * 7 + nb_cur)
    idx_h = np.full((n_inst, k), -7, dtype=np.int32)
    cnt_h = np.zeros(n_inst, dtype=np.int32)
    prev = []
    for i in range(n_inst):
        s0 = orc.select_blocks(rng.standard_normal(nb_prev), nb_prev, k, n_sink, n_local)
        prev.append(s0)
        idx_h[i, :len(s0)] = s0
        cnt_h[i] = len(s0)
    idx = torch.from_numpy(idx_h).to(dev)
    cnt = torch.from_numpy(cnt_h).to(dev)
    ctx.refresh_selection(nb_prev, nb_cur, idx, cnt)
    torch.cuda.synchronize()
    got_idx, got_cnt = idx.cpu().numpy(), cnt.cpu().numpy()
    for i in range(n_inst):
        exp = orc.refresh_selection(prev[i], nb_prev, nb_cur, k, n_sink, n_local)
        assert got_cnt[i] == len(exp)
        assert got_idx[i, :got_cnt[i]].tolist() == exp.tolist(), f"instance {i}"


@pytest.mark.parametrize("every", [4, 16])
def test_lockstep_refresh_interval(every):
    """The selection is re-made on every 4th (16th) step only; in between it is carried over while the context
    grows across block boundaries.  Every step against the oracle told to do the same.  With the long interval
    the predictor is left out in between and evaluates the full tile when a selection is due."""
    dev = _dev()
    w = small("refresh", kv_heads=3, g=4, head_dim=128, t0=1015, budget_tokens=256, hist_len=16, steps=40, calib_every=8)
    run = _run(w, dev)
    run.refresh_every = every
    predicts_always = every < run.skip_predictor_from
    K, V = kv_cache(w, dev)
    wts = orc.PredictorWeights.from_blob(predictor_weights(w), w.c1, w.c2)
    H, b = w.hist_len, w.block
    Kc = [to_f64(K[i]) for i in range(w.n_inst)]
    Vc = [to_f64(V[i]) for i in range(w.n_inst)]
    for j in range(H):
        run.warmup_calibrate(queries(w, j - H, dev), K, w.t0 - H + 1 + j)
    last = [None] * w.n_inst
    carried = 0
    for s in range(w.steps):
        t = w.t_at(s)
        nb = run.nb(t)
        q = queries(w, s, dev)
        calib = w.is_calibration_step(s)
        selects = run.selects_now(t)
        before = run.logical_history().cpu().numpy().astype(np.float64)
        if s % 2 == 0:
            run.step(q, K, V, t, calibrate=calib)
        else:
            run.step_unfused(q, K, V, t, calibrate=calib)
        torch.cuda.synchronize()
        after = run.logical_history().cpu().numpy()
        pred, idx, cnt, out = (x.cpu().numpy() for x in (run.pred, run.idx, run.cnt, run.out))
        for i in range(w.n_inst):
            qi = to_f64(q[i])
            if selects or predicts_always:                 # an advancing state stays current on every step
                assert_close(pred[i, :nb].astype(np.float64) + run.ctx.score_offset(), orc.predict(before[i], nb, wts),
                             f"step {s} inst {i} pred")
            got_idx = idx[i, :cnt[i]]
            if selects:
                exp_idx = orc.select_blocks(pred[i, :nb].astype(np.float64), nb, w.k_blocks, w.n_sink, w.n_local)
            else:
                exp_idx = orc.refresh_selection(last[i][0], last[i][1], nb, w.k_blocks, w.n_sink, w.n_local)
                carried += 1
            assert got_idx.tolist() == exp_idx.tolist(), f"step {s} inst {i}: selection differs (selects={selects})"
            last[i] = (got_idx.copy(), nb)
            ref = orc.decode_step(before[i], qi, Kc[i], Vc[i], t, wts, b=b, k=w.k_blocks, n_sink=w.n_sink,
                                  n_local=w.n_local, calibrate=calib, reuse=None if selects else (got_idx, nb))
            if not selects:
                assert ref.blocks.tolist() == got_idx.tolist()
                for h in range(w.g):
                    assert_close(out[i, h], ref.out[h], f"step {s} inst {i} head {h} out")
                row = np.zeros(run.nb_cap)
                row[:nb] = ref.row
                assert_close(after[i, H - 1], row, f"step {s} inst {i} pushed row")
            else:
                ref_out, A = orc.sparse_attention(qi, Kc[i], Vc[i], got_idx, b, t)
                for h in range(w.g):
                    assert_close(out[i, h], ref_out[h], f"step {s} inst {i} head {h} out")
    assert carried == w.n_inst * (w.steps - (w.steps + every - 1) // every)


def test_dense_layers_match_dense_attention():
    """A budget of all blocks through the same kernels: attention over the whole context (32 splits per instance)."""
    dev = _dev()
    from paper_2502_04077_amd.runner import DenseRun
    w = small("dense", layers=2, batch=1, kv_heads=2, g=4, head_dim=128, t0=9000, budget_tokens=256, hist_len=16, steps=3)
    K, V = kv_cache(w, dev)
    run = DenseRun(w, 2, dev)
    for s in range(w.steps):
        t = w.t_at(s)
        q = queries(w, s, dev)
        run.step(q, K, V, t)
        torch.cuda.synchronize()
        out = run.out.cpu().numpy()
        nb = (t + w.block - 1) // w.block
        for i in (0, w.n_inst - 1):
            ref_out, A = orc.sparse_attention(to_f64(q[i]), to_f64(K[i]), to_f64(V[i]), np.arange(nb), w.block, t)
            for h in range(w.g):
                assert_close(out[i, h], ref_out[h], f"step {s} inst {i} head {h}")
            assert_close(run.row[i, :nb].cpu().numpy(), orc.dense_row(to_f64(q[i]), to_f64(K[i]), w.block, t), "dense row")
