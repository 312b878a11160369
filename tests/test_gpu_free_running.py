"""Free-running parity on cfg4-shaped (planted) data: the GPU path and the oracle each run the same 56 decode
steps from their own warm-up, never re-synchronised.  The oracle's trajectory owes nothing to the GPU: its
history warm-up, scores, selections, attention and pushed rows are all its own float64 work.

What is asserted:
  * as long as the two selections have agreed on every earlier step, the two histories hold the same rows up to
    rounding; on the first step where an instance's selection differs, every swapped pair of blocks must lie
    within twice the score error of that step (oracle[y] - oracle[x] <= 2 max|gpu - oracle| over the candidate
    blocks): a divergence that is not a near tie resolved differently would be a wrong selection.  Target: none;
  * until then pred, out and the pushed row agree within the 1e-3 bar.
What is reported: per instance the first diverging step (if any), the overlap of the two selections per step,
and the recovery rate R_rec (Eq. 1) of each selection against the dense attention of that step.
Both predictors are run: the seeded random weights of the workload, and the centre-tap weights whose prediction
is the windowed mean of the history (well separated scores on this data).
"""
import numpy as np
import pytest
import torch

from oracle import attnpred_oracle as orc
from workloads import CONFIGS, kv_cache, n_weight_floats, predictor_weights, queries, to_f64

pytestmark = pytest.mark.gpu

STEPS = 56


def _delta_blob(c1, c2):
    w = orc.PredictorWeights.from_blob(np.zeros(n_weight_floats(c1, c2)), c1, c2)
    w.w1[0, 1, 1] = w.w2[0, 0, 1, 1] = w.w3[0] = 1.0
    return np.concatenate([w.w1.ravel(), w.b1, w.w2.ravel(), w.b2, w.w3, [w.b3]]).astype(np.float32)


def _free_run(w, blob, dev, name):
    from paper_2502_04077_amd.runner import DecodeRun
    run = DecodeRun(w, dev)
    run.set_weights(blob)
    wts = orc.PredictorWeights.from_blob(blob, w.c1, w.c2)
    K, V = kv_cache(w, dev)
    H, b, k = w.hist_len, w.block, w.k_blocks
    n = w.n_inst
    Kc = [to_f64(K[i]) for i in range(n)]
    Vc = [to_f64(V[i]) for i in range(n)]
    # warm-up on both sides, each from the same seeded queries: the last H prefill steps as dense rows
    hist = [np.zeros((H, w.nb_cap)) for _ in range(n)]
    for j in range(H):
        t = w.t0 - H + 1 + j
        q = queries(w, j - H, dev)
        run.warmup_calibrate(q, K, t)
        for i in range(n):
            hist[i] = orc.history_push(hist[i], orc.dense_row(to_f64(q[i]), Kc[i], b, t))
    first_div = [None] * n
    unexplained = []
    overlap = np.zeros((STEPS, n))
    rrec = np.zeros((STEPS, n, 2))
    worst = dict(pred=0.0, out=0.0, row=0.0)
    for s in range(STEPS):
        t = w.t_at(s)
        nb = run.nb(t)
        q = queries(w, s, dev)
        calib = w.is_calibration_step(s)
        run.step(q, K, V, t, calibrate=calib)
        torch.cuda.synchronize()
        g_pred, g_idx, g_cnt = run.pred.cpu().numpy(), run.idx.cpu().numpy(), run.cnt.cpu().numpy()
        g_out = run.out.cpu().numpy()
        g_row = run.logical_history()[:, H - 1].cpu().numpy()
        for i in range(n):
            qi = to_f64(q[i])
            ref = orc.decode_step(hist[i], qi, Kc[i], Vc[i], t, wts, b=b, k=k, n_sink=w.n_sink, n_local=w.n_local,
                                  calibrate=calib)
            hist[i] = ref.hist
            got = g_idx[i, :g_cnt[i]]
            same = got.tolist() == ref.blocks.tolist()
            overlap[s, i] = len(set(got.tolist()) & set(ref.blocks.tolist())) / len(ref.blocks)
            A = orc.attention_scores(qi, Kc[i][:t], np.arange(t)).mean(axis=0)
            rrec[s, i, 0] = orc.recovery_rate(A, orc.expand_blocks(got, b, t))
            rrec[s, i, 1] = orc.recovery_rate(A, orc.expand_blocks(ref.blocks, b, t))
            if first_div[i] is not None:
                continue                                   # the trajectories have parted: nothing to hold them to
            gp = g_pred[i, :nb].astype(np.float64) + run.ctx.score_offset()   # pred is relative to that constant
            err_all = np.abs(gp - ref.pred).max()
            assert err_all <= 1e-3 * np.abs(ref.pred).max(), f"{name} step {s} inst {i}: pred off by {err_all:.3e}"
            worst["pred"] = max(worst["pred"], err_all / np.abs(ref.pred).max())
            if not same:
                first_div[i] = s
                cand = slice(w.n_sink, nb - w.n_local)
                err = np.abs(gp[cand] - ref.pred[cand]).max()
                a = sorted(set(got.tolist()) - set(ref.blocks.tolist()))
                bb = sorted(set(ref.blocks.tolist()) - set(got.tolist()))
                gap = max(ref.pred[y] - ref.pred[x] for x in a for y in bb)
                if not gap <= 2 * err:
                    unexplained.append((i, s, gap, err))
                continue
            for h in range(w.g):
                e = np.abs(g_out[i, h] - ref.out[h]).max() / np.abs(ref.out[h]).max()
                assert e <= 1e-3, f"{name} step {s} inst {i} head {h}: out off by {e:.3e}"
                worst["out"] = max(worst["out"], e)
            e = np.abs(g_row[i, :nb] - ref.row).max() / np.abs(ref.row).max()
            assert e <= 1e-3, f"{name} step {s} inst {i}: pushed row off by {e:.3e}"
            worst["row"] = max(worst["row"], e)
    print(f"{name}: first diverging step per instance {first_div}; unexplained divergences {len(unexplained)}")
    print(f"{name}: worst relative error while in step: pred {worst['pred']:.2e}, out {worst['out']:.2e}, "
          f"row {worst['row']:.2e}")
    print(f"{name}: selection overlap per step (mean over instances), steps 0..{STEPS - 1}: "
          + " ".join(f"{x:.2f}" for x in overlap.mean(axis=1)))
    print(f"{name}: R_rec (Eq. 1) mean over steps and instances: GPU selection {rrec[..., 0].mean():.4f}, "
          f"oracle selection {rrec[..., 1].mean():.4f}, ratio {rrec[..., 0].mean() / rrec[..., 1].mean():.4f}")
    del run, K, V
    torch.cuda.empty_cache()
    return first_div, unexplained, overlap, rrec


@pytest.mark.parametrize("weights", ["windowed-mean", "random"])
def test_free_running_cfg4_shaped(weights):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    dev = torch.device("cuda:0")
    w = CONFIGS["cfg4"].with_(layers=1, batch=1, kv_heads=4, steps=STEPS, calib_every=8)
    blob = _delta_blob(w.c1, w.c2) if weights == "windowed-mean" else predictor_weights(w)
    first_div, unexplained, overlap, rrec = _free_run(w, blob, dev, f"free-running cfg4-shaped, {weights} predictor")
    assert not unexplained, f"divergences that are not near ties: {unexplained}"
    # two runs that part over a near tie keep recovering the same attention mass
    ratio = rrec[..., 0].mean() / rrec[..., 1].mean()
    assert 0.97 <= ratio <= 1.03, f"R_rec of the GPU's selections is {ratio:.4f} of the oracle's"
