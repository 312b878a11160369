"""The fused step and the calibration call under HIP graph capture.

After the first attention call of a context (which asks the runtime for occupancy figures on the host) the
library only launches kernels: no allocation, no memset node, no host synchronisation.  A captured step must
therefore replay to the same bytes as the eager call, on every replay, with other work of the program and
synchronisations in between.  The step is taken in re-base mode, which recomputes the predictor state from the
history, so that replaying it is idempotent (the pushed row lands in the same ring slot each time)."""
import pytest
import torch

from workloads import Workload, kv_cache, predictor_weights, queries

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("kw", [dict(kv_heads=3, t0=3000, budget_tokens=1024),        # split attention + combine
                                dict(kv_heads=8, batch=130, t0=700, budget_tokens=256)])   # one workgroup per instance
def test_step_and_calibration_replay_from_a_graph(kw):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    dev = torch.device("cuda:0")
    from paper_2502_04077_amd.runner import DecodeRun
    from paper_2502_04077_amd.binding import AP_PRED_REBASE
    base = dict(name="graph", layers=1, batch=1, kv_heads=3, g=4, head_dim=128, kv_dtype="bf16", t0=1000, block=16,
                hist_len=16, budget_tokens=256, n_sink=1, n_local=2, c1=8, c2=8, steps=8, calib_every=4, seed=11,
                value_scale=1.0)
    base.update(kw)
    w = Workload(**base)
    run = DecodeRun(w, dev)
    run.set_weights(predictor_weights(w))
    K, V = kv_cache(w, dev)
    for j in range(w.hist_len):
        run.warmup_calibrate(queries(w, j - w.hist_len, dev), K, w.t0 - w.hist_len + 1 + j)
    run.step(queries(w, 0, dev), K, V, w.t_at(0))          # the first calls of the context happen outside any capture
    q, t = queries(w, 1, dev), w.t_at(1)
    hist0, n0 = run.hist.clone(), run.n_pushed
    dense_row = torch.zeros_like(run.row)

    def call():
        run.ctx.step(run.hist, n0, q, K, V, t, run.out, run.idx, run.cnt, run.pred, run.pstate, AP_PRED_REBASE, run.ws)
        run.ctx.calibrate(q, K, t, dense_row, run.ws)

    nb = run.nb(t)                                         # columns past the context's blocks are not written

    def snapshot():
        torch.cuda.synchronize()
        return [x.clone() for x in (run.out, run.idx, run.cnt, run.pred[:, :nb], run.pstate[:, :nb], run.hist[..., :nb],
                                    dense_row[:, :nb])]

    call()
    want = snapshot()

    side = torch.cuda.Stream()                             # (default priority)
    graph = torch.cuda.CUDAGraph()
    run.hist.copy_(hist0)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        call()
    for replay in range(3):
        # the program's own eager work between replays: scribble over every output, restore the history
        for x in (run.out, run.pred, run.pstate, dense_row):
            x.fill_(float(replay + 7))
        run.idx.fill_(-1)
        run.cnt.fill_(-1)
        run.hist.copy_(hist0)
        other = (K[0, :64].float() @ K[0, :64].float().T).sum()      # unrelated library work
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        assert torch.isfinite(other)
        for name, a, b in zip(("out", "idx", "cnt", "pred", "pstate", "hist", "dense row"), want, got):
            assert torch.equal(a, b), f"replay {replay}: {name} differs from the eager call"
