"""K/V cache in pinned host memory with cross-token prefetching (Sec. 3.4): the staged-pool path must give
what the oracle gives for the same step - the transfer schedule changes where the bytes are, not the result."""
import numpy as np
import pytest
import torch

import oracle.attnpred_oracle as orc
from workloads import kv_cache, predictor_weights, queries, to_f64

from test_gpu_parity import ScoreStats, _ap, _dev, assert_close, check_stats, small

pytestmark = pytest.mark.gpu


def _pinned(x):
    h = torch.empty(x.shape, dtype=x.dtype, pin_memory=True)
    h.copy_(x)
    return h


def _expected_block(K, i, blk, b, t_avail):
    e = K[i, blk * b:(blk + 1) * b].clone()
    e[max(0, min(b, t_avail - blk * b)):] = 0          # rows of tokens >= t_avail are staged as zeros
    return e


@pytest.mark.parametrize("src", ["pinned", "device"])
@pytest.mark.parametrize("dtype,d,b", [("bf16", 128, 16), ("f32", 64, 8), ("bf16", 64, 32)])
def test_prefetch_blocks_and_append(src, dtype, d, b):
    """Two selections in a row: slots, block table, zero-filled future rows, the appended row, and that a block
    which stays selected is neither moved nor fetched again - all bit for bit."""
    dev = _dev()
    ap = _ap()
    n_inst, k, nb_cap = 5, 6, 40
    t_cap = nb_cap * b
    ctx = ap.Context(n_inst=n_inst, g=1, head_dim=d, block=b, hist_len=8, t_cap=t_cap, k_blocks=k, n_sink=1,
                     n_local=1, c1=4, c2=4, kv_dtype=dtype)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    g = torch.Generator(device="cpu").manual_seed(5)
    K = torch.randn((n_inst, t_cap, d), generator=g).to(tdt)
    V = torch.randn((n_inst, t_cap, d), generator=g).to(tdt)
    Ks, Vs = (_pinned(K), _pinned(V)) if src == "pinned" else (K.to(dev), V.to(dev))
    rng = np.random.default_rng(11)
    pool_K = torch.full((n_inst * k, b, d), 9.0, dtype=tdt, device=dev)
    pool_V = torch.full((n_inst * k, b, d), 9.0, dtype=tdt, device=dev)
    table = torch.full((n_inst, nb_cap), -1, dtype=torch.int32, device=dev)
    state = torch.zeros((ctx.prefetch_state_bytes() // 4,), dtype=torch.int32, device=dev)
    stride = 3 * k + 4
    assert state.numel() == n_inst * stride

    def make_selection(nb, cnt_h, keep_from=None):
        idx_h = np.full((n_inst, k), -7, dtype=np.int32)
        for i in range(n_inst):
            c = cnt_h[i]
            if not c:
                continue
            kept = [] if keep_from is None else [x for x in keep_from[i] if x >= 0 and x < nb - 1][:c // 2]
            rest = [x for x in range(nb - 1) if x not in kept]
            pick = list(rng.choice(rest, size=c - 1 - len(kept), replace=False))
            idx_h[i, :c] = np.array(sorted(kept + pick) + [nb - 1], dtype=np.int32)
        return idx_h

    holds = {}                                            # (inst, block) -> slot, as the test expects it
    content = {}                                          # (inst, block) -> (K block, V block) expected in the pool
    total_fetched = np.zeros(n_inst, dtype=np.int64)
    prev_idx = None
    for call, t_next in enumerate([29 * b + 3, 29 * b + 4, 30 * b + 1]):   # the last one opens a new block
        nb = (t_next + b - 1) // b
        cnt_h = np.array([k, k, k - 2, 0, k], dtype=np.int32)
        idx_h = make_selection(nb, cnt_h, prev_idx)
        if call == 0:
            idx_h[4, cnt_h[4] - 1] = nb - 2               # instance 4 leaves out the newest block: nothing is appended
        prev_idx = idx_h
        idx = torch.from_numpy(idx_h).to(dev)
        cnt = torch.from_numpy(cnt_h).to(dev)
        ctx.prefetch_blocks(Ks, Vs, t_next - 1, nb, idx, cnt, pool_K, pool_V, table, state)
        k_new = K[:, t_next - 1, :].contiguous().to(dev)
        v_new = V[:, t_next - 1, :].contiguous().to(dev)
        ctx.append_kv(k_new, v_new, t_next - 1, table, state, pool_K, pool_V)
        torch.cuda.synchronize()
        pk, pv, tb = pool_K.cpu(), pool_V.cpu(), table.cpu().numpy()
        st = state.cpu().numpy().reshape(n_inst, stride)
        for i in range(n_inst):
            sel = [int(x) for x in idx_h[i, :cnt_h[i]]]
            old = {blk: sl for (ii, blk), sl in holds.items() if ii == i}
            misses = [blk for blk in sel if blk not in old]
            total_fetched[i] += len(misses)
            assert st[i, 3 * k] == len(misses) and st[i, 3 * k + 1] == total_fetched[i], f"call {call} inst {i}"
            slots = []
            for blk in sel:
                sl = tb[i, blk] - i * k
                assert 0 <= sl < k and st[i, sl] == blk + 1, f"call {call} inst {i} block {blk}: bad slot"
                if blk in old:
                    assert sl == old[blk], "a block that stayed selected was moved"
                else:
                    content[(i, blk)] = (_expected_block(K, i, blk, b, t_next - 1), _expected_block(V, i, blk, b, t_next - 1))
                slots.append(sl)
            assert len(set(slots)) == len(slots), "two selected blocks share a slot"
            for blk in list(old):                         # blocks whose slot was taken over are gone
                if st[i, old[blk]] != blk + 1:
                    del holds[(i, blk)]
            for blk, sl in zip(sel, slots):
                holds[(i, blk)] = sl
            if (t_next - 1) // b in sel:                  # the appended row
                ek, ev = content[(i, (t_next - 1) // b)]
                ek[(t_next - 1) % b] = K[i, t_next - 1]
                ev[(t_next - 1) % b] = V[i, t_next - 1]
            for blk, sl in zip(sel, slots):
                ek, ev = content[(i, blk)]
                assert torch.equal(pk[i * k + sl].view(torch.uint8), ek.view(torch.uint8)), f"call {call} K inst {i} block {blk}"
                assert torch.equal(pv[i * k + sl].view(torch.uint8), ev.view(torch.uint8)), f"call {call} V inst {i} block {blk}"
        assert torch.all(pk[3 * k:4 * k] == 9.0), "an instance with an empty selection was written"
    assert total_fetched[0] < 3 * k, "nothing was re-used across the three selections"
    # zeroing the state empties the cache: the same selection is fetched in full again
    state.zero_()
    ctx.prefetch_blocks(Ks, Vs, t_next - 1, nb, idx, cnt, pool_K, pool_V, table, state)
    torch.cuda.synchronize()
    st = state.cpu().numpy().reshape(n_inst, stride)
    assert st[:, 3 * k].tolist() == cnt_h.tolist()


def test_prefetch_refuses_pageable_host_memory():
    dev = _dev()
    ap = _ap()
    ctx = ap.Context(n_inst=1, g=1, head_dim=64, block=16, hist_len=8, t_cap=64, k_blocks=2, n_sink=1, n_local=1,
                     c1=4, c2=4, kv_dtype="f32")
    pageable = torch.zeros((1, 64, 64))
    idx = torch.zeros((1, 2), dtype=torch.int32, device=dev)
    cnt = torch.zeros((1,), dtype=torch.int32, device=dev)
    pool = torch.zeros((2, 16, 64), device=dev)
    table = torch.zeros((1, 4), dtype=torch.int32, device=dev)
    state = torch.zeros((ctx.prefetch_state_bytes() // 4,), dtype=torch.int32, device=dev)
    lib = ap.load_library()
    rc = lib.ap_prefetch_blocks(ctx._h, pageable.data_ptr(), pageable.data_ptr(), 10, 1, idx.data_ptr(), cnt.data_ptr(),
                                pool.data_ptr(), pool.data_ptr(), table.data_ptr(), state.data_ptr(), None)
    assert rc == ap.AP_ERR_ARG


def test_cache_pointer_is_checked_on_every_call():
    """A cache pointer that was accepted once earns nothing: the same context is handed pinned memory (accepted),
    then pageable memory (refused), then the pinned buffer again (accepted), then - after that buffer has been
    released - pageable memory once more (refused).  Every refusal happens on the host, before any launch."""
    dev = _dev()
    ap = _ap()
    ctx = ap.Context(n_inst=1, g=1, head_dim=64, block=16, hist_len=8, t_cap=64, k_blocks=2, n_sink=1, n_local=1,
                     c1=4, c2=4, kv_dtype="f32")
    lib = ap.load_library()
    q = torch.zeros((1, 1, 64), device=dev)
    row = torch.zeros((1, ctx.nb_cap()), device=dev)
    ws = torch.zeros((max(16, ctx.workspace_bytes()),), dtype=torch.uint8, device=dev)

    def calibrate(K):
        return lib.ap_calibrate(ctx._h, q.data_ptr(), K.data_ptr(), 40, row.data_ptr(), ws.data_ptr(), None)

    pinned = torch.zeros((1, 64, 64), pin_memory=True)
    pageable = torch.zeros((1, 64, 64))
    assert calibrate(pinned) == ap.AP_OK
    assert calibrate(pageable) == ap.AP_ERR_ARG
    assert calibrate(pinned) == ap.AP_OK
    torch.cuda.synchronize()
    del pinned
    assert calibrate(pageable) == ap.AP_ERR_ARG
    on_device = torch.zeros((1, 64, 64), device=dev)
    assert calibrate(on_device) == ap.AP_OK
    torch.cuda.synchronize()


@pytest.mark.parametrize("single_calls", [False, True])
def test_offload_lockstep_vs_oracle(single_calls):
    """Every step of the prefetching schedule against the oracle started from the GPU's own history; once through
    ap_offload_begin / ap_offload_step, once composed from the single calls."""
    dev = _dev()
    from paper_2502_04077_amd.offload import OffloadRun
    w = small("offload", layers=3, batch=1, kv_heads=2, g=4, head_dim=128, t0=1010, budget_tokens=256, hist_len=16,
              steps=40, calib_every=8)
    K, V = kv_cache(w, dev)
    K_host, V_host = _pinned(K), _pinned(V)
    run = OffloadRun(w, K_host, V_host, dev, rebase_every=24, single_calls=single_calls)
    blob = predictor_weights(w)
    run.set_weights(blob)
    wts = orc.PredictorWeights.from_blob(blob, w.c1, w.c2)
    H, b = w.hist_len, w.block
    Kc = [to_f64(K[i]) for i in range(w.n_inst)]
    Vc = [to_f64(V[i]) for i in range(w.n_inst)]
    for j in range(H):
        run.warmup_calibrate(queries(w, j - H, dev), w.t0 - H + 1 + j)
    run.start(w.t_at(0))
    stats = ScoreStats()
    off = run.score_offset()
    for s in range(w.steps):
        t = w.t_at(s)
        nb = run.nb(t)
        q = queries(w, s, dev)
        calib = w.is_calibration_step(s)
        torch.cuda.synchronize()
        before = run.logical_history().cpu().numpy().astype(np.float64)
        pred, idx, cnt = (x.cpu().numpy() for x in run.staged_selection())
        run.step(q, K[:, t - 1, :].contiguous(), V[:, t - 1, :].contiguous(), t, calibrate=calib)
        torch.cuda.synchronize()
        after = run.logical_history().cpu().numpy()
        out = run.out().cpu().numpy()
        for i in range(w.n_inst):
            qi = to_f64(q[i])
            ref_pred = orc.predict(before[i], nb, wts)
            assert_close(pred[i, :nb].astype(np.float64) + off, ref_pred, f"step {s} inst {i} pred")
            got_idx = idx[i, :cnt[i]]
            exp_idx = orc.select_blocks(pred[i, :nb].astype(np.float64), nb, w.k_blocks, w.n_sink, w.n_local)
            assert got_idx.tolist() == exp_idx.tolist(), f"step {s} inst {i}: selection differs"
            stats.add(f"step {s} inst {i}", pred[i, :nb].astype(np.float64) + off, ref_pred, got_idx, nb, w.k_blocks,
                      w.n_sink, w.n_local)
            ref_out, A = orc.sparse_attention(qi, Kc[i], Vc[i], got_idx, b, t)
            for h in range(w.g):
                assert_close(out[i, h], ref_out[h], f"step {s} inst {i} head {h} out")
            ref_row = np.zeros(run.nb_cap)
            ref_row[:nb] = orc.dense_row(qi, Kc[i], b, t) if calib else orc.pooled_row(A, b)
            assert_close(after[i, H - 1], ref_row, f"step {s} inst {i} pushed row")
            assert np.array_equal(after[i, :H - 1], before[i, 1:].astype(np.float32)), "history did not shift"
    run.finish()
    check_stats("offload lock-step", stats, "small", rows=w.steps * w.n_inst)
