"""K/V cache in pinned host memory with cross-token prefetching (Sec. 3.4): the staged-pool path must give
what the oracle gives for the same step - the transfer schedule changes where the bytes are, not the result."""
import numpy as np
import pytest
import torch

import oracle.attnpred_oracle as orc
from workloads import kv_cache, predictor_weights, queries, to_f64

from test_gpu_parity import TIE_MARGIN, _ap, _dev, assert_close, small

pytestmark = pytest.mark.gpu


def _pinned(x):
    h = torch.empty(x.shape, dtype=x.dtype, pin_memory=True)
    h.copy_(x)
    return h


@pytest.mark.parametrize("src", ["pinned", "device"])
@pytest.mark.parametrize("dtype,d,b", [("bf16", 128, 16), ("f32", 64, 8), ("bf16", 64, 32)])
def test_prefetch_blocks_and_append(src, dtype, d, b):
    """Pool slots, block table, zero-filled future rows and the appended row, bit for bit."""
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
    t_next = 29 * b + 3                       # context length the selection is for; its token has index t_next - 1
    nb = (t_next + b - 1) // b
    rng = np.random.default_rng(11)
    idx_h = np.full((n_inst, k), -7, dtype=np.int32)
    cnt_h = np.array([k, k, k - 2, 0, k], dtype=np.int32)
    for i in range(n_inst):
        c = cnt_h[i]
        if c:
            pick = np.sort(rng.choice(nb - 1, size=c - 1, replace=False))
            idx_h[i, :c] = np.concatenate([pick, [nb - 1]])
    idx_h[4, cnt_h[4] - 1] = nb - 2           # instance 4 does not select the newest block: nothing is appended
    idx = torch.from_numpy(idx_h).to(dev)
    cnt = torch.from_numpy(cnt_h).to(dev)
    pool_K = torch.full((n_inst * k, b, d), 9.0, dtype=tdt, device=dev)
    pool_V = torch.full((n_inst * k, b, d), 9.0, dtype=tdt, device=dev)
    table = torch.full((n_inst, nb_cap), -1, dtype=torch.int32, device=dev)
    ctx.prefetch_blocks(Ks, Vs, t_next - 1, nb, idx, cnt, pool_K, pool_V, table)
    k_new = K[:, t_next - 1, :].contiguous().to(dev)
    v_new = V[:, t_next - 1, :].contiguous().to(dev)
    ctx.append_kv(k_new, v_new, t_next - 1, idx, cnt, pool_K, pool_V)
    torch.cuda.synchronize()
    pk, pv, tb = pool_K.cpu(), pool_V.cpu(), table.cpu().numpy()
    exp_table = np.full((n_inst, nb_cap), -1, dtype=np.int32)
    for i in range(n_inst):
        for p in range(k):
            slot = i * k + p
            if p >= cnt_h[i]:
                assert torch.all(pk[slot] == 9.0) and torch.all(pv[slot] == 9.0), "slot beyond cnt was written"
                continue
            blk = idx_h[i, p]
            exp_table[i, blk] = slot
            ek = K[i, blk * b:(blk + 1) * b].clone()
            ev = V[i, blk * b:(blk + 1) * b].clone()
            first_missing = max(0, min(b, (t_next - 1) - blk * b))      # rows of tokens >= t_avail
            ek[first_missing:] = 0
            ev[first_missing:] = 0
            if blk == nb - 1 and p == cnt_h[i] - 1:                      # the appended row
                r = (t_next - 1) % b
                ek[r] = K[i, t_next - 1]
                ev[r] = V[i, t_next - 1]
            assert torch.equal(pk[slot].view(torch.uint8), ek.view(torch.uint8)), f"K inst {i} pos {p}"
            assert torch.equal(pv[slot].view(torch.uint8), ev.view(torch.uint8)), f"V inst {i} pos {p}"
    assert np.array_equal(tb, exp_table)


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
    lib = ap.load_library()
    rc = lib.ap_prefetch_blocks(ctx._h, pageable.data_ptr(), pageable.data_ptr(), 10, 1, idx.data_ptr(), cnt.data_ptr(),
                                pool.data_ptr(), pool.data_ptr(), table.data_ptr(), None)
    assert rc == ap.AP_ERR_ARG


def test_offload_lockstep_vs_oracle():
    """Every step of the prefetching schedule against the oracle started from the GPU's own history."""
    dev = _dev()
    from paper_2502_04077_amd.offload import OffloadRun
    w = small("offload", layers=3, batch=1, kv_heads=2, g=4, head_dim=128, t0=1010, budget_tokens=256, hist_len=16,
              steps=40, calib_every=8)
    K, V = kv_cache(w, dev)
    K_host, V_host = _pinned(K), _pinned(V)
    run = OffloadRun(w, K_host, V_host, dev, rebase_every=24)
    blob = predictor_weights(w)
    run.set_weights(blob)
    wts = orc.PredictorWeights.from_blob(blob, w.c1, w.c2)
    H, b = w.hist_len, w.block
    Kc = [to_f64(K[i]) for i in range(w.n_inst)]
    Vc = [to_f64(V[i]) for i in range(w.n_inst)]
    for j in range(H):
        run.warmup_calibrate(queries(w, j - H, dev), w.t0 - H + 1 + j)
    run.start(w.t_at(0))
    near_ties = 0
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
            assert_close(pred[i, :nb], ref_pred, f"step {s} inst {i} pred")
            got_idx = idx[i, :cnt[i]]
            exp_idx = orc.select_blocks(pred[i, :nb].astype(np.float64), nb, w.k_blocks, w.n_sink, w.n_local)
            assert got_idx.tolist() == exp_idx.tolist(), f"step {s} inst {i}: selection differs"
            o_idx = orc.select_blocks(ref_pred, nb, w.k_blocks, w.n_sink, w.n_local)
            a = sorted(set(got_idx.tolist()) - set(o_idx.tolist()))
            bb = sorted(set(o_idx.tolist()) - set(got_idx.tolist()))
            if a:
                near_ties += len(a)
                gap = max(abs(ref_pred[x] - ref_pred[y]) for x in a for y in bb)
                assert gap <= TIE_MARGIN * np.abs(ref_pred).max()
            ref_out, A = orc.sparse_attention(qi, Kc[i], Vc[i], got_idx, b, t)
            for h in range(w.g):
                assert_close(out[i, h], ref_out[h], f"step {s} inst {i} head {h} out")
            ref_row = np.zeros(run.nb_cap)
            ref_row[:nb] = orc.dense_row(qi, Kc[i], b, t) if calib else orc.pooled_row(A, b)
            assert_close(after[i, H - 1], ref_row, f"step {s} inst {i} pushed row")
            assert np.array_equal(after[i, :H - 1], before[i, 1:].astype(np.float32)), "history did not shift"
    run.finish()
    print("offload lock-step: swaps against float64 scores (near ties):", near_ties)
