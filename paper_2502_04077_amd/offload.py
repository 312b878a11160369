"""Call sequencing for a K/V cache kept in pinned host memory with cross-token prefetching (Sec. 3.4 and the
timeline figure of the appendix): device buffers, streams and events only, no arithmetic of the method.

Per layer (one context per layer, as a model would own them) and decode step:

  compute stream   wait(staged) -> append the new token's K/V row to its staged block -> sparse decode over the
                   staged pool -> [calibrate from the host-resident K] -> push -> predict + select for the NEXT
                   token -> record(selected)
  copy stream      wait(selected) -> gather the next token's blocks from host memory into the pool -> record(staged)

so the transfer for layer l's next token runs while the layers after l (and, in the next step, the layers
before l) compute.  The selection for token t+1 needs the pooled row of token t, hence one pool per layer is
enough: its gather can only start after the decode that read the pool.
"""
from __future__ import annotations

import torch

from .binding import AP_PRED_ADVANCE, AP_PRED_REBASE, Context, _check, _ptr, _rptr, load_library


class _Layer:
    pass


class OffloadRun:
    def __init__(self, w, K_host, V_host, device="cuda:0", rebase_every=512, flags=0, single_calls=False):
        """w: Workload; K_host, V_host: pinned host tensors [n_inst][t_cap][d] (instances layer-major).
        single_calls: compose every layer step from the single C calls here instead of ap_offload_step."""
        if w.n_local < 1:
            raise ValueError("the newest block must be a forced local block (n_local >= 1)")
        if not (K_host.is_pinned() and V_host.is_pinned()):
            raise ValueError("K_host and V_host must be pinned host tensors")
        self.w = w
        self.dev = torch.device(device)
        self.ipl = w.batch * w.kv_heads                     # instances per layer
        self.rebase_every = rebase_every
        self.single_calls = single_calls
        self.copy_stream = torch.cuda.Stream(device=self.dev)
        self.K_host, self.V_host = K_host, V_host
        self.n_pushed = 0
        self.layers = []
        f32, i32 = torch.float32, torch.int32
        for l in range(w.layers):
            L = _Layer()
            L.ctx = Context(n_inst=self.ipl, g=w.g, head_dim=w.head_dim, block=w.block, hist_len=w.hist_len,
                            t_cap=w.t_cap, k_blocks=w.k_blocks, n_sink=w.n_sink, n_local=w.n_local, c1=w.c1, c2=w.c2,
                            kv_dtype=w.kv_dtype, flags=flags)
            R, nbc = L.ctx.hist_slots(), L.ctx.nb_cap()
            n = self.ipl
            L.hist = torch.zeros((n, R, nbc), dtype=f32, device=self.dev)
            L.pred = torch.zeros((n, nbc), dtype=f32, device=self.dev)
            L.pstate = torch.zeros((n, nbc), dtype=f32, device=self.dev)
            L.row = torch.zeros((n, nbc), dtype=f32, device=self.dev)
            L.idx = torch.zeros((n, w.k_blocks), dtype=i32, device=self.dev)
            L.cnt = torch.zeros((n,), dtype=i32, device=self.dev)
            L.out = torch.zeros((n, w.g, w.head_dim), dtype=f32, device=self.dev)
            L.ws = torch.zeros((max(16, L.ctx.workspace_bytes()),), dtype=torch.uint8, device=self.dev)
            L.pool_K = torch.zeros((n * w.k_blocks, w.block, w.head_dim), dtype=w.torch_dtype(), device=self.dev)
            L.pool_V = torch.zeros_like(L.pool_K)
            L.table = torch.zeros((n, nbc), dtype=i32, device=self.dev)
            L.state = torch.zeros((L.ctx.prefetch_state_bytes() // 4,), dtype=i32, device=self.dev)
            L.K_host = K_host[l * n:(l + 1) * n]
            L.V_host = V_host[l * n:(l + 1) * n]
            L.selected = torch.cuda.Event()
            L.staged = torch.cuda.Event()
            # addresses that never change, checked once: a 32-layer token step is bound by the host's enqueue rate
            L.handle = L.ctx._h
            L.ptrs = {n: _ptr(getattr(L, n)) for n in ("hist", "out", "idx", "cnt", "pred", "pstate", "pool_K", "pool_V",
                                                       "table", "state", "row", "ws")}
            L.ptrs["K_host"], L.ptrs["V_host"] = _rptr(L.K_host), _rptr(L.V_host)
            self.layers.append(L)
        self.R, self.nb_cap = R, nbc
        self._step_fn = load_library().ap_offload_step

    def set_weights(self, blob):
        for L in self.layers:
            L.ctx.set_weights(blob)

    def nb(self, t):
        return (t + self.w.block - 1) // self.w.block

    def _sl(self, x, l):
        return x[l * self.ipl:(l + 1) * self.ipl]

    def warmup_calibrate(self, q, t):
        """Push the dense pooled row of (q, K_host[:t]) into every layer's history (prefill tail)."""
        for l, L in enumerate(self.layers):
            L.ctx.calibrate(self._sl(q, l), L.K_host, t, L.row, L.ws)
            L.ctx.update_history(L.hist, self.n_pushed, L.row)
        self.n_pushed += 1

    def _select_and_fetch(self, L, t_next, mode, t_avail):
        """Predict + select for the token that makes the context t_next long, then stage its blocks."""
        nb_next = self.nb(t_next)
        L.ctx.predict_incremental(L.hist, self.n_pushed_layer, nb_next, self.nb(max(t_next - 1, 1)), mode, L.pstate,
                                  L.pred, L.ws)
        L.ctx.select_topk(L.pred, nb_next, L.idx, L.cnt, L.ws)
        cur = torch.cuda.current_stream(self.dev)
        L.selected.record(cur)
        self.copy_stream.wait_event(L.selected)
        with torch.cuda.stream(self.copy_stream):
            L.ctx.prefetch_blocks(L.K_host, L.V_host, t_avail, nb_next, L.idx, L.cnt, L.pool_K, L.pool_V, L.table,
                                  L.state)
            L.staged.record(self.copy_stream)

    def start(self, t_first):
        """After the warm-up pushes: select and stage the blocks of the first decode step (context t_first)."""
        self.n_pushed_layer = self.n_pushed
        for L in self.layers:
            if self.single_calls:
                self._select_and_fetch(L, t_first, AP_PRED_REBASE, t_first - 1)
            else:
                L.ctx.offload_begin(L.hist, self.n_pushed, L.K_host, L.V_host, t_first, L.idx, L.cnt, L.pred, L.pstate,
                                    L.pool_K, L.pool_V, L.table, L.state, L.ws, self.copy_stream)

    def step(self, q, k_new, v_new, t, calibrate=False):
        """One decode step at context length t (the new token has index t - 1).
        q: device [n_inst][g][d]; k_new, v_new: device [n_inst][d], the new token's K/V rows."""
        cur = torch.cuda.current_stream(self.dev)
        n_after = self.n_pushed + 1
        mode = AP_PRED_REBASE if n_after % self.rebase_every == 0 else AP_PRED_ADVANCE
        if not self.single_calls:
            qp, kp, vp = _ptr(q), _ptr(k_new), _ptr(v_new)
            q_step = self.ipl * self.w.g * self.w.head_dim * q.element_size()
            kv_step = self.ipl * self.w.head_dim * k_new.element_size()
            cs, ps, cal = cur.cuda_stream, self.copy_stream.cuda_stream, int(bool(calibrate))
            for l, L in enumerate(self.layers):
                P = L.ptrs
                _check(self._step_fn(L.handle, P["hist"], self.n_pushed, qp + l * q_step, kp + l * kv_step,
                                     vp + l * kv_step, P["K_host"], P["V_host"], t, cal, P["out"], P["idx"], P["cnt"],
                                     P["pred"], P["pstate"], mode, P["pool_K"], P["pool_V"], P["table"], P["state"],
                                     P["row"], P["ws"], cs, ps))
            self.n_pushed = n_after
            return
        for l, L in enumerate(self.layers):
            cur.wait_event(L.staged)
            L.ctx.append_kv(self._sl(k_new, l), self._sl(v_new, l), t - 1, L.table, L.state, L.pool_K, L.pool_V)
            L.ctx.set_block_table(L.table, self.ipl * self.w.k_blocks)
            L.ctx.sparse_decode(self._sl(q, l), L.pool_K, L.pool_V, t, L.idx, L.cnt, L.out, L.row, L.ws)
            if calibrate:
                L.ctx.set_block_table(None)
                L.ctx.calibrate(self._sl(q, l), L.K_host, t, L.row, L.ws)
            L.ctx.update_history(L.hist, self.n_pushed, L.row)
            self.n_pushed_layer = n_after
            if t + 1 <= self.w.t_cap:
                self._select_and_fetch(L, t + 1, mode, t)
        self.n_pushed = n_after

    def finish(self):
        """Wait for the last prefetches (their pools are about to go away)."""
        self.copy_stream.synchronize()

    def logical_history(self) -> torch.Tensor:
        """The H-row window of every instance in logical order (index H-1 = newest), [n_inst][H][nb_cap]."""
        H, R = self.w.hist_len, self.R
        slots = torch.tensor([(self.n_pushed - H + r) % R for r in range(H)], device=self.dev)
        h = torch.cat([L.hist.index_select(1, slots) for L in self.layers])
        for r in range(H):
            if self.n_pushed - H + r < 0:
                h[:, r, :] = 0
        return h

    def blocks_fetched(self) -> int:
        """Blocks copied from the full cache since the start (all layers and instances); synchronises."""
        k = self.w.k_blocks
        return int(sum(L.state.view(self.ipl, 3 * k + 4)[:, 3 * k + 1].sum().item() for L in self.layers))

    def out(self):
        return torch.cat([L.out for L in self.layers])

    def score_offset(self) -> float:
        """The constant the scores are relative to (the same for every layer: one predictor serves them all)."""
        return self.layers[0].ctx.score_offset()

    def staged_selection(self):
        """Scores and selection made for the NEXT step: pred [n_inst][nb_cap], idx [n_inst][k], cnt [n_inst]."""
        return (torch.cat([L.pred for L in self.layers]), torch.cat([L.idx for L in self.layers]),
                torch.cat([L.cnt for L in self.layers]))
