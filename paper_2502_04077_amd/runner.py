"""Device buffers and call sequencing for a Workload: allocation and bookkeeping only.

Holds the tensors one decode run needs (history ring, pred, idx, out, row, workspace) and drives
the C-ABI calls in the order of Algorithm 1.  No arithmetic of the method happens here.
"""
from __future__ import annotations

import torch

from .binding import AP_PRED_ADVANCE, AP_PRED_HOLD, AP_PRED_REBASE, AP_PRED_SKIP, AP_STEP_REUSE_SELECTION, Context


class DecodeRun:
    def __init__(self, w, device="cuda:0", incremental=True, rebase_every=512, flags=0, refresh_every=1):
        """incremental: carry the predictor's interior state across steps (ap_predict_incremental)
        and re-evaluate the full tile every `rebase_every` pushes; False evaluates the full tile
        on every step.  refresh_every: the selection is re-made on every refresh_every-th step and
        carried over (ap_refresh_selection) on the others (Sec. 3.3).  The predictor state then either
        advances on every step anyway, or - from skip_predictor_from steps between selections on - the
        predictor is left out on the steps in between and evaluates the full tile when it is needed
        (one full tile costs about as much as a dozen advances)."""
        self.w = w
        self.refresh_every = refresh_every
        self.skip_predictor_from = 12
        self.steps_done = 0
        self.incremental = incremental
        self.rebase_every = rebase_every
        self.state_n = None       # n_pushed the predictor state is valid for
        self.state_t = None       # t_cur of the call that wrote it
        self.dev = torch.device(device)
        self.ctx = Context(n_inst=w.n_inst, g=w.g, head_dim=w.head_dim, block=w.block, hist_len=w.hist_len,
                           t_cap=w.t_cap, k_blocks=w.k_blocks, n_sink=w.n_sink, n_local=w.n_local,
                           c1=w.c1, c2=w.c2, kv_dtype=w.kv_dtype, flags=flags)
        R, nbc = self.ctx.hist_slots(), self.ctx.nb_cap()
        self.R, self.nb_cap = R, nbc
        f32, i32 = torch.float32, torch.int32
        self.hist = torch.zeros((w.n_inst, R, nbc), dtype=f32, device=self.dev)
        self.pred = torch.zeros((w.n_inst, nbc), dtype=f32, device=self.dev)
        self.pstate = torch.zeros((w.n_inst, nbc), dtype=f32, device=self.dev)
        self.row = torch.zeros((w.n_inst, nbc), dtype=f32, device=self.dev)
        self.idx = torch.zeros((w.n_inst, w.k_blocks), dtype=i32, device=self.dev)
        self.cnt = torch.zeros((w.n_inst,), dtype=i32, device=self.dev)
        self.out = torch.zeros((w.n_inst, w.g, w.head_dim), dtype=f32, device=self.dev)
        self.ws = torch.zeros((max(16, self.ctx.workspace_bytes()),), dtype=torch.uint8, device=self.dev)
        self.n_pushed = 0

    def set_weights(self, blob):
        self.ctx.set_weights(blob)

    def nb(self, t):
        return (t + self.w.block - 1) // self.w.block

    def logical_history(self, instances=None) -> torch.Tensor:
        """The H-row window in logical order (index H-1 = newest) as a new tensor
        [len(instances) or n_inst][H][nb_cap]."""
        H, R = self.w.hist_len, self.R
        slots = torch.tensor([(self.n_pushed - H + r) % R for r in range(H)], device=self.dev)
        src = self.hist if instances is None else self.hist[torch.as_tensor(list(instances), device=self.dev)]
        h = src.index_select(1, slots)
        for r in range(H):
            if self.n_pushed - H + r < 0:
                h[:, r, :] = 0
        return h

    def warmup_calibrate(self, q, K, t):
        """Push the dense pooled row of (q, K[:t]) - used for the prefill tail and calibration."""
        self.ctx.calibrate(q, K, t, self.row, self.ws)
        self.ctx.update_history(self.hist, self.n_pushed, self.row)
        self.n_pushed += 1

    def _pred_mode(self, t):
        """Which predictor mode is valid now, and the bookkeeping for the next call."""
        if not self.incremental:
            return AP_PRED_REBASE
        n = self.n_pushed
        if self.state_n == n and self.state_t == t:
            mode = AP_PRED_HOLD
        elif self.state_n == n - 1 and self.state_t == t - 1 and n % self.rebase_every != 0:
            mode = AP_PRED_ADVANCE
        else:
            mode = AP_PRED_REBASE
        return mode

    def selects_now(self, t):
        """Whether the step at context length t re-makes the selection (else it carries the last one over)."""
        k = self.w.k_blocks
        return (self.steps_done % self.refresh_every == 0 or self.nb(t - 1) <= k < self.nb(t)
                or self.nb(t) <= k)

    def _step_mode(self, t, selects):
        """Predictor mode of this step; AP_PRED_SKIP on steps that carry the selection over under a long interval."""
        if not selects and self.refresh_every >= self.skip_predictor_from:
            return AP_PRED_SKIP
        return self._pred_mode(t)

    def step_unfused(self, q, K, V, t, calibrate=False):
        nb = self.nb(t)
        selects = self.selects_now(t)
        mode = self._step_mode(t, selects)
        if mode == AP_PRED_SKIP:
            pass
        elif self.incremental:
            self.ctx.predict_incremental(self.hist, self.n_pushed, nb, self.nb(max(t - 1, 1)), mode, self.pstate,
                                         self.pred, self.ws)
            self.state_n, self.state_t = self.n_pushed, t
        else:
            self.ctx.predict(self.hist, self.n_pushed, nb, self.pred, self.ws)
        if selects:
            self.ctx.select_topk(self.pred, nb, self.idx, self.cnt, self.ws)
        elif nb != self.nb(t - 1):
            self.ctx.refresh_selection(self.nb(t - 1), nb, self.idx, self.cnt)
        self.ctx.sparse_decode(q, K, V, t, self.idx, self.cnt, self.out, self.row, self.ws)
        if calibrate:
            self.ctx.calibrate(q, K, t, self.row, self.ws)
        self.ctx.update_history(self.hist, self.n_pushed, self.row)
        self.n_pushed += 1
        self.steps_done += 1
        return mode

    def step(self, q, K, V, t, calibrate=False):
        selects = self.selects_now(t)
        mode = self._step_mode(t, selects)
        flag = 0 if selects else AP_STEP_REUSE_SELECTION
        self.ctx.step(self.hist, self.n_pushed, q, K, V, t, self.out, self.idx, self.cnt, self.pred,
                      self.pstate if self.incremental else None, mode | flag, self.ws)
        if self.incremental and mode != AP_PRED_SKIP:
            self.state_n, self.state_t = self.n_pushed, t
        if calibrate:
            self.ctx.calibrate(q, K, t, self.row, self.ws)
            self.ctx.update_history(self.hist, self.n_pushed, self.row)
        self.n_pushed += 1
        self.steps_done += 1
        return mode


class DenseRun:
    """Layers that attend to the whole cache in every step (Sec. 4.1 keeps the first two layers uncompressed):
    the same attention kernel with a budget of all blocks, no history and no predictor."""

    def __init__(self, w, n_layers, device="cuda:0"):
        self.w = w
        self.dev = torch.device(device)
        self.n_inst = n_layers * w.batch * w.kv_heads
        self.ctx = Context(n_inst=self.n_inst, g=w.g, head_dim=w.head_dim, block=w.block, hist_len=w.hist_len,
                           t_cap=w.t_cap, k_blocks=w.nb_cap, n_sink=0, n_local=0, c1=w.c1, c2=w.c2,
                           kv_dtype=w.kv_dtype)
        f32, i32 = torch.float32, torch.int32
        nbc = self.ctx.nb_cap()
        self.idx = torch.zeros((self.n_inst, nbc), dtype=i32, device=self.dev)
        self.cnt = torch.zeros((self.n_inst,), dtype=i32, device=self.dev)
        self.row = torch.zeros((self.n_inst, nbc), dtype=f32, device=self.dev)
        self.out = torch.zeros((self.n_inst, w.g, w.head_dim), dtype=f32, device=self.dev)
        self.ws = torch.zeros((max(16, self.ctx.workspace_bytes()),), dtype=torch.uint8, device=self.dev)
        self.nb_listed = 0

    def step(self, q, K, V, t):
        nb = (t + self.w.block - 1) // self.w.block
        if nb != self.nb_listed:                          # all blocks: no scores are read
            self.ctx.select_topk(self.row, nb, self.idx, self.cnt, self.ws)
            self.nb_listed = nb
        self.ctx.sparse_decode(q, K, V, t, self.idx, self.cnt, self.out, self.row, self.ws)
