"""Seeded synthetic inputs for the AttentionPredictor decode hot path.

This module only *draws inputs* (shapes, seeds, value distributions, planted key
structure).  It holds none of the method's arithmetic: no softmax, pooling,
convolution, selection or attention lives here.  Both the CPU oracle's tests and
the HIP path's tests/bench take their inputs from here, so that the two sides are
compared on byte-identical tensors.

Shapes follow the paper's evaluation set-up (Sec. 4.1 "Implementation details":
history H = 64, block size b = 16, 64 prefix + 64 local tokens inside the budget)
on 7B/8B-shaped long-context decode; the values stand in for the paper's
benchmark prompts, which are not available here.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    """One decode workload.  An *instance* is one (layer, batch, KV-head) triple."""

    name: str
    layers: int
    batch: int
    kv_heads: int
    g: int                 # query heads per KV head (GQA group size)
    head_dim: int
    kv_dtype: str          # "bf16" | "f32"  (q uses the same dtype)
    t0: int                # context length when decoding starts
    block: int             # b
    hist_len: int          # H
    budget_tokens: int     # B (includes sink and local tokens)
    n_sink: int            # forced leading blocks
    n_local: int           # forced trailing blocks
    c1: int                # predictor hidden channels, first conv
    c2: int                # predictor hidden channels, second conv
    steps: int             # decode steps of the run
    calib_every: int       # M: dense calibration interval in steps
    seed: int
    value_scale: float     # q/K/V ~ N(0,1) * value_scale
    planted: bool = False  # structured keys/queries (sink, local, stripes, slashes)

    @property
    def n_inst(self) -> int:
        return self.layers * self.batch * self.kv_heads

    @property
    def k_blocks(self) -> int:
        return self.budget_tokens // self.block

    @property
    def t_cap(self) -> int:
        """Token capacity of the K/V buffers: all decode steps fit, rounded up to a block."""
        t = self.t0 + self.steps
        return (t + self.block - 1) // self.block * self.block

    @property
    def nb_cap(self) -> int:
        return self.t_cap // self.block

    def t_at(self, step: int) -> int:
        """Tokens visible to decode step `step` (0-based): the new token's K/V is appended first."""
        return self.t0 + step + 1

    def is_calibration_step(self, step: int) -> bool:
        return self.calib_every > 0 and (step + 1) % self.calib_every == 0

    def torch_dtype(self) -> torch.dtype:
        return torch.bfloat16 if self.kv_dtype == "bf16" else torch.float32

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


_S128 = 1.0 / math.sqrt(128.0)

CONFIGS = {
    # Tiny fp32 case the oracle finishes in seconds.
    "cfg0": Workload("cfg0", 1, 1, 1, 4, 64, "f32", 2048, 16, 16, 256, 1, 2, 4, 4, 32, 8, 0, 1.0),
    # One Llama-3.1-8B-shaped layer, batch 1, 32K context.
    "cfg1": Workload("cfg1", 1, 1, 8, 4, 128, "bf16", 32768, 16, 64, 1024, 4, 4, 8, 8, 256, 32, 1, _S128),
    # All 32 layers, batch 8, 32K context: the working set is far beyond any cache.
    "cfg2": Workload("cfg2", 32, 8, 8, 4, 128, "bf16", 32768, 16, 64, 1024, 4, 4, 8, 8, 128, 32, 2, _S128),
    # 128K context, 4 layers, batch 4.
    "cfg3": Workload("cfg3", 4, 4, 8, 4, 128, "bf16", 131072, 16, 64, 2048, 4, 4, 8, 8, 64, 32, 3, _S128),
    # 7B MHA shape with planted attention structure.
    "cfg4": Workload("cfg4", 8, 16, 32, 1, 128, "bf16", 32768, 16, 64, 1024, 4, 4, 8, 8, 256, 32, 4, _S128,
                     planted=True),
}


def n_weight_floats(c1: int, c2: int) -> int:
    """Length of the flat predictor blob: w1[c1][3][3], b1[c1], w2[c2][c1][3][3], b2[c2], w3[c2], b3."""
    return c1 * 9 + c1 + c2 * c1 * 9 + c2 + c2 + 1


def predictor_weights(w: Workload, sigma: float = 0.1) -> np.ndarray:
    """Random-init predictor blob, every entry ~ N(0, sigma), fp32, seeded with seed + 1000."""
    rng = np.random.default_rng(w.seed + 1000)
    return (rng.standard_normal(n_weight_floats(w.c1, w.c2)) * sigma).astype(np.float32)


def _gen(device, *seed_words: int) -> torch.Generator:
    g = torch.Generator(device=device)
    s = 0x9E3779B97F4A7C15
    for x in seed_words:
        s = (s * 6364136223846793005 + int(x) + 1442695040888963407) & 0x7FFFFFFFFFFFFFFF
    g.manual_seed(s)
    return g


# ---------------------------------------------------------------------------------------------
# Planted structure (cfg4): coordinates of head_dim reserved for each pattern.  Amplitudes are in
# logit units (queries carry a factor sqrt(head_dim) so that q.k / sqrt(d) gives them directly).
#   dim 0          sink      key 0 carries 1; every query carries A_SINK                     (re-access)
#   dim 1          stripes   16 seeded key positions per instance carry 1; queries carry A_STRIPE during the
#                            first 40 steps of every 200-step season, 0 otherwise              (seasonal)
#   dims 2..33     local     16 rotary (cos, sin) pairs with geometric wavelengths: key i carries angle
#                            theta_m * i, the query of the token at position p carries A_LOCAL * angle
#                            theta_m * p, so the logit is A_LOCAL * sum_m cos(theta_m (p - i)): a peak of
#                            16 A_LOCAL at the newest tokens that falls off within a few tens of tokens
#   dims 34..97    slashes   one-hot code of (block index mod 64) on the keys; the query carries A_SLASH on
#                            the code of (its own block index - delta) mod 64, delta seeded per instance:
#                            every 64th block lights up and the lit set moves on by one block every 16
#                            steps                                                            (sequential)
#   dims 98..127   noise     N(0,1) * value_scale
# ---------------------------------------------------------------------------------------------
_LOC0, _NLOC = 2, 16
_SL0, _SLP = 34, 64
_NOISE0 = _SL0 + _SLP
_A_SINK, _A_STRIPE, _A_LOCAL, _A_SLASH = 13.0, 10.5, 0.7, 7.0
_SEASON, _SEASON_ON = 200, 40
_N_STRIPES = 16


def _local_thetas(device) -> torch.Tensor:
    m = torch.arange(_NLOC, device=device, dtype=torch.float64)
    return 2.0 * math.pi / (32.0 * (1.66 ** m))       # wavelengths 32 .. ~64K tokens


def _slash_delta(w: Workload, inst: torch.Tensor) -> torch.Tensor:
    """Seeded per-instance offset (in blocks) of the slash family."""
    return (inst.to(torch.int64) * 2654435761 + w.seed * 97) % _SLP


def _stripe_positions(w: Workload, inst: int) -> torch.Tensor:
    """One token in each of 16 distinct seeded blocks, away from the sink and local blocks."""
    rng = np.random.default_rng([w.seed, 77, int(inst)])
    nb0 = w.t0 // w.block
    blocks = rng.choice(np.arange(8, nb0 - 8), size=_N_STRIPES, replace=False)
    return torch.from_numpy(np.sort(blocks * w.block + rng.integers(0, w.block, size=_N_STRIPES)))


def kv_cache(w: Workload, device="cpu", chunk_inst: int = 32):
    """K and V as `[n_inst][t_cap][head_dim]` in the workload's KV dtype.

    Rows at positions >= t0 are the tokens that decode steps append; they are drawn up front so
    that step s simply exposes `t_at(s)` rows.
    """
    dt = w.torch_dtype()
    K = torch.empty((w.n_inst, w.t_cap, w.head_dim), dtype=dt, device=device)
    V = torch.empty_like(K)
    for i0 in range(0, w.n_inst, chunk_inst):
        i1 = min(w.n_inst, i0 + chunk_inst)
        gk = _gen(device, w.seed, 1, i0)
        gv = _gen(device, w.seed, 2, i0)
        k = torch.randn((i1 - i0, w.t_cap, w.head_dim), generator=gk, device=device, dtype=torch.float32)
        k *= w.value_scale
        if w.planted:
            _plant_keys(w, k, i0)
        K[i0:i1] = k.to(dt)
        del k
        v = torch.randn((i1 - i0, w.t_cap, w.head_dim), generator=gv, device=device, dtype=torch.float32)
        v *= w.value_scale
        V[i0:i1] = v.to(dt)
        del v
    return K, V


def _plant_keys(w: Workload, k: torch.Tensor, i0: int) -> None:
    n, t_cap, _ = k.shape
    dev = k.device
    k[:, :, 0:_NOISE0] = 0.0
    k[:, 0, 0] = 1.0                                          # sink token
    for j in range(n):
        k[j, _stripe_positions(w, i0 + j).to(dev), 1] = 1.0   # vertical stripes
    pos = torch.arange(t_cap, device=dev)
    ang = pos.to(torch.float64)[:, None] * _local_thetas(dev)[None, :]
    k[:, :, _LOC0:_LOC0 + 2 * _NLOC:2] = torch.cos(ang).to(torch.float32)[None]
    k[:, :, _LOC0 + 1:_LOC0 + 2 * _NLOC:2] = torch.sin(ang).to(torch.float32)[None]
    code = (pos // w.block) % _SLP
    k[:, pos, _SL0 + code] = 1.0                              # block-residue code


def queries(w: Workload, step: int, device="cpu") -> torch.Tensor:
    """Query of decode step `step` (negative steps are the prefill tail used for history warm-up).

    Shape `[n_inst][g][head_dim]` in the KV dtype.
    """
    gq = _gen(device, w.seed, 3, step + 100000)
    q = torch.randn((w.n_inst, w.g, w.head_dim), generator=gq, device=device, dtype=torch.float32)
    q *= w.value_scale
    if w.planted:
        p = w.t0 + step                                       # position of the querying (newest) token
        dev = q.device
        sd = math.sqrt(w.head_dim)
        q[:, :, 0:_NOISE0] = 0.0
        q[:, :, 0] = _A_SINK * sd
        q[:, :, 1] = (_A_STRIPE * sd) if (step % _SEASON) < _SEASON_ON else 0.0
        ang = float(p) * _local_thetas(dev)
        q[:, :, _LOC0:_LOC0 + 2 * _NLOC:2] = (_A_LOCAL * sd) * torch.cos(ang).to(torch.float32)[None, None, :]
        q[:, :, _LOC0 + 1:_LOC0 + 2 * _NLOC:2] = (_A_LOCAL * sd) * torch.sin(ang).to(torch.float32)[None, None, :]
        inst = torch.arange(w.n_inst, device=dev)
        code = (p // w.block - _slash_delta(w, inst)) % _SLP
        q[inst, :, _SL0 + code] = _A_SLASH * sd
    return q.to(w.torch_dtype())


def to_f64(x: torch.Tensor) -> np.ndarray:
    """Exact widening of a (bf16 or fp32) tensor to a float64 numpy array on the host."""
    return x.detach().to("cpu", torch.float32).numpy().astype(np.float64)
