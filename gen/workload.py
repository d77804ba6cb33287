"""Seeded tensors for one layer of the LRQK decode step and its query stream.

Recipe (all draws from torch generators seeded from (config seed, layer, purpose)):

* per (batch, KV head): A_K (l x r) ~ N(0,1) fp32, B (r x d) ~ N(0, 1/r),
  K = A_K B + noise * N(0,1) rounded to the K/V dtype, V ~ N(0,1).
  Keys are therefore close to rank r, as the paper observes of real keys.
* heavy tokens are planted in factor space so a rank-r proxy can see them.
  Each query head owns a plane (e1, e2) of R^r and a pool of tokens at random
  positions; pool token p sits at phase phi_p on the plane:
      A_K[pos_p] += beta * (cos(phi_p) e1 + sin(phi_p) e2)       (before K is formed)
* the query of a head at step t is a background vector, AR(1) across steps,
  plus gamma * (cos(theta_t) b1 + sin(theta_t) b2) with b_i = B_i / |B_i|^2, so
  that its rank-r image has gamma * (cos, sin) on the head's plane.  Pool tokens
  whose phase is near theta_t get the largest scores; theta_t advances a
  fraction of the heavy window per step (drift) or jumps (re-draw).
* group_share = s > 0 makes the query heads of a KV group want some of the same tokens at the
  same steps: that fraction of every head's pool sits at the positions of the first head's
  pool (same phases) on the first head's plane, the group's queries share their phase and
  that plane, and the background queries of
  the group share a component (sqrt(s) of a draw per KV head + sqrt(1 - s) of the head's own).
  With 0 (the workloads' default) every head owns its heavy tokens and its query.
* q_hat = q B^T: the lambda = 0 closed form of the paper's decode update
  when B_K = B and B_Q is its dual basis.  It is an *input* of the hot path.

Nothing here computes scores, selections, cache decisions or attention.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np
import torch

from .configs import WorkloadConfig


def _gen(device, *keys) -> torch.Generator:
    """A generator whose seed is a fixed mix of the integer keys."""
    s = 0x9E3779B97F4A7C15
    for kx in keys:
        s = (s ^ (int(kx) + 0x632BE59BD9B4E019)) * 0xD1342543DE82EF95 % (1 << 64)
        s ^= s >> 29
    g = torch.Generator(device=device)
    g.manual_seed(s % (1 << 63))
    return g


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """uint16 view of a bf16 tensor as a numpy array on the host."""
    assert t.dtype == torch.bfloat16
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def as_numpy(t: torch.Tensor) -> np.ndarray:
    """Host numpy array with the same bits (bf16 -> uint16)."""
    if t.dtype == torch.bfloat16:
        return bf16_bits(t)
    return t.detach().cpu().contiguous().numpy()


@dataclass
class LayerData:
    cfg: WorkloadConfig
    layer: int
    A_K: torch.Tensor       # fp32 [B,Hkv,l,r]
    Bmat: torch.Tensor      # fp32 [B,Hkv,r,d]
    K: torch.Tensor         # kv dtype [B,Hkv,l,d]
    V: torch.Tensor         # kv dtype [B,Hkv,l,d]
    pool_pos: torch.Tensor  # int64 [B,Hq,P] positions of each head's pool tokens
    pool_phase: torch.Tensor  # fp64 [P]

    @property
    def liteK(self) -> torch.Tensor:
        c = self.cfg
        return self.K[:, :, c.l - c.w:, :].contiguous()

    @property
    def liteV(self) -> torch.Tensor:
        c = self.cfg
        return self.V[:, :, c.l - c.w:, :].contiguous()


def _plane(cfg: WorkloadConfig, hg: int):
    """Coordinates of R^r spanned by the plane of the hg-th query head of a group (with
    group_share > 0 the whole group looks for its heavy tokens on the first head's plane)."""
    if cfg.group_share > 0.0:
        hg = 0
    return (2 * hg) % cfg.r, (2 * hg + 1) % cfg.r


def make_layer(cfg: WorkloadConfig, layer: int = 0, device="cpu") -> LayerData:
    dev = torch.device(device)
    B, Hq, Hkv, l, r, d, G = cfg.B, cfg.Hq, cfg.Hkv, cfg.l, cfg.r, cfg.d, cfg.G
    P = cfg.pool
    assert Hq % Hkv == 0 and 0 < P * G <= l - cfg.w
    kvdt = torch.bfloat16 if cfg.kv_dtype == "bf16" else torch.float32

    A_K = torch.randn(B, Hkv, l, r, generator=_gen(dev, cfg.seed, layer, 1), device=dev,
                      dtype=torch.float32)
    Bmat = torch.randn(B, Hkv, r, d, generator=_gen(dev, cfg.seed, layer, 2), device=dev,
                       dtype=torch.float32) / math.sqrt(r)

    # pool positions: one permutation of [0, l-w) per (batch, KV head), cut into G pools
    gp = _gen("cpu", cfg.seed, layer, 3)
    pool_pos = torch.empty(B, Hq, P, dtype=torch.int64)
    n_shared = int(round(cfg.group_share * P))   # pool entries that a head shares with head 0
    shared_idx = [[None] * Hkv for _ in range(B)]
    for b in range(B):
        for kv in range(Hkv):
            perm = torch.randperm(l - cfg.w, generator=gp)[: G * P]
            for hg in range(G):
                pool_pos[b, kv * G + hg] = perm[hg * P:(hg + 1) * P]
            if n_shared > 0:
                # the same pool indices (hence phases) for every head of the group, so that the
                # heads want those tokens at the same steps
                shared = torch.randperm(P, generator=gp)[:n_shared]
                shared_idx[b][kv] = shared
                for hg in range(1, G):
                    pool_pos[b, kv * G + hg, shared] = pool_pos[b, kv * G, shared]
    pool_phase = cfg.phase_spread * 2.0 * math.pi * torch.arange(P, dtype=torch.float64) / P

    # plant the pools in factor space
    cosp = (cfg.beta * torch.cos(pool_phase)).to(torch.float32).to(dev)
    sinp = (cfg.beta * torch.sin(pool_phase)).to(torch.float32).to(dev)
    pp = pool_pos.to(dev)
    for hg in range(G):
        c1, c2 = _plane(cfg, hg)
        for b in range(B):
            for kv in range(Hkv):
                pos = pp[b, kv * G + hg]
                if hg > 0 and n_shared > 0:      # shared entries were planted with the first head
                    own = torch.ones(P, dtype=torch.bool, device=dev)
                    own[shared_idx[b][kv].to(dev)] = False
                    A_K[b, kv, pos[own], c1] += cosp[own]
                    A_K[b, kv, pos[own], c2] += sinp[own]
                else:
                    A_K[b, kv, pos, c1] += cosp
                    A_K[b, kv, pos, c2] += sinp

    gk = _gen(dev, cfg.seed, layer, 4)
    gv = _gen(dev, cfg.seed, layer, 5)
    K = torch.empty(B, Hkv, l, d, device=dev, dtype=kvdt)
    V = torch.empty(B, Hkv, l, d, device=dev, dtype=kvdt)
    for b in range(B):
        for kv in range(Hkv):
            full = A_K[b, kv] @ Bmat[b, kv]
            full += cfg.noise * torch.randn(l, d, generator=gk, device=dev, dtype=torch.float32)
            K[b, kv] = full.to(kvdt)
            V[b, kv] = torch.randn(l, d, generator=gv, device=dev, dtype=torch.float32).to(kvdt)
    return LayerData(cfg=cfg, layer=layer, A_K=A_K, Bmat=Bmat, K=K, V=V,
                     pool_pos=pool_pos, pool_phase=pool_phase)


class QueryStream:
    """Per-step queries of one layer: q [B,Hq,d] fp32 and q_hat [B,Hq,r] fp32."""

    def __init__(self, data: LayerData, device=None):
        self.data = data
        self.cfg = data.cfg
        self.dev = torch.device(device) if device is not None else data.A_K.device
        self.t = 0
        c = self.cfg
        self._g = _gen(self.dev, c.seed, data.layer, 6)
        self._gth = _gen("cpu", c.seed, data.layer, 7)
        self._bg = self._draw_background()
        self._theta0 = 2.0 * math.pi * torch.rand(c.B, c.Hq, generator=self._gth,
                                                  dtype=torch.float64) * c.phase_spread
        if c.group_share > 0.0:      # the heads of a KV group move through their pools together
            self._theta0 = self._theta0[:, ::c.G].repeat_interleave(c.G, dim=1)
        # planted directions b1, b2 per query head
        G = c.G
        b1 = torch.empty(c.B, c.Hq, c.d, dtype=torch.float32, device=self.dev)
        b2 = torch.empty_like(b1)
        Bm = data.Bmat.to(self.dev)
        for h in range(c.Hq):
            c1, c2 = _plane(c, h % G)
            r1 = Bm[:, h // G, c1, :]
            r2 = Bm[:, h // G, c2, :]
            b1[:, h] = r1 / (r1 * r1).sum(-1, keepdim=True)
            b2[:, h] = r2 / (r2 * r2).sum(-1, keepdim=True)
        self._b1, self._b2, self._Bm = b1, b2, Bm

    def _draw_background(self) -> torch.Tensor:
        """N(0,1) per query head; with group_share = s > 0 the heads of a KV group share a
        component: sqrt(s) * (one draw per KV head) + sqrt(1 - s) * (one draw per head)."""
        c = self.cfg
        own = torch.randn(c.B, c.Hq, c.d, generator=self._g, device=self.dev, dtype=torch.float32)
        if c.group_share <= 0.0:
            return own
        grp = torch.randn(c.B, c.Hkv, c.d, generator=self._g, device=self.dev,
                          dtype=torch.float32).repeat_interleave(c.G, dim=1)
        return math.sqrt(c.group_share) * grp + math.sqrt(1.0 - c.group_share) * own

    def theta(self) -> torch.Tensor:
        """Current phase of the planted query component, [B,Hq] fp64."""
        c = self.cfg
        window = 2.0 * math.pi * c.n_heavy / max(c.pool, 1)
        if c.redraw_every > 0:
            epoch, within = divmod(self.t, c.redraw_every)
            # a fresh heavy window for every epoch: hop by one and a half windows, so the new
            # window shares no pool token with the old one
            base = self._theta0 + epoch * 1.5 * window
            return base + within * c.drift * window
        return self._theta0 + self.t * c.drift * window

    def next(self):
        c = self.cfg
        if self.t > 0:
            eps = self._draw_background()
            self._bg = c.rho * self._bg + math.sqrt(max(0.0, 1.0 - c.rho * c.rho)) * eps
        th = self.theta()
        ct = (c.gamma * torch.cos(th)).to(torch.float32).to(self.dev)[..., None]
        st = (c.gamma * torch.sin(th)).to(torch.float32).to(self.dev)[..., None]
        q = (self._bg + ct * self._b1 + st * self._b2).contiguous()
        # q_hat[b,h,:] = q[b,h,:] B[b,h/G]^T in double, rounded once to fp32
        Bq = self._Bm.repeat_interleave(c.G, dim=1).double()          # [B,Hq,r,d]
        q_hat = torch.einsum("bhd,bhrd->bhr", q.double(), Bq).to(torch.float32).contiguous()
        self.t += 1
        return q, q_hat


def make_prefill_inputs(cfg: WorkloadConfig, data: LayerData, device=None):
    """Inputs of the prefill factorisation for one layer: the prompt's queries Q [B,Hq,l,d] in
    the K/V dtype (close to rank r like the keys: Q = Z C + noise with Z ~ N(0,1), C ~ N(0,1/r))
    and the N(0,1) draws A_Q0 [B,Hq,l,r], A_K0 [B,Hkv,l,r] that Alg. 1 starts from.  The keys
    are the layer's K.  Nothing of the method is computed here."""
    dev = torch.device(device) if device is not None else data.A_K.device
    B, Hq, Hkv, l, r, d = cfg.B, cfg.Hq, cfg.Hkv, cfg.l, cfg.r, cfg.d
    g = _gen(dev, cfg.seed, data.layer, 8)
    Q = torch.empty(B, Hq, l, d, device=dev, dtype=data.K.dtype)
    for b in range(B):
        for h in range(Hq):
            Z = torch.randn(l, r, generator=g, device=dev, dtype=torch.float32)
            Cm = torch.randn(r, d, generator=g, device=dev, dtype=torch.float32) / math.sqrt(r)
            full = Z @ Cm + cfg.noise * torch.randn(l, d, generator=g, device=dev,
                                                    dtype=torch.float32)
            Q[b, h] = full.to(data.K.dtype)
    A_Q0 = torch.randn(B, Hq, l, r, generator=g, device=dev, dtype=torch.float32)
    A_K0 = torch.randn(B, Hkv, l, r, generator=g, device=dev, dtype=torch.float32)
    return Q, A_Q0, A_K0
