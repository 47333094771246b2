"""Gaussian-mixture keys, values and queries.

Recipe (per head-problem = one (sequence, KV head) of one layer): M centers drawn
from N(0, I_d) and scaled to unit length; every token picks one center uniformly;
key = 3 * center + N(0, 0.5^2 I); value ~ N(0, I); every query head picks one
center of its KV head uniformly and query = 3 * center + N(0, 0.5^2 I).  Everything
is rounded to the storage dtype (bf16 unless stated).  These tensors stand in for
the KV cache of a long prompt: keys that form direction clusters of unequal size,
with queries that point at a few of them.

All draws come from a torch.Generator on the requested device seeded with
(seed, layer), so the same call reproduces the same tensors on that device type.
"""
from __future__ import annotations

import numpy as np
import torch

from .configs import Config

_SCALE = 3.0
_SIGMA = 0.5


def _gen(device, seed: int, layer: int, stream: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1_000_003 + int(layer)) * 16 + int(stream))
    return g


class MixtureWorkload:
    """Keys/values of one layer of a configuration, plus query / new-token draws."""

    def __init__(self, cfg: Config, layer: int = 0, device="cpu", dtype=torch.bfloat16,
                 extra_tokens: int = 0):
        self.cfg = cfg
        self.layer = layer
        self.device = torch.device(device)
        self.dtype = dtype
        S, H, N, d, M = cfg.S, cfg.Hkv, cfg.N, cfg.d, cfg.M
        self.N_cap = N + extra_tokens
        g = _gen(self.device, cfg.seed, layer, 0)
        centers = torch.randn(S, H, M, d, generator=g, device=self.device)
        self.centers = centers / centers.norm(dim=-1, keepdim=True)
        self.K = torch.zeros(S, H, self.N_cap, d, device=self.device, dtype=dtype)
        self.V = torch.zeros(S, H, self.N_cap, d, device=self.device, dtype=dtype)
        self.token_center = torch.zeros(S, H, self.N_cap, dtype=torch.int64,
                                        device=self.device)
        # one head-problem at a time keeps the fp32 temporaries small
        for s in range(S):
            for h in range(H):
                k, v, tc = self._draw_tokens(s, h, N, g)
                self.K[s, h, :N] = k
                self.V[s, h, :N] = v
                self.token_center[s, h, :N] = tc
        self.n_tokens = N
        self._g_new = _gen(self.device, cfg.seed, layer, 1)
        self._g_q = _gen(self.device, cfg.seed, layer, 2)

    def _draw_tokens(self, s, h, n, g):
        d, M = self.cfg.d, self.cfg.M
        tc = torch.randint(0, M, (n,), generator=g, device=self.device)
        k = _SCALE * self.centers[s, h, tc] + _SIGMA * torch.randn(
            n, d, generator=g, device=self.device)
        v = torch.randn(n, d, generator=g, device=self.device)
        return k.to(self.dtype), v.to(self.dtype), tc

    def query(self, sticky: float = 0.0) -> torch.Tensor:
        """One decode-step query, [S, Hq, d]; heads of one group draw centers
        of their own KV head independently.  With sticky > 0 a head keeps the
        center of its previous query with that probability (a stand-in for the
        slow drift of attention targets between consecutive decode steps)."""
        cfg = self.cfg
        S, Hq, G, d, M = cfg.S, cfg.Hq, cfg.G, cfg.d, cfg.M
        pick = torch.randint(0, M, (S, Hq), generator=self._g_q, device=self.device)
        if sticky > 0.0:
            keep = torch.rand(S, Hq, generator=self._g_q, device=self.device) < sticky
            last = getattr(self, "_last_pick", None)
            if last is not None:
                pick = torch.where(keep, last, pick)
            self._last_pick = pick
        kv_head = torch.arange(Hq, device=self.device) // G
        c = self.centers[torch.arange(S, device=self.device)[:, None], kv_head[None, :], pick]
        q = _SCALE * c + _SIGMA * torch.randn(S, Hq, d, generator=self._g_q,
                                              device=self.device)
        return q.to(self.dtype)

    def append_token(self) -> int:
        """Draw the key/value of one generated token per head-problem from the same
        mixture and store it at row n_tokens; returns that row."""
        cfg = self.cfg
        if self.n_tokens >= self.N_cap:
            raise RuntimeError("KV capacity exhausted")
        S, H, d, M = cfg.S, cfg.Hkv, cfg.d, cfg.M
        g = self._g_new
        tc = torch.randint(0, M, (S, H), generator=g, device=self.device)
        c = torch.gather(self.centers, 2, tc[:, :, None, None].expand(S, H, 1, d))[:, :, 0]
        k = _SCALE * c + _SIGMA * torch.randn(S, H, d, generator=g, device=self.device)
        v = torch.randn(S, H, d, generator=g, device=self.device)
        t = self.n_tokens
        self.K[:, :, t] = k.to(self.dtype)
        self.V[:, :, t] = v.to(self.dtype)
        self.token_center[:, :, t] = tc
        self.n_tokens = t + 1
        return t


def sample_init_indices(keys: torch.Tensor, C: int, seed: int, tok_begin: int = 0,
                        tok_count: int | None = None) -> torch.Tensor:
    """Random draw of the initial centroids for K-means: per head-problem, a seeded
    shuffle of the token range, of which the first C tokens whose key rows are
    pairwise bit-distinct are kept.  keys: [S, H, N_cap, d]; returns int32 [S, H, C]
    of absolute token rows.  The shuffle uses NumPy's PCG64 (host side)."""
    S, H = keys.shape[:2]
    if tok_count is None:
        tok_count = keys.shape[2] - tok_begin
    if C > tok_count:
        raise ValueError("more clusters than tokens")
    out = np.zeros((S, H, C), dtype=np.int32)
    rng = np.random.default_rng(np.random.SeedSequence([int(seed), 0xC1A5]))
    for s in range(S):
        for h in range(H):
            perm = rng.permutation(tok_count) + tok_begin
            taken: list[int] = []
            seen: set[bytes] = set()
            pos = 0
            while len(taken) < C:
                if pos >= tok_count:
                    raise ValueError("fewer than C distinct key rows in the range")
                # fetch candidates in small batches (rows may live on the GPU)
                batch = perm[pos:pos + max(C - len(taken), 8)]
                rows = keys[s, h, torch.as_tensor(batch, device=keys.device)]
                rows = rows.contiguous().view(torch.uint8).cpu().numpy()
                for j, t in enumerate(batch):
                    b = rows[j].tobytes()
                    if b not in seen:
                        seen.add(b)
                        taken.append(int(t))
                        if len(taken) == C:
                            break
                pos += len(batch)
            out[s, h] = taken
    return torch.from_numpy(out)
