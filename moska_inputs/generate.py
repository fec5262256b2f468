"""Seeded generator for the synthetic decode-step workloads.

Recipe (one independent random stream per tensor, all derived from one seed):

  mu[c,h,:]      ~ N(0, I_D)                      topic centre of chunk c on KV head h
  K_s[c,h,t,:]   = mu[c,h] + 0.5 N(0,1)           shared keys cluster round their centre
  V_s[c,h,t,:]   ~ N(0,1)
  c*[b]          ~ uniform, or Zipf(s) over ranks mapped through a seeded permutation
  q[b,hq,:]      = (mu[c*[b], hq//G] + N(0,1)) / sqrt(D)     (one per query token when T > 1)
  K_u[b,h,t,:]   = mu[c*[b],h] + 0.5 N(0,1),  V_u ~ N(0,1)
  E[h,c,:]       = mean over t of the *stored* K_s[c,h,t,:]   (chunk embedding, Sec. III-B)

Everything is rounded (round-to-nearest-even) to its storage dtype; an fp8 shared
store is quantised per (chunk, KV head) with scale = amax/448.  The stored bits are
what both the oracle and the GPU library consume.  Works on any torch device; big
tensors are produced slab by slab so peak temporary memory stays small.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional
import math
import torch

from .problem import Problem, torch_dtype

FP8_MAX = 448.0


@dataclass
class Inputs:
    prob: Problem
    Q: torch.Tensor                    # [B*T,Hq,D]     q_dtype (row b*T + t = token t of request b)
    E: torch.Tensor                    # [Hkv,C,D]      q_dtype
    Ks: torch.Tensor                   # [C,Hkv,L,D]    kv_dtype
    Vs: torch.Tensor                   # [C,Hkv,L,D]    kv_dtype
    scale_k: Optional[torch.Tensor]    # [C,Hkv] f32 (fp8 store only)
    scale_v: Optional[torch.Tensor]
    Ku: torch.Tensor                   # [B,Hkv,U,D]    q_dtype
    Vu: torch.Tensor                   # [B,Hkv,U,D]    q_dtype
    unique_len: torch.Tensor           # [B] int32, 0 <= len <= U
    cstar: torch.Tensor                # [B] int64, the chunk each request's query is aimed at

    def to(self, device) -> "Inputs":
        mv = lambda t: None if t is None else t.to(device)
        return Inputs(self.prob, mv(self.Q), mv(self.E), mv(self.Ks), mv(self.Vs), mv(self.scale_k),
                      mv(self.scale_v), mv(self.Ku), mv(self.Vu), mv(self.unique_len), mv(self.cstar))


def _gen(seed: int, stream: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1009 + stream)
    return g


def _randn(shape, g, device):
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32)


def _quantise_fp8(x: torch.Tensor):
    """x [n,Hkv,L,D] f32 -> (fp8 tensor, scale [n,Hkv] f32) with x ~= scale * fp8."""
    amax = x.abs().amax(dim=(2, 3))
    scale = (amax / FP8_MAX).clamp_min(1e-30).to(torch.float32)
    y = (x / scale[:, :, None, None]).clamp_(-FP8_MAX, FP8_MAX)
    return y.to(torch.float8_e4m3fn), scale


def generate(prob: Problem, seed: int = 20251106, device="cpu", unique_len: str = "full",
             slab_elems: int = 1 << 26) -> Inputs:
    """Draw one decode step's inputs for `prob`.  unique_len: "full" (all U) or "ragged"."""
    p = prob
    dev = torch.device(device)
    qd, kvd = torch_dtype(p.q_dtype), torch_dtype(p.kv_dtype)
    G = p.G

    mu = _randn((p.C, p.Hkv, p.D), _gen(seed, 0, dev), dev)

    # request targets c*
    g = _gen(seed, 1, dev)
    if p.popularity == "zipf":
        ranks = torch.arange(1, p.C + 1, device=dev, dtype=torch.float64)
        w = ranks.pow(-p.zipf_s)
        r = torch.multinomial((w / w.sum()).to(torch.float32), p.B, replacement=True, generator=g)
        perm = torch.randperm(p.C, generator=g, device=dev)
        cstar = perm[r]
    else:
        cstar = torch.randint(0, p.C, (p.B,), generator=g, device=dev)

    # queries
    noise = _randn((p.Bq, p.Hq, p.D), _gen(seed, 2, dev), dev)
    mu_q = mu[cstar.repeat_interleave(p.T)]            # [B*T,Hkv,D]: the tokens of a request share its target
    mu_q = mu_q.repeat_interleave(G, dim=1)            # [B*T,Hq,D]  (head hq uses KV head hq//G)
    Q = ((mu_q + noise) / math.sqrt(p.D)).to(qd)

    # shared store, slab by slab over chunks
    Ks = torch.empty((p.C, p.Hkv, p.L, p.D), dtype=kvd, device=dev)
    Vs = torch.empty_like(Ks)
    fp8 = p.kv_dtype == "fp8"
    scale_k = torch.empty((p.C, p.Hkv), dtype=torch.float32, device=dev) if fp8 else None
    scale_v = torch.empty((p.C, p.Hkv), dtype=torch.float32, device=dev) if fp8 else None
    E = torch.empty((p.Hkv, p.C, p.D), dtype=qd, device=dev)
    per_chunk = p.Hkv * p.L * p.D
    step = max(1, slab_elems // per_chunk)
    gk, gv = _gen(seed, 3, dev), _gen(seed, 4, dev)
    for c0 in range(0, p.C, step):
        c1 = min(p.C, c0 + step)
        k = mu[c0:c1, :, None, :] + 0.5 * _randn((c1 - c0, p.Hkv, p.L, p.D), gk, dev)
        v = _randn((c1 - c0, p.Hkv, p.L, p.D), gv, dev)
        if fp8:
            k8, sk = _quantise_fp8(k)
            v8, sv = _quantise_fp8(v)
            Ks[c0:c1], Vs[c0:c1] = k8, v8
            scale_k[c0:c1], scale_v[c0:c1] = sk, sv
            stored = k8.to(torch.float64) * sk[:, :, None, None].to(torch.float64)
        else:
            Ks[c0:c1], Vs[c0:c1] = k.to(kvd), v.to(kvd)
            stored = Ks[c0:c1].to(torch.float64)
        E[:, c0:c1] = stored.mean(dim=2).permute(1, 0, 2).to(qd)
        del k, v, stored

    # unique store, slab by slab over requests
    Ku = torch.empty((p.B, p.Hkv, p.U, p.D), dtype=qd, device=dev)
    Vu = torch.empty_like(Ku)
    per_req = max(1, p.Hkv * p.U * p.D)
    step = max(1, slab_elems // per_req)
    gk, gv = _gen(seed, 5, dev), _gen(seed, 6, dev)
    for b0 in range(0, p.B, step):
        b1 = min(p.B, b0 + step)
        Ku[b0:b1] = (mu[cstar[b0:b1]][:, :, None, :]
                     + 0.5 * _randn((b1 - b0, p.Hkv, p.U, p.D), gk, dev)).to(qd)
        Vu[b0:b1] = _randn((b1 - b0, p.Hkv, p.U, p.D), gv, dev).to(qd)

    if unique_len == "full":
        ulen = torch.full((p.B,), p.U, dtype=torch.int32, device=dev)
    elif unique_len == "ragged":
        ulen = torch.randint(0, p.U + 1, (p.B,), generator=_gen(seed, 7, dev), device=dev).to(torch.int32)
        if p.B >= 2:
            ulen[0] = 0                  # an empty unique context
            ulen[1] = p.U                # and a full one
    else:
        raise ValueError(unique_len)

    return Inputs(p, Q, E, Ks, Vs, scale_k, scale_v, Ku, Vu, ulen, cstar)
