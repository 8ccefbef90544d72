"""Seeded synthetic inputs for the KVM layer: shapes and value distributions of the five
benchmark workloads.  This module holds none of the layer's arithmetic; it is the one piece
both the HIP path and the CPU oracle's tests are fed from.

Everything is drawn with a seeded torch.Generator on the requested device, so a tensor made on
the GPU can be copied to the host and handed to the oracle (CPU and GPU streams differ, which
is fine: both sides always see the same tensor).

Recipes (the workload texts leave details open; the choices are fixed here):
  * mixture of Z Gaussians: per (batch, KV head) centres mu^K_z, mu^V_z ~ N(0, I); every token
    draws its component uniformly; k = mu^K_z + sigma*eps, v = mu^V_z + sigma*eps; the query
    heads of the group use the key centres, q = mu^K_z + sigma*eps (own noise), so queries hit
    their own cluster; optional per-KV-head scale ~ U(0.5, 2) on q, k, v.
  * iid N(0,1) with needles: 5% of positions copy the (k, v) pair of another uniformly chosen
    position of the same unit (after the rotary step, so the bits are identical).
  * q and k are then rotated on their first r channels (rotate-half pairing (c, c + r/2), base
    10000, absolute positions) and everything is rounded to the I/O dtype.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Optional

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    io: str                 # "f32" | "bf16"
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq: int                # prefill length T (decode: steps)
    chunk_len: int
    rope_dims: int
    budget_kind: str        # "none" | "fixed" | "sqrt" | "table"
    budget_fixed: int = 0
    budget_scale: float = 0.0
    budget_table: tuple = ()  # "table": budget per chunk index, last entry repeats
    n_bswa_chunks: int = 2
    n_sink: int = 1
    gen: str = "mog"        # "mog" | "needle" | "normal"
    n_centres: int = 8
    sigma: float = 0.3
    head_scale: bool = False
    state_rows: int = 0     # decode workload: rows of the pre-built state
    seed: int = 0x98770000


WORKLOADS = {
    # tiny fp32 layer: correctness configuration
    "tiny_f32": Workload("tiny_f32", "f32", 1, 2, 2, 64, 1024, 64, 16, "fixed", budget_fixed=64,
                         gen="mog", n_centres=8, sigma=0.3, seed=0x98770001),
    # bf16 prefill, fixed state
    "prefill_fixed": Workload("prefill_fixed", "bf16", 4, 16, 16, 128, 16384, 256, 32, "fixed", budget_fixed=512,
                              gen="mog", n_centres=64, sigma=0.5, seed=0x98770002),
    # bf16 prefill, ~sqrt(N) growth
    "prefill_sqrt": Workload("prefill_sqrt", "bf16", 2, 16, 16, 128, 65536, 256, 32, "sqrt", budget_scale=4.0,
                             gen="needle", seed=0x98770003),
    # bf16 batched decode against a pre-built state (chunk 128, window 256)
    "decode": Workload("decode", "bf16", 64, 32, 32, 128, 1000, 128, 32, "fixed", budget_fixed=2048,
                       gen="normal", state_rows=2048, seed=0x98770004),
    # bf16 training-shape forward with grouped queries: the 32k-context headline workload
    "prefill_gqa_32k": Workload("prefill_gqa_32k", "bf16", 8, 32, 8, 128, 32768, 512, 64, "fixed",
                                budget_fixed=1024, gen="mog", n_centres=256, sigma=0.3, head_scale=True,
                                seed=0x98770005),
}


def shrink(w: Workload, **kw) -> Workload:
    """A smaller copy of a workload (tests): same recipe, other sizes."""
    return replace(w, **kw)


def torch_dtype(io: str) -> torch.dtype:
    return torch.bfloat16 if io == "bf16" else torch.float32


def rope_partial(x: torch.Tensor, pos: torch.Tensor, r: int, base: float = 10000.0) -> torch.Tensor:
    """Rotate the first r channels of x [B, T, H, d] at positions pos [T] (fp32 in, fp32 out)."""
    if r == 0:
        return x
    half = r // 2
    inv = base ** (-torch.arange(half, device=x.device, dtype=torch.float32) * 2.0 / r)
    ang = pos.to(torch.float32)[:, None] * inv[None, :]                  # [T, half]
    cos, sin = ang.cos()[None, :, None, :], ang.sin()[None, :, None, :]
    x1, x2 = x[..., :half], x[..., half:r]
    out = x.clone()
    out[..., :half] = x1 * cos - x2 * sin
    out[..., half:r] = x2 * cos + x1 * sin
    return out


def make_qkv(w: Workload, device, T: Optional[int] = None, pos0: int = 0, seed_offset: int = 0):
    """q [B,T,Hq,d], k, v [B,T,Hkv,d] in the workload's I/O dtype, on `device`."""
    T = w.seq if T is None else T
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed + seed_offset)
    B, Hq, Hkv, d = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim
    G = Hq // Hkv

    def normal(*shape):
        return torch.randn(*shape, generator=gen, device=dev, dtype=torch.float32)

    if w.gen == "mog":
        Z = w.n_centres
        mu_k, mu_v = normal(B, Hkv, Z, d), normal(B, Hkv, Z, d)
        z = torch.randint(0, Z, (B, T, Hkv), generator=gen, device=dev)
        bi = torch.arange(B, device=dev)[:, None, None]
        hi = torch.arange(Hkv, device=dev)[None, None, :]
        ck, cv = mu_k[bi, hi, z], mu_v[bi, hi, z]                      # [B,T,Hkv,d]
        k = ck + w.sigma * normal(B, T, Hkv, d)
        v = cv + w.sigma * normal(B, T, Hkv, d)
        q = ck.repeat_interleave(G, dim=2) + w.sigma * normal(B, T, Hq, d)
        if w.head_scale:
            sc = 0.5 + 1.5 * torch.rand(Hkv, generator=gen, device=dev)
            k = k * sc[None, None, :, None]
            v = v * sc[None, None, :, None]
            q = q * sc.repeat_interleave(G)[None, None, :, None]
    else:
        q, k, v = normal(B, T, Hq, d), normal(B, T, Hkv, d), normal(B, T, Hkv, d)
    pos = torch.arange(pos0, pos0 + T, device=dev)
    q = rope_partial(q, pos, w.rope_dims)
    k = rope_partial(k, pos, w.rope_dims)
    dt = torch_dtype(w.io)
    q, k, v = q.to(dt), k.to(dt), v.to(dt)
    if w.gen == "needle":
        n_needle = max(1, int(0.05 * T))
        for b in range(B):
            for h in range(Hkv):
                dst = torch.randperm(T, generator=gen, device=dev)[:n_needle]
                src = torch.randint(0, T, (n_needle,), generator=gen, device=dev)
                k[b, dst, h] = k[b, src, h]
                v[b, dst, h] = v[b, src, h]
    return q.contiguous(), k.contiguous(), v.contiguous()


def make_params(w: Workload, device, plain: bool = True, T: Optional[int] = None):
    """Layer parameters and the merge gate.  plain: gamma=1, beta=0, tau=1, gate=None (timed runs).
    Otherwise seeded gamma ~ U(0.5,1.5), beta ~ N(0, 0.1^2), tau ~ U(0.5,2), g = 1 + ELU(N(0,1))."""
    if plain:
        return dict(ln_gamma=None, ln_beta=None, tau_state=None, tau_bswa=None, gate=None)
    T = w.seq if T is None else T
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed + 7919)
    Hkv, Hq, d = w.n_kv_heads, w.n_q_heads, w.head_dim
    gamma = 0.5 + torch.rand(Hkv, d, generator=gen, device=dev)
    beta = 0.1 * torch.randn(Hkv, d, generator=gen, device=dev)
    ts = 0.5 + 1.5 * torch.rand(Hq, generator=gen, device=dev)
    tb = 0.5 + 1.5 * torch.rand(Hq, generator=gen, device=dev)
    gate = 1.0 + torch.nn.functional.elu(torch.randn(w.batch, T, Hkv, generator=gen, device=dev))
    return dict(ln_gamma=gamma, ln_beta=beta, tau_state=ts, tau_bswa=tb, gate=gate.contiguous())


def make_decode_state(w: Workload, device):
    """A synthetic pre-built state for the decode workload: `state_rows` rows of N(0,1) sums, a
    full window ring of N(0,1) tokens, tokens_seen = a chunk boundary with a full window."""
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed + 104729)
    B, H, d, m = w.batch, w.n_kv_heads, w.head_dim, w.state_rows
    L = w.chunk_len * w.n_bswa_chunks
    dt = torch_dtype(w.io)
    sK = torch.randn(B, H, m, d, generator=gen, device=dev, dtype=torch.float32).to(torch.float64)
    sV = torch.randn(B, H, m, d, generator=gen, device=dev, dtype=torch.float32)
    tokens = ((m + L) // w.chunk_len + 1) * w.chunk_len
    pos = torch.arange(tokens - L, tokens, device=dev)
    wk = torch.randn(B, L, H, d, generator=gen, device=dev, dtype=torch.float32)
    wk = rope_partial(wk, pos, w.rope_dims).to(dt)
    wv = torch.randn(B, L, H, d, generator=gen, device=dev, dtype=torch.float32).to(dt)
    # ring layout [B,H,L,d]: token p sits in slot p % L
    slots = (pos % L)
    win_k = torch.empty(B, H, L, d, dtype=dt, device=dev)
    win_v = torch.empty(B, H, L, d, dtype=dt, device=dev)
    win_k[:, :, slots] = wk.permute(0, 2, 1, 3)
    win_v[:, :, slots] = wv.permute(0, 2, 1, 3)
    return dict(sK=sK.contiguous(), sV=sV.contiguous(), rho=sV.norm(dim=-1).contiguous(),
                w=torch.ones(B, H, m, device=dev), n=torch.ones(B, H, m, dtype=torch.int32, device=dev),
                win_k=win_k, win_v=win_v, win_g=torch.ones(B, H, L, device=dev),
                m=m, tokens=tokens, folds=tokens // w.chunk_len - w.n_bswa_chunks + 1)
