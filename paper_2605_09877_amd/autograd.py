"""torch.autograd front end of the layer: one differentiable call for a whole sequence.

Marshalling only.  The forward is kvm_prefill_chunked on a fresh state with the fold record
switched on; the backward is kvm_prefill_backward on that state.  Every step runs in the
library's HIP kernels.
"""
from __future__ import annotations

from typing import Optional

import torch

from .binding import KVM_BF16, KVM_BUDGET_FIXED, KVM_F32, KVMState


class _KVMAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, q, k, v, gate, ln_gamma, ln_beta, tau_state, tau_bswa, cfg: dict):
        B, T, Hq, d = q.shape
        Hkv = k.shape[2]
        st = KVMState(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d,
                      io_dtype=KVM_BF16 if q.dtype == torch.bfloat16 else KVM_F32,
                      ln_gamma=ln_gamma, ln_beta=ln_beta, tau_state=tau_state, tau_bswa=tau_bswa,
                      max_tokens=T, device=str(q.device), **cfg)
        n_folds = T // cfg["chunk_len"] + 1
        assign, score = st.trace(n_folds)
        q, k, v = q.contiguous(), k.contiguous(), v.contiguous()
        gate = None if gate is None else gate.to(torch.float32).contiguous()
        out, lse = st.prefill(q, k, v, gate, want_lse=True)
        ctx.state, ctx.record = st, (assign, score)
        ctx.save_for_backward(q, k, v, gate if gate is not None else q.new_empty(0), out, lse)
        ctx.has_gate = gate is not None
        ctx.param_shapes = tuple(None if p is None else (p.dtype, p.shape) for p in (ln_gamma, ln_beta, tau_state, tau_bswa))
        return out

    @staticmethod
    def backward(ctx, dout):
        q, k, v, gate, out, lse = ctx.saved_tensors
        assign, score = ctx.record
        g = ctx.state.backward(q, k, v, gate if ctx.has_gate else None, out, lse, dout.contiguous(), assign, score)
        ctx.state.close()
        params = []
        for name, spec in zip(("dgamma", "dbeta", "dtau_state", "dtau_bswa"), ctx.param_shapes):
            params.append(None if spec is None else g[name].to(spec[0]).reshape(spec[1]))
        return (g["dq"], g["dk"], g["dv"], g["dgate"] if ctx.has_gate else None, *params, None)


def kvm_attention(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, gate: Optional[torch.Tensor] = None, *,
                  chunk_len: int, rope_dims: int, n_bswa_chunks: int = 2, n_sink: int = 1,
                  budget_kind: int = KVM_BUDGET_FIXED, budget_fixed: int = 0, budget_scale: float = 0.0,
                  budget_table=None, ln_gamma: Optional[torch.Tensor] = None, ln_beta: Optional[torch.Tensor] = None,
                  tau_state: Optional[torch.Tensor] = None, tau_bswa: Optional[torch.Tensor] = None,
                  ln_eps: float = 1e-5, norm_eps: float = 1e-12) -> torch.Tensor:
    """The KVM layer over a whole sequence from an empty state, differentiable in q, k, v, the merge
    gate, the LN_s parameters and the temperatures.  q [B, T, Hq, d]; k, v [B, T, Hkv, d] (bf16 or
    fp32, prepared: normalised and rotated); gate [B, T, Hkv] fp32 or None.  Returns out like q."""
    cfg = dict(chunk_len=chunk_len, rope_dims=rope_dims, n_bswa_chunks=n_bswa_chunks, n_sink=n_sink,
               budget_kind=budget_kind, budget_fixed=budget_fixed, budget_scale=budget_scale,
               budget_table=budget_table, ln_eps=ln_eps, norm_eps=norm_eps)
    return _KVMAttention.apply(q, k, v, gate, ln_gamma, ln_beta, tau_state, tau_bswa, cfg)
