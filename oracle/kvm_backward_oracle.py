"""CPU oracle for the backward pass of the Key-Value Means (KVM) layer -- TEST INFRASTRUCTURE ONLY.

The paper benchmarks a backward pass ("Speed Benchmarks") without spelling it out; what it has
to compute is fixed by the forward definition ("KVM Formulation"): the gradient of a scalar
loss with respect to q, k, v, the merge gate g, the LN_s parameters and the two temperatures,
given the gradient dy of the layer's output.  This file writes that gradient out by the chain
rule, in fp64, one (batch, KV-head) unit at a time, stepping back through the forward's own
steps in reverse order: chunk attention, readout ("Readout"), fold ("Append", "Merge"),
memory key (equation "memory key").

Readings (the paper is silent on all of them):
  * The slot assignment (which tokens are appended, which row a token merges into) is a
    piecewise constant function of the inputs: it gets no gradient and is replayed as
    recorded by the forward.
  * The roundings of the materialised vectors (k-bar, s-hat^K, s-hat^V in the I/O dtype) are
    treated as the identity by the backward pass (straight through); the rounded values are
    the ones the forward used and are used here wherever the forward used them.
  * The layer's output is a materialised vector too: the backward pass reads it as the forward
    stored it, rounded to the I/O dtype (it enters through the softmax's own term, the row sums
    of dy * y).
  * A new row's radius rho = ||v|| carries gradient to the value that created it.
  * The gradient of g is reported also when the forward ran without a gate (g = 1).
  * With grouped queries the gradients of the shared keys, values and state sum over the
    query heads of the group.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module.  It
shares no code with the HIP library.  The forward steps are the ones of oracle/kvm_oracle.py,
called, not repeated.

Pinned by tests/test_backward_pins.py: central finite differences of the forward oracle (run
without rounding) for every input and parameter, and the special case without a state, which
is textbook masked softmax attention differentiated by a library's automatic differentiation.
The straight-through treatment of the roundings (bf16 / fp32 I/O) is a reading that changes no
formula, only the values the formulas are evaluated at, and no numerical pin can check it:
parity unpinned for that reading.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from oracle import kvm_oracle as ko


def layer_norm_backward(x: np.ndarray, gamma: np.ndarray, eps: float, dy: np.ndarray
                        ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Backward of y = (x - mean) / sqrt(var + eps) * gamma + beta over the last axis.

    Returns (dx, dgamma, dbeta); the parameter gradients are summed over the leading axes."""
    x = np.asarray(x, dtype=np.float64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    sigma = np.sqrt(var + eps)
    xhat = (x - mu) / sigma
    dxhat = dy * gamma
    dx = (dxhat - dxhat.mean(axis=-1, keepdims=True)
          - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True)) / sigma
    lead = tuple(range(x.ndim - 1))
    return dx, (dy * xhat).sum(axis=lead), dy.sum(axis=lead)


def value_readout_backward(sV: np.ndarray, rho: np.ndarray, eps: float, dvhat: np.ndarray
                           ) -> Tuple[np.ndarray, np.ndarray]:
    """Backward of s-hat^V = rho * s^V / max(||s^V||, eps), row-wise.  Returns (ds^V, drho)."""
    nrm = np.sqrt((sV * sV).sum(axis=-1, keepdims=True))
    den = np.maximum(nrm, eps)
    unit = sV / den
    drho = (dvhat * unit).sum(axis=-1)
    dsV = rho[:, None] * dvhat / den
    # the norm itself moves with s^V only while it is the one in the denominator
    live = nrm > eps
    dsV = dsV - np.where(live, rho[:, None] * unit * (dvhat * unit).sum(axis=-1, keepdims=True) / den, 0.0)
    return dsV, drho


def attend_backward(q, q_pos, khat, vhat, k_win, v_win, win_pos, tau_state, tau_bswa, lse, y, dy):
    """Backward of kvm_oracle.attend.  Shapes as there; lse, y its results, dy [G, nq, d].

    Returns dq [G, nq, d], dkhat [m, d], dvhat [m, d], dk_win [w, d], dv_win [w, d],
    dtau_state [G], dtau_bswa [G]."""
    G, nq, d = q.shape
    m = khat.shape[0]
    scale = 1.0 / math.sqrt(d)
    dq = np.zeros_like(q)
    dkhat, dvhat = np.zeros((m, d)), np.zeros((m, d))
    dk_win, dv_win = np.zeros_like(k_win), np.zeros_like(v_win)
    dts, dtb = np.zeros(G), np.zeros(G)
    visible = win_pos[None, :] <= q_pos[:, None]
    for h in range(G):
        delta = (dy[h] * y[h]).sum(axis=-1, keepdims=True)           # [nq, 1]
        if m:
            raw = (q[h] @ khat.T) * scale                            # logits before the temperature
            p = np.exp(tau_state[h] * raw - lse[h][:, None])
            dlogit = p * (dy[h] @ vhat.T - delta)
            dvhat += p.T @ dy[h]
            dts[h] = (dlogit * raw).sum()
            dq[h] += tau_state[h] * scale * (dlogit @ khat)
            dkhat += tau_state[h] * scale * (dlogit.T @ q[h])
        raw = (q[h] @ k_win.T) * scale
        p = np.where(visible, np.exp(tau_bswa[h] * raw - lse[h][:, None]), 0.0)
        dlogit = p * (dy[h] @ v_win.T - delta)
        dv_win += p.T @ dy[h]
        dtb[h] = (dlogit * raw).sum()
        dq[h] += tau_bswa[h] * scale * (dlogit @ k_win)
        dk_win += tau_bswa[h] * scale * (dlogit.T @ q[h])
    return dq, dkhat, dvhat, dk_win, dv_win, dts, dtb


def forward_backward_unit(cfg: ko.KVMConfig, q: np.ndarray, k: np.ndarray, v: np.ndarray,
                          g: Optional[np.ndarray], dy: np.ndarray, n_q_heads: int = 1,
                          gamma: Optional[np.ndarray] = None, beta: Optional[np.ndarray] = None,
                          tau_state: Optional[np.ndarray] = None, tau_bswa: Optional[np.ndarray] = None,
                          overrides: Optional[Dict[Tuple[int, int], int]] = None,
                          append_overrides: Optional[Dict[int, Sequence[int]]] = None,
                          round_output: bool = True, stored_output: Optional[np.ndarray] = None) -> dict:
    """Forward (from an empty state, position 0) and backward of one unit over T tokens.

    stored_output [G, T, d]: the layer's output as the caller stored it.  A backward call is
    handed that tensor, not the exact output, and the softmax term D_i = sum_c dy_ic * y_ic is taken
    over it; when given it replaces this function's own (rounded) output in that one place.

    round_output=False lets the backward read the unrounded output instead of the stored one:
    the difference between the two results is how far the rounding of the output alone moves
    each gradient, which tests use to size their bars.

    q, dy: [G, T, d]; k, v: [T, d]; g: [T] or None.  overrides / append_overrides as in
    kvm_oracle.KVMUnit (they let a test follow a run after a counted tie).
    Returns y, lse, fold_logs and the gradients dq [G,T,d], dk, dv [T,d], dg [T],
    dgamma, dbeta [d], dtau_state, dtau_bswa [G].
    """
    G, T, d = q.shape
    C, L = cfg.chunk_len, cfg.window
    unit = ko.KVMUnit(cfg, n_q_heads, gamma, beta, tau_state, tau_bswa)
    unit.overrides = dict(overrides or {})
    unit.append_overrides = dict(append_overrides or {})
    gamma_, beta_, ts, tb = unit.gamma, unit.beta, unit.tau_state, unit.tau_bswa
    k = np.asarray(k, np.float64)
    v = np.asarray(v, np.float64)
    gates = np.ones(T) if g is None else np.asarray(g, np.float64)

    # ---- forward, chunk by chunk, keeping what each chunk saw
    y, lse = np.zeros((G, T, d)), np.zeros((G, T))
    seen: List[dict] = []
    s = 0
    while s < T:
        e = min(s + C, T)
        st = unit.state
        snap = dict(s=s, e=e, sK=st.sK.copy(), sV=st.sV.copy(), rho=st.rho.copy(), n_folds=len(unit.fold_logs))
        y[:, s:e], lse[:, s:e] = unit.prefill(q[:, s:e], k[s:e], v[s:e], gates[s:e])
        snap["fold"] = unit.fold_logs[-1] if len(unit.fold_logs) > snap["n_folds"] else None
        seen.append(snap)
        s = e

    # ---- backward
    dq = np.zeros((G, T, d))
    dk, dv, dg = np.zeros((T, d)), np.zeros((T, d)), np.zeros(T)
    dgamma, dbeta = np.zeros(d), np.zeros(d)
    dts, dtb = np.zeros(G), np.zeros(G)
    m_end = unit.state.m
    dsK, dsV, drho = np.zeros((m_end, d)), np.zeros((m_end, d)), np.zeros(m_end)   # adjoint of the state sums

    for snap in reversed(seen):
        s, e = snap["s"], snap["e"]
        log = snap["fold"]
        if log is not None and cfg.budget_kind != ko.BUDGET_NONE:
            # the fold that followed this chunk, undone: its block is [e - L, e - L + C)
            lo = e - L
            blk = slice(lo, lo + C)
            kz = k[blk].copy()
            kz[:, : cfg.rope_dims] = 0.0
            kbar = ko.memory_key(k[blk], cfg, gamma_, beta_)
            dkbar = np.zeros((C, d))
            for j in range(C):
                i = int(log["assign"][j])
                t = lo + j
                if log["appended"][j]:
                    # new row: ungated copy; rho = ||v||
                    dkbar[j] = dsK[i]
                    nv = math.sqrt(float((v[t] * v[t]).sum()))
                    dv[t] += dsV[i] + (drho[i] * v[t] / nv if nv > 0.0 else 0.0)
                else:
                    dkbar[j] = gates[t] * dsK[i]
                    dv[t] += gates[t] * dsV[i]
                    dg[t] += float(dsK[i] @ kbar[j]) + float(dsV[i] @ v[t])
            dkz, dga, dbe = layer_norm_backward(kz, gamma_, cfg.ln_eps, dkbar)
            dkz[:, : cfg.rope_dims] = 0.0
            dk[blk] += dkz
            dgamma += dga
            dbeta += dbe
            m0 = int(log["m_before"])
            dsK, dsV, drho = dsK[:m0], dsV[:m0], drho[:m0]   # rows created by this fold end here

        # attention of the chunk against the state version it saw and its window
        state_then = ko.UnitState(d, snap["sK"], snap["sV"], snap["rho"])
        m = state_then.m
        assert m == dsK.shape[0]
        khat, vhat = ko.readout(state_then, cfg, gamma_, beta_)
        b = max(0, (s // C) * C + C - L)
        pos_q, pos_w = np.arange(s, e), np.arange(b, e)
        a_dq, a_dkh, a_dvh, a_dkw, a_dvw, a_dts, a_dtb = attend_backward(
            q[:, s:e], pos_q, khat, vhat, k[b:e], v[b:e], pos_w, ts, tb, lse[:, s:e],
            np.asarray(stored_output, np.float64)[:, s:e] if stored_output is not None
            else ko.round_io(y[:, s:e], cfg.io) if round_output else y[:, s:e], dy[:, s:e])
        dq[:, s:e] += a_dq
        dk[b:e] += a_dkw
        dv[b:e] += a_dvw
        dts += a_dts
        dtb += a_dtb
        if m:
            r_dsK, dga, dbe = layer_norm_backward(snap["sK"], gamma_, cfg.ln_eps, a_dkh)
            r_dsV, r_drho = value_readout_backward(snap["sV"], snap["rho"], cfg.norm_eps, a_dvh)
            dsK = dsK + r_dsK
            dsV = dsV + r_dsV
            drho = drho + r_drho
            dgamma += dga
            dbeta += dbe

    return dict(y=y, lse=lse, fold_logs=unit.fold_logs, dq=dq, dk=dk, dv=dv, dg=dg, dgamma=dgamma,
                dbeta=dbeta, dtau_state=dts, dtau_bswa=dtb, m=m_end)
