"""CPU oracle for the attention weight preparation in front of the KVM layer -- TEST
INFRASTRUCTURE ONLY.

A plain fp64 numpy statement of the paper's appendix "GPTAlpha-2 Attention weight preparation"
(value residual, token shift, LayerNorm with bias on queries and keys, rotary embedding on the
first r channels) and of the merge gate of the Method section ("KVM weight preparation":
g_t = 1 + ELU(x_t W_g)), in the paper's order.  The input projections themselves (x W_Q, x W_K,
x W_V) are not part of it: the "simple" query, key and value arrive as inputs.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module.  It
shares no code with the HIP library and imports nothing from it.

Arithmetic: fp64 throughout; the inputs are values of the I/O dtype widened to fp64, and only
the three outputs q, k, v are rounded to the I/O dtype, once, at the end.  The gate is fp32 on
the device and is not rounded here.

Readings where the paper is silent:
  * Order: value residual on the simple value first, then token shift of q, k and v (each with
    its own coefficient vector alpha), then LN_q / LN_k, then the rotation -- the order in
    which the appendix lists the equations.
  * Token shift of the first token: a_0 = a~_0 (stated); a call that continues a sequence is
    handed the previous token's simple rows instead.
  * Rotary convention (the paper fixes only the base, 10 000, and that r of the d_h channels
    rotate): channel c < r/2 pairs with channel c + r/2, angle = position * base^(-2c/r),
    absolute positions.  The same convention generates the synthetic keys of the KVM tests.
  * LayerNorm: biased variance over the d_h channels of one head, eps = 1e-5.
  * alpha, lambda, LN parameters are per head and channel ([H, d_h]); W_g has one column per
    KV head (the gate is "a scalar for each head").

Pinned by tests/test_prep_pins.py: closed forms of the shift and of the residual, torch's
layer_norm, rotation invariants (norm, relative-position property, identity at position 0),
ELU closed forms.  Exact output values for general inputs are "parity unpinned".
"""
from __future__ import annotations

from typing import Optional

import numpy as np

from .kvm_oracle import round_io


def value_residual(v: np.ndarray, v_first: Optional[np.ndarray], lam: Optional[np.ndarray]) -> np.ndarray:
    """v~_t <- (1 - lambda) v~_t + lambda v~first_t (appendix, "value residual").
    v, v_first [T, H, d]; lam [H, d] or None (no residual)."""
    if v_first is None or lam is None:
        return v.copy()
    return (1.0 - lam)[None] * v + lam[None] * v_first


def token_shift(a: np.ndarray, alpha: Optional[np.ndarray], prev: Optional[np.ndarray]) -> np.ndarray:
    """a_t = a~_t + alpha * (a~_{t-1} - a~_t), a_0 = a~_0 (appendix, "token shift").
    a [T, H, d]; alpha [H, d] or None (no shift); prev [H, d]: the simple row of the token before
    this block, or None when the block starts the sequence."""
    if alpha is None:
        return a.copy()
    out = a.copy()
    out[1:] = a[1:] + alpha[None] * (a[:-1] - a[1:])
    if prev is not None:
        out[0] = a[0] + alpha * (prev - a[0])
    return out


def layer_norm_heads(x: np.ndarray, gamma: Optional[np.ndarray], beta: Optional[np.ndarray],
                     eps: float) -> np.ndarray:
    """LayerNorm with bias over the last axis, parameters per head ("LN_q", "LN_k")."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    y = (x - mu) / np.sqrt(var + eps)
    if gamma is not None:
        y = y * gamma[None]
    if beta is not None:
        y = y + beta[None]
    return y


def rope_r(x: np.ndarray, pos: np.ndarray, r: int, base: float = 10000.0) -> np.ndarray:
    """RoPE_r: rotate channel pairs (c, c + r/2), c < r/2, of x [T, H, d] by pos * base^(-2c/r)."""
    if r == 0:
        return x.copy()
    half = r // 2
    c = np.arange(half, dtype=np.float64)
    ang = pos.astype(np.float64)[:, None] * base ** (-2.0 * c / r)[None, :]   # [T, half]
    cos, sin = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    out = x.copy()
    x1, x2 = x[..., :half], x[..., half:r]
    out[..., :half] = x1 * cos - x2 * sin
    out[..., half:r] = x2 * cos + x1 * sin
    return out


def merge_gate(x: np.ndarray, w_g: np.ndarray) -> np.ndarray:
    """g_t = 1 + ELU(x_t W_g) per KV head (Method, "merge gate").  x [T, d_model], w_g [d_model, H_kv]."""
    z = x @ w_g
    return 1.0 + np.where(z > 0.0, z, np.expm1(np.minimum(z, 0.0)))


def prepare(q_raw, k_raw, v_raw, pos, r, io, *, v_first=None, lam=None, alpha_q=None, alpha_k=None,
            alpha_v=None, lnq=(None, None), lnk=(None, None), eps=1e-5, base=10000.0,
            prev_q=None, prev_k=None, prev_v=None, x=None, w_g=None):
    """The whole preparation for one sequence: simple q [T, H_q, d], k, v [T, H_kv, d] -> the q, k,
    v the KVM layer takes (rounded to the I/O dtype) and, with x and W_g, the merge gate.
    prev_v is the previous token's value after its own value residual."""
    v = value_residual(v_raw, v_first, lam)
    q = token_shift(q_raw, alpha_q, prev_q)
    k = token_shift(k_raw, alpha_k, prev_k)
    v = token_shift(v, alpha_v, prev_v)
    q = rope_r(layer_norm_heads(q, lnq[0], lnq[1], eps), pos, r, base)
    k = rope_r(layer_norm_heads(k, lnk[0], lnk[1], eps), pos, r, base)
    g = None if x is None or w_g is None else merge_gate(x, w_g)
    return round_io(q, io), round_io(k, io), round_io(v, io), g
