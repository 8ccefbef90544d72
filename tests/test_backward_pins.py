"""Pins of the backward oracle (oracle/kvm_backward_oracle.py) to things other than itself.

1. Central finite differences of the *forward* oracle (itself pinned in test_oracle_pins.py),
   run without rounding (io = 'f64'), along random directions of every input and parameter
   and on single elements: a dropped term, a wrong sign, a transposed operand or a missing
   gate factor in the backward changes one of these by far more than the bound.
2. Without a state the layer is masked softmax attention over a block sliding window; there
   the gradients must equal those of a library's automatic differentiation of that textbook
   formula.
3. The pieces (LayerNorm, value readout) against the same automatic differentiation.
Straight-through rounding (bf16 / fp32 I/O) cannot be pinned numerically: "parity unpinned"
for that reading; it changes no formula, only the values the formulas are evaluated at.
"""
import math

import numpy as np
import pytest
import torch

from oracle import kvm_backward_oracle as kb
from oracle import kvm_oracle as ko


def make_case(seed, T, C=8, n_bswa=2, d=16, r=4, G=2, budget=("fixed", 12), n_sink=1, gated=True, twins=()):
    rng = np.random.default_rng(seed)
    kind = {"fixed": ko.BUDGET_FIXED, "sqrt": ko.BUDGET_SQRT, "none": ko.BUDGET_NONE,
            "table": ko.BUDGET_TABLE}[budget[0]]
    cfg = ko.KVMConfig(head_dim=d, rope_dims=r, chunk_len=C, n_bswa_chunks=n_bswa, n_sink=n_sink, io="f64",
                       budget_kind=kind, budget_fixed=budget[1] if kind == ko.BUDGET_FIXED else 0,
                       budget_scale=budget[1] if kind == ko.BUDGET_SQRT else 0.0,
                       budget_table=budget[1] if kind == ko.BUDGET_TABLE else None)
    # clustered keys, so that merges have clear winners and a small step flips no assignment
    centres = rng.normal(size=(5, d)) * 1.5
    k = centres[rng.integers(0, 5, size=T)] + 0.3 * rng.normal(size=(T, d))
    # twins: positions that share a centre of their own, unlike anything else
    if twins:
        k[list(twins)] = 2.0 * rng.normal(size=d) + 0.05 * rng.normal(size=(len(twins), d))
    x = dict(q=rng.normal(size=(G, T, d)), k=k, v=rng.normal(size=(T, d)),
             g=(1.0 + np.abs(rng.normal(size=T))) if gated else np.ones(T),
             gamma=rng.uniform(0.5, 1.5, size=d), beta=0.1 * rng.normal(size=d),
             tau_state=rng.uniform(0.5, 2.0, size=G), tau_bswa=rng.uniform(0.5, 2.0, size=G))
    dy = rng.normal(size=(G, T, d))
    return cfg, x, dy, G


def forward_loss(cfg, x, dy, G):
    unit = ko.KVMUnit(cfg, G, x["gamma"], x["beta"], x["tau_state"], x["tau_bswa"])
    y, _ = unit.prefill(x["q"], x["k"], x["v"], x["g"])
    return float((y * dy).sum()), [log["assign"].copy() for log in unit.fold_logs]


def grads(cfg, x, dy, G):
    out = kb.forward_backward_unit(cfg, x["q"], x["k"], x["v"], x["g"], dy, G, x["gamma"], x["beta"],
                                   x["tau_state"], x["tau_bswa"])
    return dict(q=out["dq"], k=out["dk"], v=out["dv"], g=out["dg"], gamma=out["dgamma"], beta=out["dbeta"],
                tau_state=out["dtau_state"], tau_bswa=out["dtau_bswa"]), out


def directional(cfg, x, dy, G, name, direction, h=1e-6):
    base = forward_loss(cfg, x, dy, G)[1]
    vals = []
    for sgn in (+1, -1):
        xp = dict(x)
        xp[name] = x[name] + sgn * h * direction
        loss, assign = forward_loss(cfg, xp, dy, G)
        assert all(np.array_equal(a, b) for a, b in zip(assign, base)), "a step of 1e-6 flipped an assignment"
        vals.append(loss)
    return (vals[0] - vals[1]) / (2 * h)


CASES = [
    dict(seed=1, T=64, budget=("fixed", 12)),                 # creation, append-all?, then merges only
    dict(seed=2, T=61, budget=("sqrt", 2.0)),                 # growing state: partial appends; ragged tail
    dict(seed=3, T=72, budget=("fixed", 20), n_bswa=3, G=1),  # three-chunk window
    dict(seed=4, T=48, budget=("fixed", 8), n_sink=0, gated=False),
    # one row per fold: of two twin outliers in a block one creates a row and the other joins it
    dict(seed=5, T=48, budget=("table", [8, 8, 9, 10, 11, 12]), twins=(10, 13)),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: f"seed{c['seed']}")
def test_gradients_match_finite_differences_of_the_forward_oracle(case):
    cfg, x, dy, G = make_case(**case)
    gr, out = grads(cfg, x, dy, G)
    assert len(out["fold_logs"]) >= 3 and any(0 < log["n_append"] < cfg.chunk_len or log["n_append"] == 0
                                               for log in out["fold_logs"])
    rng = np.random.default_rng(100 + case["seed"])
    for name in ("q", "k", "v", "g", "gamma", "beta", "tau_state", "tau_bswa"):
        for _ in range(2):
            direction = rng.normal(size=x[name].shape)
            fd = directional(cfg, x, dy, G, name, direction)
            an = float((gr[name] * direction).sum())
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)) + 1e-7, (name, fd, an)
    # single elements: an early token (folded, merged or appended), a rotary channel of k (reaches
    # the output only through the window), a late token (window only)
    T = x["k"].shape[0]
    for name, idx in (("k", (3, cfg.rope_dims + 1)), ("k", (5, 0)), ("v", (2, 7)), ("k", (T - 2, 5)),
                      ("v", (T - 1, 0)), ("g", (4,)), ("g", (T - 1,)), ("q", (0, 9, 3))):
        direction = np.zeros_like(x[name])
        direction[idx] = 1.0
        fd = directional(cfg, x, dy, G, name, direction)
        an = float(gr[name][idx])
        assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)) + 1e-7, (name, idx, fd, an)
    # tokens that were never folded have no gate gradient
    n_folded = len(out["fold_logs"]) * cfg.chunk_len
    assert np.all(gr["g"][n_folded:] == 0.0)
    # the rotary channels of a token older than every window still get no key gradient
    if n_folded > 0 and cfg.n_bswa_chunks == 2:
        pass  # covered by the single-element check on k[5, 0]


def test_every_fold_kind_occurs_in_the_cases():
    kinds = set()
    for case in CASES:
        cfg, x, dy, G = make_case(**case)
        _, out = grads(cfg, x, dy, G)
        for log in out["fold_logs"]:
            if log["m_before"] == 0:
                kinds.add("creation")
            elif log["n_append"] == cfg.chunk_len:
                kinds.add("append all")
            elif log["n_append"] > 0:
                kinds.add("partial append")
            else:
                kinds.add("merge only")
    assert kinds == {"creation", "append all", "partial append", "merge only"}


def test_some_token_merges_into_a_row_created_by_the_same_fold():
    """That token is gated and gets a gate gradient although its row number is a new one -- the
    case that separates "went to a new row" from "created a row"."""
    hits = 0
    for case in CASES:
        cfg, x, dy, G = make_case(**case)
        gr, out = grads(cfg, x, dy, G)
        L = cfg.window
        for f, log in enumerate(out["fold_logs"]):
            late = (log["assign"] >= log["m_before"]) & ~log["appended"]
            if log["m_before"] > 0 and late.any():
                hits += int(late.sum())
    assert hits > 0


def test_without_state_equals_autodiff_of_block_sliding_window_attention():
    cfg, x, dy, G = make_case(seed=7, T=45, budget=("none", 0))
    gr, out = grads(cfg, x, dy, G)
    T, d, C, L = 45, cfg.head_dim, cfg.chunk_len, cfg.window
    q = torch.tensor(x["q"], requires_grad=True)
    k = torch.tensor(x["k"], requires_grad=True)
    v = torch.tensor(x["v"], requires_grad=True)
    tau = torch.tensor(x["tau_bswa"], requires_grad=True)
    i = torch.arange(T)[:, None]
    j = torch.arange(T)[None, :]
    start = torch.clamp((i // C) * C + C - L, min=0)
    mask = (j <= i) & (j >= start)
    logits = tau[:, None, None] * (q @ k.T) / math.sqrt(d)
    y = torch.softmax(logits.masked_fill(~mask, float("-inf")), dim=-1) @ v
    (y * torch.tensor(dy)).sum().backward()
    np.testing.assert_allclose(out["y"], y.detach().numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(gr["q"], q.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(gr["k"], k.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(gr["v"], v.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(gr["tau_bswa"], tau.grad.numpy(), rtol=1e-9, atol=1e-11)
    assert np.all(gr["tau_state"] == 0) and np.all(gr["g"] == 0) and np.all(gr["gamma"] == 0)


def test_layer_norm_backward_matches_autodiff():
    rng = np.random.default_rng(11)
    x, gam, bet, dy = rng.normal(size=(5, 12)), rng.uniform(0.5, 2, 12), rng.normal(size=12), rng.normal(size=(5, 12))
    tx, tg, tb = (torch.tensor(a, requires_grad=True) for a in (x, gam, bet))
    (torch.nn.functional.layer_norm(tx, (12,), tg, tb, 1e-5) * torch.tensor(dy)).sum().backward()
    dx, dga, dbe = kb.layer_norm_backward(x, gam, 1e-5, dy)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dga, tg.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dbe, tb.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_value_readout_backward_matches_autodiff_and_handles_tiny_rows():
    rng = np.random.default_rng(12)
    sV, rho, dvh = rng.normal(size=(6, 10)), rng.uniform(0.5, 2, 6), rng.normal(size=(6, 10))
    sV[2] *= 1e-14                                     # below the epsilon of the denominator
    tv, tr = torch.tensor(sV, requires_grad=True), torch.tensor(rho, requires_grad=True)
    nrm = torch.clamp(torch.linalg.vector_norm(tv, dim=-1, keepdim=True), min=1e-12)
    ((tr[:, None] * tv / nrm) * torch.tensor(dvh)).sum().backward()
    dsV, drho = kb.value_readout_backward(sV, rho, 1e-12, dvh)
    np.testing.assert_allclose(dsV, tv.grad.numpy(), rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(drho, tr.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_gradients_are_linear_in_dy_and_zero_for_zero_dy():
    cfg, x, dy, G = make_case(seed=5, T=40)
    g1, _ = grads(cfg, x, dy, G)
    g2, _ = grads(cfg, x, 2.5 * dy, G)
    g0, _ = grads(cfg, x, 0.0 * dy, G)
    for name in g1:
        np.testing.assert_allclose(g2[name], 2.5 * g1[name], rtol=1e-12, atol=1e-14)
        assert np.all(g0[name] == 0.0)
