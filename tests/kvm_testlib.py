"""Shared machinery of the GPU parity tests: run the CPU oracle on the same tensors the HIP
library saw, unit by unit, and compare to the bars stated in each test.

Tie protocol.  Slot assignments must agree exactly.  Where they do not, the oracle's own scores
decide: if the library's choice lies within 1e-4 of the oracle's best score (its fp32
matrix-core accumulation rounds differently from the oracle's fp64 sum) the event is counted
as a tie, the oracle is re-run for that unit with that one choice overridden (the oracle checks
the 1e-4 margin itself and refuses anything else), and the comparison goes on.  Any other
disagreement fails.
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import kvm_oracle as ko

F32_EPS = dict(ln_eps=float(np.float32(1e-5)), norm_eps=float(np.float32(1e-12)))
ORACLE_BUDGET = {"none": ko.BUDGET_NONE, "fixed": ko.BUDGET_FIXED, "sqrt": ko.BUDGET_SQRT,
                 "table": ko.BUDGET_TABLE}


def oracle_cfg(w) -> ko.KVMConfig:
    return ko.KVMConfig(head_dim=w.head_dim, rope_dims=w.rope_dims, chunk_len=w.chunk_len,
                        n_bswa_chunks=w.n_bswa_chunks, n_sink=w.n_sink, io=w.io,
                        budget_kind=ORACLE_BUDGET[w.budget_kind], budget_fixed=w.budget_fixed,
                        budget_scale=w.budget_scale,
                        budget_table=list(w.budget_table) if w.budget_kind == "table" else None, **F32_EPS)


def f64(t) -> np.ndarray:
    return t.detach().to("cpu", torch.float64).numpy()


def unit_inputs(w, q, k, v, params, b, h):
    """Slices of one (batch, KV head) unit as fp64 numpy, laid out for the oracle."""
    G = w.n_q_heads // w.n_kv_heads
    qs = f64(q[b, :, h * G:(h + 1) * G]).transpose(1, 0, 2)         # [G, T, d]
    g = params.get("gate")
    return dict(q=qs, k=f64(k[b, :, h]), v=f64(v[b, :, h]), g=None if g is None else f64(g[b, :, h]))


def make_oracle_unit(w, params, h) -> ko.KVMUnit:
    G = w.n_q_heads // w.n_kv_heads
    pick = lambda key, sl: None if params.get(key) is None else f64(params[key][sl])
    return ko.KVMUnit(oracle_cfg(w), G, pick("ln_gamma", h), pick("ln_beta", h),
                      pick("tau_state", slice(h * G, (h + 1) * G)), pick("tau_bswa", slice(h * G, (h + 1) * G)))


def run_oracle_following(w, params, h, drive, gpu_assign, max_rounds=50):
    """Run `drive(unit)` (which feeds tokens and returns outputs) and compare the fold logs with
    gpu_assign [F, C] (the library's trace for this unit).  Ties are overridden and the run is
    repeated.  Returns (outputs of drive, unit, number of counted ties)."""
    overrides, app_overrides, ties = {}, {}, 0
    for _ in range(max_rounds):
        unit = make_oracle_unit(w, params, h)
        unit.overrides, unit.append_overrides = dict(overrides), dict(app_overrides)
        out = drive(unit)
        bad = None
        for f, log in enumerate(unit.fold_logs):
            ga = gpu_assign[f]
            if not np.array_equal(log["assign"], ga):
                bad = (f, log, ga)
                break
        if bad is None:
            assert len(unit.fold_logs) == gpu_assign.shape[0] or len(unit.fold_logs) <= gpu_assign.shape[0]
            return out, unit, ties
        f, log, ga = bad
        m0 = log["m_before"]
        gpu_app = sorted(int(j) for j in np.nonzero(ga >= m0)[0]) if m0 > 0 else None
        ora_app = sorted(int(j) for j in np.nonzero(log["appended"])[0]) if m0 > 0 else None
        ties += 1
        if m0 > 0 and gpu_app != ora_app:
            app_overrides[f] = gpu_app        # the oracle raises unless it is a boundary tie
        else:
            j = int(np.nonzero(log["assign"] != ga)[0][0])
            overrides[(f, j)] = int(ga[j])    # the oracle raises unless within the margin
    raise AssertionError("tie protocol did not converge")


def check_outputs(w, y_gpu: np.ndarray, y_ref: np.ndarray, what=""):
    """fp32: max-abs <= 1e-4.  bf16: per output row, max-abs error <= 2e-2 * max(row max-abs of
    the reference, 1e-3)."""
    err = np.abs(y_gpu - y_ref)
    if w.io == "f32":
        assert err.max() <= 1e-4, f"{what}: fp32 max-abs error {err.max():.3e}"
        return float(err.max())
    row_err = err.max(axis=-1)
    bound = 2e-2 * np.maximum(np.abs(y_ref).max(axis=-1), 1e-3)
    worst = float((row_err / bound).max())
    assert worst <= 1.0, f"{what}: bf16 row error is {worst:.3f} x the 2e-2 relative bound"
    return worst


def check_state(w, exp: dict, unit: ko.KVMUnit, b: int, h: int):
    """Exported library state of unit (b, h) against the oracle's."""
    st = unit.state
    m = st.m
    assert exp["m"] == m
    sK = exp["sK"][b, h].cpu().numpy()
    # both sides add exact products g * k-bar to an fp64 sum in position order
    np.testing.assert_array_equal(sK, st.sK)
    np.testing.assert_allclose(exp["sV"][b, h].cpu().numpy(), st.sV, rtol=2e-5, atol=1e-5)
    np.testing.assert_allclose(exp["rho"][b, h].cpu().numpy(), st.rho, rtol=1e-6)
    np.testing.assert_allclose(exp["w"][b, h].cpu().numpy(), st.w, rtol=1e-5)
    np.testing.assert_array_equal(exp["n"][b, h].cpu().numpy(), st.n)
    khat, vhat = ko.readout(st, unit.cfg, unit.gamma, unit.beta)
    kh_gpu, vh_gpu = f64(exp["khat"][b, h]), f64(exp["vhat"][b, h])
    n_diff = int((kh_gpu != khat).sum())
    # LN_s is done in fp64 on both sides; a rounding flip needs a value within ~1e-15 of a tie
    assert n_diff <= max(1, khat.size // 100000), f"{n_diff} of {khat.size} key readout elements differ"
    tol = 2.0 ** -7 if w.io == "bf16" else 1e-5
    np.testing.assert_allclose(vh_gpu, vhat, rtol=tol, atol=tol * 1e-2)
