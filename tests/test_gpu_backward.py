"""Parity of kvm_prefill_backward (through the C ABI) with the backward oracle, unit by unit, on
seeded inputs: every gradient, element by element.

Bars.  fp32 I/O: max-abs error <= 1e-4 * max(1, max-abs of the reference tensor) (the gradients
are fp32 sums of up to (m + L) * G * C products of O(1) numbers); 1e-3 for the temperature and
LN_s gradients, which are sums over every row of the sequence of terms of both signs whose
absolute values add up to some 1e2..1e3 times the result, so that fp32 rounding of the terms
(and the order in which token sums are taken apart again) shows at the 1e-4 level.  bf16 I/O: max-abs error <= 2e-2 *
max-abs of the reference tensor of the unit (of the whole tensor for the parameter gradients).
The backward call is handed the forward's output as the library stored it (bf16); the oracle is
handed that very tensor for the softmax term D_i = sum_c dy_ic y_ic (`stored_output`), so both
sides differentiate from the same stored values and the bar covers only what the bf16 kernels
themselves round: P^T and dS^T as bf16 operands of the second products (2^-9 relative per term)
and the bf16 store of dq, dk, dv (2^-9 of the element).  The bar is relative to the tensor, not
to the row, because a row's gradient is a sum of terms of both signs whose rounding errors scale
with the terms, not with the sum.  Slot assignments follow the forward's record under the tie
protocol of kvm_testlib.
"""
import numpy as np
import pytest
import torch

import kvm_testlib as tl
from oracle import kvm_backward_oracle as kb

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def kvm():
    import paper_2605_09877_amd as pkg
    return pkg


def synth():
    from paper_2605_09877_amd import synth as s
    return s


def oracle_unit_following(w, params, u, dy, h, gpu_assign, **kw):
    """forward_backward_unit with the library's counted ties overridden, under the same ceiling on
    their number as the forward tests (see kvm_testlib)."""
    G = w.n_q_heads // w.n_kv_heads
    pick = lambda key, sl: None if params.get(key) is None else tl.f64(params[key][sl])
    overrides, app_overrides, ties = {}, {}, tl.Ties()
    ceiling = tl.tie_ceiling(w, gpu_assign.shape[0])
    while True:
        res = kb.forward_backward_unit(
            tl.oracle_cfg(w), u["q"], u["k"], u["v"], u["g"], dy, G, pick("ln_gamma", h), pick("ln_beta", h),
            pick("tau_state", slice(h * G, (h + 1) * G)), pick("tau_bswa", slice(h * G, (h + 1) * G)),
            overrides=overrides, append_overrides=app_overrides, **kw)
        assert len(res["fold_logs"]) == gpu_assign.shape[0]
        bad = None
        for f, log in enumerate(res["fold_logs"]):
            if not np.array_equal(log["assign"], gpu_assign[f]):
                bad = (f, log, gpu_assign[f])
                break
        if bad is None:
            res["ties"] = ties
            return res
        f, log, ga = bad
        m0 = log["m_before"]
        gpu_app = sorted(int(j) for j in np.nonzero(ga >= m0)[0]) if m0 > 0 else None
        ora_app = sorted(int(j) for j in np.nonzero(log["appended"])[0]) if m0 > 0 else None
        if m0 > 0 and gpu_app != ora_app:
            assert f not in app_overrides
            ties.append += 1
            app_overrides[f] = gpu_app
        else:
            j = int(np.nonzero(log["assign"] != ga)[0][0])
            assert (f, j) not in overrides
            ties.merge += 1
            overrides[(f, j)] = int(ga[j])
        assert ties.total <= ceiling, f"{ties}: more than the {ceiling} allowed"


def check(w, name, got, ref, f32_bar=1e-4):
    err = np.abs(got - ref)
    top = float(np.abs(ref).max())
    if w.io == "f32":
        assert err.max() <= f32_bar * max(1.0, top), f"{name}: fp32 max-abs error {err.max():.3e} (reference max {top:.3e})"
        return
    worst = float(err.max() / (2e-2 * top + 1e-6))
    assert worst <= 1.0, f"{name}: bf16 error is {worst:.3f} x the 2e-2 bound"


def run_backward_case(w, plain, units=None, split=None):
    """Forward with the fold record on, backward, and the oracle on every unit (or on the sampled
    `units`: then the gradients summed over all units -- LN_s, temperatures -- are not checked)."""
    pkg, sy = kvm(), synth()
    q, k, v = sy.make_qkv(w, DEV)
    params = sy.make_params(w, DEV, plain=plain)
    gate = params["gate"]
    gen = torch.Generator(device=DEV)
    gen.manual_seed(w.seed + 31337)
    dout = torch.randn(q.shape, generator=gen, device=DEV, dtype=torch.float32).to(q.dtype)
    st = pkg.state_for(w, device=DEV, **params)
    assign, score = st.trace(w.seq // w.chunk_len + 1)
    if split is None:
        out, lse = st.prefill(q, k, v, gate, want_lse=True)
    else:  # the forward in two calls (the second starts on a chunk boundary); one backward over all of it
        parts = [st.prefill(q[:, lo:hi].contiguous(), k[:, lo:hi].contiguous(), v[:, lo:hi].contiguous(),
                            None if gate is None else gate[:, lo:hi].contiguous(), want_lse=True)
                 for lo, hi in ((0, split), (split, w.seq))]
        out = torch.cat([p[0] for p in parts], dim=1).contiguous()
        lse = torch.cat([p[1] for p in parts], dim=1).contiguous()
    g = st.backward(q, k, v, gate, out, lse, dout, assign, score)
    torch.cuda.synchronize()
    ga_all = assign[:st.folds].cpu().numpy()
    G = w.n_q_heads // w.n_kv_heads
    d = w.head_dim
    sums = dict(dgamma=np.zeros((w.n_kv_heads, d)), dbeta=np.zeros((w.n_kv_heads, d)),
                dtau_state=np.zeros(w.n_q_heads), dtau_bswa=np.zeros(w.n_q_heads))
    kinds = set()
    all_units = [(b, h) for b in range(w.batch) for h in range(w.n_kv_heads)]
    for key in ("dq", "dk", "dv", "dgate", "dgamma", "dbeta", "dtau_state", "dtau_bswa"):
        assert bool(torch.isfinite(g[key].float()).all()), f"{key} has non-finite entries"
    for (b, h) in (all_units if units is None else units):
        u = tl.unit_inputs(w, q, k, v, params, b, h)
        dy = tl.f64(dout[b, :, h * G:(h + 1) * G]).transpose(1, 0, 2)
        y_stored = tl.f64(out[b, :, h * G:(h + 1) * G]).transpose(1, 0, 2)
        res = oracle_unit_following(w, params, u, dy, h, ga_all[:, b, h], stored_output=y_stored)
        assert res["m"] == st.rows and len(res["fold_logs"]) == st.folds
        for log in res["fold_logs"]:
            kinds.add("creation" if log["m_before"] == 0 else "append all" if log["n_append"] == w.chunk_len
                      else "partial append" if log["n_append"] > 0 else "merge only")
        what = f"unit {(b, h)}"
        check(w, f"dq {what}", tl.f64(g["dq"][b, :, h * G:(h + 1) * G]).transpose(1, 0, 2), res["dq"])
        check(w, f"dk {what}", tl.f64(g["dk"][b, :, h]), res["dk"])
        check(w, f"dv {what}", tl.f64(g["dv"][b, :, h]), res["dv"])
        check(w, f"dgate {what}", tl.f64(g["dgate"][b, :, h]), res["dg"])
        sums["dgamma"][h] += res["dgamma"]
        sums["dbeta"][h] += res["dbeta"]
        sums["dtau_state"][h * G:(h + 1) * G] += res["dtau_state"]
        sums["dtau_bswa"][h * G:(h + 1) * G] += res["dtau_bswa"]
    if units is None:
        for name, ref in sums.items():
            check(w, name, tl.f64(g[name]), ref, f32_bar=1e-3)
    return kinds


def test_f32_backward_fixed_budget_with_parameters():
    w = synth().shrink(synth().WORKLOADS["tiny_f32"], batch=2, seq=64 * 9 + 17)
    kinds = run_backward_case(w, plain=False)
    assert {"creation", "merge only"} <= kinds


def test_f32_backward_growing_state_grouped_queries():
    w = synth().shrink(synth().WORKLOADS["tiny_f32"], n_q_heads=4, n_kv_heads=2, seq=64 * 12, budget_kind="sqrt",
                       budget_scale=4.0, n_sink=2)
    kinds = run_backward_case(w, plain=False)
    assert "partial append" in kinds


def test_f32_backward_plain_parameters_three_chunk_window():
    w = synth().shrink(synth().WORKLOADS["tiny_f32"], seq=64 * 8, n_bswa_chunks=3, budget_fixed=160)
    kinds = run_backward_case(w, plain=True)
    assert "append all" in kinds or "partial append" in kinds


def test_f32_backward_without_state():
    w = synth().shrink(synth().WORKLOADS["tiny_f32"], seq=64 * 4 + 5, budget_kind="none")
    run_backward_case(w, plain=False)


def test_bf16_backward_d128():
    w = synth().shrink(synth().WORKLOADS["prefill_fixed"], batch=1, n_q_heads=4, n_kv_heads=2, seq=128 * 7 + 64,
                       chunk_len=128, budget_fixed=192)
    run_backward_case(w, plain=False)


def test_bf16_backward_grouped_queries_growing_state_ragged_tail():
    w = synth().shrink(synth().WORKLOADS["prefill_sqrt"], batch=1, n_q_heads=8, n_kv_heads=2, seq=256 * 6 + 100,
                       chunk_len=256, budget_scale=8.0)
    kinds = run_backward_case(w, plain=True)
    assert "partial append" in kinds


def test_bf16_backward_short_chunks_three_chunk_window():
    w = synth().shrink(synth().WORKLOADS["prefill_gqa_32k"], batch=2, n_q_heads=4, n_kv_heads=2, seq=64 * 11 + 7,
                       chunk_len=64, n_bswa_chunks=3, budget_fixed=96, rope_dims=32)
    run_backward_case(w, plain=False)


@pytest.mark.parametrize("seq", [64 + 5, 128, 64 * 3])
def test_f32_backward_of_short_sequences(seq):
    """No fold at all (shorter than the window), exactly one window (one fold, after the last
    chunk, that no query sees), and one chunk more."""
    w = synth().shrink(synth().WORKLOADS["tiny_f32"], seq=seq)
    run_backward_case(w, plain=False)


def test_f32_backward_head_dim_128_table_budget_no_sinks():
    w = synth().shrink(synth().WORKLOADS["tiny_f32"], head_dim=128, rope_dims=32, seq=64 * 7 + 9, n_sink=0,
                       budget_kind="table", budget_table=(0, 64, 70, 70, 100, 101))
    kinds = run_backward_case(w, plain=False)
    assert "partial append" in kinds


def test_bf16_backward_head_dim_64_on_the_vector_kernels():
    w = synth().shrink(synth().WORKLOADS["prefill_fixed"], batch=1, n_q_heads=4, n_kv_heads=2, head_dim=64, rope_dims=16,
                       seq=64 * 6 + 30, chunk_len=64, budget_fixed=96)
    run_backward_case(w, plain=False)


def test_bf16_backward_of_one_window():
    w = synth().shrink(synth().WORKLOADS["prefill_fixed"], batch=1, n_q_heads=2, n_kv_heads=2, seq=512, chunk_len=256)
    run_backward_case(w, plain=False)


@pytest.mark.parametrize("name,n_units", [("prefill_gqa_32k", 2), ("prefill_fixed", 2), ("prefill_sqrt", 1)])
def test_full_size_backward_sampled_units(name, n_units):
    """The prefill workloads at full size, in the configuration bench.py times (plain parameters,
    no gate): the library runs the whole backward pass, the oracle replays the last (and the
    first) (batch, KV head) unit over all chunks and folds."""
    w = synth().WORKLOADS[name]
    units = [(w.batch - 1, w.n_kv_heads - 1), (0, 0)][:n_units]
    run_backward_case(w, plain=True, units=units)


def test_backward_after_a_forward_in_two_calls():
    w = synth().shrink(synth().WORKLOADS["prefill_fixed"], batch=1, n_q_heads=4, n_kv_heads=2, seq=128 * 6 + 50,
                       chunk_len=128, budget_fixed=200)
    run_backward_case(w, plain=False, split=128 * 3)


def test_autograd_front_end_returns_the_library_gradients():
    """kvm_attention(...).backward() hands torch the tensors kvm_prefill_backward wrote."""
    pkg, sy = kvm(), synth()
    w = sy.shrink(sy.WORKLOADS["tiny_f32"], seq=64 * 5 + 11)
    q, k, v = sy.make_qkv(w, DEV)
    params = sy.make_params(w, DEV, plain=False)
    leaves = dict(q=q, k=k, v=v, gate=params["gate"], ln_gamma=params["ln_gamma"], ln_beta=params["ln_beta"],
                  tau_state=params["tau_state"], tau_bswa=params["tau_bswa"])
    leaves = {n: t.clone().requires_grad_(True) for n, t in leaves.items()}
    out = pkg.kvm_attention(leaves["q"], leaves["k"], leaves["v"], leaves["gate"], chunk_len=w.chunk_len,
                            rope_dims=w.rope_dims, n_bswa_chunks=w.n_bswa_chunks, n_sink=w.n_sink,
                            budget_fixed=w.budget_fixed, ln_gamma=leaves["ln_gamma"], ln_beta=leaves["ln_beta"],
                            tau_state=leaves["tau_state"], tau_bswa=leaves["tau_bswa"])
    gen = torch.Generator(device=DEV)
    gen.manual_seed(5)
    dout = torch.randn(out.shape, generator=gen, device=DEV)
    out.backward(dout)
    st = pkg.state_for(w, device=DEV, **params)
    assign, score = st.trace(w.seq // w.chunk_len + 1)
    o2, lse = st.prefill(q, k, v, params["gate"], want_lse=True)
    g = st.backward(q, k, v, params["gate"], o2, lse, dout, assign, score)
    torch.testing.assert_close(out.detach(), o2, rtol=0, atol=0)
    for name, key in (("q", "dq"), ("k", "dk"), ("v", "dv"), ("gate", "dgate")):
        torch.testing.assert_close(leaves[name].grad, g[key], rtol=0, atol=0)
    # parameter gradients are summed with atomics: equal to the last bits only
    for name, key in (("ln_gamma", "dgamma"), ("ln_beta", "dbeta"), ("tau_state", "dtau_state"), ("tau_bswa", "dtau_bswa")):
        torch.testing.assert_close(leaves[name].grad, g[key], rtol=1e-5, atol=1e-6)


def test_backward_on_a_stream_of_the_callers_choice():
    """Forward and backward enqueued on a stream other than the default one, with the caller's own
    work before and after them on that stream and no host synchronisation in between: the
    library's second stream is forked from and joined to the caller's stream, so the results are
    those of the default stream (to the bit, where no atomics are involved)."""
    pkg, sy = kvm(), synth()
    w = sy.shrink(sy.WORKLOADS["prefill_gqa_32k"], batch=1, n_q_heads=8, n_kv_heads=2, seq=128 * 9 + 70, chunk_len=128,
                  budget_fixed=256)
    q, k, v = sy.make_qkv(w, DEV)
    params = sy.make_params(w, DEV, plain=False)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(11)
    dout0 = torch.randn(q.shape, generator=gen, device=DEV, dtype=torch.float32)

    def both(stream):
        with torch.cuda.stream(stream):
            dout = (dout0 * 0.5).to(q.dtype)  # the caller's own kernel ahead of the library's
            st = pkg.state_for(w, device=DEV, **params)
            assign, score = st.trace(w.seq // w.chunk_len + 1)
            out, lse = st.prefill(q, k, v, params["gate"], want_lse=True)
            g = st.backward(q, k, v, params["gate"], out, lse, dout, assign, score)
            after = {n: t.float() * 2.0 for n, t in g.items()}  # and one behind them
            again = st.backward(q, k, v, params["gate"], out, lse, dout, assign, score)  # the state is only read
        stream.synchronize()
        for name in ("dq", "dk", "dv", "dgate"):
            torch.testing.assert_close(again[name], g[name], rtol=0, atol=0)
        return after

    torch.cuda.synchronize()
    ref = both(torch.cuda.current_stream())
    got = both(torch.cuda.Stream())
    for name in ("dq", "dk", "dv", "dgate"):
        torch.testing.assert_close(got[name], ref[name], rtol=0, atol=0)
    for name in ("dgamma", "dbeta", "dtau_state", "dtau_bswa"):
        torch.testing.assert_close(got[name], ref[name], rtol=1e-5, atol=1e-5)


def test_backward_rejects_a_state_that_did_not_run_this_prefill():
    pkg, sy = kvm(), synth()
    from paper_2605_09877_amd import binding
    w = sy.shrink(sy.WORKLOADS["tiny_f32"], seq=256)
    q, k, v = sy.make_qkv(w, DEV)
    st = pkg.state_for(w, device=DEV)
    assign, score = st.trace(8)
    out, lse = st.prefill(q, k, v, None, want_lse=True)
    with pytest.raises(binding.KVMError):
        st.backward(q[:, :128].contiguous(), k[:, :128].contiguous(), v[:, :128].contiguous(), None,
                    out[:, :128].contiguous(), lse[:, :128].contiguous(), out[:, :128].contiguous(), assign, score)
