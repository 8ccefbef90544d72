"""Parity of the HIP library (through its C ABI) with the CPU oracle, element by element, on
seeded inputs shaped like the benchmark workloads but small enough for the oracle.

Bars: state sizes and slot assignments exact (ties inside a 1e-4 score margin are counted, see
kvm_testlib); outputs max-abs 1e-4 in fp32, 2e-2 relative per row in bf16; key sums exact.
"""
import numpy as np
import pytest
import torch

import kvm_testlib as tl
from oracle import kvm_oracle as ko

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def kvm():
    import paper_2605_09877_amd as pkg
    return pkg


def synth():
    from paper_2605_09877_amd import synth as s
    return s


def run_prefill_case(w, plain, split=None, decode_tail=0, check_lse=True, units=None, tweak=None, case=None,
                     widen=None, knobs=None, mutate=None):
    """Prefill (optionally in two calls, optionally finishing with decode steps) on the GPU and in
    the oracle; compare sizes, assignments, scores, outputs, lse and the final state.  widen: the
    library is handed q, k, v, gate, out and lse as views of wider buffers (element strides through
    kvm_strides) instead of dense tensors.  knobs: {kvm_debug_set knob: value} applied to the state.
    mutate(q, k, v): edits the generated tensors in place before either side sees them.
    Returns (Ties, state)."""
    pkg, sy = kvm(), synth()
    q, k, v = sy.make_qkv(w, DEV)
    if mutate is not None:
        mutate(q, k, v)
    params = sy.make_params(w, DEV, plain=plain)
    if tweak is not None:
        tweak(params)
    gate = params["gate"]
    st = pkg.state_for(w, device=DEV, **params)
    for knob, value in (knobs or {}).items():
        st.debug_set(knob, value)
    T = w.seq
    Tp = T - decode_tail
    n_trace = T // w.chunk_len + 1
    assign, score = st.trace(n_trace)
    cuts = [0, Tp] if split is None else [0, split, Tp]
    outs, lses = [], []
    for lo, hi in zip(cuts, cuts[1:]):
        g = None if gate is None else gate[:, lo:hi].contiguous()
        if widen is None:
            o, l = st.prefill(q[:, lo:hi].contiguous(), k[:, lo:hi].contiguous(), v[:, lo:hi].contiguous(), g,
                              want_lse=True)
        else:
            o, l = widen(st, q[:, lo:hi], k[:, lo:hi], v[:, lo:hi], g)
        outs.append(o)
        lses.append(l)
    for t in range(Tp, T):
        g = None if gate is None else gate[:, t].contiguous()
        outs.append(st.decode(q[:, t].contiguous(), k[:, t].contiguous(), v[:, t].contiguous(), g)[:, None])
    torch.cuda.synchronize()
    y_gpu = torch.cat(outs, dim=1)
    lse_gpu = torch.cat(lses, dim=1)
    assert st.tokens == T
    n_folds = st.folds
    exp = st.export()
    torch.cuda.synchronize()
    ga_all = assign[:n_folds].cpu().numpy()
    gs_all = score[:n_folds].cpu().numpy()
    G = w.n_q_heads // w.n_kv_heads
    total_ties, worst = tl.Ties(), 0.0
    if units is None:
        units = [(b, h) for b in range(w.batch) for h in range(w.n_kv_heads)]
    for (b, h) in units:
        u = tl.unit_inputs(w, q, k, v, params, b, h)

        def drive(unit):
            ys, ls = [], []
            for lo, hi in zip(cuts, cuts[1:]):
                y, l = unit.prefill(u["q"][:, lo:hi], u["k"][lo:hi], u["v"][lo:hi],
                                    None if u["g"] is None else u["g"][lo:hi])
                ys.append(y)
                ls.append(l)
            for t in range(Tp, T):
                y, l = unit.decode(u["q"][:, t], u["k"][t], u["v"][t], None if u["g"] is None else u["g"][t])
                ys.append(y[:, None])
            return np.concatenate(ys, axis=1), np.concatenate(ls, axis=1)

        (y_ref, lse_ref), unit, ties = tl.run_oracle_following(w, params, h, drive, ga_all[:, b, h])
        total_ties += ties
        assert len(unit.fold_logs) == n_folds
        assert unit.state.m == st.rows
        # scores the library reports: append score and winning merge score, fp32 accumulation
        for f, log in enumerate(unit.fold_logs):
            for col, key in ((0, "s_max"), (1, "best")):
                got, want = gs_all[f, b, h, :, col], log[key]
                ok = ~np.isnan(got) & ~np.isnan(want)
                np.testing.assert_allclose(got[ok], want[ok], rtol=1e-5, atol=1e-4)
        yg = tl.f64(y_gpu[b, :, h * G:(h + 1) * G]).transpose(1, 0, 2)
        worst = max(worst, tl.check_outputs(w, yg, y_ref, f"{w.name} unit {(b, h)}"))
        if check_lse:
            lg = tl.f64(lse_gpu[b, :, h * G:(h + 1) * G]).T
            tol = 1e-4 if w.io == "f32" else 2e-2
            np.testing.assert_allclose(lg, lse_ref[:, :Tp], atol=tol, rtol=tol * 1e-1)
        tl.check_state(w, exp, unit, b, h)
    import inspect
    tl.record_parity(case or inspect.stack()[1].function + f"[{w.name},T={w.seq}]", len(units), total_ties, worst,
                     w.io)
    return total_ties, st


def test_tiny_f32_layer_full():
    """Workload 1 at full size: fp32, B1 H2 d64 T1024 C64, 64 fixed slots, r = 16."""
    w = synth().WORKLOADS["tiny_f32"]
    ties, st = run_prefill_case(w, plain=True)
    assert st.rows == 64 and st.folds == 15
    assert ties.total == 0


def test_tiny_f32_layer_with_gate_affine_and_temperatures():
    w = synth().WORKLOADS["tiny_f32"]
    run_prefill_case(synth().shrink(w, seq=640 + 23), plain=False)


@pytest.mark.parametrize("plain", [True, False])
def test_bf16_fixed_budget_prefill(plain):
    """Workload 2 shape, shrunk: creation -> 256 rows, append-all -> 512, then pure merges;
    ragged tail (T not a multiple of C)."""
    w = synth().shrink(synth().WORKLOADS["prefill_fixed"], batch=2, n_q_heads=2, n_kv_heads=2, seq=2560 + 77)
    ties, st = run_prefill_case(w, plain=plain)
    assert st.rows == 512


def test_bf16_negative_temperatures():
    """Learned temperatures may be negative: one sign per region and head, in every combination
    (the matrix-core kernel flips the sign of its query fragments when it changes region)."""
    w = synth().shrink(synth().WORKLOADS["prefill_fixed"], batch=1, n_q_heads=4, n_kv_heads=2, seq=1536 + 40)

    def tweak(params):
        params["tau_state"] *= torch.tensor([1.0, -1.0, 1.0, -1.0], device=DEV)
        params["tau_bswa"] *= torch.tensor([1.0, 1.0, -1.0, -1.0], device=DEV)

    run_prefill_case(w, plain=False, tweak=tweak)


def test_bf16_long_chunks_prefill():
    """C = 1024: a block's merge targets no longer fit one scan round of the accumulate pass."""
    w = synth().shrink(synth().WORKLOADS["prefill_fixed"], batch=1, n_q_heads=2, n_kv_heads=2, chunk_len=1024,
                       budget_fixed=1536, seq=6 * 1024 + 50)
    ties, st = run_prefill_case(w, plain=False)
    assert st.rows == 1536


def test_bf16_three_window_blocks_with_state():
    """n_bswa = 3: a 768-token window over a 512-row state on the matrix-core path."""
    w = synth().shrink(synth().WORKLOADS["prefill_fixed"], batch=1, n_q_heads=2, n_kv_heads=2, n_bswa_chunks=3,
                       seq=3072 + 45)
    ties, st = run_prefill_case(w, plain=False)
    assert st.rows == 512


def test_bf16_saturating_budget_table():
    """A saturating schedule given as a table (one budget per chunk; the last entry repeats):
    growth by whole blocks, then by a few rows, then none."""
    table = (256, 256, 512, 640, 700, 720, 730, 736, 736)
    w = synth().shrink(synth().WORKLOADS["prefill_fixed"], batch=1, n_q_heads=2, n_kv_heads=2,
                       budget_kind="table", budget_table=table, seq=12 * 256 + 19)
    ties, st = run_prefill_case(w, plain=False)
    assert st.rows == 736


def test_bf16_sqrt_growth_prefill():
    """Workload 3 shape, shrunk: rows stay 256 until e = 4096, then grow by a few rows per fold
    (partial appends + re-scoring against the new rows); needle duplicates in the data."""
    w = synth().shrink(synth().WORKLOADS["prefill_sqrt"], batch=1, n_q_heads=2, n_kv_heads=2, seq=6144)
    ties, st = run_prefill_case(w, plain=True)
    assert st.rows == ko.expected_rows(tl.oracle_cfg(w), w.seq)[-1] == 4 * 79


def test_bf16_gqa_training_shape_prefill():
    """Workload 5 shape, shrunk: 4 query heads per KV head, C = 512, 1024 rows, per-head scales."""
    w = synth().shrink(synth().WORKLOADS["prefill_gqa_32k"], batch=1, n_q_heads=8, n_kv_heads=2, seq=4096)
    ties, st = run_prefill_case(w, plain=False)
    assert st.rows == 1024


def test_split_prefill_then_decode_matches_oracle():
    """Continuation from the window ring, and a partial chunk completed token by token."""
    w = synth().shrink(synth().WORKLOADS["prefill_fixed"], batch=1, n_q_heads=2, n_kv_heads=2, seq=1024 + 300,
                       chunk_len=128, budget_fixed=256)
    run_prefill_case(w, plain=False, split=512, decode_tail=300 - 128 + 45, check_lse=True)


@pytest.mark.parametrize("n_q,n_kv", [(8, 2), (8, 1), (4, 2), (6, 2)])
def test_bf16_grouped_query_decode(n_q, n_kv):
    """Decode steps with grouped queries: a workgroup takes four query heads of a KV head together
    (groups of 4 and 8), two (group of 2), or one (group of 3)."""
    w = synth().shrink(synth().WORKLOADS["prefill_fixed"], batch=2, n_q_heads=n_q, n_kv_heads=n_kv, seq=512 + 140,
                       chunk_len=128, budget_fixed=256)
    run_prefill_case(w, plain=False, decode_tail=140, check_lse=True)


def test_f32_split_and_decode():
    w = synth().shrink(synth().WORKLOADS["tiny_f32"], seq=512 + 100)
    run_prefill_case(w, plain=False, split=192, decode_tail=100)


def test_no_state_is_block_sliding_window():
    w = synth().shrink(synth().WORKLOADS["prefill_fixed"], batch=1, n_q_heads=2, n_kv_heads=1, seq=1024 + 64,
                       budget_kind="none", n_bswa_chunks=3, chunk_len=128)
    ties, st = run_prefill_case(w, plain=False)
    assert st.rows == 0 and st.folds == 0


def test_short_inputs():
    """T below one chunk, and exactly one chunk."""
    for seq in (5, 64):
        w = synth().shrink(synth().WORKLOADS["tiny_f32"], seq=seq)
        run_prefill_case(w, plain=False)
    w = synth().shrink(synth().WORKLOADS["prefill_fixed"], batch=1, n_q_heads=1, n_kv_heads=1, seq=37)
    run_prefill_case(w, plain=True)


# ----------------------------------------------------------------------------- degenerate inputs
def _few_distinct_tokens(n_distinct):
    """Every token of a sequence is one of n_distinct (k, v) pairs, in rotation: memory keys repeat,
    so scores tie exactly -- between tokens (append selection: the lower position goes first) and,
    once rows built from the same tokens exist, between rows (merge: the lowest row wins)."""
    def mutate(q, k, v):
        T = k.shape[1]
        idx = torch.arange(T, device=k.device) % n_distinct
        k.copy_(k[:, :n_distinct][:, idx])
        v.copy_(v[:, :n_distinct][:, idx])
    return mutate


def _zero_stretch(lo, hi):
    """Tokens lo .. hi-1 have k = 0 and v = 0: LN_s of a constant vector (variance 0), rows of
    radius 0, value sums of norm 0."""
    def mutate(q, k, v):
        k[:, lo:hi] = 0
        v[:, lo:hi] = 0
    return mutate


FOLD_PATHS = {"kernel per step": {0: 2}, "one launch": {0: 1}}     # KVM_DEBUG_FOLD_PATH


@pytest.mark.parametrize("path", list(FOLD_PATHS))
def test_bf16_exact_ties_between_tokens_and_between_rows(path):
    w = synth().shrink(synth().WORKLOADS["prefill_fixed"], batch=1, n_q_heads=2, n_kv_heads=2, seq=2048,
                       chunk_len=128, budget_kind="sqrt", budget_scale=6.0)
    ties, st = run_prefill_case(w, plain=False, mutate=_few_distinct_tokens(5), knobs=FOLD_PATHS[path])
    assert ties.total == 0      # exact ties are decided by the stated order, not counted as near-ties


def test_f32_exact_ties_between_tokens_and_between_rows():
    w = synth().shrink(synth().WORKLOADS["tiny_f32"], seq=768, budget_kind="sqrt", budget_scale=4.0)
    ties, st = run_prefill_case(w, plain=False, mutate=_few_distinct_tokens(3))
    assert ties.total == 0


@pytest.mark.parametrize("path", list(FOLD_PATHS))
def test_bf16_zero_keys_and_values(path):
    """A stretch of all-zero tokens that covers whole blocks (state creation from zeros included in
    the second case) and is later merged into and attended: no NaN, no Inf, parity as usual."""
    w = synth().shrink(synth().WORKLOADS["prefill_fixed"], batch=1, n_q_heads=2, n_kv_heads=2, seq=1536,
                       chunk_len=128, budget_fixed=192)
    for lo, hi in ((300, 700), (0, 256)):
        ties, st = run_prefill_case(w, plain=False, mutate=_zero_stretch(lo, hi), knobs=FOLD_PATHS[path])
        exp = st.export()
        for name in ("khat", "vhat", "sV", "rho"):
            assert torch.isfinite(exp[name].float()).all(), name


def test_f32_zero_keys_and_values():
    w = synth().shrink(synth().WORKLOADS["tiny_f32"], seq=640)
    run_prefill_case(w, plain=False, mutate=_zero_stretch(0, 200))


@pytest.mark.parametrize("path", list(FOLD_PATHS))
def test_bf16_every_channel_rotary_all_memory_keys_equal(path):
    """rope_dims = head_dim: zero_r removes every channel, so every memory key is LN_s of the zero
    vector (= beta) and every similarity is the same number: the fold is decided by the tie rules
    alone (lowest eligible row; appended tokens by position)."""
    w = synth().shrink(synth().WORKLOADS["prefill_fixed"], batch=1, n_q_heads=2, n_kv_heads=2, seq=1536 + 20,
                       chunk_len=128, rope_dims=128, budget_kind="sqrt", budget_scale=6.0)
    ties, st = run_prefill_case(w, plain=False, knobs=FOLD_PATHS[path])
    assert ties.total == 0


def test_f32_every_channel_rotary_all_memory_keys_equal():
    w = synth().shrink(synth().WORKLOADS["tiny_f32"], seq=700, rope_dims=64, budget_kind="sqrt", budget_scale=4.0)
    ties, st = run_prefill_case(w, plain=False)
    assert ties.total == 0


@pytest.mark.parametrize("n_sink", [0, 3])
@pytest.mark.parametrize("path", list(FOLD_PATHS))
def test_bf16_sink_counts(path, n_sink):
    """No sink row at all, and three: the rows below n_sink never receive a token but count for the
    append score."""
    w = synth().shrink(synth().WORKLOADS["prefill_fixed"], batch=1, n_q_heads=2, n_kv_heads=2, seq=2048 + 31,
                       chunk_len=128, budget_fixed=200, n_sink=n_sink)
    ties, st = run_prefill_case(w, plain=False, knobs=FOLD_PATHS[path])
    exp = st.export()
    if n_sink:
        assert int(exp["n"][:, :, :n_sink].max()) == 1      # a sink row holds its creator only


@pytest.mark.parametrize("split", [0, 1, 4])
def test_bf16_units_not_a_multiple_of_eight(split):
    """3 sequences x 3 KV heads = 9 units (workgroup -> unit mappings that deal units round robin
    over the accelerator dies have a ragged last round; the batch cannot be halved either), two
    query heads per KV head; on the kernel-per-step path and on the one-launch path with one and
    with four workgroups per unit."""
    from paper_2605_09877_amd import binding
    w = synth().shrink(synth().WORKLOADS["prefill_fixed"], batch=3, n_q_heads=6, n_kv_heads=3, seq=2048 + 64 + 9,
                       chunk_len=128, budget_kind="sqrt", budget_scale=7.0)
    knobs = {binding.KVM_DEBUG_FOLD_PATH: 2} if split == 0 else \
        {binding.KVM_DEBUG_FOLD_PATH: 1, binding.KVM_DEBUG_FOLD_SPLIT: split}
    run_prefill_case(w, plain=False, split=1024, decode_tail=9, knobs=knobs)


def test_bf16_budget_of_one_block_and_a_single_fold():
    """A budget equal to the block length (the state is created full and never grows: every later
    block merges whole), and a sequence that ends right after its first fold."""
    w = synth().shrink(synth().WORKLOADS["prefill_fixed"], batch=1, n_q_heads=2, n_kv_heads=2, seq=1280,
                       chunk_len=128, budget_fixed=128)
    ties, st = run_prefill_case(w, plain=False)
    assert st.rows == 128
    w = synth().shrink(w, seq=256)          # T = L: attention over the window only, then one fold
    ties, st = run_prefill_case(w, plain=False)
    assert st.folds == 1 and st.rows == 128


def test_bf16_head_dim_64_generic_kernels():
    w = synth().shrink(synth().WORKLOADS["prefill_fixed"], batch=1, n_q_heads=2, n_kv_heads=1, head_dim=64,
                       rope_dims=16, seq=768 + 10, chunk_len=96, budget_fixed=160)
    run_prefill_case(w, plain=False)


# ----------------------------------------------------------------------------- fold alone
@pytest.mark.parametrize("io,d,C,m0,budget", [("f32", 64, 64, 64, 80), ("bf16", 128, 256, 300, 340),
                                               ("bf16", 128, 128, 128, 128), ("bf16", 64, 64, 100, 130),
                                               ("bf16", 128, 1024, 700, 900), ("f32", 128, 576, 200, 200),
                                               # a few new rows: selection, creation and the second
                                               # scoring pass run in one launch
                                               ("bf16", 128, 256, 300, 310), ("bf16", 64, 64, 100, 112),
                                               ("f32", 128, 128, 200, 207), ("bf16", 128, 250, 300, 301)])
def test_state_fold_entry_point(io, d, C, m0, budget):
    """kvm_state_fold on an imported state: partial append + re-score + merge in one call."""
    pkg, sy = kvm(), synth()
    w = sy.shrink(sy.WORKLOADS["prefill_fixed"], io=io, batch=2, n_q_heads=2, n_kv_heads=2, head_dim=d,
                  rope_dims=d // 4, chunk_len=C, budget_fixed=budget, seq=4 * C)
    params = sy.make_params(w, DEV, plain=False, T=C)
    st = pkg.state_for(w, device=DEV, max_tokens=64 * C, **params)
    gen = torch.Generator(device=DEV).manual_seed(1234)
    B, H = w.batch, w.n_kv_heads
    dt = sy.torch_dtype(io)
    imp = dict(sK=torch.randn(B, H, m0, d, generator=gen, device=DEV, dtype=torch.float32).double() * 3,
               sV=torch.randn(B, H, m0, d, generator=gen, device=DEV),
               rho=0.5 + torch.rand(B, H, m0, generator=gen, device=DEV),
               w=torch.ones(B, H, m0, device=DEV), n=torch.ones(B, H, m0, dtype=torch.int32, device=DEV),
               m=m0, tokens=0, folds=1)
    st.import_(imp)
    kb = torch.randn(B, C, H, d, generator=gen, device=DEV).to(dt)
    vb = torch.randn(B, C, H, d, generator=gen, device=DEV).to(dt)
    # plant duplicates of state rows and of each other
    kb[:, 5] = kb[:, 3]
    e = 16 * C
    assign, score = st.fold(kb, vb, params["gate"], e=e)
    exp = st.export()
    torch.cuda.synchronize()
    assert st.rows == min(budget, m0 + C)
    all_ties = tl.Ties()
    for b in range(B):
        for h in range(H):
            unit = tl.make_oracle_unit(w, params, h)
            s0 = ko.UnitState(d)
            s0.sK, s0.sV = imp["sK"][b, h].cpu().numpy().copy(), tl.f64(imp["sV"][b, h]).copy()
            s0.rho, s0.w = tl.f64(imp["rho"][b, h]).copy(), np.ones(m0)
            s0.n, s0.members = np.ones(m0, dtype=np.int64), [[-1] for _ in range(m0)]
            unit.state = s0
            ga = assign[b, h].cpu().numpy()
            ov, app_ov, ties = None, None, tl.Ties()
            for _ in range(4):
                import copy
                trial = copy.deepcopy(s0)
                log = ko.fold(trial, tl.f64(kb[b, :, h]), tl.f64(vb[b, :, h]), tl.f64(params["gate"][b, :, h]),
                              e, unit.cfg, unit.gamma, unit.beta, overrides=ov, append_override=app_ov)
                if np.array_equal(log["assign"], ga):
                    break
                ga_app = sorted(np.nonzero(ga >= m0)[0].tolist())
                if ga_app != sorted(np.nonzero(log["appended"])[0].tolist()):
                    ties.append += 1
                    app_ov = ga_app
                else:
                    ties.merge += 1
                    j = int(np.nonzero(log["assign"] != ga)[0][0])
                    ov = dict(ov or {})
                    ov[j] = int(ga[j])
            else:
                raise AssertionError("assignments differ beyond ties")
            # one fold: no tie in fp32; in bf16 at most one (tl.tie_ceiling)
            assert ties.total <= tl.tie_ceiling(w, 1), ties
            all_ties += ties
            unit.state = trial
            tl.check_state(w, exp, unit, b, h)
            gs = score[b, h].cpu().numpy()
            ok = ~np.isnan(gs[:, 0])
            np.testing.assert_allclose(gs[ok, 0], log["s_max"][ok], rtol=1e-5, atol=1e-4)
    tl.record_parity(f"state_fold[{io},d{d},C{C},{m0}->{budget}]", B * H, all_ties, 0.0, io)


# ----------------------------------------------------------------------------- decode workload shape
def test_decode_against_prebuilt_state():
    """Workload 4 shape, shrunk: imported state + full window ring, successive decode steps with
    a fold when a chunk completes."""
    pkg, sy = kvm(), synth()
    w = sy.shrink(sy.WORKLOADS["decode"], batch=3, n_q_heads=4, n_kv_heads=2, state_rows=320, budget_fixed=320,
                  seq=140)
    pre = sy.make_decode_state(w, DEV)
    st = pkg.state_for(w, device=DEV, max_tokens=pre["tokens"] + w.seq + w.chunk_len)
    assign, _ = st.trace(4)
    # trace slots are indexed by the state's lifetime fold count: start it at 0 for this test
    st.import_(dict(pre, folds=0))
    q, k, v = sy.make_qkv(w, DEV, T=w.seq, pos0=pre["tokens"])
    outs = [st.decode(q[:, t].contiguous(), k[:, t].contiguous(), v[:, t].contiguous()) for t in range(w.seq)]
    torch.cuda.synchronize()
    y_gpu = torch.stack(outs, dim=1)
    n_folds = st.folds
    assert n_folds == 1
    ga = assign[:n_folds].cpu().numpy()
    G = w.n_q_heads // w.n_kv_heads
    L = w.chunk_len * w.n_bswa_chunks
    t0 = pre["tokens"]
    all_ties, worst = tl.Ties(), 0.0
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            def drive(unit):
                s0 = unit.state
                s0.sK = pre["sK"][b, h].cpu().numpy().copy()
                s0.sV = tl.f64(pre["sV"][b, h]).copy()
                s0.rho = tl.f64(pre["rho"][b, h]).copy()
                s0.w, s0.n = np.ones(w.state_rows), np.ones(w.state_rows, dtype=np.int64)
                s0.members = [[-1] for _ in range(w.state_rows)]
                unit.t = t0
                # history: only the last L tokens exist; earlier ones are never read again
                unit.k_hist = np.zeros((t0, w.head_dim))
                unit.v_hist = np.zeros((t0, w.head_dim))
                unit.g_hist = np.ones(t0)
                pos = np.arange(t0 - L, t0)
                unit.k_hist[pos] = tl.f64(pre["win_k"][b, h])[pos % L]
                unit.v_hist[pos] = tl.f64(pre["win_v"][b, h])[pos % L]
                ys = [unit.decode(tl.f64(q[b, t, h * G:(h + 1) * G]), tl.f64(k[b, t, h]), tl.f64(v[b, t, h]))[0]
                      for t in range(w.seq)]
                return np.stack(ys, axis=1)

            y_ref, unit, ties = tl.run_oracle_following(w, {}, h, drive, ga[:, b, h])
            all_ties += ties
            worst = max(worst, tl.check_outputs(w, tl.f64(y_gpu[b, :, h * G:(h + 1) * G]).transpose(1, 0, 2), y_ref,
                                                "decode"))
    tl.record_parity("decode_against_prebuilt_state", w.batch * w.n_kv_heads, all_ties, worst, w.io)


# ----------------------------------------------------------------------------- checkpoint, growth, errors
def test_export_import_roundtrip_and_grow():
    pkg, sy = kvm(), synth()
    w = sy.shrink(sy.WORKLOADS["prefill_sqrt"], batch=1, n_q_heads=2, n_kv_heads=2, seq=8192, gen="normal")
    q, k, v = sy.make_qkv(w, DEV)
    full = pkg.state_for(w, device=DEV)
    y_full = full.prefill(q, k, v)
    T1 = 4096
    a = pkg.state_for(w, device=DEV, max_tokens=T1)          # capacity for the first part only
    y1 = a.prefill(q[:, :T1].contiguous(), k[:, :T1].contiguous(), v[:, :T1].contiguous())
    with pytest.raises(pkg.KVMError) as ei:
        a.prefill(q[:, T1:].contiguous(), k[:, T1:].contiguous(), v[:, T1:].contiguous())
    assert ei.value.status == pkg.KVM_ERR_CAPACITY
    assert a.tokens == T1                                     # the failed call enqueued nothing
    a.grow(w.seq)
    y2 = a.prefill(q[:, T1:].contiguous(), k[:, T1:].contiguous(), v[:, T1:].contiguous())
    torch.cuda.synchronize()
    assert torch.equal(torch.cat([y1, y2], dim=1), y_full)
    assert a.rows == full.rows
    # checkpoint: export after T1, import into a fresh state, continue
    b_ = pkg.state_for(w, device=DEV)
    b_.prefill(q[:, :T1].contiguous(), k[:, :T1].contiguous(), v[:, :T1].contiguous())
    snap = b_.export()
    c_ = pkg.state_for(w, device=DEV)
    c_.import_(snap)
    y3 = c_.prefill(q[:, T1:].contiguous(), k[:, T1:].contiguous(), v[:, T1:].contiguous())
    torch.cuda.synchronize()
    assert torch.equal(y3, y_full[:, T1:])
    ea, ec = full.export(), c_.export()
    for key in ("sK", "sV", "rho", "n", "khat", "vhat"):
        assert torch.equal(ea[key], ec[key]), key


def test_fold_is_deterministic():
    """Two runs over the same input leave bit-identical states (no atomics-order dependence)."""
    pkg, sy = kvm(), synth()
    w = sy.shrink(sy.WORKLOADS["prefill_fixed"], batch=2, n_q_heads=2, n_kv_heads=2, seq=2048)
    q, k, v = sy.make_qkv(w, DEV)
    exps = []
    for _ in range(2):
        st = pkg.state_for(w, device=DEV)
        y = st.prefill(q, k, v)
        exps.append((y, st.export()))
    torch.cuda.synchronize()
    assert torch.equal(exps[0][0], exps[1][0])
    for key in ("sK", "sV", "khat", "vhat", "n"):
        assert torch.equal(exps[0][1][key], exps[1][1][key])


# ----------------------------------------------------------------------------- strided operands
def _widened(st, q, k, v, g):
    """q, k, v as slices of one fused-projection buffer [B, T, H_q + 2 H_kv (+ 1 spare head), d],
    out, gate and lse as slices of wider buffers too: every kvm_strides field differs from the
    dense layout."""
    B, T, Hq, d = q.shape
    Hkv = k.shape[2]
    fused = torch.full((B, T + 3, Hq + 2 * Hkv + 1, d), float("nan"), dtype=q.dtype, device=q.device)
    fused[:, 1:T + 1, :Hq] = q
    fused[:, 1:T + 1, Hq:Hq + Hkv] = k
    fused[:, 1:T + 1, Hq + Hkv + 1:] = v          # a spare head between k and v
    qv, kv, vv = fused[:, 1:T + 1, :Hq], fused[:, 1:T + 1, Hq:Hq + Hkv], fused[:, 1:T + 1, Hq + Hkv + 1:]
    assert not qv.is_contiguous() and not kv.is_contiguous() and not vv.is_contiguous()
    out_w = torch.zeros((B, T, Hq + 2, d), dtype=q.dtype, device=q.device)
    lse_w = torch.zeros((B, T + 1, Hq + 3), dtype=torch.float32, device=q.device)
    gv = None
    if g is not None:
        g_w = torch.full((B, T, Hkv + 2), float("nan"), dtype=torch.float32, device=q.device)
        g_w[:, :, 1:Hkv + 1] = g
        gv = g_w[:, :, 1:Hkv + 1]
    o, l = st.prefill(qv, kv, vv, gv, out=out_w[:, :, 1:Hq + 1], lse=lse_w[:, :T, 2:Hq + 2])
    torch.cuda.synchronize()
    # nothing outside the views was written
    assert float(out_w[:, :, 0].abs().max()) == 0.0 and float(out_w[:, :, Hq + 1].abs().max()) == 0.0
    assert float(lse_w[:, T].abs().max()) == 0.0 and float(lse_w[:, :, :2].abs().max()) == 0.0
    return o.contiguous(), l.contiguous()


def test_bf16_strided_operands_matrix_core_path():
    """kvm_strides on the matrix-core path (bf16, d = 128): q, k, v are slices of a fused
    projection buffer, out / gate / lse slices of wider buffers; two calls, so that the second
    one's window reaches back into the ring; partial appends (growth budget) and plain merges."""
    w = synth().shrink(synth().WORKLOADS["prefill_sqrt"], batch=2, n_q_heads=4, n_kv_heads=2, seq=5376 + 31)
    ties, st = run_prefill_case(w, plain=False, split=2560, widen=_widened)
    assert st.rows == ko.expected_rows(tl.oracle_cfg(w), w.seq)[-1]


def test_bf16_strided_operands_gqa_long_chunks():
    """The same with the headline workload's shape (four query heads per KV head, C = 512)."""
    w = synth().shrink(synth().WORKLOADS["prefill_gqa_32k"], batch=1, n_q_heads=8, n_kv_heads=2, seq=3072 + 9)
    ties, st = run_prefill_case(w, plain=False, widen=_widened)
    assert st.rows == 1024


def test_f32_strided_operands_generic_path():
    """kvm_strides on the generic kernels (fp32, d = 64)."""
    w = synth().shrink(synth().WORKLOADS["tiny_f32"], batch=2, seq=640 + 23)
    ties, st = run_prefill_case(w, plain=False, split=256, widen=_widened)
    assert ties.total == 0


# ----------------------------------------------------------------------------- the two fold paths
@pytest.mark.parametrize("waves,split", [(8, 1), (16, 1), (8, 2), (8, 4), (16, 2), (8, 8)])
@pytest.mark.parametrize("shape", ["fixed", "sqrt", "gqa"])
def test_fold_paths_agree(shape, waves, split):
    """bf16 / d = 128 states fold with one launch per run of folds (one workgroup per unit); the
    kernel-per-step path they can be switched to (kvm_debug_set) must take the same decisions:
    assignments, row counts and key sums equal to the bit (both score with the same matrix-core
    arithmetic and add exact products in fp64), value sums to the bit too (same adds in the same
    order); radii and the value readout may differ in the last fp32 bit (sums over a row's
    channels are taken in another order), outputs accordingly.  split > 1: a unit's rows are shared
    among that many workgroups of the launch, which settle every token's winner by an exchange."""
    pkg, sy = kvm(), synth()
    from paper_2605_09877_amd import binding
    w = {"fixed": sy.shrink(sy.WORKLOADS["prefill_fixed"], batch=2, n_q_heads=2, n_kv_heads=2, seq=3072 + 77),
         "sqrt": sy.shrink(sy.WORKLOADS["prefill_sqrt"], batch=1, n_q_heads=2, n_kv_heads=2, seq=6144),
         "gqa": sy.shrink(sy.WORKLOADS["prefill_gqa_32k"], batch=1, n_q_heads=8, n_kv_heads=2, seq=4096 + 512)}[shape]
    q, k, v = sy.make_qkv(w, DEV)
    params = sy.make_params(w, DEV, plain=False)
    res = []
    for path in (1, 2):
        st = pkg.state_for(w, device=DEV, **params)
        st.debug_set(binding.KVM_DEBUG_FOLD_PATH, path)
        st.debug_set(binding.KVM_DEBUG_FOLD_WAVES, waves)
        st.debug_set(binding.KVM_DEBUG_FOLD_SPLIT, split)
        assign, score = st.trace(w.seq // w.chunk_len + 1)
        y = st.prefill(q, k, v, params["gate"])
        torch.cuda.synchronize()
        res.append((y, assign[:st.folds].clone(), score[:st.folds].clone(), st.export(), st.rows, st.folds))
    a, b = res
    assert a[4] == b[4] and a[5] == b[5]
    assert torch.equal(a[1], b[1]), "assignments differ between the fold paths"
    # scores: equal where both paths use the matrix cores; a token that moved to a row appended
    # in the same fold was scored against it on the vector ALU by the kernel-per-step path
    assert torch.equal(torch.isnan(a[2]), torch.isnan(b[2]))
    torch.testing.assert_close(torch.nan_to_num(a[2], nan=0.0), torch.nan_to_num(b[2], nan=0.0), rtol=1e-5, atol=1e-4)
    for key in ("sK", "sV", "n", "w", "khat"):
        assert torch.equal(a[3][key], b[3][key]), key
    torch.testing.assert_close(a[3]["rho"], b[3]["rho"], rtol=1e-6, atol=0)
    torch.testing.assert_close(a[3]["vhat"].float(), b[3]["vhat"].float(), rtol=2 ** -7, atol=1e-6)
    torch.testing.assert_close(a[0].float(), b[0].float(), rtol=2e-2, atol=2e-2)


@pytest.mark.parametrize("waves,split", [(8, 1), (16, 1), (8, 4), (16, 2)])
@pytest.mark.parametrize("case", ["fixed", "sqrt", "gqa", "decode_tail", "table", "three_blocks"])
def test_one_launch_fold_path_against_the_oracle(case, waves, split):
    """The one-launch fold path (kvm_debug_set; not the default), both workgroup shapes, against
    the oracle to the bars of the other tests: plain merges, append-all, partial appends with the
    second scoring pass, folds in place during decode steps, a budget table, a three-block window."""
    from paper_2605_09877_amd import binding
    sy = synth()
    knobs = {binding.KVM_DEBUG_FOLD_PATH: 1, binding.KVM_DEBUG_FOLD_WAVES: waves, binding.KVM_DEBUG_FOLD_SPLIT: split}
    if case == "fixed":
        w = sy.shrink(sy.WORKLOADS["prefill_fixed"], batch=2, n_q_heads=2, n_kv_heads=2, seq=2560 + 77)
        run_prefill_case(w, plain=False, knobs=knobs)
    elif case == "sqrt":
        w = sy.shrink(sy.WORKLOADS["prefill_sqrt"], batch=1, n_q_heads=2, n_kv_heads=2, seq=6144)
        run_prefill_case(w, plain=True, knobs=knobs)
    elif case == "gqa":
        w = sy.shrink(sy.WORKLOADS["prefill_gqa_32k"], batch=1, n_q_heads=8, n_kv_heads=2, seq=4096)
        run_prefill_case(w, plain=False, knobs=knobs)
    elif case == "decode_tail":
        w = sy.shrink(sy.WORKLOADS["prefill_fixed"], batch=1, n_q_heads=2, n_kv_heads=2, seq=1024 + 300,
                      chunk_len=128, budget_fixed=256)
        run_prefill_case(w, plain=False, split=512, decode_tail=300 - 128 + 45, knobs=knobs)
    elif case == "table":
        table = (256, 256, 512, 640, 700, 720, 730, 736, 736)
        w = sy.shrink(sy.WORKLOADS["prefill_fixed"], batch=1, n_q_heads=2, n_kv_heads=2, budget_kind="table",
                      budget_table=table, seq=12 * 256 + 19)
        run_prefill_case(w, plain=False, knobs=knobs)
    else:
        w = sy.shrink(sy.WORKLOADS["prefill_fixed"], batch=1, n_q_heads=2, n_kv_heads=2, n_bswa_chunks=3, seq=3072 + 45)
        run_prefill_case(w, plain=False, knobs=knobs)
