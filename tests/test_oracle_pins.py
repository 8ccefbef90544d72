"""Pins for the CPU oracle: what the paper and the mathematics fix, independent of the oracle.

Each test names the passage it leans on.  Brute-force helpers in this file are written
with explicit loops from the equations and share no code with oracle/kvm_oracle.py.

Parity unpinned: the paper prints no numeric outputs, so the exact output values for
general inputs, and the readings listed in the oracle's header (tie order, LN statistics
over the zeroed channels, sink inclusion in the append score, GQA), rest on the special
cases, invariants and brute-force replays below and not on published numbers.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import kvm_oracle as ko

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers
def rng(seed):
    return np.random.default_rng(seed)


def brute_softmax_attention(q_u, keys, vals, scales):
    """Textbook softmax attention for one query: explicit loops, max-subtracted."""
    d = len(q_u)
    logits = []
    for kk, sc in zip(keys, scales):
        dot = 0.0
        for c in range(d):
            dot += q_u[c] * kk[c]
        logits.append(sc * dot / math.sqrt(d))
    mx = max(logits)
    ws = [math.exp(l - mx) for l in logits]
    z = sum(ws)
    y = [0.0] * len(vals[0])
    for wgt, vv in zip(ws, vals):
        for c in range(len(vv)):
            y[c] += wgt / z * vv[c]
    return np.array(y), mx + math.log(z)


def brute_ln(x, gamma, beta, eps):
    d = len(x)
    mu = sum(x) / d
    var = sum((xi - mu) ** 2 for xi in x) / d
    return np.array([(x[c] - mu) / math.sqrt(var + eps) * gamma[c] + beta[c] for c in range(d)])


def make_unit(cfg, G=1, seed=0, gated=False, affine=False, taus=False, T=None, standardise=False):
    r = rng(seed)
    d = cfg.head_dim
    q = r.normal(size=(G, T, d))
    k = r.normal(size=(T, d))
    v = r.normal(size=(T, d))
    if standardise:
        k = (k - k.mean(-1, keepdims=True)) / k.std(-1, keepdims=True)
    q, k, v = (ko.round_io(a, cfg.io) for a in (q, k, v))
    g = 1.0 + np.where((z := r.normal(size=T)) > 0, z, np.exp(z) - 1.0) if gated else None
    gamma = r.uniform(0.5, 1.5, size=d) if affine else None
    beta = r.normal(scale=0.1, size=d) if affine else None
    ts = r.uniform(0.5, 2.0, size=G) if taus else None
    tb = r.uniform(0.5, 2.0, size=G) if taus else None
    unit = ko.KVMUnit(cfg, G, gamma, beta, ts, tb)
    return unit, q, k, v, g


# ----------------------------------------------------------------------------- primitives
def test_round_bf16_matches_library_conversion():
    r = rng(1)
    x = np.concatenate([r.normal(size=4096) * 10.0 ** r.integers(-6, 6, size=4096),
                        # exact ties between two bf16 neighbours, both parities
                        np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(2.0 + 2.0 ** -7), 0.0, -0.0])])
    x = x.astype(np.float32).astype(np.float64)
    ref = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(ko.round_bf16(x), ref)


def test_layer_norm_matches_library_and_loops():
    r = rng(2)
    x = r.normal(size=(5, 16)) * 3 + 1
    gamma, beta = r.uniform(0.5, 1.5, 16), r.normal(size=16)
    got = ko.layer_norm(x, gamma, beta, 1e-5)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x), (16,), torch.from_numpy(gamma),
                                         torch.from_numpy(beta), 1e-5).numpy()
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    for i in range(5):
        np.testing.assert_allclose(got[i], brute_ln(list(x[i]), gamma, beta, 1e-5), atol=1e-12)


def test_memory_key_zeroes_rotary_channels_before_ln():
    """Equation "memory key": LN_s is applied to k with its first r channels set to 0,
    statistics over all d_h channels."""
    cfg = ko.KVMConfig(head_dim=8, rope_dims=4, chunk_len=4, io="f32")
    r = rng(3)
    k = r.normal(size=8)
    gamma, beta = r.uniform(0.5, 1.5, 8), r.normal(size=8)
    kz = [0.0] * 4 + list(k[4:])
    want = brute_ln(kz, gamma, beta, cfg.ln_eps).astype(np.float32).astype(np.float64)
    np.testing.assert_array_equal(ko.memory_key(k[None], cfg, gamma, beta)[0], want)
    # changing the rotary channels of k cannot change the memory key
    k2 = k.copy()
    k2[:4] += 7.0
    np.testing.assert_array_equal(ko.memory_key(k2[None], cfg, gamma, beta),
                                  ko.memory_key(k[None], cfg, gamma, beta))


# ----------------------------------------------------------------------------- P1 / P1' / P2
def test_no_compression_equals_textbook_causal_attention():
    """Budget >= T appends every overflow token, so nothing is merged.  With r = 0,
    row-standardised keys, gamma = 1, beta = 0 and equal temperatures, LN_s is the identity
    (up to its eps) and rho * v / ||v|| = v: the layer is exact causal softmax attention."""
    T, d, C = 40, 8, 4
    cfg = ko.KVMConfig(head_dim=d, rope_dims=0, chunk_len=C, io="f32",
                       budget_kind=ko.BUDGET_FIXED, budget_fixed=10 * T, ln_eps=1e-30)
    unit, q, k, v, _ = make_unit(cfg, G=2, seed=4, T=T, standardise=True)
    y, lse = unit.prefill(q, k, v)
    for h in range(2):
        for u in range(T):
            want, want_lse = brute_softmax_attention(q[h, u], k[:u + 1], v[:u + 1], [1.0] * (u + 1))
            np.testing.assert_allclose(y[h, u], want, atol=5e-6)
            assert abs(lse[h, u] - want_lse) < 5e-6
    assert unit.state.m == T - cfg.window + C      # the fold after the last chunk has run too


def test_no_compression_general_parameters_brute_force():
    """Same, any r, gamma, beta, tau: every key older than the window is replaced by
    tau_state * LN_s(zero_r(k_j)), window keys are tau_bswa * k_t; rho * v/||v|| = v."""
    T, d, C, r_ = 36, 8, 4, 4
    cfg = ko.KVMConfig(head_dim=d, rope_dims=r_, chunk_len=C, n_bswa_chunks=2, io="f32",
                       budget_kind=ko.BUDGET_FIXED, budget_fixed=10 * T)
    unit, q, k, v, g = make_unit(cfg, G=2, seed=5, T=T, gated=True, affine=True, taus=True)
    y, lse = unit.prefill(q, k, v, g)
    L = cfg.window
    for h in range(2):
        for u in range(T):
            s = (u // C) * C
            b = max(0, s + C - L)
            keys, vals, scales = [], [], []
            for j in range(0, b):
                kz = [0.0] * r_ + list(k[j, r_:])
                kb = brute_ln(kz, unit.gamma, unit.beta, cfg.ln_eps).astype(np.float32).astype(np.float64)
                # LN_s of a one-token row is LN_s applied again to the stored memory key
                kh = brute_ln(list(kb), unit.gamma, unit.beta, cfg.ln_eps).astype(np.float32)
                keys.append(kh.astype(np.float64)); vals.append(v[j]); scales.append(unit.tau_state[h])
            for t in range(b, u + 1):
                keys.append(k[t]); vals.append(v[t]); scales.append(unit.tau_bswa[h])
            want, want_lse = brute_softmax_attention(q[h, u], keys, vals, scales)
            np.testing.assert_allclose(y[h, u], want, atol=2e-6)
            assert abs(lse[h, u] - want_lse) < 2e-6


def test_no_state_equals_block_sliding_window_attention():
    """With no compressed state the layer is n_bswa-block BSWA: query u sees [b, u]."""
    T, d, C = 30, 8, 4          # T not a multiple of C: trailing partial chunk
    cfg = ko.KVMConfig(head_dim=d, rope_dims=4, chunk_len=C, n_bswa_chunks=3, io="f32",
                       budget_kind=ko.BUDGET_NONE)
    unit, q, k, v, _ = make_unit(cfg, G=1, seed=6, T=T, taus=True)
    y, _ = unit.prefill(q, k, v)
    for u in range(T):
        b = max(0, (u // C) * C + C - cfg.window)
        want, _ = brute_softmax_attention(q[0, u], k[b:u + 1], v[b:u + 1], [unit.tau_bswa[0]] * (u + 1 - b))
        np.testing.assert_allclose(y[0, u], want, atol=1e-12)
    assert unit.state.m == 0


# ----------------------------------------------------------------------------- P11 mask geometry
def read_mask_golden():
    rows = {}
    with open(os.path.join(GOLDEN, "mask_c3_l6.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            u, b, last, st = line.split()
            rows[int(u)] = (int(b), int(last), [] if st == "-" else [int(x) for x in st.split(",")])
    return rows


@pytest.mark.parametrize("budget_kind", [ko.BUDGET_NONE, ko.BUDGET_FIXED])
def test_mask_geometry_c3_l6(budget_kind):
    """One-hot values make the support of each output row the set of visible tokens."""
    T, d, C = 12, 16, 3
    cfg = ko.KVMConfig(head_dim=d, rope_dims=4, chunk_len=C, n_bswa_chunks=2, io="f32",
                       budget_kind=budget_kind, budget_fixed=3)
    r = rng(7)
    q, k = r.normal(size=(1, T, d)), r.normal(size=(T, d))
    v = np.eye(d)[:T]
    y, _ = ko.KVMUnit(cfg).prefill(q, k, v)
    for u, (b, last, covered) in read_mask_golden().items():
        want = set(range(b, last + 1))
        if budget_kind != ko.BUDGET_NONE:
            want |= set(covered)
        assert set(np.nonzero(y[0, u] > 0)[0].tolist()) == want, u


# ----------------------------------------------------------------------------- P3, P6, P7, P9 fold
def run_fold_case(seed, gated, n_rows=6, n_tok=10, d=8, r_=2, S=1, budget=6):
    cfg = ko.KVMConfig(head_dim=d, rope_dims=r_, chunk_len=n_tok, io="f32", n_sink=S,
                       budget_kind=ko.BUDGET_FIXED, budget_fixed=budget)
    r = rng(seed)
    gamma, beta = r.uniform(0.5, 1.5, d), r.normal(scale=0.1, size=d)
    st = ko.UnitState(d)
    k0, v0 = r.normal(size=(n_rows, d)), r.normal(size=(n_rows, d))
    ko.fold(st, k0, v0, None, 2 * n_tok, ko.KVMConfig(head_dim=d, rope_dims=r_, chunk_len=n_rows, io="f32",
                                                      budget_kind=ko.BUDGET_FIXED, budget_fixed=budget),
            gamma, beta, positions=list(range(n_rows)))
    k1, v1 = r.normal(size=(n_tok, d)), r.normal(size=(n_tok, d))
    g = r.uniform(0.2, 3.0, size=n_tok) if gated else None
    return cfg, st, k0, v0, k1, v1, g, gamma, beta


@pytest.mark.parametrize("seed", [10, 11, 12])
def test_merge_targets_by_exhaustive_loops(seed):
    """Equation for pi_e(j): argmax over rows i >= S of k-bar_j . LN_s(s^K_i), every score
    against the pre-merge state.  Recomputed here with scalar loops."""
    cfg, st, k0, v0, k1, v1, g, gamma, beta = run_fold_case(seed, gated=True)
    pre_sK = st.sK.copy()
    log = ko.fold(st, k1, v1, g, 3 * cfg.chunk_len, cfg, gamma, beta)
    assert log["n_append"] == 0
    d = cfg.head_dim
    for j in range(k1.shape[0]):
        kz = [0.0] * cfg.rope_dims + list(k1[j, cfg.rope_dims:])
        kb = brute_ln(kz, gamma, beta, cfg.ln_eps).astype(np.float32).astype(np.float64)
        best, best_i = -1e300, -1
        for i in range(cfg.n_sink, pre_sK.shape[0]):
            kh = brute_ln(list(pre_sK[i]), gamma, beta, cfg.ln_eps).astype(np.float32).astype(np.float64)
            sc = sum(kb[c] * kh[c] for c in range(d))
            if sc > best:
                best, best_i = sc, i
        assert log["assign"][j] == best_i
        assert abs(log["best"][j] - best) < 1e-12


@pytest.mark.parametrize("gated", [False, True])
def test_state_rows_are_weighted_means_of_their_members(gated):
    """s^K_i / w_i is the g-weighted mean of the memory keys assigned to row i (creator
    weight 1); with g = 1 it is the arithmetic mean s^K_i / n_i.  Same for values."""
    cfg, st, k0, v0, k1, v1, g, gamma, beta = run_fold_case(20, gated)
    n0 = k0.shape[0]
    log = ko.fold(st, k1, v1, g, 3 * cfg.chunk_len, cfg, gamma, beta,
                  positions=list(range(n0, n0 + k1.shape[0])))
    cfg0 = ko.KVMConfig(head_dim=cfg.head_dim, rope_dims=cfg.rope_dims, chunk_len=n0, io="f32")
    kb_all = np.concatenate([ko.memory_key(k0, cfg0, gamma, beta), ko.memory_key(k1, cfg, gamma, beta)])
    v_all = np.concatenate([v0, v1])
    g_all = np.concatenate([np.ones(n0), np.ones(len(k1)) if g is None else g])
    for i in range(st.m):
        mem = [i] + [n0 + j for j in range(len(k1)) if log["assign"][j] == i]
        assert sorted(st.members[i]) == sorted(mem)
        wts = np.array([1.0] + [g_all[p] for p in mem[1:]])
        mean_k = sum(wt * kb_all[p] for wt, p in zip(wts, mem)) / wts.sum()
        mean_v = sum(wt * v_all[p] for wt, p in zip(wts, mem)) / wts.sum()
        np.testing.assert_allclose(st.sK[i] / st.w[i], mean_k, atol=1e-12)
        np.testing.assert_allclose(st.sV[i] / st.w[i], mean_v, atol=1e-12)
        assert st.n[i] == len(mem)
        if not gated:
            np.testing.assert_allclose(st.sK[i] / st.n[i], kb_all[mem].mean(0), atol=1e-12)


def test_radii_and_sinks_are_frozen_and_readout_has_stored_radius():
    """rho_i is set at row creation only; sink rows never receive a merge; the value readout
    has norm rho_i whatever was merged."""
    cfg, st, k0, v0, k1, v1, g, gamma, beta = run_fold_case(21, gated=True)
    rho0, sK0, sV0 = st.rho.copy(), st.sK[0].copy(), st.sV[0].copy()
    np.testing.assert_allclose(rho0, np.linalg.norm(v0, axis=1), atol=1e-13)
    for rep in range(4):
        r = rng(100 + rep)
        ko.fold(st, r.normal(size=k1.shape), r.normal(size=v1.shape), g, (3 + rep) * cfg.chunk_len,
                cfg, gamma, beta)
    np.testing.assert_array_equal(st.rho, rho0)
    np.testing.assert_array_equal(st.sK[0], sK0)
    np.testing.assert_array_equal(st.sV[0], sV0)
    assert st.n[0] == 1 and st.n.sum() == k0.shape[0] + 5 * 0 + 4 * k1.shape[0]
    _, vhat = ko.readout(st, cfg, gamma, beta)
    np.testing.assert_allclose(np.linalg.norm(vhat, axis=1), st.rho, rtol=1e-6)


def test_sink_is_attended_but_never_a_merge_target():
    """A token identical to the sink's creator would win row 0 if sinks were eligible."""
    cfg, st, k0, v0, k1, v1, g, gamma, beta = run_fold_case(22, gated=False)
    k1[3] = k0[0]
    log = ko.fold(st, k1, v1, None, 3 * cfg.chunk_len, cfg, gamma, beta)
    assert log["assign"][3] >= cfg.n_sink
    assert (log["assign"] >= cfg.n_sink).all()


# ----------------------------------------------------------------------------- append selection
def test_append_takes_the_least_similar_tokens_then_merges_the_rest_into_updated_state():
    """Section "Append" + "Merge": with room for n rows, the n tokens with the smallest
    s_j = max_i k-bar_j . s-hat^K_i are appended (ascending position); the others may merge
    into rows appended in the same step."""
    d, r_, n_rows, n_tok = 8, 2, 5, 9
    cfg = ko.KVMConfig(head_dim=d, rope_dims=r_, chunk_len=n_tok, io="f32",
                       budget_kind=ko.BUDGET_FIXED, budget_fixed=n_rows + 3)
    r = rng(30)
    gamma, beta = np.ones(d), np.zeros(d)
    st = ko.UnitState(d)
    k0, v0 = r.normal(size=(n_rows, d)), r.normal(size=(n_rows, d))
    st.append_rows(ko.memory_key(k0, cfg, gamma, beta), v0, list(range(n_rows)))
    k1, v1 = r.normal(size=(n_tok, d)), r.normal(size=(n_tok, d))
    k1[7] = k1[2] * 1.0001          # near-duplicate pair: if 2 is appended, 7 should merge into it
    kb = ko.memory_key(k1, cfg, gamma, beta)
    khat = np.stack([brute_ln(list(row), gamma, beta, cfg.ln_eps) for row in st.sK]).astype(np.float32)
    s = np.array([max(float(kb[j] @ khat[i].astype(np.float64)) for i in range(n_rows)) for j in range(n_tok)])
    # force token 2 to be among the least similar by checking the brute-force ranking itself
    want_app = sorted(sorted(range(n_tok), key=lambda j: (s[j], j))[:3])
    log = ko.fold(st, k1, v1, None, 3 * n_tok, cfg, gamma, beta)
    assert log["n_append"] == 3 and st.m == n_rows + 3
    assert [j for j in range(n_tok) if log["appended"][j]] == want_app
    assert [int(log["assign"][j]) for j in want_app] == [n_rows, n_rows + 1, n_rows + 2]
    np.testing.assert_allclose(log["s_max"], s, atol=1e-12)
    for a, j in enumerate(want_app):
        np.testing.assert_allclose(st.sV[n_rows + a] - sum(v1[p] for p in range(n_tok)
                                   if log["assign"][p] == n_rows + a and p != j), v1[j], atol=1e-12)
        assert abs(st.rho[n_rows + a] - np.linalg.norm(v1[j])) < 1e-13
    if 2 in want_app and 7 not in want_app:
        assert log["assign"][7] == log["assign"][2]


def test_remaining_token_merges_into_a_row_appended_in_the_same_step():
    """"The merge targets include ... any rows appended in the same step": two identical
    outlier tokens, room for one new row -> the earlier one is appended, the later one
    merges into that new row."""
    d, n_rows, n_tok = 8, 4, 6
    cfg = ko.KVMConfig(head_dim=d, rope_dims=2, chunk_len=n_tok, io="f32",
                       budget_kind=ko.BUDGET_FIXED, budget_fixed=n_rows + 1)
    r = rng(32)
    gamma, beta = np.ones(d), np.zeros(d)
    a = np.array([0, 0, 3.0, -3.0, 2.0, -2.0, 1.0, -1.0])
    b = np.array([0, 0, 1.0, 1.0, -3.0, -3.0, 2.0, 2.0])      # orthogonal to a after centring
    st = ko.UnitState(d)
    k0 = a + 0.05 * r.normal(size=(n_rows, d))
    st.append_rows(ko.memory_key(k0, cfg, gamma, beta), r.normal(size=(n_rows, d)), list(range(n_rows)))
    k1 = a + 0.05 * r.normal(size=(n_tok, d))
    k1[1] = b
    k1[4] = b
    k1[4, :2] = 5.0                                             # rotary channels are ignored
    v1 = r.normal(size=(n_tok, d))
    log = ko.fold(st, k1, v1, None, 3 * n_tok, cfg, gamma, beta)
    assert log["n_append"] == 1
    assert log["appended"].tolist() == [False, True, False, False, False, False]
    assert log["assign"][1] == n_rows and log["assign"][4] == n_rows
    np.testing.assert_allclose(st.sV[n_rows], v1[1] + v1[4], atol=1e-13)
    assert abs(st.rho[n_rows] - np.linalg.norm(v1[1])) < 1e-13


def test_append_tie_prefers_lower_position_and_merge_tie_prefers_lower_row():
    d, n_rows, n_tok = 8, 4, 6
    cfg = ko.KVMConfig(head_dim=d, rope_dims=0, chunk_len=n_tok, io="f32",
                       budget_kind=ko.BUDGET_FIXED, budget_fixed=n_rows + 1)
    r = rng(31)
    gamma, beta = np.ones(d), np.zeros(d)
    st = ko.UnitState(d)
    k0 = r.normal(size=(n_rows, d))
    k0[3] = k0[2]                                   # rows 2 and 3 identical -> merge ties
    st.append_rows(ko.memory_key(k0, cfg, gamma, beta), r.normal(size=(n_rows, d)), list(range(n_rows)))
    k1 = r.normal(size=(n_tok, d))
    k1[4] = k1[1]                                   # tokens 1 and 4 identical -> equal s_j
    log = ko.fold(st, k1, r.normal(size=(n_tok, d)), None, 3 * n_tok, cfg, gamma, beta)
    order = sorted(range(n_tok), key=lambda j: (log["s_max"][j], j))
    assert log["s_max"][1] == log["s_max"][4]
    if order[0] in (1, 4):
        assert log["appended"][1] and not log["appended"][4]
    assert 3 not in [int(a) for j, a in enumerate(log["assign"]) if not log["appended"][j]]


# ----------------------------------------------------------------------------- P12 duplicates
def test_exact_duplicate_joins_its_own_row_and_leaves_the_key_readout_unchanged():
    """With gamma = 1, beta = 0 every normalised key has the same norm, so a token whose
    memory key equals a one-member row's key scores highest there (Cauchy-Schwarz); the
    sum 2 * k-bar normalises to the same s-hat^K."""
    cfg, st, k0, v0, k1, v1, g, _, _ = run_fold_case(40, gated=False)
    d = cfg.head_dim
    gamma, beta = np.ones(d), np.zeros(d)
    st = ko.UnitState(d)
    cfg0 = ko.KVMConfig(head_dim=d, rope_dims=cfg.rope_dims, chunk_len=len(k0), io="f32")
    st.append_rows(ko.memory_key(k0, cfg0, gamma, beta), v0, list(range(len(k0))))
    k1[5] = k0[4]
    k1[5, :cfg.rope_dims] += 3.0                    # rotary channels do not matter
    kh_before, _ = ko.readout(st, cfg, gamma, beta)
    log = ko.fold(st, k1, v1, None, 3 * cfg.chunk_len, cfg, gamma, beta)
    assert log["assign"][5] == 4
    if (log["assign"] == 4).sum() == 1:
        kh_after, _ = ko.readout(st, cfg, gamma, beta)
        np.testing.assert_allclose(kh_after[4], kh_before[4], atol=1e-5)


# ----------------------------------------------------------------------------- P5 budget
def test_state_size_follows_the_growth_budget():
    """M*(e) = max(m, min(B(e), m + C)), n_append = min(M* - m, |Omega|); creation gives C.
    Expected sizes below are worked by hand for each schedule."""
    # fixed budget 512, C = 256, L = 512: folds at e = 512 (creation -> 256), 768 (-> 512), then flat
    cfg = ko.KVMConfig(head_dim=8, rope_dims=0, chunk_len=256, budget_kind=ko.BUDGET_FIXED, budget_fixed=512)
    assert ko.expected_rows(cfg, 2048) == [256, 512, 512, 512, 512, 512, 512]
    # fixed budget 64 = C: creation then never grows
    cfg = ko.KVMConfig(head_dim=8, rope_dims=0, chunk_len=64, budget_kind=ko.BUDGET_FIXED, budget_fixed=64)
    assert ko.expected_rows(cfg, 1024) == [64] * 15
    # budget below C: creation still copies a whole chunk
    cfg = ko.KVMConfig(head_dim=8, rope_dims=0, chunk_len=64, budget_kind=ko.BUDGET_FIXED, budget_fixed=10)
    assert ko.expected_rows(cfg, 512) == [64] * 7
    # 4 * ceil(sqrt(e)), C = 256: stays 256 while 4*ceil(sqrt(e)) <= 256 i.e. e <= 4096;
    # 4*ceil(sqrt(4352)) = 4*66 = 264; reaches 512 at e = 16384 and 1024 at e = 65536
    cfg = ko.KVMConfig(head_dim=8, rope_dims=0, chunk_len=256, budget_kind=ko.BUDGET_SQRT, budget_scale=4.0)
    rows = ko.expected_rows(cfg, 65536)
    ends = [512 + 256 * i for i in range(len(rows))]
    by_e = dict(zip(ends, rows))
    assert len(rows) == 255 and by_e[512] == 256 and by_e[4096] == 256 and by_e[4352] == 264
    assert by_e[16384] == 512 and by_e[65536] == 1024
    assert all(b >= a for a, b in zip(rows, rows[1:]))
    # no state at all
    cfg = ko.KVMConfig(head_dim=8, rope_dims=0, chunk_len=4, budget_kind=ko.BUDGET_NONE)
    assert ko.expected_rows(cfg, 64) == []
    # exact integer ceil-sqrt
    for e in [1, 2, 3, 4, 5, 15, 16, 17, 4095, 4096, 4097, 10 ** 12, 10 ** 12 + 1]:
        n = ko.ceil_sqrt(e)
        assert n * n >= e and (n - 1) * (n - 1) < e


def test_run_state_sizes_match_integer_replay():
    T, C = 96, 4
    for kind, kw in [(ko.BUDGET_FIXED, dict(budget_fixed=10)), (ko.BUDGET_SQRT, dict(budget_scale=2.0)),
                     (ko.BUDGET_TABLE, dict(budget_table=[0, 4, 5, 5, 9, 30, 31, 31])),
                     # budgets below the rows the state already has: it neither grows nor shrinks
                     (ko.BUDGET_FIXED, dict(budget_fixed=2)),
                     (ko.BUDGET_TABLE, dict(budget_table=[0, 4, 7, 3, 3, 9, 1]))]:
        cfg = ko.KVMConfig(head_dim=8, rope_dims=2, chunk_len=C, io="f32", budget_kind=kind, **kw)
        unit, q, k, v, _ = make_unit(cfg, seed=50, T=T)
        unit.prefill(q, k, v)
        got = [lg["m_after"] for lg in unit.fold_logs]
        m, want = 0, []
        for e in range(2 * C, T + 1, C):            # replay written out here, not via the oracle
            if m == 0:
                m = C
            else:
                if kind == ko.BUDGET_FIXED:
                    B = kw["budget_fixed"]
                elif kind == ko.BUDGET_SQRT:
                    B = int(2.0 * math.ceil(math.sqrt(e)))
                else:
                    tb = kw["budget_table"]
                    B = tb[min(e // C - 1, len(tb) - 1)]
                m = max(m, min(B, m + C))
            want.append(m)
        assert got == want
        assert all(lg["m_after"] - lg["m_before"] == lg["n_append"] for lg in unit.fold_logs)
        assert all(int(lg["appended"].sum()) == lg["n_append"] >= 0 for lg in unit.fold_logs)
        assert unit.state.m == want[-1] == len(unit.state.rho)


# ----------------------------------------------------------------------------- P4 softmax
def test_constant_values_give_constant_output():
    """Softmax rows sum to 1: with every value equal to the all-ones vector, rho = sqrt(d),
    s-hat^V = 1 and every output is the all-ones vector."""
    T, d, C = 48, 8, 4
    cfg = ko.KVMConfig(head_dim=d, rope_dims=2, chunk_len=C, io="f32",
                       budget_kind=ko.BUDGET_FIXED, budget_fixed=6)
    unit, q, k, _, g = make_unit(cfg, G=2, seed=60, T=T, gated=True, taus=True, affine=True)
    y, _ = unit.prefill(q, k, np.ones((T, d)), g)
    np.testing.assert_allclose(y, 1.0, atol=1e-6)


def test_lse_is_log_of_summed_exponentials_over_state_and_window():
    T, d, C = 40, 8, 4
    cfg = ko.KVMConfig(head_dim=d, rope_dims=2, chunk_len=C, io="f32",
                       budget_kind=ko.BUDGET_FIXED, budget_fixed=6)
    unit, q, k, v, g = make_unit(cfg, G=1, seed=61, T=T, gated=True, taus=True)
    probe = ko.KVMUnit(cfg, 1, None, None, unit.tau_state, unit.tau_bswa)
    y, lse = unit.prefill(q, k, v, g)
    # replay up to the last chunk to obtain the state that chunk saw, then brute-force it
    probe.prefill(q[:, :T - C], k[:T - C], v[:T - C], g[:T - C])
    khat, vhat = ko.readout(probe.state, cfg, probe.gamma, probe.beta)
    u = T - 2
    b = T - cfg.window
    keys = list(khat) + list(k[b:u + 1])
    vals = list(vhat) + list(v[b:u + 1])
    scales = [unit.tau_state[0]] * len(khat) + [unit.tau_bswa[0]] * (u + 1 - b)
    want, want_lse = brute_softmax_attention(q[0, u], keys, vals, scales)
    np.testing.assert_allclose(y[0, u], want, atol=1e-12)
    assert abs(lse[0, u] - want_lse) < 1e-12


# ----------------------------------------------------------------------------- P8 invariances
def test_readout_ignores_row_scale_and_row_order():
    """Normalising before readout makes a row's scale irrelevant ("equivalent to taking the
    weighted mean"); state rows are a set, so permuting non-sink rows changes nothing."""
    T, d, C = 40, 8, 4
    cfg = ko.KVMConfig(head_dim=d, rope_dims=2, chunk_len=C, io="f32",
                       budget_kind=ko.BUDGET_FIXED, budget_fixed=8, ln_eps=1e-12)
    unit, q, k, v, g = make_unit(cfg, G=1, seed=70, T=T, gated=True)
    unit.prefill(q[:, :T - C], k[:T - C], v[:T - C], g[:T - C])
    base = ko.KVMUnit(cfg)
    import copy
    twin = copy.deepcopy(unit)
    y0, _ = unit.prefill(q[:, T - C:], k[T - C:], v[T - C:], g[T - C:])
    sc = rng(71).uniform(0.5, 4.0, size=twin.state.m)
    perm = np.concatenate([[0], 1 + rng(72).permutation(twin.state.m - 1)])
    twin.state.sK = (twin.state.sK * sc[:, None])[perm]
    twin.state.sV = (twin.state.sV * sc[:, None])[perm]
    twin.state.rho = twin.state.rho[perm]
    y1, _ = twin.prefill(q[:, T - C:], k[T - C:], v[T - C:], g[T - C:])
    np.testing.assert_allclose(y1, y0, atol=2e-6)


# ----------------------------------------------------------------------------- P10 self-consistency
@pytest.mark.parametrize("io", ["f32", "bf16"])
def test_split_prefill_and_decode_reproduce_one_shot_prefill(io):
    T, d, C = 56, 8, 4
    cfg = ko.KVMConfig(head_dim=d, rope_dims=4, chunk_len=C, io=io,
                       budget_kind=ko.BUDGET_SQRT, budget_scale=1.5)
    a, q, k, v, g = make_unit(cfg, G=2, seed=80, T=T, gated=True, affine=True, taus=True)
    y_all, lse_all = a.prefill(q, k, v, g)
    mk = lambda: ko.KVMUnit(cfg, 2, a.gamma, a.beta, a.tau_state, a.tau_bswa)
    b_ = mk()
    T1 = 24
    y1, _ = b_.prefill(q[:, :T1], k[:T1], v[:T1], g[:T1])
    y2, _ = b_.prefill(q[:, T1:], k[T1:], v[T1:], g[T1:])
    np.testing.assert_allclose(np.concatenate([y1, y2], axis=1), y_all, atol=1e-12)
    c_ = mk()
    T0 = 18                                          # partial chunk, completed by decode
    yp, _ = c_.prefill(q[:, :T0], k[:T0], v[:T0], g[:T0])
    ys = [c_.decode(q[:, t], k[t], v[t], g[t])[0] for t in range(T0, T)]
    # a matmul over one row and over C rows may round differently in the last bits
    np.testing.assert_allclose(np.concatenate([yp, np.stack(ys, axis=1)], axis=1), y_all, atol=1e-12)
    np.testing.assert_array_equal(c_.state.sK, a.state.sK)
    assert [lg["assign"].tolist() for lg in c_.fold_logs] == [lg["assign"].tolist() for lg in a.fold_logs]


def test_bf16_contract_rounds_only_the_materialised_vectors():
    """Memory keys and readout rows are bf16 values; the state sums are not rounded."""
    d, C, T = 8, 4, 24
    cfg = ko.KVMConfig(head_dim=d, rope_dims=2, chunk_len=C, io="bf16",
                       budget_kind=ko.BUDGET_FIXED, budget_fixed=4)
    unit, q, k, v, g = make_unit(cfg, seed=90, T=T, gated=True)
    unit.prefill(q, k, v, g)
    khat, vhat = ko.readout(unit.state, cfg, unit.gamma, unit.beta)
    for arr in (khat, vhat, ko.memory_key(k, cfg, unit.gamma, unit.beta)):
        np.testing.assert_array_equal(arr, ko.round_bf16(arr))
    assert not np.array_equal(unit.state.sK, ko.round_bf16(unit.state.sK))


def test_override_is_refused_outside_the_tie_margin():
    cfg, st, k0, v0, k1, v1, g, gamma, beta = run_fold_case(95, gated=False)
    import copy
    st2 = copy.deepcopy(st)
    log = ko.fold(st, k1, v1, None, 3 * cfg.chunk_len, cfg, gamma, beta)
    j = int(np.nanargmax(log["margin"]))
    other = 1 if log["assign"][j] != 1 else 2
    with pytest.raises(ValueError):
        ko.fold(st2, k1, v1, None, 3 * cfg.chunk_len, cfg, gamma, beta, overrides={j: other})


def _append_boundary_case():
    """Five rows, nine tokens, room for three new rows; token b is token a scaled by 1 + 1e-7,
    so their memory keys (LN_s is scale invariant) and append scores agree to ~1e-7 while the
    other scores lie far apart.  a and b are placed on the selection boundary by brute force."""
    d, r_, n_rows, n_tok = 8, 2, 5, 9
    cfg = ko.KVMConfig(head_dim=d, rope_dims=r_, chunk_len=n_tok, io="f32",
                       budget_kind=ko.BUDGET_FIXED, budget_fixed=n_rows + 3)
    gamma, beta = np.ones(d), np.zeros(d)
    for seed in range(200, 260):
        r = rng(seed)
        st = ko.UnitState(d)
        k0, v0 = r.normal(size=(n_rows, d)), r.normal(size=(n_rows, d))
        st.append_rows(ko.memory_key(k0, cfg, gamma, beta), v0, list(range(n_rows)))
        k1, v1 = r.normal(size=(n_tok, d)), r.normal(size=(n_tok, d))
        # brute-force append scores (scalar loops, equation for s_j)
        def scores(kblk):
            out = []
            for j in range(n_tok):
                kz = [0.0] * r_ + list(kblk[j, r_:])
                kb = brute_ln(kz, gamma, beta, cfg.ln_eps).astype(np.float32).astype(np.float64)
                best = -1e300
                for i in range(n_rows):
                    kh = brute_ln(list(st.sK[i]), gamma, beta, cfg.ln_eps).astype(np.float32).astype(np.float64)
                    best = max(best, sum(kb[c] * kh[c] for c in range(d)))
                out.append(best)
            return np.array(out)
        s = scores(k1)
        order = sorted(range(n_tok), key=lambda j: (s[j], j))
        a = order[2]                       # the last token taken
        b = order[3]                       # the first token left out: make it a's near twin
        k1[b] = k1[a] * (1.0 + 1e-7)
        s = scores(k1)
        order = sorted(range(n_tok), key=lambda j: (s[j], j))
        gaps_ok = all(abs(s[j] - s[a]) > 1e-2 for j in range(n_tok) if j not in (a, b))
        if set(order[2:4]) == {a, b} and abs(s[a] - s[b]) < 1e-5 and gaps_ok:
            return cfg, st, k1, v1, gamma, beta, s, order
    raise AssertionError("no seed gave a clean boundary pair")


def test_append_override_is_honoured_only_inside_the_tie_margin():
    """"Append": A_e is the n_append tokens with the smallest s_j.  The oracle lets a test swap
    tokens in and out of A_e only when their scores lie within 1e-4 of the boundary score (the
    n_append-th smallest); the accepted set is then what gets appended, in ascending position."""
    import copy
    cfg, st, k1, v1, gamma, beta, s, order = _append_boundary_case()
    n_rows, n_tok, e = st.m, k1.shape[0], 3 * k1.shape[0]
    own = sorted(order[:3])
    log = ko.fold(copy.deepcopy(st), k1, v1, None, e, cfg, gamma, beta)
    assert sorted(np.nonzero(log["appended"])[0].tolist()) == own
    # inside the margin: the boundary pair swapped
    taken, left = order[2], order[3]
    alt = sorted(set(own) - {taken} | {left})
    st_alt = copy.deepcopy(st)
    log_alt = ko.fold(st_alt, k1, v1, None, e, cfg, gamma, beta, append_override=alt)
    assert sorted(np.nonzero(log_alt["appended"])[0].tolist()) == alt
    assert [int(log_alt["assign"][j]) for j in alt] == [n_rows, n_rows + 1, n_rows + 2]
    for a_, j in enumerate(alt):           # the new rows were created from the override's tokens
        assert abs(st_alt.rho[n_rows + a_] - np.linalg.norm(v1[j])) < 1e-13
    assert not log_alt["appended"][taken] and log_alt["assign"][taken] >= cfg.n_sink
    # the same set as the oracle's own choice is a no-op
    log_same = ko.fold(copy.deepcopy(st), k1, v1, None, e, cfg, gamma, beta, append_override=list(reversed(own)))
    np.testing.assert_array_equal(log_same["assign"], log["assign"])
    # outside the margin: any swap that involves a token far from the boundary
    far_out = order[-1]
    far_in = order[0]
    for bad in (sorted(set(own) - {taken} | {far_out}), sorted(set(own) - {far_in} | {left}),
                sorted(set(own) - {far_in} | {far_out})):
        with pytest.raises(ValueError, match="tie margin"):
            ko.fold(copy.deepcopy(st), k1, v1, None, e, cfg, gamma, beta, append_override=bad)
    # wrong sizes, repeated tokens
    for bad in (own[:2], own + [left], [own[0], own[0], own[1]]):
        with pytest.raises(ValueError, match="wrong size"):
            ko.fold(copy.deepcopy(st), k1, v1, None, e, cfg, gamma, beta, append_override=bad)


def test_append_override_margin_is_measured_from_the_boundary_score():
    """A token 5e-5 above the boundary may be swapped in; one 2e-4 above may not (margin 1e-4)."""
    import copy
    cfg, st, k1, v1, gamma, beta, s, order = _append_boundary_case()
    e = 3 * k1.shape[0]
    own = sorted(order[:3])
    taken, left = order[2], order[3]

    # the left-out token's append score is moved by a chosen amount: its raw key is pushed along
    # the state key it scores highest against
    khat, _ = ko.readout(st, cfg, gamma, beta)
    kb = ko.memory_key(k1, cfg, gamma, beta)
    sim = kb @ khat.T
    i_star = int(np.argmax(sim[left]))
    for delta, ok in ((5e-5, True), (2e-4, False)):
        # find a scale of the raw key's component along khat[i*] that lifts s_left by ~delta
        k_mod = k1.copy()
        lo, hi = 0.0, 1.0
        for _ in range(60):
            mid = 0.5 * (lo + hi)
            k_try = k1.copy()
            k_try[left, cfg.rope_dims:] += mid * khat[i_star, cfg.rope_dims:]
            s_try = (ko.memory_key(k_try, cfg, gamma, beta) @ khat.T).max(axis=1)
            if s_try[left] - s[taken] < delta:
                lo = mid
            else:
                hi = mid
        k_mod[left, cfg.rope_dims:] += hi * khat[i_star, cfg.rope_dims:]
        s_mod = (ko.memory_key(k_mod, cfg, gamma, beta) @ khat.T).max(axis=1)
        gap = s_mod[left] - s_mod[taken]
        assert abs(gap - delta) < 2e-5, gap
        alt = sorted(set(own) - {taken} | {left})
        if ok:
            log = ko.fold(copy.deepcopy(st), k_mod, v1, None, e, cfg, gamma, beta, append_override=alt)
            assert sorted(np.nonzero(log["appended"])[0].tolist()) == alt
        else:
            with pytest.raises(ValueError, match="tie margin"):
                ko.fold(copy.deepcopy(st), k_mod, v1, None, e, cfg, gamma, beta, append_override=alt)


def test_merge_override_is_honoured_inside_the_tie_margin():
    """Two state rows with the same key sums score alike; the lowest row wins by default and an
    override to its twin is accepted (margin 0 <= 1e-4), then that row receives the token."""
    import copy
    cfg, st, k0, v0, k1, v1, g, gamma, beta = run_fold_case(96, gated=False)
    st.sK[4] = st.sK[2]
    base = copy.deepcopy(st)
    log = ko.fold(copy.deepcopy(base), k1, v1, None, 3 * cfg.chunk_len, cfg, gamma, beta)
    js = [j for j in range(k1.shape[0]) if log["assign"][j] == 2]
    assert js and not (log["assign"] == 4).any()
    j = js[0]
    st2 = copy.deepcopy(base)
    log2 = ko.fold(st2, k1, v1, None, 3 * cfg.chunk_len, cfg, gamma, beta, overrides={j: 4})
    assert log2["assign"][j] == 4 and st2.n[4] == 2
    np.testing.assert_allclose(st2.sV[4], base.sV[4] + v1[j], atol=1e-13)
