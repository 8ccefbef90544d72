"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (plain
parameters, no gate): the HIP path runs the whole workload, the oracle replays sampled
(batch, KV head) units -- first, last and a seeded random one -- over all chunks and folds.
Units are independent, so a sampled unit checks every step of the path at its real shape."""
import numpy as np
import pytest
import torch

import kvm_testlib as tl
from test_gpu_parity import run_prefill_case, synth, kvm

pytestmark = pytest.mark.gpu


def sample_units(w, n_random=1):
    units = [(0, 0), (w.batch - 1, w.n_kv_heads - 1)]
    r = np.random.default_rng(w.seed)
    while len(units) < 2 + n_random:
        cand = (int(r.integers(w.batch)), int(r.integers(w.n_kv_heads)))
        if cand not in units:
            units.append(cand)
    return units


@pytest.mark.parametrize("name,rows", [("prefill_fixed", 512), ("prefill_sqrt", 1024), ("prefill_gqa_32k", 1024)])
def test_full_size_prefill_sampled_units(name, rows):
    w = synth().WORKLOADS[name]
    ties, st = run_prefill_case(w, plain=True, units=sample_units(w), check_lse=True)
    assert st.rows == rows
    assert st.folds == w.seq // w.chunk_len - 1
    print(f"{name}: ties counted in sampled units: {ties}")


@pytest.mark.parametrize("name,split", [("prefill_gqa_32k", 4), ("prefill_sqrt", 8)])
def test_full_size_prefill_with_rows_shared_among_workgroups(name, split):
    """The one-launch fold with a unit's rows shared among `split` workgroups (kvm_debug_set), at
    full size and beside the attention launches: 256 workgroups that wait for each other's winners
    at every fold while the chip is busy with other kernels."""
    from paper_2605_09877_amd import binding
    w = synth().WORKLOADS[name]
    ties, st = run_prefill_case(w, plain=True, units=sample_units(w), check_lse=True,
                                knobs={binding.KVM_DEBUG_FOLD_PATH: 1, binding.KVM_DEBUG_FOLD_SPLIT: split})
    assert st.fold_path == 1 and st.folds == w.seq // w.chunk_len - 1 and ties.total == 0


def test_full_size_decode_sampled_units():
    """Batched decode workload at full size: 64 x 32 heads, 2048 rows + 256-token window, all of
    its 1000 successive steps (seven folds); sampled units replayed by the oracle."""
    pkg, sy = kvm(), synth()
    w = sy.WORKLOADS["decode"]
    assert w.seq == 1000
    pre = sy.make_decode_state(w, "cuda:0")
    st = pkg.state_for(w, device="cuda:0", max_tokens=pre["tokens"] + 2 * w.seq)
    assign, _ = st.trace(8)
    st.import_(dict(pre, folds=0))
    q, k, v = sy.make_qkv(w, "cuda:0", T=w.seq, pos0=pre["tokens"])
    outs = [st.decode(q[:, t].contiguous(), k[:, t].contiguous(), v[:, t].contiguous()) for t in range(w.seq)]
    torch.cuda.synchronize()
    y_gpu = torch.stack(outs, dim=1)
    assert st.folds == 7 and st.rows == 2048
    ga = assign[:7].cpu().numpy()
    L, t0 = w.chunk_len * w.n_bswa_chunks, pre["tokens"]
    all_ties, worst, units = tl.Ties(), 0.0, sample_units(w)
    for (b, h) in units:
        def drive(unit):
            s0 = unit.state
            s0.sK = pre["sK"][b, h].cpu().numpy().copy()
            s0.sV = tl.f64(pre["sV"][b, h]).copy()
            s0.rho = tl.f64(pre["rho"][b, h]).copy()
            s0.w, s0.n = np.ones(w.state_rows), np.ones(w.state_rows, dtype=np.int64)
            s0.members = [[-1] for _ in range(w.state_rows)]
            unit.t = t0
            unit.k_hist = np.zeros((t0, w.head_dim))
            unit.v_hist = np.zeros((t0, w.head_dim))
            unit.g_hist = np.ones(t0)
            pos = np.arange(t0 - L, t0)
            unit.k_hist[pos] = tl.f64(pre["win_k"][b, h])[pos % L]
            unit.v_hist[pos] = tl.f64(pre["win_v"][b, h])[pos % L]
            ys = [unit.decode(tl.f64(q[b, t, h:h + 1]), tl.f64(k[b, t, h]), tl.f64(v[b, t, h]))[0]
                  for t in range(w.seq)]
            return np.stack(ys, axis=1)

        y_ref, unit, ties = tl.run_oracle_following(w, {}, h, drive, ga[:, b, h])
        all_ties += ties
        worst = max(worst, tl.check_outputs(w, tl.f64(y_gpu[b, :, h:h + 1]).transpose(1, 0, 2), y_ref,
                                            f"decode unit {(b, h)}"))
    tl.record_parity("full_size_decode[1000 steps]", len(units), all_ties, worst, w.io)


def test_paper_speed_benchmark_shape_growth_budget_sampled_units():
    """The configuration bench.py --sweep times (the paper's "Speed Benchmarks" shape): 8 sequences
    x 32 heads (no grouping), head_dim 128, 256-token chunks, a budget of 16 * ceil(sqrt(e)) rows
    (1456 rows after 8192 tokens).  At this size the library runs the prefill chunk by chunk with
    folds in place against a large, growing state, a schedule the other workloads do not take;
    sampled units are replayed by the oracle over all 32 chunks and 31 folds."""
    sy = synth()
    w = sy.shrink(sy.WORKLOADS["prefill_fixed"], name="paper_shape_sqrt", batch=8, n_q_heads=32, n_kv_heads=32,
                  head_dim=128, chunk_len=256, rope_dims=32, seq=8192, budget_kind="sqrt", budget_scale=16.0)
    ties, st = run_prefill_case(w, plain=True, units=sample_units(w), check_lse=True)
    assert st.rows == 16 * 91 and st.folds == 31          # ceil(sqrt(8192)) = 91


def test_full_budget_is_exact_causal_attention_over_memory_keys():
    """The sweep's comparator: a budget that never fills, so every block is appended whole and a
    query attends every earlier token (as its memory key once it has left the window)."""
    sy = synth()
    w = sy.shrink(sy.WORKLOADS["prefill_fixed"], name="paper_shape_full", batch=2, n_q_heads=4, n_kv_heads=4,
                  head_dim=128, chunk_len=256, rope_dims=32, seq=4096, budget_kind="fixed", budget_fixed=4096 + 256)
    ties, st = run_prefill_case(w, plain=True, units=[(0, 0), (1, 3)], check_lse=True)
    # every token of the blocks folded so far (all but the last window block) has a row of its own
    assert st.rows == 4096 - 512 + 256 and ties.total == 0
