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
