"""kvm_decode_step_multi: one decode launch over sequences that live in different states, each at
its own position and with its own number of state rows.  Every sequence is checked against the CPU
oracle driven on its own (prefill of its prompt, then token by token), to the same bars as the
single-state tests.
"""
import numpy as np
import pytest
import torch

import kvm_testlib as tl

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def kvm():
    import paper_2605_09877_amd as pkg
    return pkg


def synth():
    from paper_2605_09877_amd import synth as s
    return s


def run_ragged(base, batches, prompts, n_dec, plain):
    """States with `batches[i]` sequences and a prompt of `prompts[i]` tokens each, sharing one
    configuration and one set of layer parameters; n_dec decode steps over all of them at once."""
    pkg, sy = kvm(), synth()
    from paper_2605_09877_amd import binding
    shared = sy.make_params(base, DEV, plain=plain)
    states, data = [], []
    for i, (B, Tp) in enumerate(zip(batches, prompts)):
        w = sy.shrink(base, batch=B, seq=Tp + n_dec, seed=base.seed + 101 * i)
        q, k, v = sy.make_qkv(w, DEV)
        params = dict(shared)
        params["gate"] = None if plain else sy.make_params(w, DEV, plain=False)["gate"]
        st = pkg.state_for(w, device=DEV, **params)
        assign, score = st.trace(w.seq // w.chunk_len + 1)
        g = params["gate"]
        o = st.prefill(q[:, :Tp].contiguous(), k[:, :Tp].contiguous(), v[:, :Tp].contiguous(),
                       None if g is None else g[:, :Tp].contiguous())
        o = o[0] if isinstance(o, tuple) else o
        states.append(st)
        data.append(dict(w=w, q=q, k=k, v=v, params=params, Tp=Tp, outs=[o], assign=assign))
    rows_seen = set()
    for t in range(n_dec):
        qs = torch.cat([d["q"][:, d["Tp"] + t] for d in data]).contiguous()
        ks = torch.cat([d["k"][:, d["Tp"] + t] for d in data]).contiguous()
        vs = torch.cat([d["v"][:, d["Tp"] + t] for d in data]).contiguous()
        gs = None if plain else torch.cat([d["params"]["gate"][:, d["Tp"] + t] for d in data]).contiguous()
        out = binding.decode_multi(states, qs, ks, vs, gs)
        s = 0
        for d, st in zip(data, states):
            B = d["w"].batch
            d["outs"].append(out[s:s + B][:, None])
            s += B
        rows_seen.add(tuple(st.rows for st in states))
    torch.cuda.synchronize()
    all_ties, worst, n_units = tl.Ties(), 0.0, 0
    for d, st in zip(data, states):
        w, Tp = d["w"], d["Tp"]
        assert st.tokens == w.seq
        y_gpu = torch.cat(d["outs"], dim=1)
        ga_all = d["assign"][:st.folds].cpu().numpy()
        exp = st.export()
        G = w.n_q_heads // w.n_kv_heads
        for b in range(w.batch):
            for h in range(w.n_kv_heads):
                u = tl.unit_inputs(w, d["q"], d["k"], d["v"], d["params"], b, h)

                def drive(unit):
                    y, _ = unit.prefill(u["q"][:, :Tp], u["k"][:Tp], u["v"][:Tp], None if u["g"] is None else u["g"][:Tp])
                    ys = [y]
                    for t in range(Tp, w.seq):
                        yt, _ = unit.decode(u["q"][:, t], u["k"][t], u["v"][t], None if u["g"] is None else u["g"][t])
                        ys.append(yt[:, None])
                    return np.concatenate(ys, axis=1)

                y_ref, unit, ties = tl.run_oracle_following(w, d["params"], h, drive, ga_all[:, b, h])
                assert len(unit.fold_logs) == st.folds and unit.state.m == st.rows
                yg = tl.f64(y_gpu[b, :, h * G:(h + 1) * G]).transpose(1, 0, 2)
                worst = max(worst, tl.check_outputs(w, yg, y_ref, f"state with prompt {Tp}, unit {(b, h)}"))
                all_ties += ties
                n_units += 1
                tl.check_state(w, exp, unit, b, h)
    tl.record_parity(f"ragged_decode[{base.name},{base.io}]", n_units, all_ties, worst, base.io)
    return states, rows_seen


def test_ragged_decode_growing_states_bf16():
    """Square-root budget: three states whose prompts end at different places, so that they differ
    in state rows and window fill, and fold at different steps (with small appends)."""
    base = synth().shrink(synth().WORKLOADS["prefill_sqrt"], n_q_heads=4, n_kv_heads=2, chunk_len=128)
    states, rows_seen = run_ragged(base, batches=(1, 2, 1), prompts=(128 * 9, 128 * 20 + 57, 300), n_dec=200, plain=False)
    assert len({st.rows for st in states}) == 3 and len({st.tokens for st in states}) == 3
    assert len(rows_seen) > 2  # folds happened during the decode steps, at different steps


def test_ragged_decode_fixed_budget_f32():
    base = synth().shrink(synth().WORKLOADS["tiny_f32"])
    run_ragged(base, batches=(2, 1), prompts=(64 * 5 + 3, 64), n_dec=140, plain=True)


def test_ragged_decode_rejects_mismatched_states():
    pkg, sy = kvm(), synth()
    from paper_2605_09877_amd import binding
    w1 = sy.shrink(sy.WORKLOADS["prefill_fixed"], batch=1, n_q_heads=2, n_kv_heads=2, seq=512)
    w2 = sy.shrink(w1, chunk_len=128)
    s1, s2 = pkg.state_for(w1, device=DEV), pkg.state_for(w2, device=DEV)
    dt = torch.bfloat16
    q = torch.zeros(2, 2, 128, dtype=dt, device=DEV)
    with pytest.raises(binding.KVMError):
        binding.decode_multi([s1, s2], q, q.clone(), q.clone())
    with pytest.raises(binding.KVMError):
        binding.decode_multi([s1, s1], q, q.clone(), q.clone())
