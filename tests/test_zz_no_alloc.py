"""kvm_decode_step_multi_static, the allocation-free variant of kvm_decode_step_multi (its
per-sequence descriptor table lives in a device array inside the library): called through the C
ABI on two batches in a row, the second smaller than the first, and checked against
kvm_decode_step_multi on twin states.  Both run the same attention and fold kernels, so outputs
and states must agree to the bit, which is inside every bar of the parity tests.  Decode steps run
across a chunk boundary, so folds (with small appends) happen on both sides.
"""
import ctypes as C

import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def build_states(pkg, sy, base, batches, prompts, n_dec, shared):
    states, data = [], []
    for i, (B, Tp) in enumerate(zip(batches, prompts)):
        w = sy.shrink(base, batch=B, seq=Tp + n_dec, seed=base.seed + 101 * i)
        q, k, v = sy.make_qkv(w, DEV)
        gate = sy.make_params(w, DEV, plain=False)["gate"]
        params = dict(shared, gate=gate)
        st = pkg.state_for(w, device=DEV, **params)
        st.prefill(q[:, :Tp].contiguous(), k[:, :Tp].contiguous(), v[:, :Tp].contiguous(), gate[:, :Tp].contiguous())
        states.append(st)
        data.append(dict(q=q, k=k, v=v, gate=gate, Tp=Tp))
    return states, data


def step_inputs(data, t):
    cat = lambda key: torch.cat([d[key][:, d["Tp"] + t] for d in data]).contiguous()
    return cat("q"), cat("k"), cat("v"), cat("gate")


def run_both(base, batches, prompts, n_dec):
    import paper_2605_09877_amd as pkg
    from paper_2605_09877_amd import binding, synth as sy
    shared = {k: v for k, v in sy.make_params(base, DEV, plain=False).items() if k != "gate"}
    ref_states, data = build_states(pkg, sy, base, batches, prompts, n_dec, shared)
    new_states, _ = build_states(pkg, sy, base, batches, prompts, n_dec, shared)
    n = sum(batches)
    out_new = torch.empty((n, base.n_q_heads, base.head_dim), dtype=ref_states[0].dtype, device=DEV)
    folds0 = [st.folds for st in ref_states]
    for t in range(n_dec):
        q, k, v, g = step_inputs(data, t)
        out_ref = binding.decode_multi(ref_states, q, k, v, g)
        out_new.fill_(float("nan"))
        binding.decode_multi_static(new_states, q, k, v, g, out=out_new)
        assert torch.equal(out_ref, out_new), f"step {t}: outputs differ"
    torch.cuda.synchronize()
    assert any(st.folds > f0 for st, f0 in zip(ref_states, folds0)), "no fold happened during the steps"
    for a, b in zip(ref_states, new_states):
        assert (a.rows, a.tokens, a.folds) == (b.rows, b.tokens, b.folds)
        ea, eb = a.export(), b.export()
        for key in ("sK", "sV", "rho", "w", "n", "khat", "vhat", "win_k", "win_v", "win_g"):
            assert torch.equal(ea[key], eb[key]), key


def test_static_ragged_decode_two_calls_second_smaller():
    from paper_2605_09877_amd import synth as sy
    base = sy.shrink(sy.WORKLOADS["prefill_sqrt"], n_q_heads=4, n_kv_heads=2, chunk_len=128)
    # five sequences in three states at different positions and sizes; then, with the table still
    # holding that call's entries, two sequences in one state
    run_both(base, batches=(1, 3, 1), prompts=(128 * 9, 128 * 20 + 57, 300), n_dec=90)
    run_both(base, batches=(2,), prompts=(128 * 5 + 100,), n_dec=40)


def test_static_ragged_decode_f32_many_states():
    """More states than one descriptor launch carries (32): 40 single-sequence fp32 states."""
    from paper_2605_09877_amd import synth as sy
    base = sy.shrink(sy.WORKLOADS["tiny_f32"])
    run_both(base, batches=(1,) * 40, prompts=tuple(64 * 2 + 3 * i for i in range(40)), n_dec=70)


def test_static_ragged_decode_rejects_more_sequences_than_the_table_holds():
    import paper_2605_09877_amd as pkg
    from paper_2605_09877_amd import binding, synth as sy
    w = sy.shrink(sy.WORKLOADS["tiny_f32"], batch=binding.KVM_STATIC_MAX_SEQUENCES + 1, n_q_heads=1, n_kv_heads=1,
                  seq=64)
    st = pkg.state_for(w, device=DEV)
    x = torch.zeros((w.batch, 1, w.head_dim), dtype=torch.float32, device=DEV)
    with pytest.raises(binding.KVMError) as ei:
        binding.decode_multi_static([st], x, x.clone(), x.clone(), out=torch.empty_like(x))
    assert ei.value.status == binding.KVM_ERR_LIMIT and "4097" in str(ei.value)
    assert st.tokens == 0
