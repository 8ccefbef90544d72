"""Parity of kvm_prepare_qkv (through the C ABI) with the weight-preparation oracle, element by
element, on seeded inputs: every feature on, a continued call, ragged row counts, both dtypes.
Bars: fp32 outputs max-abs 1e-4 (rows are LayerNorm outputs, magnitude ~1..4); bf16 outputs
within one bf16 ulp of the oracle's rounded value (2^-7 relative, plus 1e-2 absolute near zero);
gate rtol 1e-4 (fp32 dot over d_model terms against fp64)."""
import numpy as np
import pytest
import torch

from oracle import prep_oracle as po

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def f64(t):
    return None if t is None else t.detach().to("cpu", torch.float64).numpy()


def run_case(io, B, T, Hq, Hkv, d, r, dm, pos0, seed, with_prev, features=True):
    from paper_2605_09877_amd import binding as kb
    dt = torch.bfloat16 if io == "bf16" else torch.float32
    gen = torch.Generator(device=DEV).manual_seed(seed)
    rnd = lambda *s: torch.randn(*s, generator=gen, device=DEV)
    uni = lambda *s: torch.rand(*s, generator=gen, device=DEV)
    q, k, v, vf = (rnd(B, T, Hq, d) * 1.5).to(dt), (rnd(B, T, Hkv, d) + 0.3).to(dt), rnd(B, T, Hkv, d).to(dt), \
        rnd(B, T, Hkv, d).to(dt)
    x = rnd(B, T, dm).to(dt) if dm else None
    P = dict(alpha_q=uni(Hq, d), alpha_k=uni(Hkv, d), alpha_v=uni(Hkv, d), lambda_v=uni(Hkv, d),
             lnq_gamma=0.5 + uni(Hq, d), lnq_beta=0.1 * rnd(Hq, d), lnk_gamma=0.5 + uni(Hkv, d),
             lnk_beta=0.1 * rnd(Hkv, d), w_gate=rnd(dm, Hkv) / dm ** 0.5 if dm else None) if features else \
        dict(w_gate=rnd(dm, Hkv) / dm ** 0.5 if dm else None)
    prev = dict(prev_q=rnd(B, Hq, d).to(dt), prev_k=rnd(B, Hkv, d).to(dt), prev_v=rnd(B, Hkv, d).to(dt)) \
        if with_prev else {}
    qo, ko_, vo, g = kb.prepare_qkv(q, k, v, rope_dims=r, pos0=pos0, v_first=vf if features else None, x=x,
                                    **prev, **P)
    torch.cuda.synchronize()
    pos = np.arange(pos0, pos0 + T)
    for b in range(B):
        rq, rk, rv, rg = po.prepare(
            f64(q[b]), f64(k[b]), f64(v[b]), pos, r, io, v_first=f64(vf[b]) if features else None,
            lam=f64(P.get("lambda_v")), alpha_q=f64(P.get("alpha_q")), alpha_k=f64(P.get("alpha_k")),
            alpha_v=f64(P.get("alpha_v")), lnq=(f64(P.get("lnq_gamma")), f64(P.get("lnq_beta"))),
            lnk=(f64(P.get("lnk_gamma")), f64(P.get("lnk_beta"))),
            prev_q=f64(prev["prev_q"][b]) if with_prev else None, prev_k=f64(prev["prev_k"][b]) if with_prev else None,
            prev_v=f64(prev["prev_v"][b]) if with_prev else None, x=f64(x[b]) if dm else None, w_g=f64(P["w_gate"]))
        for got, ref, name in ((qo[b], rq, "q"), (ko_[b], rk, "k"), (vo[b], rv, "v")):
            got = f64(got)
            if io == "f32":
                assert np.abs(got - ref).max() <= 1e-4, name
            else:
                assert np.all(np.abs(got - ref) <= 2.0 ** -7 * np.abs(ref) + 1e-2), name
                # and most elements are the very same bf16 value
                assert np.mean(got == ref) > 0.97, (name, np.mean(got == ref))
        if dm:
            np.testing.assert_allclose(f64(g[b]), rg, rtol=1e-4, atol=1e-5)
        else:
            assert g is None


def test_prep_bf16_all_features_long_positions():
    """d 128, r 64 (the 32k-context workload's heads), positions near 32k, gate from a 1024-wide x."""
    run_case("bf16", B=2, T=300, Hq=8, Hkv=2, d=128, r=64, dm=1024, pos0=32000, seed=1, with_prev=True)


def test_prep_bf16_plain_start_of_sequence():
    """No shift, residual or LN parameters; first token unshifted; r 32; rows that do not fill the last wave."""
    run_case("bf16", B=1, T=37, Hq=3, Hkv=3, d=128, r=32, dm=0, pos0=0, seed=2, with_prev=False, features=False)


def test_prep_f32_d64():
    run_case("f32", B=2, T=65, Hq=4, Hkv=2, d=64, r=16, dm=96, pos0=5000, seed=3, with_prev=True)


def test_prep_heads_not_a_multiple_of_eight_and_no_rotation():
    run_case("bf16", B=1, T=50, Hq=5, Hkv=5, d=64, r=0, dm=264, pos0=7, seed=4, with_prev=False)


def test_prep_rejects_bad_arguments():
    from paper_2605_09877_amd import binding as kb
    q = torch.zeros(1, 4, 2, 128, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(kb.KVMError):
        kb.prepare_qkv(q, q.clone(), q.clone(), rope_dims=48)          # half = 24 channels: 3 lanes
    with pytest.raises(kb.KVMError):
        kb.prepare_qkv(q, q.clone(), q.clone(), rope_dims=32, x=torch.zeros(1, 4, 64, dtype=torch.bfloat16, device=DEV))
