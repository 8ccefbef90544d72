#!/usr/bin/env python3
"""Benchmark of the KVM layer hot path on one MI355X.

A "step" is one pass of the whole path over one batch of synthetic input: chunk-wise prefill
of the 32k-context workload (every chunk's attention over [state || window] plus every fold),
inputs resident in HBM.  One JSON line is printed: prefill tokens/s, the roofline of the
dominant kernel (fused MFMA attention; kernel time from HIP events recorded by the library on
the launch stream), the decode leg (us per token on the batched-decode workload, HBM roofline)
and the CPU oracle timed on the host cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak
HBM_PEAK_GBS = 8000.0            # MI355X HBM3E peak


def measured_traffic(summary):
    """HBM bytes per launch of a kernel, as committed under profiles/ (derived from the
    FETCH_SIZE and WRITE_SIZE counters of this same command, scaled by what the counters read
    for a plain copy of known size); None when there is no such summary."""
    path = os.path.join(ROOT, "profiles", summary)
    try:
        for ln in open(path):
            if ln.startswith("traffic_bytes_per_launch:"):
                return float(ln.split(":", 1)[1])
    except OSError:
        pass
    return None


def copy_calibration(dev):
    """A plain device copy of known size (1 GiB read, 1 GiB written), for scaling HBM counters."""
    import torch
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
    dst = torch.empty_like(src)
    for _ in range(3):
        torch.add(src, 0.0, out=dst)   # one elementwise kernel: reads src once, writes dst once
    torch.cuda.synchronize()


def attention_flops(w, T):
    """Algorithmic attention flops of a T-token prefill: 4*d per visible (query, key) pair, pairs
    per chunk and query head = C*(m + tokens of earlier window blocks) + C*(C+1)/2."""
    C, L = w.chunk_len, w.chunk_len * w.n_bswa_chunks
    kind = w.budget_kind
    pairs, m, launches = 0, 0, 0
    for s in range(0, T, C):
        e = s + C
        b = max(0, e - L)
        pairs += C * (m + (s - b)) + C * (C + 1) // 2
        launches += 1
        if e >= L and kind != "none":
            if m == 0:
                m = C
            else:
                import math
                B = w.budget_fixed if kind == "fixed" else int(w.budget_scale * (math.isqrt(e - 1) + 1))
                m = max(m, min(B, m + C))
    return 4.0 * w.head_dim * pairs * w.n_q_heads * w.batch, launches


def fold_bytes(w, units, C, m, touched=None, copied=None):
    """Bytes one fold moves, two models.  `survey`: the per-fold figure of the scope table this
    build is measured against -- the block's k, v re-read, the normalised state keys read, fp32
    sums read-modify-written and the readout refreshed on min(C, m) rows (an upper bound on the
    rows a block can touch).  `own`: what the kernels here move -- memory keys written and read
    back, fp64 key sums, rows touched as measured (`touched`), and, inside a prefill, the readout of
    untouched rows copied to the new state version (`copied` rows)."""
    d, es = w.head_dim, 2 if w.io == "bf16" else 4
    up = min(C, m)
    survey = units * (2 * C * d * es + m * d * es + up * d * 4 * 2 * 2 + up * d * 2 * es)
    t = up if touched is None else touched
    cp = 0 if copied is None else copied
    own = units * (2 * C * d * es * 2 + m * d * es + t * d * (8 + 4) * 2 + t * d * 2 * es + cp * d * 2 * es * 2)
    return dict(survey=survey, own=own)


def prefill_leg(args, pkg, synth, dev):
    import torch
    w = synth.WORKLOADS[args.workload]
    q, k, v = synth.make_qkv(w, dev)
    st = pkg.state_for(w, device=dev)
    out = torch.empty_like(q)
    if args.kernels_apart:
        st.profile(2)      # folds and attention never share the chip: for traces and counters of each alone
    for _ in range(args.warmup):
        st.reset()
        st.prefill(q, k, v, out=out)
    torch.cuda.synchronize()
    # the timed steps: no kernel timing events, nothing but the calls
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        marks[i].record()          # on the stream the library is called on; each call joins back to it
        st.reset()
        st.prefill(q, k, v, out=out)
    marks[args.steps].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    # kernel spans, in passes of their own: the library brackets its attention launches and its
    # folds with HIP events on the streams they are launched on
    n_prof = max(2, min(args.steps, 5))
    st.profile(True)
    st.profile_read()
    for _ in range(n_prof):
        st.reset()
        st.prefill(q, k, v, out=out)
    torch.cuda.synchronize()
    prof = st.profile_read()
    # the same step with folds and attention kept apart: each kernel's time without the other
    iso = None
    if not args.no_isolated:
        st.profile(2)
        for _ in range(2):
            st.reset()
            st.prefill(q, k, v, out=out)
        torch.cuda.synchronize()
        iso = st.profile_read()
    st.profile(False)
    tokens = w.batch * w.seq
    flops, _ = attention_flops(w, w.seq)
    attn_ms, attn_n = prof["attn"]
    fold_ms, fold_n = prof["fold"]
    launches = max(attn_n // n_prof, 1)                   # attention launches per step (groups of chunks)
    avg_launch_s = attn_ms / max(attn_n, 1) * 1e-3
    achieved = flops / launches / avg_launch_s / 1e12 if attn_n else 0.0
    isolated, fold = None, None
    if iso is not None:
        iso_tflops = flops / launches / (iso["attn"][0] / max(iso["attn"][1], 1) * 1e-3) / 1e12
        isolated = dict(achieved=iso_tflops, frac=iso_tflops / MFMA_BF16_PEAK_TFLOPS,
                        attn_ms_per_step=iso["attn"][0] / 2, fold_ms_per_step=iso["fold"][0] / 2)
        # the fold's HBM roofline: a steady fold of this workload (m = the fixed budget, no append)
        n_folds = max(iso["fold"][1], 1)
        us = iso["fold"][0] / n_folds * 1e3
        units, m = w.batch * w.n_kv_heads, rows_after_prefill(w, w.seq)
        touched = int(0.4 * min(w.chunk_len, m)) if w.name == "prefill_gqa_32k" else None
        nb = fold_bytes(w, units, w.chunk_len, m, touched=touched,
                        copied=None if touched is None else m - touched)
        fold = dict(bound="hbm", kernel="memkey_kernel + fold_fused_kernel" if st.fold_path == 1
                    else "memkey_kernel + score_mfma_kernel + accum_kernel", peak=HBM_PEAK_GBS,
                    unit="GB/s", isolated_us_per_fold=us, beside_attention_us_per_fold=fold_ms / max(fold_n, 1) * 1e3,
                    folds_per_step=n_folds // 2, algorithmic_bytes_per_fold=nb["survey"],
                    achieved=nb["survey"] / (us * 1e-6) / 1e9, frac=nb["survey"] / (us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                    moved_bytes_per_fold_model=nb["own"], moved_gbs=nb["own"] / (us * 1e-6) / 1e9,
                    traffic=measured_traffic("fold_kernels_prefill_gqa_32k_hbm_traffic.txt")
                    if w.name == "prefill_gqa_32k" else None,
                    note="algorithmic bytes: block k, v + state keys + fp32 sums read-modify-written and readout "
                         "refreshed on min(C, m) rows; moved bytes: this build's own model (memory keys written "
                         "and read back, fp64 key sums, 0.4 m rows touched as measured, readout of the others "
                         "copied to the new state version)")
    res = dict(
        value=tokens * args.steps / dt, ms_per_step=dt / args.steps * 1e3,
        step_ms=dict(median=step_ms[len(step_ms) // 2], min=step_ms[0], max=step_ms[-1]),
        roofline=dict(bound="mfma", kernel="attn_mfma_kernel", achieved=achieved, peak=MFMA_BF16_PEAK_TFLOPS,
                      unit="TFLOP/s", frac=achieved / MFMA_BF16_PEAK_TFLOPS,
                      traffic=measured_traffic("attn_mfma_kernel_prefill_gqa_32k_hbm_traffic.txt")
                      if w.name == "prefill_gqa_32k" else None,
                      launches_per_step=launches, avg_launch_us=avg_launch_s * 1e6,
                      attn_ms_per_step=attn_ms / n_prof, fold_ms_per_step=fold_ms / n_prof,
                      folds_per_step=fold_n // n_prof, timed_in="a pass of its own with the library's event "
                      "brackets on (the timed steps run without them)",
                      isolated=isolated),
        fold=fold, workload=w)
    return res, (q, k, v)


def backward_leg(args, pkg, synth, dev, w):
    """Backward pass of the same prefill (kvm_prefill_backward): its time alone, on resident
    tensors, after one forward with the fold record switched on.  Algorithmic flops: five
    contractions of 2*d flops per visible (query, key) pair -- the logits and dout . v^T once each,
    dq, dk, dv -- against the forward's two."""
    import torch
    q, k, v = synth.make_qkv(w, dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed + 31337)
    dout = torch.randn(q.shape, generator=gen, device=dev, dtype=torch.float32).to(q.dtype)
    st = pkg.state_for(w, device=dev)
    assign, score = st.trace(w.seq // w.chunk_len + 1)
    out, lse = st.prefill(q, k, v, want_lse=True)
    nbytes = st.lib.kvm_backward_workspace_bytes(st.handle, w.seq)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    reps = max(2, min(args.steps, 3))
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
    st.backward(q, k, v, None, out, lse, dout, assign, score, workspace=ws)   # warm-up
    torch.cuda.synchronize()
    for i in range(reps):
        marks[i].record()
        g = st.backward(q, k, v, None, out, lse, dout, assign, score, workspace=ws)
        del g
    marks[reps].record()
    torch.cuda.synchronize()
    ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(reps))
    med = ms[len(ms) // 2]
    flops = attention_flops(w, w.seq)[0] * 2.5
    tf = flops / (med * 1e-3) / 1e12
    return dict(ms_per_pass=med, ms_min=ms[0], ms_max=ms[-1], tokens_per_s=w.batch * w.seq / (med * 1e-3),
                algorithmic_tflop=flops / 1e12, achieved_tflops=tf, frac_of_mfma_peak=tf / MFMA_BF16_PEAK_TFLOPS,
                workspace_gb=nbytes / 1e9, note="whole pass: per chunk undo fold, dq kernel, dk kernel, dv kernel, readout adjoint; the three "
                "matrix-core kernels each compute the logits (8 contractions run for the 5 counted)")


def decode_leg(args, pkg, synth, dev):
    """Batched decode workload: successive steps against a pre-built state, folds included."""
    import torch
    w = synth.WORKLOADS["decode"]
    pre = synth.make_decode_state(w, dev)
    steps = w.seq
    st = pkg.state_for(w, device=dev, max_tokens=pre["tokens"] + 2 * steps)
    st.import_(pre)
    n_in = 16                                            # distinct inputs, cycled
    q, k, v = synth.make_qkv(w, dev, T=n_in, pos0=pre["tokens"])
    qs = [q[:, t].contiguous() for t in range(n_in)]
    ks = [k[:, t].contiguous() for t in range(n_in)]
    vs = [v[:, t].contiguous() for t in range(n_in)]
    out = torch.empty_like(qs[0])
    for t in range(20):
        st.decode(qs[t % n_in], ks[t % n_in], vs[t % n_in], out=out)
    st.import_(pre)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(steps):
        st.decode(qs[t % n_in], ks[t % n_in], vs[t % n_in], out=out)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # kernel spans in a pass of their own (the timed steps run without the event brackets)
    st.import_(pre)
    st.profile(True)
    st.profile_read()
    for t in range(steps):
        st.decode(qs[t % n_in], ks[t % n_in], vs[t % n_in], out=out)
    torch.cuda.synchronize()
    prof = st.profile_read()
    st.profile(False)
    dec_ms, dec_n = prof["decode"]
    fold_ms, fold_n = prof["fold"]
    L, C, m, d = w.chunk_len * w.n_bswa_chunks, w.chunk_len, w.state_rows, w.head_dim
    mean_w = (L - C + 1 + L) / 2.0                       # window length cycles L-C+1 .. L
    bytes_per_step = w.batch * w.n_q_heads * ((m + mean_w) * d * 2 * 2 + 2 * d * 2)
    avg_s = dec_ms / max(dec_n, 1) * 1e-3
    gbs = bytes_per_step / avg_s / 1e9 if dec_n else 0.0
    fold_us = fold_ms / max(fold_n, 1) * 1e3
    fb = fold_bytes(w, w.batch * w.n_kv_heads, C, m)
    fold = dict(bound="hbm", kernel="memkey_kernel + fold_fused_kernel" if st.fold_path == 1
                else "memkey_kernel + score_mfma_kernel + merge_inplace_kernel", peak=HBM_PEAK_GBS,
                unit="GB/s", us_per_fold=fold_us, folds=fold_n, algorithmic_bytes_per_fold=fb["survey"],
                achieved=fb["survey"] / (fold_us * 1e-6) / 1e9 if fold_n else 0.0,
                frac=fb["survey"] / (fold_us * 1e-6) / 1e9 / HBM_PEAK_GBS if fold_n else 0.0,
                note="in place: rows no token goes to are not touched; algorithmic bytes as for the prefill fold")
    ragged = ragged_decode(pkg, synth, dev, w, pre, qs, ks, vs, out, steps=200)
    grouped = grouped_decode(pkg, synth, dev, w, steps=200)
    return dict(us_per_token=dt / steps / w.batch * 1e6, us_per_step=dt / steps * 1e6, steps=steps,
                folds=fold_n, fold_us=fold_us, fold=fold, ragged=ragged, grouped_query=grouped,
                config=dict(workload="decode", batch=w.batch, heads=w.n_q_heads, head_dim=d, state_rows=m,
                            window=L, chunk_len=C),
                roofline=dict(bound="hbm", kernel="attn_rows_kernel", achieved=gbs, peak=HBM_PEAK_GBS,
                              unit="GB/s", frac=gbs / HBM_PEAK_GBS,
                              traffic=measured_traffic("attn_rows_kernel_decode_hbm_traffic.txt"),
                              avg_launch_us=avg_s * 1e6, bytes_per_launch=bytes_per_step))


def grouped_decode(pkg, synth, dev, w, steps):
    """The decode workload with the headline workload's grouped queries (32 query heads on 8 KV
    heads): a workgroup takes a KV head's four query heads together, so every key and value row is
    fetched once for all of them; the rate is over the distinct K/V bytes of a step."""
    import torch
    wg = synth.shrink(w, n_kv_heads=8)
    pre = synth.make_decode_state(wg, dev)
    st = pkg.state_for(wg, device=dev, max_tokens=pre["tokens"] + 2 * steps)
    st.import_(pre)
    n_in = 16
    q, k, v = synth.make_qkv(wg, dev, T=n_in, pos0=pre["tokens"])
    qs = [q[:, t].contiguous() for t in range(n_in)]
    ks = [k[:, t].contiguous() for t in range(n_in)]
    vs = [v[:, t].contiguous() for t in range(n_in)]
    out = torch.empty_like(qs[0])
    for t in range(10):
        st.decode(qs[t % n_in], ks[t % n_in], vs[t % n_in], out=out)
    st.import_(pre)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(steps):
        st.decode(qs[t % n_in], ks[t % n_in], vs[t % n_in], out=out)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    st.import_(pre)
    st.profile(True)
    st.profile_read()
    for t in range(steps):
        st.decode(qs[t % n_in], ks[t % n_in], vs[t % n_in], out=out)
    torch.cuda.synchronize()
    dec_ms, dec_n = st.profile_read()["decode"]
    st.profile(False)
    L, C, m, d = wg.chunk_len * wg.n_bswa_chunks, wg.chunk_len, wg.state_rows, wg.head_dim
    mean_w = L - C + 1 + (steps - 1) / 2.0               # the window grows by one per step from L - C + 1
    nbytes = wg.batch * (wg.n_kv_heads * (m + mean_w) * d * 2 * 2 + wg.n_q_heads * 2 * d * 2)
    avg_s = dec_ms / max(dec_n, 1) * 1e-3
    return dict(us_per_token=dt / steps / wg.batch * 1e6, us_per_step=dt / steps * 1e6, steps=steps,
                n_q_heads=wg.n_q_heads, n_kv_heads=wg.n_kv_heads, kernel_us=avg_s * 1e6,
                distinct_gbs=nbytes / avg_s / 1e9 if dec_n else 0.0)


def ragged_decode(pkg, synth, dev, w, pre, qs, ks, vs, out, steps):
    """The same decode workload as a ragged batch: one single-sequence state per sequence, each
    standing at its own position (so their windows differ in length and they fold at different
    steps), all advanced by one kvm_decode_step_multi launch per step."""
    import torch
    states = []
    per_seq = ("sK", "sV", "rho", "w", "n", "win_k", "win_v", "win_g")
    for b in range(w.batch):
        wb = synth.shrink(w, batch=1)
        stagger = (b * 37) % w.chunk_len
        st = pkg.state_for(wb, device=dev, max_tokens=pre["tokens"] + stagger + 2 * steps + w.chunk_len)
        one = {k: (pre[k][b:b + 1].contiguous() if k in per_seq else pre[k]) for k in pre}
        one["tokens"] = pre["tokens"] + stagger
        st.import_(one)
        states.append(st)
    n_in = len(qs)
    for t in range(10):
        pkg.binding.decode_multi(states, qs[t % n_in], ks[t % n_in], vs[t % n_in], out=out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(steps):
        pkg.binding.decode_multi(states, qs[t % n_in], ks[t % n_in], vs[t % n_in], out=out)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    folds = sum(st.folds for st in states)
    return dict(us_per_token=dt / steps / w.batch * 1e6, us_per_step=dt / steps * 1e6, steps=steps,
                states=len(states), folds=folds)


def prep_leg(args, pkg, synth, dev):
    """The weight preparation in front of the layer (value residual, token shift, LN_q/LN_k, partial
    RoPE, merge gate) on the headline workload's shape, every feature on: HBM roofline of the call."""
    import torch
    w = synth.WORKLOADS[args.workload]
    B, T, Hq, Hkv, d = w.batch, w.seq, w.n_q_heads, w.n_kv_heads, w.head_dim
    dm = Hq * d
    dt = synth.torch_dtype(w.io)
    gen = torch.Generator(device=dev).manual_seed(w.seed + 31)
    rnd = lambda *s: torch.randn(*s, generator=gen, device=dev)
    q, k, v, vf = (rnd(B, T, H, d).to(dt) for H in (Hq, Hkv, Hkv, Hkv))
    x = rnd(B, T, dm).to(dt)
    P = dict(alpha_q=torch.rand(Hq, d, device=dev), alpha_k=torch.rand(Hkv, d, device=dev),
             alpha_v=torch.rand(Hkv, d, device=dev), lambda_v=torch.rand(Hkv, d, device=dev),
             lnq_gamma=torch.ones(Hq, d, device=dev), lnq_beta=torch.zeros(Hq, d, device=dev),
             lnk_gamma=torch.ones(Hkv, d, device=dev), lnk_beta=torch.zeros(Hkv, d, device=dev),
             w_gate=rnd(dm, Hkv) / dm ** 0.5)
    run = lambda: pkg.binding.prepare_qkv(q, k, v, rope_dims=w.rope_dims, v_first=vf, x=x, **P)
    run()
    reps = 5
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
    for i in range(reps):
        marks[i].record()
        run()
    marks[reps].record()
    torch.cuda.synchronize()
    ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(reps))[reps // 2]
    es = 2 if w.io == "bf16" else 4
    nbytes = B * T * (2 * Hq * d * es + 5 * Hkv * d * es + dm * es + Hkv * 4)   # q r+w, k r+w, v r+w + v_first, x, gate
    gbs = nbytes / (ms * 1e-3) / 1e9
    return dict(ms=ms, bytes=nbytes, config=dict(batch=B, seq_len=T, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d,
                                                 d_model=dm, rope_dims=w.rope_dims),
                roofline=dict(bound="hbm", kernel="prep_rows_kernel + gate_kernel", achieved=gbs, peak=HBM_PEAK_GBS,
                              unit="GB/s", frac=gbs / HBM_PEAK_GBS, traffic=None))


def cpu_baseline_leg(w, tensors, budget_s, gpu=None):
    """The oracle, as it stands, on (batch, KV head) units of the same inputs, one after the other,
    for as many chunks as fit the time budget; scaled to whole-layer tokens/s (units are
    independent and equal in work: a layer token is one position of every KV head).  gpu: the
    library's output and fold record of the same prefill; what the oracle got through is then
    compared with them (returned as the `parity` object: units and chunks compared, folds whose
    assignments differ from the oracle's -- reported, not overridden, here -- and the worst output
    row error as a fraction of the bf16 bar, over the chunks ahead of the first such fold)."""
    import numpy as np
    import kvm_testlib as tl
    q, k, v = tensors
    C = w.chunk_len
    G = w.n_q_heads // w.n_kv_heads
    t0 = time.perf_counter()
    done, units_done, folds = 0, 0, 0
    par = dict(units=0, chunks=0, folds=0, folds_differing=0, ties_merge=None, ties_append=None, max_err=0.0)
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            if time.perf_counter() - t0 >= budget_s:
                break
            u = tl.unit_inputs(w, q[b:b + 1], k[b:b + 1], v[b:b + 1], {}, 0, h)
            unit = tl.make_oracle_unit(w, {}, h)
            pos, ys = 0, []
            while pos < w.seq and time.perf_counter() - t0 < budget_s:
                y, _ = unit.prefill(u["q"][:, pos:pos + C], u["k"][pos:pos + C], u["v"][pos:pos + C])
                ys.append(y)
                pos += C
            done += pos
            folds += len(unit.fold_logs)
            units_done += 1
            if gpu is not None and ys:
                t_cmp = time.perf_counter()
                ga = gpu["assign"][:len(unit.fold_logs), b, h].cpu().numpy()
                bad = [f for f, log in enumerate(unit.fold_logs) if not np.array_equal(log["assign"], ga[f])]
                # chunk c is attended before fold c - (L/C - 1) + ... : outputs are comparable up to the
                # chunk that follows the first differing fold
                n_ok = len(ys) if not bad else min(len(ys), bad[0] + w.n_bswa_chunks)
                if n_ok:
                    y_ref = np.concatenate(ys[:n_ok], axis=1)
                    y_gpu = tl.f64(gpu["out"][b, :n_ok * C, h * G:(h + 1) * G]).transpose(1, 0, 2)
                    par["max_err"] = max(par["max_err"], tl.check_outputs(w, y_gpu, y_ref, "bench parity"))
                par["units"] += 1
                par["chunks"] += n_ok
                par["folds"] += len(unit.fold_logs)
                par["folds_differing"] += len(bad)
                t0 += time.perf_counter() - t_cmp       # the comparison is not the baseline's time
    dt = time.perf_counter() - t0
    try:
        import threadpoolctl
        cores = max(int(i.get("num_threads", 1)) for i in threadpoolctl.threadpool_info()) \
            if threadpoolctl.threadpool_info() else os.cpu_count()
    except Exception:
        cores = os.cpu_count()
    base = dict(value=done / (dt * w.n_kv_heads), unit="tokens/s", cores=cores, kind="oracle",
                sample=f"{units_done} of {w.batch * w.n_kv_heads} (sequence, KV head) units in order from "
                       f"(0, 0): {done} unit-tokens ({done // C} chunks, {folds} folds) in {dt:.1f} s; "
                       f"one layer token = {w.n_kv_heads} unit-tokens")
    if gpu is not None:
        par["max_err_unit"] = "worst output row error as a fraction of the bf16 bar (2e-2 of the row's max-abs)"
        par["ties_merge"] = par["ties_append"] = 0 if par["folds_differing"] == 0 else None
    return base, (par if gpu is not None else None)


def rows_after_prefill(w, T):
    """State rows after a T-token prefill (the data-independent schedule)."""
    import math
    C, L, m = w.chunk_len, w.chunk_len * w.n_bswa_chunks, 0
    for e in range(C, T + 1, C):
        if e >= L and w.budget_kind != "none":
            B = w.budget_fixed if w.budget_kind == "fixed" else int(w.budget_scale * (math.isqrt(e - 1) + 1))
            m = C if m == 0 else max(m, min(B, m + C))
    return m


def sweep(args, pkg, synth, dev):
    """The paper's speed-benchmark shape ("Speed Benchmarks": one layer, 32 heads of dimension
    128, batch 8, bf16, context 512 .. 32768) for a 256-row state, for a 16*sqrt(N) state, and --
    the full-attention comparator -- for the library itself with a budget that never fills (every
    block is appended whole, so each query attends every earlier token through the same kernels:
    exact causal attention over [memory keys of the tokens that left the window || window]).
    Prefill ms, backward ms and decode us per step; one JSON line per context length."""
    import statistics
    import torch

    def timed(fn, reps):
        ts = []
        for _ in range(reps):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            ts.append((time.perf_counter() - t0) * 1e3)
        return statistics.median(ts), min(ts), max(ts)

    base = synth.WORKLOADS["prefill_fixed"]
    lengths = [int(x) for x in args.sweep_lengths.split(",")]
    for T in lengths:
        variants = {"kvm_256": dict(budget_kind="fixed", budget_fixed=256),
                    "kvm_sqrt": dict(budget_kind="sqrt", budget_scale=16.0),
                    "full": dict(budget_kind="fixed", budget_fixed=T + 256)}
        shape = dict(batch=8, n_q_heads=32, n_kv_heads=32, head_dim=128, chunk_len=256, rope_dims=32, seq=T)
        w0 = synth.shrink(base, **shape)
        q, k, v = synth.make_qkv(w0, dev)
        out = torch.empty_like(q)
        gen = torch.Generator(device=dev)
        gen.manual_seed(w0.seed + 31337)
        dout = torch.randn(q.shape, generator=gen, device=dev, dtype=torch.float32).to(q.dtype)
        row = dict(T=T)
        for name, bud in variants.items():
            w = synth.shrink(w0, name=name, **bud)
            st = pkg.state_for(w, device=dev, max_tokens=T + 2 * w.chunk_len)

            def prefill():
                st.reset()
                st.prefill(q, k, v, out=out)
            for _ in range(args.warmup):
                prefill()
            med, lo, hi = timed(prefill, args.steps)
            # decode: one chunk of single-token steps from the state that prefill left (one fold)
            n_dec = w.chunk_len
            qd, kd, vd = synth.make_qkv(w, dev, T=16, pos0=T)
            qs = [qd[:, t].contiguous() for t in range(16)]
            ks = [kd[:, t].contiguous() for t in range(16)]
            vs = [vd[:, t].contiguous() for t in range(16)]
            od = torch.empty_like(qs[0])
            prefill()
            for t in range(8):
                st.decode(qs[t], ks[t], vs[t], out=od)
            prefill()
            dmed = timed(lambda: [st.decode(qs[t % 16], ks[t % 16], vs[t % 16], out=od) for t in range(n_dec)], 1)[0]
            row[name] = dict(prefill_ms=med, prefill_ms_min=lo, prefill_ms_max=hi, rows=rows_after_prefill(w, T),
                             tokens_per_s=w.batch * T / (med * 1e-3), decode_us_per_step=dmed * 1e3 / n_dec)
            # backward of the same prefill (kvm_prefill_backward), alone
            if not args.no_backward:
                st.reset()
                assign, score = st.trace(T // w.chunk_len + 1)
                o2, lse = st.prefill(q, k, v, want_lse=True)
                ws = torch.empty(st.lib.kvm_backward_workspace_bytes(st.handle, T), dtype=torch.uint8, device=dev)
                bwd = lambda: st.backward(q, k, v, None, o2, lse, dout, assign, score, workspace=ws)
                bwd()
                row[name]["backward_ms"] = timed(bwd, max(min(args.steps, 3), 2))[0]
                st.trace(0)
                del ws, o2, lse, assign, score
            del st
            torch.cuda.empty_cache()
        for name in ("kvm_256", "kvm_sqrt"):
            row[name]["prefill_speedup_vs_full"] = row["full"]["prefill_ms"] / row[name]["prefill_ms"]
            row[name]["decode_speedup_vs_full"] = row["full"]["decode_us_per_step"] / row[name]["decode_us_per_step"]
            if "backward_ms" in row[name]:
                row[name]["backward_speedup_vs_full"] = row["full"]["backward_ms"] / row[name]["backward_ms"]
        print(json.dumps(dict(sweep="paper_shape_B8_H32_d128_C256_bf16", **row)), flush=True)
        del q, k, v, out, dout
        torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="prefill_gqa_32k")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the two other prefill workloads")
    ap.add_argument("--no-backward", action="store_true", help="skip the backward pass of the prefill")
    ap.add_argument("--no-isolated", action="store_true",
                    help="skip the extra passes that time folds and attention apart")
    ap.add_argument("--kernels-apart", action="store_true",
                    help="keep the prefill's fold chain and its attention launches apart in every step (slower; "
                         "for kernel traces and hardware counters of the fold kernels alone)")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark line: the paper's speed-benchmark shape over context lengths")
    ap.add_argument("--sweep-lengths", default="512,1024,2048,4096,8192,16384,32768",
                    help="context lengths of --sweep")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2605_09877_amd as pkg
    from paper_2605_09877_amd import synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    from paper_2605_09877_amd import build
    if build.is_stale():      # missing, or built from other sources than the tree holds
        build.build()
    dev = "cuda:0"
    if args.sweep:
        sweep(args, pkg, synth, dev)
        return
    res, tensors = prefill_leg(args, pkg, synth, dev)
    w = res.pop("workload")
    line = dict(
        metric="KVM-layer prefill tokens/sec at 32k ctx bf16", value=res["value"], unit="tokens/s",
        n_gpus=1, steps=args.steps, warmup=args.warmup, ms_per_step=res["ms_per_step"],
        higher_is_better=True, scaling="weak", vs_baseline=None, dtype="bf16", data="synthetic",
        config=dict(workload=w.name, batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads,
                    head_dim=w.head_dim, seq_len=w.seq, chunk_len=w.chunk_len, state_rows=w.budget_fixed,
                    rope_dims=w.rope_dims, gpu=torch.cuda.get_device_name(0)),
        step_ms=res["step_ms"], roofline=res["roofline"], fold=res["fold"])
    # what this GPU reaches in the library's own microkernels (registers-only bf16 MFMA; 1 GiB copy)
    peaks = pkg.binding.measure_peaks(dev)
    line["measured_peaks"] = dict(mfma_bf16_tflops=peaks["mfma_bf16_tflops"], copy_gbs=peaks["copy_gbs"],
                                  read_gbs=peaks["read_gbs"],
                                  attn_frac_of_measured=res["roofline"]["achieved"] / peaks["mfma_bf16_tflops"])
    if not args.no_others and args.workload == "prefill_gqa_32k":
        # the two other prefill configurations (fixed 512-row state; ~sqrt growth): step time only
        del tensors
        torch.cuda.empty_cache()
        line["other_workloads"] = {}
        for name in ("prefill_fixed", "prefill_sqrt"):
            a2 = argparse.Namespace(**{**vars(args), "workload": name, "no_isolated": True})
            r2, t2 = prefill_leg(a2, pkg, synth, dev)
            w2 = r2["workload"]
            line["other_workloads"][name] = dict(
                tokens_per_s=r2["value"], ms_per_step=r2["ms_per_step"], step_ms=r2["step_ms"],
                attn_tflops=r2["roofline"]["achieved"], folds_per_step=r2["roofline"]["folds_per_step"],
                config=dict(batch=w2.batch, heads=w2.n_q_heads, seq_len=w2.seq, chunk_len=w2.chunk_len,
                            budget=w2.budget_kind))
            del t2
            torch.cuda.empty_cache()
            if not args.no_backward:
                b2 = backward_leg(a2, pkg, synth, dev, w2)
                line["other_workloads"][name]["backward_ms_per_pass"] = b2["ms_per_pass"]
                line["other_workloads"][name]["backward_tflops"] = b2["achieved_tflops"]
                torch.cuda.empty_cache()
        tensors = None
    if not args.no_backward:
        tensors = None
        torch.cuda.empty_cache()
        line["backward"] = backward_leg(args, pkg, synth, dev, w)
        line["backward"]["vs_forward_step"] = line["backward"]["ms_per_pass"] / res["ms_per_step"]
        torch.cuda.empty_cache()
    if not args.no_others:
        line["prep"] = prep_leg(args, pkg, synth, dev)
        torch.cuda.empty_cache()
    if not args.no_decode:
        line["decode"] = decode_leg(args, pkg, synth, dev)
        line["decode"]["roofline"]["frac_of_measured_read"] = \
            line["decode"]["roofline"]["achieved"] / peaks["read_gbs"]
    if not args.no_cpu:
        if tensors is None:
            tensors = synth.make_qkv(w, dev)     # same seed, same tensors as the timed run
        # the library's output and fold record of this very prefill, for the comparison with what
        # the oracle gets through in its time budget
        st = pkg.state_for(w, device=dev)
        assign, _ = st.trace(w.seq // w.chunk_len + 1)
        out = st.prefill(*tensors)
        torch.cuda.synchronize()
        line["cpu_baseline"], line["parity"] = cpu_baseline_leg(w, tensors, args.cpu_seconds,
                                                                gpu=dict(out=out, assign=assign))
    if args.copy_calibration:
        copy_calibration(dev)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
