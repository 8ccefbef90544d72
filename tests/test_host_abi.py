"""CPU-side checks of the C ABI: the library loads, exports every symbol the header declares,
and its host logic (growth schedule, sizing, argument and capacity errors) behaves -- without
launching anything on a GPU.  Error paths return before any kernel or HIP call is made, so a
placeholder device pointer is enough here."""
import ctypes as C
import os
import re

import pytest

from oracle import kvm_oracle as ko
from paper_2605_09877_amd import binding as kb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_DEV_PTR = 0x10000000  # 256-byte aligned, never dereferenced by the calls below


def cfg(**kw):
    base = dict(batch=2, n_q_heads=4, n_kv_heads=2, head_dim=128, rope_dims=32, chunk_len=256,
                n_bswa_chunks=2, n_sink=1, io_dtype=kb.KVM_BF16, budget_kind=kb.KVM_BUDGET_FIXED,
                budget_fixed=512, budget_scale=0.0, budget_table=None, budget_table_len=0,
                ln_eps=1e-5, norm_eps=1e-12, ln_gamma=None, ln_beta=None, tau_state=None, tau_bswa=None)
    base.update(kw)
    return kb.kvm_config(**base)


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "kvm.h")).read()
    declared = set(re.findall(r"\b(kvm_[a-z0-9_]+)\s*\(", header))
    declared -= {"kvm_status"}
    assert declared == set(kb.EXPORTS), declared ^ set(kb.EXPORTS)
    lib = kb.load_library()
    for name in declared:
        assert getattr(lib, name) is not None
    assert lib.kvm_strerror(kb.KVM_ERR_CAPACITY).decode().startswith("state buffer too small")
    assert lib.kvm_strerror(0).decode() == "ok"


@pytest.mark.parametrize("kind,kw,okw", [
    (kb.KVM_BUDGET_FIXED, dict(budget_fixed=512), dict(budget_kind=ko.BUDGET_FIXED, budget_fixed=512)),
    (kb.KVM_BUDGET_FIXED, dict(budget_fixed=10), dict(budget_kind=ko.BUDGET_FIXED, budget_fixed=10)),
    (kb.KVM_BUDGET_SQRT, dict(budget_scale=4.0), dict(budget_kind=ko.BUDGET_SQRT, budget_scale=4.0)),
    (kb.KVM_BUDGET_SQRT, dict(budget_scale=16.0), dict(budget_kind=ko.BUDGET_SQRT, budget_scale=16.0)),
    (kb.KVM_BUDGET_SQRT, dict(budget_scale=2.5), dict(budget_kind=ko.BUDGET_SQRT, budget_scale=2.5)),
    (kb.KVM_BUDGET_NONE, {}, dict(budget_kind=ko.BUDGET_NONE)),
])
def test_growth_schedule_matches_oracle_and_closed_forms(kind, kw, okw):
    lib = kb.load_library()
    c = cfg(budget_kind=kind, **kw)
    oc = ko.KVMConfig(head_dim=128, rope_dims=32, chunk_len=256, **okw)
    for T in (0, 255, 256, 511, 512, 768, 4096, 4352, 16384, 65536, 65537):
        rows = ko.expected_rows(oc, T)
        assert lib.kvm_state_rows_for(C.byref(c), T) == (rows[-1] if rows else 0), T
    if kind == kb.KVM_BUDGET_SQRT and kw["budget_scale"] == 4.0:
        # worked by hand: 4*ceil(sqrt(e)) <= 256 up to e = 4096; 4*66 at 4352; 512 at 16384; 1024 at 65536
        got = [lib.kvm_state_rows_for(C.byref(c), T) for T in (4096, 4352, 16384, 65536)]
        assert got == [256, 264, 512, 1024]


def test_table_budget_and_bad_configs():
    lib = kb.load_library()
    table = (C.c_int64 * 6)(0, 256, 300, 300, 900, 901)
    c = cfg(budget_kind=kb.KVM_BUDGET_TABLE, budget_table=C.cast(table, C.POINTER(C.c_int64)), budget_table_len=6)
    oc = ko.KVMConfig(head_dim=128, rope_dims=32, chunk_len=256, budget_kind=ko.BUDGET_TABLE,
                      budget_table=list(table))
    for T in (512, 768, 1024, 1280, 1536, 4096):
        assert lib.kvm_state_rows_for(C.byref(c), T) == ko.expected_rows(oc, T)[-1]
    for bad in (dict(head_dim=96), dict(n_q_heads=3), dict(chunk_len=0), dict(n_sink=256), dict(io_dtype=7),
                dict(rope_dims=129), dict(budget_kind=9), dict(batch=0)):
        assert lib.kvm_state_bytes(C.byref(cfg(**bad)), 4096) == 0, bad
        assert lib.kvm_state_rows_for(C.byref(cfg(**bad)), 4096) == -1, bad


def test_state_bytes_cover_the_layout():
    lib = kb.load_library()
    c = cfg()
    U, d, C_, L, m = 4, 128, 256, 512, 512
    slots = 16   # readout versions kept: 2 x 8-chunk attention groups
    need = U * m * d * (8 + 4 + slots * (2 + 2)) + U * m * 12 + 2 * U * L * d * 2 + U * L * 4 + 8 * U * C_ * d * 2 + U * C_ * 20
    # fewer units than compute units: the table through which up to 8 workgroups that share a unit's
    # rows exchange each token's winner (two parities x two 64-bit words per token)
    need += U * 2 * 8 * 2 * C_ * 8
    got = lib.kvm_state_bytes(C.byref(c), 8192)
    assert need <= got <= need + 17 * 256
    assert lib.kvm_state_bytes(C.byref(cfg(budget_kind=kb.KVM_BUDGET_SQRT, budget_scale=4.0)), 65536) > \
        lib.kvm_state_bytes(C.byref(cfg(budget_kind=kb.KVM_BUDGET_SQRT, budget_scale=4.0)), 4096)


def test_argument_and_capacity_errors_before_any_launch():
    lib = kb.load_library()
    c = cfg(budget_kind=kb.KVM_BUDGET_SQRT, budget_scale=4.0)
    h = C.c_void_p()
    nbytes = lib.kvm_state_bytes(C.byref(c), 4096)
    assert lib.kvm_state_init(C.byref(h), C.byref(c), FAKE_DEV_PTR, nbytes - 1, 4096) == kb.KVM_ERR_CAPACITY
    assert lib.kvm_state_init(C.byref(h), C.byref(c), FAKE_DEV_PTR + 8, nbytes, 4096) == kb.KVM_ERR_ARG
    assert lib.kvm_state_init(C.byref(h), C.byref(c), None, nbytes, 4096) == kb.KVM_ERR_ARG
    assert lib.kvm_state_init(C.byref(h), C.byref(c), FAKE_DEV_PTR, nbytes, 4096) == kb.KVM_OK
    v = C.c_int64(-1)
    assert lib.kvm_state_rows(h, C.byref(v)) == 0 and v.value == 0
    assert lib.kvm_state_capacity(h, C.byref(v)) == 0 and v.value == 256
    assert lib.kvm_state_tokens(h, C.byref(v)) == 0 and v.value == 0
    p = FAKE_DEV_PTR
    # budget over this call (rows 264 at e = 4352) exceeds the 256-row buffer: refused up front
    assert lib.kvm_prefill_chunked(h, p, p, p, None, p, None, 8192, None, None) == kb.KVM_ERR_CAPACITY
    assert lib.kvm_state_tokens(h, C.byref(v)) == 0 and v.value == 0
    assert lib.kvm_prefill_chunked(h, p, p, p, None, p, None, 0, None, None) == kb.KVM_ERR_ARG
    assert lib.kvm_prefill_chunked(h, None, p, p, None, p, None, 256, None, None) == kb.KVM_ERR_ARG
    assert lib.kvm_prefill_chunked(h, p + 2, p, p, None, p, None, 256, None, None) == kb.KVM_ERR_ARG
    st = kb.kvm_strides(*([128] * 18))
    st.q_t = 100                                         # not a multiple of 8 elements
    assert lib.kvm_prefill_chunked(h, p, p, p, None, p, None, 256, C.byref(st), None) == kb.KVM_ERR_ARG
    # every stride the kernels take on trust is checked up front: a token or head stride shorter
    # than a row, a negative stride, a k/v token stride whose tile offsets leave 32 bits, and lse
    # strides that cannot address B * T * H_q distinct floats
    names = [f for f, _ in kb.kvm_strides._fields_]

    def strides(**kw):
        dense = dict(q_b=256 * 512, q_t=512, q_h=128, k_b=256 * 256, k_t=256, k_h=128, v_b=256 * 256, v_t=256,
                     v_h=128, o_b=256 * 512, o_t=512, o_h=128, g_b=512, g_t=2, g_h=1, lse_b=1024, lse_t=4, lse_h=1)
        dense.update(kw)
        return kb.kvm_strides(*[dense[n] for n in names])

    for bad in (dict(k_t=64), dict(v_h=64), dict(q_t=-512), dict(o_b=-8), dict(k_t=(1 << 23) + 8),
                dict(v_t=(1 << 23) + 8)):
        assert lib.kvm_prefill_chunked(h, p, p, p, None, p, None, 256, C.byref(strides(**bad)), None) \
            == kb.KVM_ERR_ARG, bad
    for bad in (dict(lse_h=0), dict(lse_t=-4), dict(lse_b=0)):
        assert lib.kvm_prefill_chunked(h, p, p, p, None, p, p, 256, C.byref(strides(**bad)), None) \
            == kb.KVM_ERR_ARG, bad
    assert lib.kvm_prefill_chunked(h, p, p, p, p, p, None, 256, C.byref(strides(g_t=-2)), None) == kb.KVM_ERR_ARG
    assert lib.kvm_state_tokens(h, C.byref(v)) == 0 and v.value == 0      # nothing was consumed
    # debugging knobs: unknown knob refused, known ones accepted and reset by 0
    assert lib.kvm_debug_set(h, kb.KVM_DEBUG_KNOBS, 1) == kb.KVM_ERR_ARG
    assert lib.kvm_debug_set(h, -1, 1) == kb.KVM_ERR_ARG
    assert lib.kvm_debug_set(None, kb.KVM_DEBUG_FOLD_PATH, 1) == kb.KVM_ERR_ARG
    assert lib.kvm_debug_set(h, kb.KVM_DEBUG_FOLD_CHAINS, 2) == kb.KVM_OK
    assert lib.kvm_debug_set(h, kb.KVM_DEBUG_FOLD_CHAINS, 0) == kb.KVM_OK
    # the allocation-free decode refuses what its fixed scratch cannot describe, before any HIP call
    hs = (C.c_void_p * 1)(h)
    assert lib.kvm_decode_step_multi_static(hs, 0, p, p, p, None, p, None) == kb.KVM_ERR_ARG
    assert lib.kvm_decode_step_multi_static(None, 1, p, p, p, None, p, None) == kb.KVM_ERR_ARG
    assert lib.kvm_state_fold(h, p, p, None, 255, 512, None, None, None) == kb.KVM_ERR_ARG
    assert lib.kvm_decode_step(h, p, None, p, None, p, None) == kb.KVM_ERR_ARG
    assert lib.kvm_state_grow(h, FAKE_DEV_PTR, 16, 65536, None) == kb.KVM_ERR_CAPACITY
    assert lib.kvm_state_import(h, None, None, None, None, None, None, None, None, 100000, 0, 0, None) \
        == kb.KVM_ERR_ARG
    assert lib.kvm_state_destroy(h) == 0


def test_backward_argument_and_state_errors_before_any_launch():
    lib = kb.load_library()
    c = cfg()
    h = C.c_void_p()
    assert lib.kvm_state_init(C.byref(h), C.byref(c), FAKE_DEV_PTR, lib.kvm_state_bytes(C.byref(c), 4096), 4096) == 0
    p = FAKE_DEV_PTR
    grads = kb.kvm_grads(*([p] * 8))
    assert lib.kvm_backward_workspace_bytes(None, 1024) == 0
    assert lib.kvm_backward_workspace_bytes(h, 0) == 0
    nbytes = lib.kvm_backward_workspace_bytes(h, 1024)
    # the work arrays hold at least the fp32 accumulators of dk and dv and the sums' copies
    U, d, T, M = 4, 128, 1024, 512
    assert nbytes >= 2 * U * T * d * 4 + U * M * d * (8 + 4 + 4 + 4)
    args = lambda **kw: [kw.get("st", h), kw.get("q", p), p, p, None, p, kw.get("lse", p), p, p, p,
                         kw.get("grads", C.byref(grads)), kw.get("T", 1024), kw.get("ws", p), kw.get("n", nbytes), None]
    # the state is empty: it has not run a prefill of 1024 tokens
    assert lib.kvm_prefill_backward(*args()) == kb.KVM_ERR_STATE
    assert lib.kvm_prefill_backward(*args(q=None)) == kb.KVM_ERR_ARG
    assert lib.kvm_prefill_backward(*args(lse=None)) == kb.KVM_ERR_ARG
    assert lib.kvm_prefill_backward(*args(grads=None)) == kb.KVM_ERR_ARG
    assert lib.kvm_prefill_backward(*args(T=0)) == kb.KVM_ERR_ARG
    assert lib.kvm_prefill_backward(*args(st=None)) == kb.KVM_ERR_ARG
    missing = kb.kvm_grads(p, p, p, p, None, p, p, p)
    assert lib.kvm_prefill_backward(*args(grads=C.byref(missing))) == kb.KVM_ERR_ARG
    assert lib.kvm_state_destroy(h) == 0


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(kb, "_lib", None)
    monkeypatch.setattr(kb, "LIB_PATH", str(tmp_path / "libkvm.so"))
    with pytest.raises(FileNotFoundError):
        kb.load_library()


def test_host_logic_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """The library's host side (argument checks, growth replay, plans, sizes) is compiled again with
    AddressSanitizer and UBSan -- host code only, kernels left out -- and this file's other tests
    run against that build in a child process: a stray write or a signed overflow in the host
    logic ends the child with a sanitizer report."""
    import subprocess
    import sys
    from paper_2605_09877_amd import build
    lib, runtime = build.build_host_checked(str(tmp_path))
    runner = (
        "import sys, pytest\n"
        "import paper_2605_09877_amd.binding as kb\n"
        f"kb.LIB_PATH = {lib!r}\n"
        "sys.exit(pytest.main(['-x', '-q', '-p', 'no:cacheprovider', '-k', 'not sanitizers and not loudly', "
        f"{os.path.abspath(__file__)!r}]))\n")
    env = dict(os.environ, PYTHONPATH=ROOT + os.pathsep + os.path.join(ROOT, "tests"),
               ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=0:halt_on_error=1:abort_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    env["LD_PRELOAD"] = (env.get("LD_PRELOAD", "") + " " + runtime).strip()
    r = subprocess.run([sys.executable, "-c", runner], env=env, capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert " passed" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
