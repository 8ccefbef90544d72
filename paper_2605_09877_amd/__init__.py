"""MI355X-native Key-Value Means (KVM) attention layer: HIP kernels behind a C ABI (libkvm.so)
and a thin ctypes binding.  Entry points carry the names of include/kvm.h."""
from .binding import (KVM_BF16, KVM_BUDGET_FIXED, KVM_BUDGET_NONE, KVM_BUDGET_SQRT, KVM_BUDGET_TABLE,
                      KVM_ERR_ARG, KVM_ERR_CAPACITY, KVM_ERR_HIP, KVM_ERR_STATE, KVM_ERR_UNSUPPORTED, KVM_F32,
                      KVM_OK, EXPORTS, KVMError, KVMState, kvm_config, kvm_strides, load_library)
from .autograd import kvm_attention


def kvm_state_init(**kw) -> KVMState:
    """Allocate a device buffer of kvm_state_bytes() and bind an empty state to it."""
    return KVMState(**kw)


def kvm_prefill_chunked(state: KVMState, q, k, v, gate=None, out=None, lse=None):
    return state.prefill(q, k, v, gate, out, lse)


def kvm_decode_step(state: KVMState, q, k, v, gate=None, out=None):
    return state.decode(q, k, v, gate, out)


def kvm_state_fold(state: KVMState, k_blk, v_blk, gate_blk=None, *, e: int):
    return state.fold(k_blk, v_blk, gate_blk, e=e)


def state_for(w, *, max_tokens=None, device="cuda:0", **params) -> KVMState:
    """A state configured like synth.Workload `w`; params: ln_gamma, ln_beta, tau_state, tau_bswa."""
    kind = {"none": KVM_BUDGET_NONE, "fixed": KVM_BUDGET_FIXED, "sqrt": KVM_BUDGET_SQRT,
            "table": KVM_BUDGET_TABLE}[w.budget_kind]
    return KVMState(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim,
                    rope_dims=w.rope_dims, chunk_len=w.chunk_len, n_bswa_chunks=w.n_bswa_chunks,
                    n_sink=w.n_sink, io_dtype=KVM_BF16 if w.io == "bf16" else KVM_F32, budget_kind=kind,
                    budget_fixed=w.budget_fixed, budget_scale=w.budget_scale,
                    budget_table=list(w.budget_table) if w.budget_kind == "table" else None,
                    max_tokens=w.seq if max_tokens is None else max_tokens, device=device,
                    **{k: v for k, v in params.items() if k in ("ln_gamma", "ln_beta", "tau_state", "tau_bswa")})
