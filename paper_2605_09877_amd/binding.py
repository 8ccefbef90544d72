"""Thin ctypes binding of libkvm.so: same entry points as include/kvm.h, torch tensors in.

Argument marshalling only -- every step of the layer runs in the library's HIP kernels.
torch is used for device memory and the current stream.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvm.so")

KVM_F32, KVM_BF16 = 0, 1
KVM_BUDGET_NONE, KVM_BUDGET_FIXED, KVM_BUDGET_SQRT, KVM_BUDGET_TABLE = 0, 1, 2, 3
KVM_OK, KVM_ERR_ARG, KVM_ERR_CAPACITY, KVM_ERR_STATE, KVM_ERR_HIP, KVM_ERR_UNSUPPORTED = 0, -1, -2, -3, -4, -5
KVM_ERR_LIMIT = -6
KVM_STATIC_MAX_SEQUENCES = 4096

EXPORTS = [
    "kvm_strerror", "kvm_last_hip_error", "kvm_state_rows_for", "kvm_state_bytes", "kvm_state_init",
    "kvm_state_destroy", "kvm_prefill_chunked", "kvm_decode_step", "kvm_decode_multi_workspace_bytes",
    "kvm_decode_step_multi", "kvm_decode_step_multi_static", "kvm_state_fold", "kvm_state_rows",
    "kvm_state_tokens", "kvm_state_capacity", "kvm_state_folds", "kvm_state_fold_path", "kvm_state_trace", "kvm_state_grow",
    "kvm_state_export", "kvm_state_import", "kvm_state_profile", "kvm_state_profile_read",
    "kvm_measure_mfma_bf16_peak", "kvm_measure_copy_peak", "kvm_measure_read_peak", "kvm_prepare_scratch_bytes", "kvm_prepare_qkv",
    "kvm_backward_workspace_bytes", "kvm_prefill_backward", "kvm_debug_set",
]
(KVM_DEBUG_FOLD_PATH, KVM_DEBUG_FOLD_WAVES, KVM_DEBUG_PREFILL_SCHEDULE, KVM_DEBUG_FOLD_CHAINS, KVM_DEBUG_MERGE_COPY,
 KVM_DEBUG_BACKWARD_PATH, KVM_DEBUG_FOLD_SPLIT) = range(7)
KVM_DEBUG_KNOBS = 8  # number of knobs the library knows of; kvm_debug_set refuses any index from here on


class kvm_config(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("rope_dims", C.c_int32), ("chunk_len", C.c_int32), ("n_bswa_chunks", C.c_int32),
        ("n_sink", C.c_int32), ("io_dtype", C.c_int32), ("budget_kind", C.c_int32),
        ("budget_fixed", C.c_int64), ("budget_scale", C.c_double),
        ("budget_table", C.POINTER(C.c_int64)), ("budget_table_len", C.c_int64),
        ("ln_eps", C.c_float), ("norm_eps", C.c_float),
        ("ln_gamma", C.c_void_p), ("ln_beta", C.c_void_p), ("tau_state", C.c_void_p), ("tau_bswa", C.c_void_p),
    ]


class kvm_prep_params(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("rope_dims", C.c_int32), ("io_dtype", C.c_int32), ("d_model", C.c_int32), ("ln_eps", C.c_float),
        ("rope_base", C.c_double),
        ("alpha_q", C.c_void_p), ("alpha_k", C.c_void_p), ("alpha_v", C.c_void_p), ("lambda_v", C.c_void_p),
        ("lnq_gamma", C.c_void_p), ("lnq_beta", C.c_void_p), ("lnk_gamma", C.c_void_p), ("lnk_beta", C.c_void_p),
        ("w_gate", C.c_void_p),
    ]


class kvm_grads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("dq", "dk", "dv", "dgate", "dgamma", "dbeta", "dtau_state", "dtau_bswa")]


class kvm_strides(C.Structure):
    _fields_ = [(n, C.c_int64) for n in (
        "q_b", "q_t", "q_h", "k_b", "k_t", "k_h", "v_b", "v_t", "v_h",
        "o_b", "o_t", "o_h", "g_b", "g_t", "g_h", "lse_b", "lse_t", "lse_h")]


class KVMError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(what)


_lib = None


def load_library() -> C.CDLL:
    """Load libkvm.so built in-tree.  There is no fallback: without it nothing here works."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2605_09877_amd.build` (needs hipcc)")
    lib = C.CDLL(LIB_PATH)
    vp, i64, i32 = C.c_void_p, C.c_int64, C.c_int32
    lib.kvm_strerror.restype = C.c_char_p
    lib.kvm_strerror.argtypes = [C.c_int]
    lib.kvm_last_hip_error.restype = C.c_char_p
    lib.kvm_state_rows_for.restype = i64
    lib.kvm_state_rows_for.argtypes = [C.POINTER(kvm_config), i64]
    lib.kvm_state_bytes.restype = C.c_size_t
    lib.kvm_state_bytes.argtypes = [C.POINTER(kvm_config), i64]
    lib.kvm_state_init.argtypes = [C.POINTER(vp), C.POINTER(kvm_config), vp, C.c_size_t, i64]
    lib.kvm_state_destroy.argtypes = [vp]
    lib.kvm_prefill_chunked.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, C.POINTER(kvm_strides), vp]
    lib.kvm_decode_step.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    lib.kvm_decode_multi_workspace_bytes.restype = C.c_size_t
    lib.kvm_decode_multi_workspace_bytes.argtypes = [i64]
    lib.kvm_decode_step_multi.argtypes = [C.POINTER(vp), i32, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
    lib.kvm_decode_step_multi_static.argtypes = [C.POINTER(vp), i32, vp, vp, vp, vp, vp, vp]
    lib.kvm_state_fold.argtypes = [vp, vp, vp, vp, i32, i64, vp, vp, vp]
    for name in ("kvm_state_rows", "kvm_state_tokens", "kvm_state_capacity", "kvm_state_folds", "kvm_state_fold_path"):
        getattr(lib, name).argtypes = [vp, C.POINTER(i64)]
    lib.kvm_state_trace.argtypes = [vp, vp, vp, i64]
    lib.kvm_state_grow.argtypes = [vp, vp, C.c_size_t, i64, vp]
    lib.kvm_state_export.argtypes = [vp] * 12
    lib.kvm_state_import.argtypes = [vp] * 9 + [i64, i64, i64, vp]
    lib.kvm_debug_set.argtypes = [vp, C.c_int, C.c_int]
    lib.kvm_state_profile.argtypes = [vp, C.c_int]
    lib.kvm_state_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64)]
    lib.kvm_prepare_scratch_bytes.restype = C.c_size_t
    lib.kvm_prepare_scratch_bytes.argtypes = [C.POINTER(kvm_prep_params), i64]
    lib.kvm_prepare_qkv.argtypes = [C.POINTER(kvm_prep_params)] + [vp] * 13 + [i64, i64, vp]
    lib.kvm_backward_workspace_bytes.restype = C.c_size_t
    lib.kvm_backward_workspace_bytes.argtypes = [vp, i64]
    lib.kvm_prefill_backward.argtypes = [vp] * 10 + [C.POINTER(kvm_grads), i64, vp, C.c_size_t, vp]
    lib.kvm_measure_mfma_bf16_peak.argtypes = [C.c_int, vp, C.POINTER(C.c_double), vp]
    lib.kvm_measure_copy_peak.argtypes = [vp, vp, C.c_size_t, C.POINTER(C.c_double), vp]
    lib.kvm_measure_read_peak.argtypes = [vp, C.c_size_t, vp, C.POINTER(C.c_double), vp]
    _lib = lib
    return lib


def _check(status: int, what: str) -> None:
    if status != KVM_OK:
        lib = load_library()
        msg = lib.kvm_strerror(status).decode()
        if status in (KVM_ERR_HIP, KVM_ERR_LIMIT):
            msg += " (" + lib.kvm_last_hip_error().decode() + ")"
        raise KVMError(status, f"{what}: {msg}")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def prepare_qkv(q_raw, k_raw, v_raw, *, rope_dims: int, pos0: int = 0, v_first=None, x=None, prev_q=None,
                prev_k=None, prev_v=None, alpha_q=None, alpha_k=None, alpha_v=None, lambda_v=None,
                lnq_gamma=None, lnq_beta=None, lnk_gamma=None, lnk_beta=None, w_gate=None,
                ln_eps: float = 0.0, rope_base: float = 0.0):
    """kvm_prepare_qkv on [B, T, H, d] tensors: returns (q, k, v, gate or None)."""
    lib = load_library()
    B, T, Hq, d = q_raw.shape
    Hkv = k_raw.shape[2]
    io = KVM_BF16 if q_raw.dtype == torch.bfloat16 else KVM_F32
    f32 = lambda t: None if t is None else t.to(torch.float32).contiguous()
    prm = [f32(t) for t in (alpha_q, alpha_k, alpha_v, lambda_v, lnq_gamma, lnq_beta, lnk_gamma, lnk_beta, w_gate)]
    p = kvm_prep_params(B, Hq, Hkv, d, rope_dims, io, 0 if x is None else x.shape[-1], ln_eps, rope_base,
                        *[_ptr(t) for t in prm])
    tens = [t if t is None else t.contiguous() for t in (q_raw, k_raw, v_raw, v_first, x, prev_q, prev_k, prev_v)]
    q, k, v = torch.empty_like(tens[0]), torch.empty_like(tens[1]), torch.empty_like(tens[2])
    gate = None if x is None else torch.empty(B, T, Hkv, dtype=torch.float32, device=q_raw.device)
    nbytes = lib.kvm_prepare_scratch_bytes(C.byref(p), T)
    if nbytes == 0:
        raise KVMError(KVM_ERR_ARG, "kvm_prepare_scratch_bytes: invalid preparation parameters")
    scratch = torch.empty(nbytes, dtype=torch.uint8, device=q_raw.device)
    _check(lib.kvm_prepare_qkv(C.byref(p), *[_ptr(t) for t in tens], _ptr(q), _ptr(k), _ptr(v), _ptr(gate),
                               _ptr(scratch), T, pos0, _stream()), "kvm_prepare_qkv")
    return q, k, v, gate


def measure_peaks(device="cuda:0", copy_bytes: int = 1 << 30, iters: int = 20000) -> dict:
    """kvm_measure_mfma_bf16_peak, kvm_measure_copy_peak and kvm_measure_read_peak on `device`:
    {"mfma_bf16_tflops", "copy_gbs", "read_gbs"}."""
    lib = load_library()
    with torch.cuda.device(device):
        src = torch.ones(copy_bytes // 4, dtype=torch.float32, device=device)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        tf, gb, rd = C.c_double(), C.c_double(), C.c_double()
        _check(lib.kvm_measure_mfma_bf16_peak(iters, dst.data_ptr(), C.byref(tf), _stream()),
               "kvm_measure_mfma_bf16_peak")
        _check(lib.kvm_measure_copy_peak(src.data_ptr(), dst.data_ptr(), copy_bytes, C.byref(gb), _stream()),
               "kvm_measure_copy_peak")
        _check(lib.kvm_measure_read_peak(src.data_ptr(), copy_bytes, dst.data_ptr(), C.byref(rd), _stream()),
               "kvm_measure_read_peak")
    return dict(mfma_bf16_tflops=tf.value, copy_gbs=gb.value, read_gbs=rd.value)


def _io_dtype(io: int) -> torch.dtype:
    return torch.bfloat16 if io == KVM_BF16 else torch.float32


class KVMState:
    """A bound state: owns the device buffer and the parameter tensors the handle points to."""

    def __init__(self, *, batch: int, n_q_heads: int, n_kv_heads: int, head_dim: int, rope_dims: int,
                 chunk_len: int, n_bswa_chunks: int = 2, n_sink: int = 1, io_dtype: int = KVM_BF16,
                 budget_kind: int = KVM_BUDGET_FIXED, budget_fixed: int = 0, budget_scale: float = 0.0,
                 budget_table: Optional[Sequence[int]] = None, ln_eps: float = 1e-5, norm_eps: float = 1e-12,
                 ln_gamma: Optional[torch.Tensor] = None, ln_beta: Optional[torch.Tensor] = None,
                 tau_state: Optional[torch.Tensor] = None, tau_bswa: Optional[torch.Tensor] = None,
                 max_tokens: int, device: str = "cuda:0"):
        self.lib = load_library()
        self.device = torch.device(device)
        self._keep = []

        def dev_f32(t, shape):
            if t is None:
                return None
            t = t.to(device=self.device, dtype=torch.float32).contiguous()
            assert tuple(t.shape) == shape, (tuple(t.shape), shape)
            self._keep.append(t)
            return t

        self.ln_gamma = dev_f32(ln_gamma, (n_kv_heads, head_dim))
        self.ln_beta = dev_f32(ln_beta, (n_kv_heads, head_dim))
        self.tau_state = dev_f32(tau_state, (n_q_heads,))
        self.tau_bswa = dev_f32(tau_bswa, (n_q_heads,))
        table = None
        if budget_table is not None:
            table = (C.c_int64 * len(budget_table))(*[int(x) for x in budget_table])
            self._keep.append(table)
        self.cfg = kvm_config(
            batch, n_q_heads, n_kv_heads, head_dim, rope_dims, chunk_len, n_bswa_chunks, n_sink, io_dtype,
            budget_kind, int(budget_fixed), float(budget_scale),
            C.cast(table, C.POINTER(C.c_int64)) if table is not None else None,
            0 if table is None else len(budget_table), ln_eps, norm_eps,
            _ptr(self.ln_gamma), _ptr(self.ln_beta), _ptr(self.tau_state), _ptr(self.tau_bswa))
        self.io = io_dtype
        self.dtype = _io_dtype(io_dtype)
        self.handle = C.c_void_p()
        self.buf = None
        self._bind(max_tokens, first=True)
        self._trace = None

    # ---- binding / growth
    def _alloc(self, max_tokens: int) -> torch.Tensor:
        nbytes = self.lib.kvm_state_bytes(C.byref(self.cfg), max_tokens)
        if nbytes == 0:
            raise KVMError(KVM_ERR_ARG, "kvm_state_bytes: bad config")
        return torch.empty(nbytes, dtype=torch.uint8, device=self.device)

    def _bind(self, max_tokens: int, first: bool) -> None:
        buf = self._alloc(max_tokens)
        _check(self.lib.kvm_state_init(C.byref(self.handle), C.byref(self.cfg), buf.data_ptr(), buf.numel(),
                                       max_tokens), "kvm_state_init")
        self.buf = buf
        self.max_tokens = max_tokens

    def grow(self, new_max_tokens: int) -> None:
        """kvm_state_grow into a freshly allocated, larger buffer."""
        buf = self._alloc(new_max_tokens)
        with torch.cuda.device(self.device):
            _check(self.lib.kvm_state_grow(self.handle, buf.data_ptr(), buf.numel(), new_max_tokens, _stream()),
                   "kvm_state_grow")
        old = self.buf
        self.buf = buf
        self.max_tokens = new_max_tokens
        old.record_stream(torch.cuda.current_stream(self.device))

    def close(self) -> None:
        if self.handle:
            self.lib.kvm_state_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- introspection
    def _i64(self, fn) -> int:
        v = C.c_int64()
        _check(fn(self.handle, C.byref(v)), fn.__name__)
        return v.value

    @property
    def rows(self) -> int:
        return self._i64(self.lib.kvm_state_rows)

    @property
    def tokens(self) -> int:
        return self._i64(self.lib.kvm_state_tokens)

    @property
    def capacity(self) -> int:
        return self._i64(self.lib.kvm_state_capacity)

    @property
    def folds(self) -> int:
        return self._i64(self.lib.kvm_state_folds)

    @property
    def fold_path(self) -> int:
        """1: a run of folds is one launch (one workgroup per unit); 2: one kernel per fold step."""
        return self._i64(self.lib.kvm_state_fold_path)

    def rows_for(self, max_tokens: int) -> int:
        return self.lib.kvm_state_rows_for(C.byref(self.cfg), max_tokens)

    # ---- the hot path
    def _chk(self, t: torch.Tensor, shape, dtype, name: str) -> torch.Tensor:
        if t.device != self.device or t.dtype != dtype or tuple(t.shape) != tuple(shape) or not t.is_contiguous():
            raise ValueError(f"{name}: want contiguous {dtype} {tuple(shape)} on {self.device}, "
                             f"got {t.dtype} {tuple(t.shape)} on {t.device}")
        return t

    def _chk_view(self, t: torch.Tensor, shape, dtype, name: str) -> torch.Tensor:
        """Like _chk, but any strides are allowed as long as the last axis is contiguous."""
        if t.device != self.device or t.dtype != dtype or tuple(t.shape) != tuple(shape) or \
                (t.dim() > 3 and t.stride(-1) != 1):
            raise ValueError(f"{name}: want {dtype} {tuple(shape)} on {self.device} with a contiguous last axis, "
                             f"got {t.dtype} {tuple(t.shape)} strides {t.stride()} on {t.device}")
        return t

    def prefill(self, q, k, v, gate=None, out=None, lse=None, want_lse=False):
        """kvm_prefill_chunked.  q [B,T,Hq,d], k/v [B,T,Hkv,d], gate [B,T,Hkv] fp32 or None.  The
        tensors may be views of wider buffers (say slices of one fused projection output): their
        element strides go to the library as kvm_strides; head_dim must be contiguous."""
        c = self.cfg
        T = q.shape[1]
        self._chk_view(q, (c.batch, T, c.n_q_heads, c.head_dim), self.dtype, "q")
        self._chk_view(k, (c.batch, T, c.n_kv_heads, c.head_dim), self.dtype, "k")
        self._chk_view(v, (c.batch, T, c.n_kv_heads, c.head_dim), self.dtype, "v")
        if gate is not None:
            self._chk_view(gate, (c.batch, T, c.n_kv_heads), torch.float32, "gate")
        if out is None:
            out = torch.empty((c.batch, T, c.n_q_heads, c.head_dim), dtype=self.dtype, device=self.device)
        self._chk_view(out, q.shape, self.dtype, "out")
        if lse is None and want_lse:
            lse = torch.empty((c.batch, T, c.n_q_heads), dtype=torch.float32, device=self.device)
        if lse is not None:
            self._chk_view(lse, (c.batch, T, c.n_q_heads), torch.float32, "lse")
        bth = lambda t, n: (0, 0, 0) if t is None else (t.stride(0), t.stride(1), t.stride(2))
        strides = kvm_strides(*bth(q, 4), *bth(k, 4), *bth(v, 4), *bth(out, 4), *bth(gate, 3), *bth(lse, 3))
        with torch.cuda.device(self.device):
            _check(self.lib.kvm_prefill_chunked(self.handle, q.data_ptr(), k.data_ptr(), v.data_ptr(), _ptr(gate),
                                                out.data_ptr(), _ptr(lse), T, C.byref(strides), _stream()),
                   "kvm_prefill_chunked")
        return (out, lse) if (want_lse or lse is not None) else out

    def decode(self, q, k, v, gate=None, out=None):
        """kvm_decode_step.  q [B,Hq,d], k/v [B,Hkv,d], gate [B,Hkv] fp32 or None."""
        c = self.cfg
        self._chk(q, (c.batch, c.n_q_heads, c.head_dim), self.dtype, "q")
        self._chk(k, (c.batch, c.n_kv_heads, c.head_dim), self.dtype, "k")
        self._chk(v, (c.batch, c.n_kv_heads, c.head_dim), self.dtype, "v")
        if gate is not None:
            self._chk(gate, (c.batch, c.n_kv_heads), torch.float32, "gate")
        if out is None:
            out = torch.empty_like(q)
        self._chk(out, q.shape, self.dtype, "out")
        # a decode step is a few microseconds of GPU work: entering a device context costs as much,
        # so it is entered only when another device is current
        if torch.cuda.current_device() == self.device.index:
            _check(self.lib.kvm_decode_step(self.handle, q.data_ptr(), k.data_ptr(), v.data_ptr(), _ptr(gate),
                                            out.data_ptr(), _stream()), "kvm_decode_step")
        else:
            with torch.cuda.device(self.device):
                _check(self.lib.kvm_decode_step(self.handle, q.data_ptr(), k.data_ptr(), v.data_ptr(), _ptr(gate),
                                                out.data_ptr(), _stream()), "kvm_decode_step")
        return out

    def fold(self, k_blk, v_blk, gate_blk=None, *, e: int):
        """kvm_state_fold.  k_blk/v_blk [B,C,Hkv,d]; returns (assign [B,Hkv,C] int32, score [B,Hkv,C,2])."""
        c = self.cfg
        n = k_blk.shape[1]
        self._chk(k_blk, (c.batch, n, c.n_kv_heads, c.head_dim), self.dtype, "k_blk")
        self._chk(v_blk, (c.batch, n, c.n_kv_heads, c.head_dim), self.dtype, "v_blk")
        if gate_blk is not None:
            self._chk(gate_blk, (c.batch, n, c.n_kv_heads), torch.float32, "gate_blk")
        assign = torch.empty((c.batch, c.n_kv_heads, n), dtype=torch.int32, device=self.device)
        score = torch.empty((c.batch, c.n_kv_heads, n, 2), dtype=torch.float32, device=self.device)
        with torch.cuda.device(self.device):
            _check(self.lib.kvm_state_fold(self.handle, k_blk.data_ptr(), v_blk.data_ptr(), _ptr(gate_blk), n, e,
                                           assign.data_ptr(), score.data_ptr(), _stream()), "kvm_state_fold")
        return assign, score

    def reset(self) -> None:
        """Back to the empty state (m = 0, no tokens seen) in the same buffer; no device work."""
        _check(self.lib.kvm_state_import(self.handle, *([None] * 8), 0, 0, 0, None), "kvm_state_import")

    def debug_set(self, knob: int, value: int) -> None:
        """kvm_debug_set: force one of the library's own choices (0 gives it back)."""
        _check(self.lib.kvm_debug_set(self.handle, knob, value), "kvm_debug_set")

    def profile(self, enable) -> None:
        """kvm_state_profile: False/0 off, True/1 on, 2 on with folds and attention kept apart."""
        _check(self.lib.kvm_state_profile(self.handle, int(enable)), "kvm_state_profile")

    def profile_read(self) -> dict:
        """kvm_state_profile_read: {"attn": (ms, launches), "fold": (...), "decode": (...)}."""
        ms = (C.c_double * 3)()
        cnt = (C.c_int64 * 3)()
        _check(self.lib.kvm_state_profile_read(self.handle, ms, cnt), "kvm_state_profile_read")
        return {k: (ms[i], cnt[i]) for i, k in enumerate(("attn", "fold", "decode"))}

    def backward(self, q, k, v, gate, out, lse, dout, assign, score, workspace=None) -> dict:
        """kvm_prefill_backward for the prefill this state has just run (one call, from empty, over
        exactly these tensors).  Returns the gradients as a dict of fresh tensors."""
        c = self.cfg
        T = q.shape[1]
        self._chk(q, (c.batch, T, c.n_q_heads, c.head_dim), self.dtype, "q")
        self._chk(k, (c.batch, T, c.n_kv_heads, c.head_dim), self.dtype, "k")
        self._chk(v, (c.batch, T, c.n_kv_heads, c.head_dim), self.dtype, "v")
        self._chk(out, q.shape, self.dtype, "out")
        self._chk(dout, q.shape, self.dtype, "dout")
        self._chk(lse, (c.batch, T, c.n_q_heads), torch.float32, "lse")
        if gate is not None:
            self._chk(gate, (c.batch, T, c.n_kv_heads), torch.float32, "gate")
        if assign is not None:
            if (assign.dtype != torch.int32 or not assign.is_contiguous() or assign.device != self.device
                    or tuple(assign.shape[1:]) != (c.batch, c.n_kv_heads, c.chunk_len) or assign.shape[0] < self.folds):
                raise ValueError("assign: want the contiguous int32 [folds, B, Hkv, C] record of kvm_state_trace")
            if (score is None or score.dtype != torch.float32 or not score.is_contiguous()
                    or tuple(score.shape) != tuple(assign.shape) + (2,)):
                raise ValueError("score: want the fp32 [folds, B, Hkv, C, 2] record of kvm_state_trace")
        f32 = dict(dtype=torch.float32, device=self.device)
        g = dict(dq=torch.empty_like(q), dk=torch.empty_like(k), dv=torch.empty_like(v),
                 dgate=torch.empty((c.batch, T, c.n_kv_heads), **f32),
                 dgamma=torch.empty((c.n_kv_heads, c.head_dim), **f32),
                 dbeta=torch.empty((c.n_kv_heads, c.head_dim), **f32),
                 dtau_state=torch.empty((c.n_q_heads,), **f32), dtau_bswa=torch.empty((c.n_q_heads,), **f32))
        nbytes = self.lib.kvm_backward_workspace_bytes(self.handle, T)
        if workspace is None or workspace.numel() < nbytes:
            workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        grads = kvm_grads(*[g[n].data_ptr() for n in ("dq", "dk", "dv", "dgate", "dgamma", "dbeta", "dtau_state",
                                                        "dtau_bswa")])
        with torch.cuda.device(self.device):
            _check(self.lib.kvm_prefill_backward(self.handle, q.data_ptr(), k.data_ptr(), v.data_ptr(), _ptr(gate),
                                                 out.data_ptr(), lse.data_ptr(), dout.data_ptr(), _ptr(assign), _ptr(score),
                                                 C.byref(grads), T, workspace.data_ptr(), workspace.numel(),
                                                 _stream()), "kvm_prefill_backward")
        workspace.record_stream(torch.cuda.current_stream(self.device))
        return g

    # ---- tracing, checkpoint
    def trace(self, max_folds: int):
        """kvm_state_trace: returns (assign [F,B,Hkv,C] int32, score [F,B,Hkv,C,2] fp32) filled by later folds."""
        c = self.cfg
        assign = torch.full((max_folds, c.batch, c.n_kv_heads, c.chunk_len), -1, dtype=torch.int32, device=self.device)
        score = torch.zeros((max_folds, c.batch, c.n_kv_heads, c.chunk_len, 2), dtype=torch.float32,
                            device=self.device)
        _check(self.lib.kvm_state_trace(self.handle, assign.data_ptr(), score.data_ptr(), max_folds),
               "kvm_state_trace")
        self._trace = (assign, score)
        return assign, score

    def export(self) -> dict:
        """kvm_state_export into fresh tensors."""
        c = self.cfg
        B, H, d, m, L = c.batch, c.n_kv_heads, c.head_dim, self.rows, c.chunk_len * c.n_bswa_chunks
        dev = self.device
        o = dict(
            sK=torch.empty((B, H, m, d), dtype=torch.float64, device=dev),
            sV=torch.empty((B, H, m, d), dtype=torch.float32, device=dev),
            rho=torch.empty((B, H, m), dtype=torch.float32, device=dev),
            w=torch.empty((B, H, m), dtype=torch.float32, device=dev),
            n=torch.empty((B, H, m), dtype=torch.int32, device=dev),
            khat=torch.empty((B, H, m, d), dtype=self.dtype, device=dev),
            vhat=torch.empty((B, H, m, d), dtype=self.dtype, device=dev),
            win_k=torch.empty((B, H, L, d), dtype=self.dtype, device=dev),
            win_v=torch.empty((B, H, L, d), dtype=self.dtype, device=dev),
            win_g=torch.empty((B, H, L), dtype=torch.float32, device=dev),
        )
        with torch.cuda.device(dev):
            _check(self.lib.kvm_state_export(self.handle, *[o[k].data_ptr() for k in (
                "sK", "sV", "rho", "w", "n", "khat", "vhat", "win_k", "win_v", "win_g")], _stream()),
                "kvm_state_export")
        o.update(m=m, tokens=self.tokens, folds=self.folds)
        return o

    def import_(self, o: dict) -> None:
        """kvm_state_import from the dict export() returns (khat/vhat are recomputed)."""
        c = self.cfg
        B, H, d, L = c.batch, c.n_kv_heads, c.head_dim, c.chunk_len * c.n_bswa_chunks
        m = int(o["m"])
        ptrs = []
        for key, dt, shape in (("sK", torch.float64, (B, H, m, d)), ("sV", torch.float32, (B, H, m, d)),
                               ("rho", torch.float32, (B, H, m)), ("w", torch.float32, (B, H, m)),
                               ("n", torch.int32, (B, H, m)), ("win_k", self.dtype, (B, H, L, d)),
                               ("win_v", self.dtype, (B, H, L, d)), ("win_g", torch.float32, (B, H, L))):
            t = o.get(key)
            ptrs.append(None if t is None else self._chk(t, shape, dt, key).data_ptr())
        with torch.cuda.device(self.device):
            _check(self.lib.kvm_state_import(self.handle, *ptrs, m, int(o["tokens"]), int(o.get("folds", 0)),
                                             _stream()), "kvm_state_import")


_multi_workspace: dict = {}


def decode_multi(states, q, k, v, gate=None, out=None):
    """kvm_decode_step_multi: one token for every sequence of every state in `states` (each state at
    its own position and state size).  q [N,Hq,d], k/v [N,Hkv,d], gate [N,Hkv] fp32 or None, with
    N = sum of the states' batches, rows in the order of `states`."""
    first = states[0]
    c = first.cfg
    n = sum(st.cfg.batch for st in states)
    first._chk(q, (n, c.n_q_heads, c.head_dim), first.dtype, "q")
    first._chk(k, (n, c.n_kv_heads, c.head_dim), first.dtype, "k")
    first._chk(v, (n, c.n_kv_heads, c.head_dim), first.dtype, "v")
    if gate is not None:
        first._chk(gate, (n, c.n_kv_heads), torch.float32, "gate")
    if out is None:
        out = torch.empty_like(q)
    first._chk(out, q.shape, first.dtype, "out")
    nbytes = first.lib.kvm_decode_multi_workspace_bytes(n)
    ws = _multi_workspace.get((str(first.device), nbytes))
    if ws is None:
        ws = _multi_workspace[(str(first.device), nbytes)] = torch.empty(nbytes, dtype=torch.uint8, device=first.device)
    handles = (C.c_void_p * len(states))(*[st.handle for st in states])
    with torch.cuda.device(first.device):
        _check(first.lib.kvm_decode_step_multi(handles, len(states), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                               _ptr(gate), out.data_ptr(), ws.data_ptr(), nbytes, _stream()),
               "kvm_decode_step_multi")
    return out



def decode_multi_static(states, q, k, v, gate=None, *, out):
    """kvm_decode_step_multi_static: decode_multi without a workspace and without any allocation
    (here neither: the caller passes `out`)."""
    first = states[0]
    c = first.cfg
    n = sum(st.cfg.batch for st in states)
    first._chk(q, (n, c.n_q_heads, c.head_dim), first.dtype, "q")
    first._chk(k, (n, c.n_kv_heads, c.head_dim), first.dtype, "k")
    first._chk(v, (n, c.n_kv_heads, c.head_dim), first.dtype, "v")
    if gate is not None:
        first._chk(gate, (n, c.n_kv_heads), torch.float32, "gate")
    first._chk(out, q.shape, first.dtype, "out")
    handles = (C.c_void_p * len(states))(*[st.handle for st in states])
    with torch.cuda.device(first.device):
        _check(first.lib.kvm_decode_step_multi_static(handles, len(states), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                                      _ptr(gate), out.data_ptr(), _stream()),
               "kvm_decode_step_multi_static")
    return out
