"""CPU oracle for the Key-Value Means (KVM) layer -- TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy statement of what one KVM attention layer computes for
one (batch, KV-head) unit: chunk-wise attention over [compressed state || block
sliding window] and the fold of each evicted block into the state.  It follows the
paper's Method section ("KVM Formulation": chunks and attention regions, weight
preparation, readout, append, merge, budget) step by step, in the paper's order
and notation.  Nothing here is blocked, fused or reordered.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
module.  It shares no code with the HIP library and imports nothing from it.

Arithmetic: everything is fp64.  The only roundings are the ones the layer's
contract fixes -- vectors that are *materialised in the I/O dtype* (fp32 or bf16):
the inputs q, k, v themselves, the memory keys k-bar, and the readout rows s-hat^K
and s-hat^V.  They are rounded to the I/O dtype (round to nearest even) at exactly
those points and widened back to fp64.  The state sums s^K, s^V, the radii rho and
the gate g are never rounded here.

Readings of the paper taken where it is silent (each is listed in the design
notes of the repository too):
  * LN_s statistics run over all d_h channels, the zeroed rotary ones included
    (equation "memory key").
  * eps of LN_s = 1e-5, eps_norm = 1e-12 unless given.
  * The append score s_j is a max over all current rows, sinks included, with no
    temperature; the merge argmax is over rows i >= S (equations of "Append" and
    "Merge").
  * Ties: argmax takes the lowest row index; append selection takes the lower
    token position; appended rows are stored in ascending position order.
  * Creation copies the whole first overflow block (m = C) even when the budget is
    smaller; afterwards M* never drops below m.
  * The budget argument e is the end of the chunk that has just been attended.
  * GQA (not in the paper): state, window, gate and LN_s belong to the KV head; the
    query heads of a group share them; temperatures are per query head.
  * A trailing partial chunk attends with b = max(0, s + C - L) and is not folded.

Pinned by tests/test_oracle_pins.py against brute force, closed forms and the
special cases that reduce to textbook attention.  Exact output values for general
inputs are "parity unpinned" (the paper prints no numbers): see that test file.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

BUDGET_NONE = 0   # no compressed state at all: the layer is pure block-sliding-window attention
BUDGET_FIXED = 1  # B(e) = budget_fixed
BUDGET_SQRT = 2   # B(e) = floor(budget_scale * ceil(sqrt(e)))
BUDGET_TABLE = 3  # B(e) = budget_table[e // C - 1] (last entry repeats)

TIE_MARGIN = 1e-4


# --------------------------------------------------------------------------- rounding
def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp64 values to bfloat16 (nearest, ties to even); return them widened to fp64.

    Goes fp64 -> fp32 -> bf16.  The first step can only move a value onto a bf16 tie
    if it was within 2^-29 relative of it; that double rounding is ignored.
    """
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    out = u.astype(np.uint32).view(np.float32)
    out = np.where(np.isfinite(f), out, f)
    return out.astype(np.float64)


def round_io(x: np.ndarray, io: str) -> np.ndarray:
    """Round to the I/O dtype ('f32' or 'bf16'); result is fp64.  'f64' rounds nothing (used
    by the pins that differentiate the layer numerically)."""
    if io == "f64":
        return np.asarray(x, dtype=np.float64)
    if io == "bf16":
        return round_bf16(x)
    if io == "f32":
        return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)
    raise ValueError(f"unknown io dtype {io!r}")


# --------------------------------------------------------------------------- config
@dataclass
class KVMConfig:
    """Per-layer constants (section "KVM Formulation": C, L = n_bswa*C, r, S, budget)."""
    head_dim: int
    rope_dims: int
    chunk_len: int
    n_bswa_chunks: int = 2
    n_sink: int = 1
    io: str = "f32"
    budget_kind: int = BUDGET_FIXED
    budget_fixed: int = 0
    budget_scale: float = 0.0
    budget_table: Optional[Sequence[int]] = None
    ln_eps: float = 1e-5
    norm_eps: float = 1e-12

    @property
    def window(self) -> int:
        return self.n_bswa_chunks * self.chunk_len


def ceil_sqrt(e: int) -> int:
    """Smallest integer n with n*n >= e (exact integer arithmetic)."""
    if e <= 0:
        return 0
    return math.isqrt(e - 1) + 1


def budget(cfg: KVMConfig, e: int) -> int:
    """State budget B(e) in rows ("We choose n_append as follows" paragraph)."""
    if cfg.budget_kind == BUDGET_NONE:
        return 0
    if cfg.budget_kind == BUDGET_FIXED:
        return int(cfg.budget_fixed)
    if cfg.budget_kind == BUDGET_SQRT:
        return int(math.floor(cfg.budget_scale * ceil_sqrt(e)))
    if cfg.budget_kind == BUDGET_TABLE:
        idx = min(max(e // cfg.chunk_len - 1, 0), len(cfg.budget_table) - 1)
        return int(cfg.budget_table[idx])
    raise ValueError("bad budget kind")


def n_append_for(cfg: KVMConfig, m: int, e: int, n_overflow: int) -> int:
    """M*(e) = max(m, min(B(e), m + C)); n_append = min(M* - m, |Omega_e|)."""
    m_star = max(m, min(budget(cfg, e), m + cfg.chunk_len))
    return min(m_star - m, n_overflow)


# --------------------------------------------------------------------------- LN_s, memory keys
def layer_norm(x: np.ndarray, gamma: np.ndarray, beta: np.ndarray, eps: float) -> np.ndarray:
    """Standard LayerNorm with bias over the last axis (biased variance)."""
    x = np.asarray(x, dtype=np.float64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * gamma + beta


def memory_key(k: np.ndarray, cfg: KVMConfig, gamma: np.ndarray, beta: np.ndarray) -> np.ndarray:
    """k-bar = LN_s(k with the first r channels zeroed), materialised in the I/O dtype."""
    kz = np.array(k, dtype=np.float64, copy=True)
    kz[..., : cfg.rope_dims] = 0.0
    return round_io(layer_norm(kz, gamma, beta, cfg.ln_eps), cfg.io)


# --------------------------------------------------------------------------- state
@dataclass
class UnitState:
    """Compressed state of one (batch, KV-head) unit.

    sK, sV: running gated sums (rows x d).  rho: radius fixed at row creation.
    w = 1 + sum of gates merged into the row, n = number of tokens in the row and
    members = their positions: diagnostics the layer itself never reads.
    """
    d: int
    sK: np.ndarray = field(default=None)
    sV: np.ndarray = field(default=None)
    rho: np.ndarray = field(default=None)
    w: np.ndarray = field(default=None)
    n: np.ndarray = field(default=None)
    members: List[List[int]] = field(default_factory=list)

    def __post_init__(self):
        if self.sK is None:
            self.sK = np.zeros((0, self.d))
            self.sV = np.zeros((0, self.d))
            self.rho = np.zeros((0,))
            self.w = np.zeros((0,))
            self.n = np.zeros((0,), dtype=np.int64)

    @property
    def m(self) -> int:
        return self.sK.shape[0]

    def append_rows(self, kbar: np.ndarray, v: np.ndarray, positions: Sequence[int]) -> None:
        """New rows take the ungated memory key and value; rho = ||v||_2 (row-wise)."""
        self.sK = np.concatenate([self.sK, kbar], axis=0)
        self.sV = np.concatenate([self.sV, v], axis=0)
        self.rho = np.concatenate([self.rho, np.sqrt((v * v).sum(axis=-1))])
        self.w = np.concatenate([self.w, np.ones(len(positions))])
        self.n = np.concatenate([self.n, np.ones(len(positions), dtype=np.int64)])
        self.members.extend([[int(p)] for p in positions])


def readout(state: UnitState, cfg: KVMConfig, gamma: np.ndarray, beta: np.ndarray
            ) -> Tuple[np.ndarray, np.ndarray]:
    """JIT normalisation ("Readout"): s-hat^K = LN_s(s^K); s-hat^V = rho * s^V / max(||s^V||, eps).

    Both are materialised in the I/O dtype.
    """
    khat = round_io(layer_norm(state.sK, gamma, beta, cfg.ln_eps), cfg.io)
    nrm = np.sqrt((state.sV * state.sV).sum(axis=-1, keepdims=True))
    vhat = round_io(state.rho[:, None] * state.sV / np.maximum(nrm, cfg.norm_eps), cfg.io)
    return khat, vhat


# --------------------------------------------------------------------------- fold
def _argmax_lowest(row: np.ndarray) -> int:
    """Index of the maximum; the lowest index among exact ties (np.argmax does this)."""
    return int(np.argmax(row))


def fold(state: UnitState, k_blk: np.ndarray, v_blk: np.ndarray, g_blk: Optional[np.ndarray],
         e: int, cfg: KVMConfig, gamma: np.ndarray, beta: np.ndarray,
         positions: Optional[Sequence[int]] = None,
         overrides: Optional[Dict[int, int]] = None,
         append_override: Optional[Sequence[int]] = None) -> dict:
    """Fold one overflow block Omega_e into the state ("Append" then "Merge").

    k_blk, v_blk: [n, d] I/O-dtype values (as fp64); g_blk: [n] gates or None (g = 1).
    e: end of the chunk just attended (argument of the budget).
    overrides: {token index in block: slot}.  Only honoured when that slot's score is
    within TIE_MARGIN of the token's best eligible score, otherwise ValueError.
    append_override: the set of tokens to append instead of the oracle's own choice.  Only
    honoured when it has n_append tokens and swaps tokens whose s_j lie within TIE_MARGIN of
    the selection boundary, otherwise ValueError.  Both let a test keep following a run
    after a counted tie; they never change what is correct.

    Returns a log: assign[n] (slot per token; appended tokens get their new row id),
    s_max[n] (append score, or NaN at creation), best[n] and margin[n] (merge score and
    its lead over the runner-up; NaN for appended tokens), n_append, m_before, m_after.
    """
    n_tok, d = k_blk.shape
    S = cfg.n_sink
    if positions is None:
        positions = list(range(n_tok))
    g = np.ones(n_tok) if g_blk is None else np.asarray(g_blk, dtype=np.float64)
    kbar = memory_key(k_blk, cfg, gamma, beta)
    v_blk = np.asarray(v_blk, dtype=np.float64)
    log = dict(m_before=state.m, e=e, assign=np.full(n_tok, -1, dtype=np.int64),
               s_max=np.full(n_tok, np.nan), best=np.full(n_tok, np.nan),
               margin=np.full(n_tok, np.nan), appended=np.zeros(n_tok, dtype=bool))

    if cfg.budget_kind == BUDGET_NONE:
        log.update(n_append=0, m_after=0)
        return log

    # State creation: the first overflow block is copied, ungated, in position order.
    if state.m == 0:
        state.append_rows(kbar, v_blk, positions)
        log["assign"][:] = np.arange(n_tok)
        log["appended"][:] = True
        log.update(n_append=n_tok, m_after=state.m)
        return log

    m = state.m
    # Append: score every overflow token against the *current* normalised state keys.
    khat, _ = readout(state, cfg, gamma, beta)
    sim = kbar @ khat.T                              # [n, m]
    s_max = sim.max(axis=1)
    log["s_max"][:] = s_max
    n_app = n_append_for(cfg, m, e, n_tok)
    # the n_app smallest scores; equal scores -> lower position first
    order = sorted(range(n_tok), key=lambda j: (s_max[j], j))
    chosen = sorted(order[:n_app])
    if append_override is not None and sorted(append_override) != chosen:
        alt = sorted(int(j) for j in append_override)
        if len(alt) != n_app or len(set(alt)) != n_app or n_app == 0 or n_app == n_tok:
            raise ValueError("append override has the wrong size")
        boundary = s_max[order[n_app - 1]]
        swapped = set(alt) ^ set(chosen)
        if any(abs(s_max[j] - boundary) > TIE_MARGIN for j in swapped):
            raise ValueError("append override is not within the tie margin")
        chosen = alt
    if n_app > 0:
        state.append_rows(kbar[chosen], v_blk[chosen], [positions[j] for j in chosen])
        for a, j in enumerate(chosen):
            log["assign"][j] = m + a
            log["appended"][j] = True

    # Merge: remaining tokens pick argmax over rows i >= S of the updated, not yet
    # merged state s_+ (one logits matrix, then one scatter).
    rest = [j for j in range(n_tok) if not log["appended"][j]]
    if rest:
        khat_plus, _ = readout(state, cfg, gamma, beta)
        logits = kbar[rest] @ khat_plus.T            # [n_rest, m + n_app]
        logits[:, :S] = -np.inf
        for row, j in zip(logits, rest):
            i = _argmax_lowest(row)
            top = row[i]
            if row.shape[0] - S > 1:
                second = np.partition(row, -2)[-2]
            else:
                second = -np.inf
            if overrides and j in overrides and overrides[j] != i:
                alt = int(overrides[j])
                if not (S <= alt < row.shape[0]) or top - row[alt] > TIE_MARGIN:
                    raise ValueError(f"override for token {j} -> {alt} is not within the tie margin")
                i = alt
            log["assign"][j] = i
            log["best"][j] = top
            log["margin"][j] = top - second
        for j in rest:                               # scatter-add, ascending position
            i = int(log["assign"][j])
            state.sK[i] += g[j] * kbar[j]
            state.sV[i] += g[j] * v_blk[j]
            state.w[i] += g[j]
            state.n[i] += 1
            state.members[i].append(int(positions[j]))
    log.update(n_append=n_app, m_after=state.m)
    return log


# --------------------------------------------------------------------------- attention
def attend(q: np.ndarray, q_pos: np.ndarray, khat: np.ndarray, vhat: np.ndarray,
           k_win: np.ndarray, v_win: np.ndarray, win_pos: np.ndarray,
           tau_state: np.ndarray, tau_bswa: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """One softmax over [state rows || window tokens] for each query ("Readout").

    q: [G, nq, d]; q_pos: [nq] absolute positions; khat, vhat: [m, d] (m may be 0);
    k_win, v_win: [w, d] with absolute positions win_pos[w]; tau_*: [G].
    logit = tau_state * q.khat_i / sqrt(d) for state rows (always visible) and
            tau_bswa  * q.k_t   / sqrt(d) for window tokens with t <= position of q.
    Returns y [G, nq, d] and the log-sum-exp of the logits [G, nq].
    """
    G, nq, d = q.shape
    m = khat.shape[0]
    y = np.zeros((G, nq, d))
    lse = np.zeros((G, nq))
    visible = win_pos[None, :] <= q_pos[:, None]          # [nq, w]
    for h in range(G):
        ls = tau_state[h] * (q[h] @ khat.T) / math.sqrt(d) if m else np.zeros((nq, 0))
        lw = tau_bswa[h] * (q[h] @ k_win.T) / math.sqrt(d)
        lw = np.where(visible, lw, -np.inf)
        logits = np.concatenate([ls, lw], axis=1)
        mx = logits.max(axis=1, keepdims=True)
        p = np.exp(logits - mx)
        z = p.sum(axis=1, keepdims=True)
        vals = np.concatenate([vhat, v_win], axis=0) if m else v_win
        y[h] = (p / z) @ vals
        lse[h] = (mx + np.log(z))[:, 0]
    return y, lse


# --------------------------------------------------------------------------- the layer, one unit
class KVMUnit:
    """One (batch, KV-head) unit of the layer: its state, its window, its token count.

    prefill() and decode() may be interleaved; a fold happens exactly when a chunk
    completes with e >= L, on the block [e - L, e - L + C).
    """

    def __init__(self, cfg: KVMConfig, n_q_heads: int = 1,
                 gamma: Optional[np.ndarray] = None, beta: Optional[np.ndarray] = None,
                 tau_state: Optional[np.ndarray] = None, tau_bswa: Optional[np.ndarray] = None):
        d = cfg.head_dim
        self.cfg = cfg
        self.G = n_q_heads
        self.gamma = np.ones(d) if gamma is None else np.asarray(gamma, dtype=np.float64)
        self.beta = np.zeros(d) if beta is None else np.asarray(beta, dtype=np.float64)
        self.tau_state = np.ones(n_q_heads) if tau_state is None else np.asarray(tau_state, np.float64)
        self.tau_bswa = np.ones(n_q_heads) if tau_bswa is None else np.asarray(tau_bswa, np.float64)
        self.state = UnitState(d)
        self.t = 0                                 # tokens seen
        # every token's k, v, g is kept here; the window is a view [b, t) of it
        self.k_hist = np.zeros((0, d))
        self.v_hist = np.zeros((0, d))
        self.g_hist = np.zeros((0,))
        self.fold_logs: List[dict] = []
        self.overrides: Dict[Tuple[int, int], int] = {}   # (fold index, token in block) -> slot
        self.append_overrides: Dict[int, Sequence[int]] = {}  # fold index -> appended tokens

    # -- helpers
    def _push(self, k, v, g):
        n = k.shape[0]
        self.k_hist = np.concatenate([self.k_hist, np.asarray(k, np.float64)], axis=0)
        self.v_hist = np.concatenate([self.v_hist, np.asarray(v, np.float64)], axis=0)
        gg = np.ones(n) if g is None else np.asarray(g, np.float64)
        self.g_hist = np.concatenate([self.g_hist, gg])

    def _window_start(self, u: int) -> int:
        C, L = self.cfg.chunk_len, self.cfg.window
        s = (u // C) * C
        return max(0, s + C - L)

    def _attend_rows(self, q_rows: np.ndarray, lo: int, hi: int):
        """Queries at positions [lo, hi) (all inside one chunk) against state + window."""
        b = self._window_start(lo)
        khat, vhat = readout(self.state, self.cfg, self.gamma, self.beta)
        win_pos = np.arange(b, hi)
        return attend(q_rows, np.arange(lo, hi), khat, vhat,
                      self.k_hist[b:hi], self.v_hist[b:hi], win_pos,
                      self.tau_state, self.tau_bswa)

    def _maybe_fold(self):
        C, L = self.cfg.chunk_len, self.cfg.window
        e = self.t
        if e % C != 0 or e < L or self.cfg.budget_kind == BUDGET_NONE:
            return
        lo = e - L
        idx = len(self.fold_logs)
        ov = {j: s for (f, j), s in self.overrides.items() if f == idx} or None
        log = fold(self.state, self.k_hist[lo:lo + C], self.v_hist[lo:lo + C],
                   self.g_hist[lo:lo + C], e, self.cfg, self.gamma, self.beta,
                   positions=list(range(lo, lo + C)), overrides=ov,
                   append_override=self.append_overrides.get(idx))
        self.fold_logs.append(log)

    # -- public
    def prefill(self, q: np.ndarray, k: np.ndarray, v: np.ndarray, g: Optional[np.ndarray] = None):
        """q: [G, T, d]; k, v: [T, d]; g: [T] or None.  The running token count must be a
        multiple of C on entry.  Returns y [G, T, d], lse [G, T]."""
        C = self.cfg.chunk_len
        if self.t % C != 0:
            raise ValueError("prefill must start on a chunk boundary")
        T = k.shape[0]
        t0 = self.t
        self._push(k, v, g)
        y = np.zeros((self.G, T, self.cfg.head_dim))
        lse = np.zeros((self.G, T))
        s = t0
        while s < t0 + T:
            e = min(s + C, t0 + T)
            y[:, s - t0:e - t0], lse[:, s - t0:e - t0] = self._attend_rows(q[:, s - t0:e - t0], s, e)
            self.t = e
            self._maybe_fold()
            s = e
        return y, lse

    def decode(self, q: np.ndarray, k: np.ndarray, v: np.ndarray, g: Optional[float] = None):
        """One token: q [G, d], k, v [d].  Returns y [G, d], lse [G]."""
        self._push(k[None, :], v[None, :], None if g is None else np.array([g]))
        u = self.t
        y, lse = self._attend_rows(q[:, None, :], u, u + 1)
        self.t = u + 1
        self._maybe_fold()
        return y[:, 0], lse[:, 0]


def expected_rows(cfg: KVMConfig, T: int) -> List[int]:
    """State size after each fold of a T-token run, by integer replay of the budget rule."""
    C, L = cfg.chunk_len, cfg.window
    rows, m = [], 0
    e = C
    while e <= T:
        if e >= L and cfg.budget_kind != BUDGET_NONE:
            if m == 0:
                m = C
            else:
                m = max(m, min(budget(cfg, e), m + C))
            rows.append(m)
        e += C
    return rows
