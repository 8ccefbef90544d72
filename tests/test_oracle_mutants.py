"""Planted mistakes in the oracle: each one must fail the pin suite.

A copy of an oracle file (the forward, its backward pass, the weight preparation) with one line changed (a dropped term, a wrong sign or index, a
missing rounding, a check removed) is put in a scratch directory together with the pin tests,
and the pins are run against it in a child process.  A mutant that survives means the pins do
not fix that part of the oracle.  Everything here runs on the CPU.
"""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# (what is broken, text in the oracle, replacement); the file and the pins that must catch it are
# attached below
FORWARD = [
    ("sinks become merge targets", "logits[:, :S] = -np.inf", "pass"),
    ("gate dropped from the key sum", "state.sK[i] += g[j] * kbar[j]", "state.sK[i] += kbar[j]"),
    ("gate dropped from the value sum", "state.sV[i] += g[j] * v_blk[j]", "state.sV[i] += v_blk[j]"),
    ("rotary channels not zeroed", "kz[..., : cfg.rope_dims] = 0.0", "pass"),
    ("most similar tokens appended", "key=lambda j: (s_max[j], j))", "key=lambda j: (-s_max[j], j))"),
    ("window mask lets two future tokens in", "win_pos[None, :] <= q_pos[:, None]",
     "win_pos[None, :] < q_pos[:, None] + 2"),
    ("state logits take the window temperature", "ls = tau_state[h]", "ls = tau_bswa[h]"),
    ("window logits not divided by sqrt(d)", "lw = tau_bswa[h] * (q[h] @ k_win.T) / math.sqrt(d)",
     "lw = tau_bswa[h] * (q[h] @ k_win.T)"),
    ("radius not applied to the value readout", "vhat = round_io(state.rho[:, None] * state.sV",
     "vhat = round_io(state.sV"),
    ("window starts a block early", "return max(0, s + C - L)", "return max(0, s - L)"),
    ("wrong block folded", "lo = e - L\n", "lo = e - L + C\n"),
    ("merge scored against the state before the append",
     "khat_plus, _ = readout(state, cfg, gamma, beta)", "khat_plus = khat"),
    ("state may shrink below its rows", "m_star = max(m, min(budget(cfg, e), m + cfg.chunk_len))",
     "m_star = min(budget(cfg, e), m + cfg.chunk_len)"),
    ("budget taken at the start of the chunk", "return int(math.floor(cfg.budget_scale * ceil_sqrt(e)))",
     "return int(math.floor(cfg.budget_scale * ceil_sqrt(e - cfg.chunk_len)))"),
    ("appended rows are gated", "state.append_rows(kbar[chosen], v_blk[chosen]",
     "state.append_rows(kbar[chosen]*g[chosen][:,None], v_blk[chosen]"),
    ("unbiased variance in LN_s", "var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)",
     "var = ((x - mu) ** 2).sum(axis=-1, keepdims=True)/(x.shape[-1]-1)"),
    ("key readout not rounded to the I/O dtype",
     "khat = round_io(layer_norm(state.sK, gamma, beta, cfg.ln_eps), cfg.io)",
     "khat = layer_norm(state.sK, gamma, beta, cfg.ln_eps)"),
    ("state keys not normalised", "khat = round_io(layer_norm(state.sK, gamma, beta, cfg.ln_eps), cfg.io)",
     "khat = round_io(state.sK, cfg.io)"),
    ("append override accepted at any distance",
     "if any(abs(s_max[j] - boundary) > TIE_MARGIN for j in swapped):", "if False:"),
    ("append override margin measured from the smallest score",
     "boundary = s_max[order[n_app - 1]]", "boundary = s_max[order[0]]"),
    ("append override of any size accepted",
     "if len(alt) != n_app or len(set(alt)) != n_app or n_app == 0 or n_app == n_tok:", "if False:"),
    ("append override ignored", "        chosen = alt\n", "        pass\n"),
    ("merge override accepted at any distance",
     "if not (S <= alt < row.shape[0]) or top - row[alt] > TIE_MARGIN:", "if not (S <= alt < row.shape[0]):"),
    ("merge override ignored", "                i = alt\n", "                pass\n"),
    ("radius follows the merged values", "state.sV[i] += g[j] * v_blk[j]",
     "state.sV[i] += g[j] * v_blk[j]; state.rho[i] = np.sqrt((state.sV[i] ** 2).sum())"),
    ("append score skips the sink rows", "s_max = sim.max(axis=1)", "s_max = sim[:, S:].max(axis=1)"),
    ("softmax without the window's values", "vals = np.concatenate([vhat, v_win], axis=0) if m else v_win",
     "vals = np.concatenate([vhat, 0 * v_win], axis=0) if m else v_win"),
    ("state logits not divided by sqrt(d)", "ls = tau_state[h] * (q[h] @ khat.T) / math.sqrt(d) if m",
     "ls = tau_state[h] * (q[h] @ khat.T) if m"),
    ("log-sum-exp without the maximum", "lse[h] = (mx + np.log(z))[:, 0]", "lse[h] = np.log(z)[:, 0]"),
    ("a query sees its own successor", "visible = win_pos[None, :] <= q_pos[:, None]",
     "visible = win_pos[None, :] <= q_pos[:, None] + 1"),
    ("a query does not see itself", "visible = win_pos[None, :] <= q_pos[:, None]",
     "visible = win_pos[None, :] < q_pos[:, None]"),
    ("square-root budget rounds down", "return math.isqrt(e - 1) + 1", "return math.isqrt(e)"),
    ("LN_s epsilon outside the root", "return (x - mu) / np.sqrt(var + eps) * gamma + beta",
     "return (x - mu) / (np.sqrt(var) + eps) * gamma + beta"),
    ("LN_s bias dropped", "return (x - mu) / np.sqrt(var + eps) * gamma + beta",
     "return (x - mu) / np.sqrt(var + eps) * gamma"),
    ("value readout divides by the squared norm", "nrm = np.sqrt((state.sV * state.sV).sum(axis=-1, keepdims=True))",
     "nrm = (state.sV * state.sV).sum(axis=-1, keepdims=True)"),
    ("bf16 rounding truncates", "u = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)",
     "u = u & np.uint64(0xFFFF0000)"),
    ("bf16 ties round away from zero", "u = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)",
     "u = (u + np.uint64(0x8000)) & np.uint64(0xFFFF0000)"),
]

BACKWARD = [
    ("radius gradient dropped from the creator's value", "dv[t] += dsV[i] + (drho[i] * v[t] / nv if nv > 0.0 else 0.0)",
     "dv[t] += dsV[i]"),
    ("value term dropped from the gate gradient", "dg[t] += float(dsK[i] @ kbar[j]) + float(dsV[i] @ v[t])",
     "dg[t] += float(dsK[i] @ kbar[j])"),
    ("key term dropped from the gate gradient", "dg[t] += float(dsK[i] @ kbar[j]) + float(dsV[i] @ v[t])",
     "dg[t] += float(dsV[i] @ v[t])"),
    ("rotary channels receive a memory-key gradient", "dkz[:, : cfg.rope_dims] = 0.0", "pass"),
    ("gate factor missing on a merged key", "dkbar[j] = gates[t] * dsK[i]", "dkbar[j] = dsK[i]"),
    ("gate factor missing on a merged value", "dv[t] += gates[t] * dsV[i]", "dv[t] += dsV[i]"),
    ("creator's key gradient gated", "dkbar[j] = dsK[i]\n", "dkbar[j] = gates[t] * dsK[i]\n"),
    ("rows of the undone fold keep their adjoint", "dsK, dsV, drho = dsK[:m0], dsV[:m0], drho[:m0]",
     "dsK, dsV, drho = dsK[:m0], dsV[:m0] * 0 + dsV[:m0], drho[:m0] * 2"),
    ("softmax term D dropped", "dlogit = p * (dy[h] @ v_win.T - delta)", "dlogit = p * (dy[h] @ v_win.T)"),
    ("state logits' temperature missing from dq", "dq[h] += tau_state[h] * scale * (dlogit @ khat)",
     "dq[h] += scale * (dlogit @ khat)"),
    ("window temperature gradient takes scaled logits", "dtb[h] = (dlogit * raw).sum()",
     "dtb[h] = (dlogit * raw * tau_bswa[h]).sum()"),
    ("LayerNorm backward without the projection on x-hat",
     "          - xhat * (dxhat * xhat).mean(axis=-1, keepdims=True)) / sigma", "          ) / sigma"),
    ("LayerNorm backward without the mean term", "dx = (dxhat - dxhat.mean(axis=-1, keepdims=True)", "dx = (dxhat"),
    ("value readout backward without the norm's own derivative",
     "live = nrm > eps", "live = nrm > np.inf"),
    ("radius adjoint dropped from the readout", "drho = drho + r_drho", "drho = drho"),
    ("LN_s parameter gradient of the readout dropped", "            dgamma += dga\n            dbeta += dbe\n\n    return",
     "            pass\n\n    return"),
    ("window key gradient transposed operand", "dk_win += tau_bswa[h] * scale * (dlogit.T @ q[h])",
     "dk_win += tau_bswa[h] * scale * (dlogit.T @ dy[h])"),
    ("state value gradient without probabilities", "dvhat += p.T @ dy[h]", "dvhat += (p > 0).T @ dy[h]"),
]

PREP = [
    ("value residual weights swapped", "return (1.0 - lam)[None] * v + lam[None] * v_first",
     "return lam[None] * v + (1.0 - lam)[None] * v_first"),
    ("token shift looks ahead", "out[1:] = a[1:] + alpha[None] * (a[:-1] - a[1:])",
     "out[:-1] = a[:-1] + alpha[None] * (a[1:] - a[:-1])"),
    ("token shift sign", "out[1:] = a[1:] + alpha[None] * (a[:-1] - a[1:])", "out[1:] = a[1:] - alpha[None] * (a[:-1] - a[1:])"),
    ("continued call ignores the previous row", "out[0] = a[0] + alpha * (prev - a[0])", "pass"),
    ("rotation pairs adjacent channels", "x1, x2 = x[..., :half], x[..., half:r]",
     "x1, x2 = x[..., 0:r:2], x[..., 1:r:2]"),
    ("rotation sign", "out[..., :half] = x1 * cos - x2 * sin", "out[..., :half] = x1 * cos + x2 * sin"),
    ("rotation frequency exponent", "base ** (-2.0 * c / r)", "base ** (-1.0 * c / r)"),
    ("gate without the offset", "return 1.0 + np.where(z > 0.0, z, np.expm1(np.minimum(z, 0.0)))",
     "return np.where(z > 0.0, z, np.expm1(np.minimum(z, 0.0)))"),
    ("gate's negative branch linear", "np.expm1(np.minimum(z, 0.0))", "np.minimum(z, 0.0)"),
    ("shift applied before the value residual", "    v = value_residual(v_raw, v_first, lam)\n    q = token_shift(q_raw, alpha_q, prev_q)\n"
     "    k = token_shift(k_raw, alpha_k, prev_k)\n    v = token_shift(v, alpha_v, prev_v)\n",
     "    q = token_shift(q_raw, alpha_q, prev_q)\n    k = token_shift(k_raw, alpha_k, prev_k)\n"
     "    v = value_residual(token_shift(v_raw, alpha_v, prev_v), v_first, lam)\n"),
    ("rotation before the normalisation", "q = rope_r(layer_norm_heads(q, lnq[0], lnq[1], eps), pos, r, base)",
     "q = layer_norm_heads(rope_r(q, pos, r, base), lnq[0], lnq[1], eps)"),
    ("unbiased variance in LN_q / LN_k", "var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)",
     "var = ((x - mu) ** 2).sum(axis=-1, keepdims=True) / (x.shape[-1] - 1)"),
]

# (oracle file, the pin file that must catch its mutants)
MUTANTS = ([(m, "kvm_oracle.py", "test_oracle_pins.py") for m in FORWARD]
           + [(m, "kvm_backward_oracle.py", "test_backward_pins.py") for m in BACKWARD]
           + [(m, "prep_oracle.py", "test_prep_pins.py") for m in PREP])


def run_pins_against(tmp, idx):
    (what, old, new), oracle_file, pin_file = MUTANTS[idx]
    box = os.path.join(tmp, f"m{idx}")
    os.makedirs(os.path.join(box, "tests"))
    shutil.copytree(os.path.join(ROOT, "oracle"), os.path.join(box, "oracle"),
                    ignore=shutil.ignore_patterns("__pycache__", "*.so", "*.o"))
    src = open(os.path.join(ROOT, "oracle", oracle_file)).read()
    assert old in src, f"mutant {idx} ({what}): {oracle_file} no longer contains {old!r}"
    with open(os.path.join(box, "oracle", oracle_file), "w") as f:
        f.write(src.replace(old, new, 1))
    shutil.copy(os.path.join(ROOT, "tests", pin_file), os.path.join(box, "tests"))
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(box, "tests", "golden"))
    env = dict(os.environ, PYTHONPATH=box, OMP_NUM_THREADS="1")
    r = subprocess.run([sys.executable, "-m", "pytest", "tests/" + pin_file, "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=box, env=env, capture_output=True, text=True)
    return r.returncode, (r.stdout + r.stderr)[-2000:]


@pytest.fixture(scope="module")
def verdicts(tmp_path_factory):
    tmp = str(tmp_path_factory.mktemp("mutants"))
    with ThreadPoolExecutor(max_workers=4) as ex:
        return list(ex.map(lambda i: run_pins_against(tmp, i), range(len(MUTANTS))))


@pytest.mark.parametrize("oracle_file,pin_file", [("kvm_oracle.py", "test_oracle_pins.py"),
                                                  ("kvm_backward_oracle.py", "test_backward_pins.py"),
                                                  ("prep_oracle.py", "test_prep_pins.py")])
def test_the_unchanged_oracle_passes_in_the_same_harness(tmp_path, oracle_file, pin_file):
    """The harness itself: the same copy-and-run with nothing changed is green."""
    MUTANTS.append((("nothing", "import", "import"), oracle_file, pin_file))
    try:
        rc, out = run_pins_against(str(tmp_path), len(MUTANTS) - 1)
    finally:
        MUTANTS.pop()
    assert rc == 0, out


@pytest.mark.parametrize("idx", range(len(MUTANTS)), ids=[f"{m[1][:-3]}: {m[0][0]}" for m in MUTANTS])
def test_planted_mistake_fails_a_pin(verdicts, idx):
    rc, out = verdicts[idx]
    assert rc == 1, f"mutant survived (or the run broke, rc={rc}): {MUTANTS[idx][0][0]}\n{out}"
