"""Planted mistakes in the oracle: each one must fail the pin suite.

A copy of oracle/kvm_oracle.py with one line changed (a dropped term, a wrong sign or index, a
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

# (what is broken, text in the oracle, replacement)
MUTANTS = [
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
]


def run_pins_against(tmp, idx):
    what, old, new = MUTANTS[idx]
    src = open(os.path.join(ROOT, "oracle", "kvm_oracle.py")).read()
    assert old in src, f"mutant {idx} ({what}): the oracle no longer contains {old!r}"
    box = os.path.join(tmp, f"m{idx}")
    os.makedirs(os.path.join(box, "oracle"))
    os.makedirs(os.path.join(box, "tests"))
    open(os.path.join(box, "oracle", "__init__.py"), "w").close()
    with open(os.path.join(box, "oracle", "kvm_oracle.py"), "w") as f:
        f.write(src.replace(old, new, 1))
    shutil.copy(os.path.join(ROOT, "tests", "test_oracle_pins.py"), os.path.join(box, "tests"))
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(box, "tests", "golden"))
    env = dict(os.environ, PYTHONPATH=box, OMP_NUM_THREADS="1")
    r = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q",
                        "-p", "no:cacheprovider"], cwd=box, env=env, capture_output=True, text=True)
    return r.returncode, (r.stdout + r.stderr)[-2000:]


@pytest.fixture(scope="module")
def verdicts(tmp_path_factory):
    tmp = str(tmp_path_factory.mktemp("mutants"))
    with ThreadPoolExecutor(max_workers=4) as ex:
        return list(ex.map(lambda i: run_pins_against(tmp, i), range(len(MUTANTS))))


def test_the_unchanged_oracle_passes_in_the_same_harness(tmp_path):
    """The harness itself: the same copy-and-run with nothing changed is green."""
    MUTANTS.append(("nothing", "TIE_MARGIN = 1e-4", "TIE_MARGIN = 1e-4"))
    try:
        rc, out = run_pins_against(str(tmp_path), len(MUTANTS) - 1)
    finally:
        MUTANTS.pop()
    assert rc == 0, out


@pytest.mark.parametrize("idx", range(len(MUTANTS)), ids=[m[0] for m in MUTANTS])
def test_planted_mistake_fails_a_pin(verdicts, idx):
    rc, out = verdicts[idx]
    assert rc == 1, f"mutant survived (or the run broke, rc={rc}): {MUTANTS[idx][0]}\n{out}"
