import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def _has_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def pytest_collection_modifyitems(config, items):
    if _has_gpu():
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture(scope="session", autouse=True)
def _library_built():
    """Tests load the in-tree libkvm.so; it is compiled here when it does not exist or was built
    from other sources than the tree holds (a digest of the sources is kept beside it), so that a
    stale binary is never tested against new sources."""
    from paper_2605_09877_amd import build
    if build.is_stale():
        build.build()
    yield


def pytest_sessionfinish(session, exitstatus):
    """Parity statistics of the GPU tests that ran (units compared, counted ties by kind, worst
    output error relative to its bar), as one JSON file next to the other GPU-run artefacts."""
    try:
        import kvm_testlib as tl
    except Exception:
        return
    if not tl.PARITY_LOG:
        return
    import json
    out = os.path.join(ROOT, "gpurun_out")
    os.makedirs(out, exist_ok=True)
    total = dict(cases=len(tl.PARITY_LOG), units=sum(r["units"] for r in tl.PARITY_LOG),
                 ties_merge=sum(r["ties_merge"] for r in tl.PARITY_LOG),
                 ties_append=sum(r["ties_append"] for r in tl.PARITY_LOG),
                 max_err=max(r["max_err"] for r in tl.PARITY_LOG))
    with open(os.path.join(out, "parity_stats.json"), "w") as f:
        json.dump(dict(total=total, cases=tl.PARITY_LOG,
                       note="max_err: fp32 max-abs error; bf16 worst row error as a fraction of the "
                            "2e-2 relative bound"), f, indent=1)
    print("\nparity: " + json.dumps(total))
