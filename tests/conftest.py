import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionfinish(session, exitstatus):
    """After a run that compared GPU results with the oracle: write the worst error per
    workload and tensor class to gpurun_out/parity_errors.txt (the tracked copy lives in
    profiles/)."""
    try:
        from tests import parity_util
    except Exception:
        return
    if not parity_util.RECORD:
        return
    out = os.path.join(ROOT, "gpurun_out")
    os.makedirs(out, exist_ok=True)
    lines = ["# worst error per workload and tensor class over every comparison of this pytest run",
             "# (HIP library through the C ABI against the CPU fp64 oracle, storage-model mode for bf16 workloads)",
             "# command: python -m pytest tests -m gpu   exit status: %s" % int(exitstatus),
             "# columns: workload | tensor class | worst l2-relative | worst max-norm relative | l2 bar"]
    for wl in sorted(parity_util.RECORD):
        for cls, (e2, em, bar) in sorted(parity_util.RECORD[wl].items()):
            lines.append(f"{wl} | {cls} | {e2:.3e} | {em:.3e} | {bar:.3e}")
    with open(os.path.join(out, "parity_errors.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")
