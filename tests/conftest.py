import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionfinish(session, exitstatus):
    """After a session with GPU parity comparisons: one summary per configuration in the session's output folder (what
    was compared, what mismatched, how many residual masses lie outside 1e-5 relative)."""
    try:
        from tests import parity
    except Exception:
        return
    if not parity.RECORDS:
        return
    out_dir = os.path.join(ROOT, os.environ.get("SPECVERIFY_TEST_OUTPUT", "gpurun_out"))
    os.makedirs(out_dir, exist_ok=True)
    groups = {}
    for rep in parity.RECORDS:
        label = rep.get("label", "")
        cfg = label.split("/", 1)[0]
        if not cfg.startswith("cfg"):
            continue
        key = "/".join(p for p in label.split("/")[1:] if not p.startswith(("seed", "call")))
        groups.setdefault(cfg, {}).setdefault(key, []).append(rep)
    for cfg, rows in groups.items():
        lines = ["GPU path against the CPU oracle, " + cfg + ": written by tests/conftest.py at the end of "
                 "`python -m pytest tests -m gpu -q` (every comparison of that session, summed over seeds / calls)",
                 "tolerances: tau, Y exact unless a uniform lies within %g of a decision boundary (excused, counted); "
                 "|dS| <= %g S + %g w" % (parity.MARGIN, parity.S_RTOL, parity.S_FLOOR), "",
                 "%-34s %9s %8s %8s %8s %10s %9s %12s %12s %12s %8s" % (
                     "case", "sequences", "tau_miss", "Y_miss", "excused", "unexcused", "S_rows",
                     "S_out_1e-5", "max_dS/w", "max_w_rel", "mean_tau")]
        for key in sorted(rows):
            reps = rows[key]
            n = sum(r["n"] for r in reps)
            lines.append("%-34s %9d %8d %8d %8d %10d %9d %12d %12.2e %12.2e %8.3f" % (
                key or "-", n, sum(r["tau_mismatch"] for r in reps), sum(r["y_mismatch"] for r in reps),
                sum(r["excused"] for r in reps), sum(r["unexcused"] for r in reps),
                sum(r["S_rows"] for r in reps), sum(r["S_rows_outside_1e-5_rel"] for r in reps),
                max(r["max_dS_over_w"] for r in reps), max(r["max_w_rel_err"] for r in reps),
                sum(r["mean_tau"] * r["n"] for r in reps) / max(n, 1)))
        with open(os.path.join(out_dir, "parity_%s.txt" % cfg), "w") as f:
            f.write("\n".join(lines) + "\n")
