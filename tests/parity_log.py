"""Record of measured parity errors (test infrastructure).

Every GPU-vs-oracle comparison appends one row here; at the end of the session the rows are
written as a table to parity_errors.txt in the run's output folder (OUT_DIR below; also printed
with `pytest -s`), so that the measured errors, not only pass/fail, are on record.
"""
import os

ROWS = []
current_test = ""
OUT_DIR = "gpurun_out"      # relative to the repository root

HEADER = "%-78s %-5s %-4s %10s %10s %10s %10s %10s" % (
    "test", "what", "out", "rel_l2", "max_abs", "max|ref|", "abs_tol", "|bnd|/|ref|")


def add(name, out, rel, max_abs, max_ref, tol, bound_ratio=None):
    row = "%-78s %-5s %-4s %10.3e %10.3e %10.3e %10.3e %10s" % (
        current_test[:78], name, out, rel, max_abs, max_ref, tol,
        "-" if bound_ratio is None else "%.3e" % bound_ratio)
    ROWS.append(row)
    print(row, flush=True)


def write():
    if not ROWS:
        return
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    out_dir = os.path.join(root, OUT_DIR)
    try:
        os.makedirs(out_dir, exist_ok=True)
        with open(os.path.join(out_dir, "parity_errors.txt"), "w") as f:
            f.write(HEADER + "\n")
            f.write("\n".join(ROWS) + "\n")
    except OSError:
        pass
