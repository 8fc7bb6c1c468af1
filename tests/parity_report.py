"""Turns the error record of a GPU test session (gpurun_out/parity_errors.json, written by tests/conftest.py) into
the markdown table of the design doc: per workload and output, the worst measured figures.

    python tests/parity_report.py [path/to/parity_errors.json]
"""
import collections
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def family(case: str) -> str:
    """Workload a test case belongs to (the case labels of tests/test_gpu_*.py)."""
    head = case.split(" ")[0]
    for key in ("480p", "720p", "train55k", "train56k", "stress", "mid"):
        if head.startswith(key):
            return key
    return "small grids (tiny, ragged, variants)"


def main():
    path = sys.argv[1] if len(sys.argv) > 1 else os.path.join(ROOT, "gpurun_out", "parity_errors.json")
    recs = json.load(open(path))
    groups = collections.defaultdict(list)
    for r in recs:
        groups[(r["dtype"], family(r["case"]), r["output"])].append(r)
    order = {"O": 0, "LSE": 1, "dQ": 2, "dK": 3, "dV": 4}
    print(f"{len(recs)} checked outputs in {path}\n")
    print("| dtype | workload | output | checks | values compared | worst max-abs err | at max\\|ref\\| | worst err where \\|ref\\| ≤ 1 "
          "| worst element ratio | worst rel. Frobenius | rule asserted |")
    print("|---|---|---|---|---|---|---|---|---|---|---|")
    for key in sorted(groups, key=lambda k: (k[0], k[1], order.get(k[2], 9))):
        v = groups[key]
        w = max(v, key=lambda r: r["max_abs_err"])
        rules = sorted({r.get("rule", "max-abs tol") for r in v})
        print("| %s | %s | %s | %d | %.3g | %.2e | %.2f | %s | %s | %.1e | %s |" % (
            key[0], key[1], key[2], len(v), sum(r["n_values"] for r in v), w["max_abs_err"], w["max_abs_ref"],
            "%.2e" % max(r.get("max_abs_err_where_ref_le_1", 0.0) for r in v) if key[2] != "LSE" else "–",
            "%.2f" % max(r.get("worst_elementwise_ratio", 0.0) for r in v) if key[2] != "LSE" else "–",
            max(r["rel_frobenius"] for r in v), "; ".join(rules)))


if __name__ == "__main__":
    main()
