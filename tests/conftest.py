import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionfinish(session, exitstatus):
    """Per-tensor parity table of the GPU layer tests that ran in this session (error, floor, verdict), written where a GPU
    run's results are collected: parity_table.md holds every tensor, parity_summary.md one line per case plus every tensor
    that is not simply within tolerance (the committed copy of the latter is profiles/parity.md)."""
    try:
        from tests import layer_harness as LH
    except Exception:
        return
    rows = LH.PARITY_ROWS
    if not rows:
        return
    out = os.path.join(ROOT, "gpurun_out")
    os.makedirs(out, exist_ok=True)
    head = ("| case | tensor | max err / rms(ref) | rms-relative err | tolerance | floor: max err / rms(ref) | floor: rms-relative err | verdict |\n"
            "|---|---|---|---|---|---|---|---|\n")
    line = lambda case, name, e, r, tol, fl, fr, verdict: (
        f"| {case} | {name} | {e:.4f} | {r:.5f} | {tol:g} | {'' if fl is None else f'{fl:.4f}'} | {'' if fr is None else f'{fr:.5f}'} | {verdict} |\n")
    with open(os.path.join(out, "parity_table.md"), "w") as f:
        f.write(head)
        for row in rows:
            f.write(line(*row))
    cases = {}
    for row in rows:
        cases.setdefault(row[0], []).append(row)
    with open(os.path.join(out, "parity_summary.md"), "w") as f:
        f.write("| case | tensors | within tolerance | format-limited | failed | largest error / tolerance | largest rms-relative error |\n|---|---|---|---|---|---|---|\n")
        for case, rs in cases.items():
            n = lambda v: sum(1 for r in rs if r[7] == v)
            f.write(f"| {case} | {len(rs)} | {n('ok')} | {n('FORMAT-LIMITED')} | {n('FAIL')} | {max(r[2] / r[4] for r in rs):.2f} | {max(r[3] for r in rs):.5f} |\n")
        f.write("\nTensors beyond the tolerance (format-limited or failed):\n\n" + head)
        for row in rows:
            if row[7] != "ok":
                f.write(line(*row))
