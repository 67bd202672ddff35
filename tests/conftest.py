import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_terminal_summary(terminalreporter):
    """Measured parity errors of the run: the comparisons closest to their bars on the terminal, every
    comparison in the file $MTNLG_PARITY_LOG names (tab-separated)."""
    try:
        from parity import RECORDS
    except ImportError:
        return
    RECORDS = [r for r in RECORDS if "planted_mistake" not in r[0]]   # those comparisons are meant to fail
    if not RECORDS:
        return
    path = os.environ.get("MTNLG_PARITY_LOG")
    if path:
        with open(path, "w") as f:
            f.write("test\ttensor\trel_fro\ttol\telementwise_ratio\telements\n")
            for r in RECORDS:
                f.write("%s\t%s\t%.3e\t%.1e\t%.3f\t%d\n" % r)
    tr = terminalreporter
    tr.section("parity: comparisons closest to their bars (of %d)" % len(RECORDS))
    worst = sorted(RECORDS, key=lambda r: -max(r[2] / r[3], r[4] if r[4] == r[4] else 0.0))[:12]
    for test, what, err, tol, ratio, n in worst:
        tr.write_line("%-28s rel_fro %.2e (bar %.0e)  element %.2f of allowance  %s" %
                      (what[:28], err, tol, ratio, test.split("::")[-1][:60]))
