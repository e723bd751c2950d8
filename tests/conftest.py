import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    config.addinivalue_line("markers", "slow: full-size parity case whose oracle leg takes minutes of CPU time")


def pytest_terminal_summary(terminalreporter):
    """Largest per-row relative error any bf16 / 4-bit parity check of this run saw (the bar is helpers.BF16_ROW_REL_L2)."""
    try:
        import helpers
    except ImportError:
        return
    for dtype, worst in sorted(helpers.WORST_ROW.items()):
        for err, what, index, shape in worst:
            terminalreporter.write_line(f"worst rows of the parity checks, {dtype} stage: rel-L2 {err:.3e} "
                                        f"at row {index} of {shape} ({what})")
