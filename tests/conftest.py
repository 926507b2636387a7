import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def have_gpu() -> bool:
    import torch
    return torch.cuda.is_available()


def pytest_terminal_summary(terminalreporter):
    """Parity statistics of the GPU tests (largest errors, how many streams were compared exactly, how many
    decisions fell inside the stated tie / threshold margins), printed even in quiet runs."""
    parity = sys.modules.get("parity")
    if parity is None or not getattr(parity, "STATS_LOG", None):
        return
    terminalreporter.section("GPU parity statistics")
    for tag, stats in parity.STATS_LOG:
        shown = {k: (float(f"{v:.3g}") if isinstance(v, float) else v) for k, v in stats.items()}
        if "alpha_err" not in stats:          # WISV rounds: exemption counts always shown, zero included
            shown.setdefault("exempt_tie", 0)
            shown.setdefault("exempt_tau", 0)
        terminalreporter.write_line(f"{tag}: {shown}")
