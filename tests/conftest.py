import sys
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir() -> Path:
    return ROOT / "tests" / "golden"


def pytest_terminal_summary(terminalreporter):
    """Report the worst plain relative error any GPU parity assertion of this run has seen."""
    mod = sys.modules.get("gpu_common")
    if mod is not None and mod.WORST_PLAIN_REL["value"] > 0:
        terminalreporter.write_line(
            f"worst plain relative error over all GPU parity assertions: {mod.WORST_PLAIN_REL['value']:.3e} "
            f"({mod.WORST_PLAIN_REL['what']}); bar {mod.PLAIN_REL_TOL:.0e}.  Over outputs not cancelled by more than 8x: "
            f"{mod.WORST_PLAIN_REL['solid']:.3e} ({mod.WORST_PLAIN_REL['solid_what']}); bar {mod.SOLID_REL_TOL:.0e}")
