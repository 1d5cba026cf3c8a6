import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")


@pytest.fixture(autouse=True)
def _admission_counter_matches_slots(request, monkeypatch):
    """Every counter read-back of a GPU test also checks the device's admission counter (the figure the
    load-factor limit bounds) against live + deleted slots."""
    if request.node.get_closest_marker("gpu") is None:
        yield
        return
    from paper_2505_12663_amd import EmbeddingTable
    plain = EmbeddingTable.stats

    def checked(self):
        st = plain(self)
        assert st["occupied"] == st["live"] + st["tombstones"], st
        return st

    monkeypatch.setattr(EmbeddingTable, "stats", checked)
    yield
