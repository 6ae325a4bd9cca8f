import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


import pytest


@pytest.fixture(autouse=True)
def _default_tuning(request):
    """The library's measurement knobs are process-wide: whatever a GPU test sets is put back to the
    defaults when the test ends, also when it fails half-way."""
    yield
    if request.node.get_closest_marker("gpu") is None:
        return
    from paper_2603_12145_amd import binding as b
    L = b.lib()
    L.mi355env_tune_rollout(0, 1)
    L.mi355env_tune_rollout_chunk(0)
    L.mi355env_tune_rollout_split(0)
    L.mi355env_tune_rollout_pace(0)
    L.mi355env_tune_measure_pace(1)
    L.mi355env_tune_cartpole_split(0)
    L.mi355env_tune_step_kernel(1)
    L.mi355env_tune_paged_stores(2)
    L.mi355env_tune_pixels(0, 0)
    L.mi355env_tune_frame_trajectory(2)
    L.mi355env_tune_plane_path(2)


@pytest.fixture
def l3_report(request):
    """Collects one row per workload of the level-3 rollout comparison; the rows are printed as one
    table at the end of the session (below), whether or not output capture is on."""
    rows = request.config.__dict__.setdefault("_l3_rows", [])
    return rows.append


def pytest_terminal_summary(terminalreporter, exitstatus, config):
    rows = getattr(config, "_l3_rows", None)
    if not rows:
        return
    tr = terminalreporter
    tr.section("level-3 rollout comparison: HIP path vs CPU oracle, matched seeds and actions")
    head = ("workload", "mode", "episodes", "env-steps", "max error", "result")
    table = [head] + [tuple(str(r[k]) for k in head) for r in rows]
    width = [max(len(row[c]) for row in table) for c in range(len(head))]
    for row in table:
        tr.write_line("  ".join(cell.ljust(w) for cell, w in zip(row, width)))
