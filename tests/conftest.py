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
    L.mi355env_tune_paged_stores(2)
    L.mi355env_tune_pixels(0, 0)
    L.mi355env_tune_frame_trajectory(2)
    L.mi355env_tune_plane_path(2)
