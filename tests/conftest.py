import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs the HIP path through the C-ABI)")


def pytest_collection_modifyitems(config, items):
    """GPU tests are skipped when no device is visible, so a plain `pytest tests` works anywhere."""
    try:
        import torch
        have_gpu = torch.cuda.is_available()
    except Exception:
        have_gpu = False
    if have_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU visible")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture(autouse=True, scope="session")
def _guard_words_checked_when_a_job_closes():
    """Every job a test closes first has its guard words counted (adore_check_guards): 0 damaged, or -1 when the job
    was laid out without them.  With ADORE_GUARD_WORDS=1 in the environment the whole GPU suite runs on the debug
    layout and any kernel that writes past the end of a workspace region fails the test that ran it."""
    from paper_2407_02328_amd import binding
    plain_close = binding.Adore.close

    def close(self):
        if getattr(self, "handle", None):
            damaged = self.check_guards()
            assert damaged <= 0, f"{damaged} guard words of the workspace were overwritten"
        plain_close(self)

    binding.Adore.close = close
    yield
    binding.Adore.close = plain_close
