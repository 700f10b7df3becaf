import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def read_golden(name):
    """Rows of whitespace-separated integers from tests/golden/<name>; '#' starts a comment."""
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if line:
                rows.append([int(t) for t in line.split()])
    return rows


@pytest.fixture(scope="session")
def golden():
    return read_golden


@pytest.fixture(autouse=True, scope="module")
def _release_the_default_workspace_after_each_module():
    """The default context's workspace only grows (a test with T in the paper's slots can leave it at 200 GiB):
    after every GPU test module it is released, and torch's cached blocks with it, so that no module depends on
    what ran before it."""
    yield
    binding = sys.modules.get("paper_2411_02581_amd.binding")
    torch = sys.modules.get("torch")
    if binding is None or torch is None or getattr(binding, "_lib", None) is None or not torch.cuda.is_available():
        return
    torch.cuda.synchronize()
    binding.tuna_release()             # refuses while persistent plans are alive; then nothing is freed
    torch.cuda.empty_cache()
