import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    import oracle as o
    o.build()
    return o


def pytest_sessionfinish(session, exitstatus):
    """Hand back what the HIP library keeps between layers (buffer cache, pinned cold tier, the
    chunk loader's copy stream) while the HIP runtime is still up: nothing of the library's is
    then alive when the process exits."""
    mod = sys.modules.get("paper_2605_09402_amd")
    if mod is None or getattr(mod, "_lib", None) is None:
        return
    try:
        import torch
        if torch.cuda.is_available():
            torch.cuda.synchronize()
            mod.atlas_release_cache()
    except Exception as exc:   # never turn a finished session into an error
        print("atlas_release_cache at session end:", exc, file=sys.stderr)
