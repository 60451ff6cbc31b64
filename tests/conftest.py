import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
for p in (ROOT, os.path.join(ROOT, "oracle"), os.path.dirname(os.path.abspath(__file__))):
    if p not in sys.path:
        sys.path.insert(0, p)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except Exception:
        has_gpu = False
    if has_gpu:
        return
    skip = pytest.mark.skip(reason="no GPU in this environment")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture(autouse=True)
def _oracle_progress(request, capsys):
    """The oracle's prompt pass over thousands of rows at 7B / 13B width takes minutes on the host
    cores: print a line every 20 s past pytest's capture, so that a watcher sees the run is alive."""
    if "gpu" not in request.keywords:
        yield
        return
    import time

    import pass_oracle as O
    last = [time.time()]

    def tick(done, total):
        if time.time() - last[0] >= 20.0:
            last[0] = time.time()
            with capsys.disabled():
                print(f"\n[{request.node.name}] oracle prompt pass {done}/{total} rows", flush=True)

    O.set_progress(tick)
    yield
    O.set_progress(None)
