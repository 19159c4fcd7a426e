import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """Load the HIP library if it is built; build it only if nothing is built and a selected
    test needs it (the GPU tests and the boundary checks of test_abi.py).  The oracle's pins
    import nothing of the product and run on a machine without hipcc."""
    needs = any(it.get_closest_marker("gpu") is not None or it.fspath.basename == "test_abi.py" for it in items)
    if needs:
        import __graft_entry__
        __graft_entry__.ensure_built()
