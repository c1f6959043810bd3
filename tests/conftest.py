import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
# streams beyond HIP's hardware queues per process (four by default) share a queue with another stream and take
# turns with it; the test process keeps many streams alive over its run, so the limit is raised well above them
os.environ["GPU_MAX_HW_QUEUES"] = str(max(32, int(os.environ.get("GPU_MAX_HW_QUEUES") or 0)))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_sessionstart(session):
    """Tests load the library that is built; only if none is there it is built first."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    if not os.path.exists(os.path.join(root, "paper_2509_11076_amd", "libss.so")):
        from paper_2509_11076_amd.build import build_library
        build_library(verbose=False)
