import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

# the library reads its planner override variables (which the tests use to force every kernel family onto small
# shapes) only if this is set before its first call
os.environ["FLASHRNN_PLAN_OVERRIDES"] = "1"


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
