import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_runtest_logstart(nodeid, location):
    # One unbuffered line per test on the real stderr (pytest captures the tests' own output and, into a file or a
    # pipe, buffers its progress dots): a harness that watches for output sees each test start, and a hang names its test.
    sys.__stderr__.write(f"[{time.strftime('%H:%M:%S')}] {nodeid}\n")
    sys.__stderr__.flush()
