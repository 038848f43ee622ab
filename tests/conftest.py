import os
import sys

import torch  # noqa: F401  -- before anything loads libtcx.so: torch must bring up its own HIP runtime first

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


import __graft_entry__  # noqa: E402

__graft_entry__.ensure_built()          # a fresh checkout has no library yet; an existing one is loaded as it is


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
