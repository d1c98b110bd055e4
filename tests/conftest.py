import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


from paper_2406_10707_amd import build as _build_lib  # noqa: E402

_build_lib.ensure_built()      # loads what is built; rebuilds only a missing or outdated library


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")
