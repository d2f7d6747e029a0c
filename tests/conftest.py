import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_addoption(parser):
    parser.addoption("--artopk-option", action="append", default=[], metavar="NAME=VALUE",
                     help="route switch applied to every context the GPU tests create unless a test sets its own "
                          "(guess_min_n, update_tiles_min_n, leader_first, nontemporal, stage_tiles); the routes "
                          "give identical results, so the suite may be run on any of them (its checks of which route ran "
                          "are then off)")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")
    for item in config.getoption("--artopk-option"):
        from tests import gpu_util

        name, value = item.split("=", 1)
        if name not in gpu_util._OPTION_KEYS:
            raise pytest.UsageError(f"--artopk-option: unknown switch {name!r}")
        gpu_util.OPTIONS[name] = int(value)
        gpu_util.FORCED.add(name)
