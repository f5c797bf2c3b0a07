"""Runs the oracle's pins and the planner's tests against builds made with CPU sanitizers.
Started by tests/test_sanitizers.py in a process of its own (the address sanitizer's runtime has to be
loaded before everything else):  python sanitized_runner.py <oracle.so> <planner.so>"""
import ctypes
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(HERE))
sys.path.insert(0, HERE)

import pytest  # noqa: E402

import oracle  # noqa: E402
from paper_2512_17910_amd import planner  # noqa: E402


def main() -> int:
    o = ctypes.CDLL(sys.argv[1])
    o.oracle_num_threads.restype = ctypes.c_int
    oracle._lib = o
    planner.use_planner_library(ctypes.CDLL(sys.argv[2]))
    return int(pytest.main(["-x", "-q", "-p", "no:cacheprovider", os.path.join(HERE, "test_oracle_pins.py"),
                            os.path.join(HERE, "test_planner_pins.py")]))


if __name__ == "__main__":
    sys.exit(main())
