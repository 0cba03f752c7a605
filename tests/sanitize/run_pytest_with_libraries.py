"""Runs pytest on the given files with the package bound to another build of the C-ABI library and
the oracle bound to another build of its C code (the sanitizer builds of tests/test_sanitized_host.py).

    python run_pytest_with_libraries.py <libtaper_attn.so> <libtaper_oracle.so> <pytest arguments...>
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from paper_2605_06914_amd import binding  # noqa: E402

binding.LIB_PATH = os.path.abspath(sys.argv[1])
import oracle.oracle as oracle_front  # noqa: E402

oracle_front._LIB = os.path.abspath(sys.argv[2])
oracle_front.build = lambda force=False: oracle_front._LIB  # (already built, with other flags)

import pytest  # noqa: E402

rc = pytest.main(sys.argv[3:])
mapped = sorted({line.split()[-1] for line in open("/proc/self/maps") if line.rstrip().endswith(".so") and "taper" in line})
print("libraries mapped:", " ".join(mapped))
sys.exit(rc)
