"""Runs CPU test files against instrumented builds of the two native libraries.

usage: run_checked.py <libotf build> <oracle build> <test file>...

The HIP library's binding and the oracle's ctypes front each load a shared library from a path
they hold in a module attribute; this script points both at builds compiled with
-fsanitize=undefined in trap mode (no runtime library, so they load into an ordinary interpreter;
undefined behaviour ends the process with SIGILL) and then runs pytest on the named files in this
process.  TEST INFRASTRUCTURE ONLY."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)


def main(argv):
    libotf, liboracle, files = argv[1], argv[2], argv[3:]
    from paper_1407_4764_amd import binding
    from oracle import otf_oracle
    binding.LIB_PATH = libotf
    otf_oracle._LIB = liboracle                      # newer than the source: build() leaves it alone
    import pytest
    rc = pytest.main(["-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"] + files)
    loaded = open("/proc/self/maps").read()
    for path in (libotf, liboracle):
        if os.path.realpath(path) not in loaded:
            print("the tests never loaded %s" % path)
            return 3
    return int(rc)


if __name__ == "__main__":
    sys.exit(main(sys.argv))
