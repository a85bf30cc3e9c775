"""Compile the C++ oracle into ``oracle/libwd_oracle.so`` with the host compiler.

TEST INFRASTRUCTURE ONLY.  Run as ``python -m oracle.build``.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = [os.path.join(HERE, "wd_oracle.cpp"), os.path.join(HERE, "wdc_oracle.cpp")]
HEADERS = [os.path.join(HERE, "wd_oracle.h"), os.path.join(HERE, "wdc_oracle.h")]
LIBRARY = os.path.join(HERE, "libwd_oracle.so")


def build(force: bool = True) -> str:
    """Compile the oracle; returns the path of the shared library."""
    if not force and os.path.exists(LIBRARY) and os.path.getmtime(LIBRARY) >= max(
        os.path.getmtime(f) for f in SOURCES + HEADERS
    ):
        return LIBRARY
    cmd = [
        os.environ.get("CXX", "g++"), "-O2", "-std=c++17", "-fPIC", "-shared",
        "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
        "-o", LIBRARY + ".tmp", *SOURCES,
    ]
    subprocess.run(cmd, check=True)
    os.replace(LIBRARY + ".tmp", LIBRARY)
    return LIBRARY


if __name__ == "__main__":
    print(build())
    sys.exit(0)
