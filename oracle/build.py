"""Compile the CPU oracle (plain C, gcc) into oracle/libmw_oracle.so.

Test infrastructure only: run by the test suite, the smoke check and the
build step; nothing in the product path depends on it.
"""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "mw_oracle.c")
LIB = os.path.join(HERE, "libmw_oracle.so")


def sanitizers() -> str:
    """ORACLE_SANITIZE=1: the oracle built with AddressSanitizer and UndefinedBehaviorSanitizer
    (-O1 -g), as a library of its own; ORACLE_SANITIZE=<list> names the sanitizers (e.g.
    "undefined", which needs no preloaded runtime).  A process that loads the address-sanitized
    library must start with the sanitizer's runtime preloaded (see README)."""
    v = os.environ.get("ORACLE_SANITIZE", "").strip()
    if v in ("", "0"):
        return ""
    return "address,undefined" if v == "1" else v


def build(force: bool = False) -> str:
    san = sanitizers()
    lib = LIB if not san else os.path.join(HERE, "libmw_oracle_san.so")
    if (not force and not san and os.path.exists(lib)
            and os.path.getmtime(lib) >= os.path.getmtime(SRC)):
        return lib
    opt = ["-O2"] if not san else ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=" + san,
                                   "-fno-sanitize-recover=undefined"]
    tmp = lib + ".tmp%d" % os.getpid()
    subprocess.check_call(["gcc", "-std=c99"] + opt + ["-Wall", "-Wextra", "-fPIC", "-shared",
                           "-ffp-contract=off", SRC, "-o", tmp, "-lm"])
    os.replace(tmp, lib)
    return lib


if __name__ == "__main__":
    print(build(force=True))
