"""Runs tests/host_sanitizers.py (the oracle and the host side of the C ABI under AddressSanitizer and
UndefinedBehaviorSanitizer) when KLA_RUN_SANITIZERS=1: it recompiles the library, which takes a minute."""
import os
import subprocess
import sys

import pytest


@pytest.mark.skipif(os.environ.get("KLA_RUN_SANITIZERS") != "1", reason="set KLA_RUN_SANITIZERS=1 to run (recompiles the library)")
def test_host_sanitizers():
    here = os.path.dirname(os.path.abspath(__file__))
    subprocess.check_call([sys.executable, os.path.join(here, "host_sanitizers.py")])
