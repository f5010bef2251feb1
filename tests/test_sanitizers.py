"""The CPU sanitizer mode: the oracle and the host side of the C ABI under AddressSanitizer and
UndefinedBehaviorSanitizer (see tests/sanitize/build_and_run.py).  No GPU is used."""
import importlib.util
import os
import shutil

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
spec = importlib.util.spec_from_file_location("sanitize_build_and_run", os.path.join(HERE, "sanitize", "build_and_run.py"))
sanitize = importlib.util.module_from_spec(spec)
spec.loader.exec_module(sanitize)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not found")
def test_oracle_runs_clean_under_asan_and_ubsan():
    rc, out = sanitize.oracle()
    assert rc == 0 and "oracle sanitize: ok" in out, out[-3000:]


@pytest.mark.skipif(not os.path.exists(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")), reason="hipcc not found")
def test_host_argument_checks_run_clean_under_asan_and_ubsan():
    rc, out = sanitize.abi()
    assert rc == 0 and "abi sanitize: ok" in out, out[-3000:]
