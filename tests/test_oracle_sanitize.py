"""Host sanitizer run of the C oracle: dream_oracle.c + oracle/selftest.c built as one executable under
AddressSanitizer and UBSan (gcc), every entry point called on exact-size heap buffers.  No GPU involved."""
import shutil

import pytest

import oracle


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
def test_selftest_is_clean_under_address_and_ub_sanitizers():
    r = oracle.build_sanitized(run_selftest=True)   # raises with the sanitizer report if anything fires
    assert "oracle selftest ok" in r["selftest_output"]
