"""CPU sanitizer leg: the oracle and the host side of the C ABI layer under AddressSanitizer
and UndefinedBehaviorSanitizer.  Both are built as stand-alone executables (a sanitized shared
library cannot be loaded into an unsanitized Python), run here on the CPU, and must finish
without a single report.  The same two commands by hand:
    python -m oracle.build --sanitize
    python -m paper_2505_19602_amd.build --sanitize
"""
from oracle import build as oracle_build
from paper_2505_19602_amd import build as hip_build


def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers():
    out = oracle_build.run_sanitized()
    assert "oracle sanitizer run complete" in out


def test_abi_host_layer_is_clean_under_address_and_undefined_behaviour_sanitizers():
    out = hip_build.run_sanitized()
    assert "0 failed expectations" in out
