"""The host-only sources (exact construction and point discovery of the library, the oracle's C loops) built
with AddressSanitizer + UndefinedBehaviorSanitizer and walked through by their self-test programs.
CPU only; about twenty seconds, most of it compilation."""
from paper_2512_18453_amd import build


def test_host_sources_are_clean_under_address_and_undefined_behaviour_sanitizers():
    out = build.sanitize_selftest()
    assert out[0].endswith("host_selftest: ok"), out
    assert out[1].startswith("conv_oracle_selftest: ok"), out
