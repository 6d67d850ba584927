"""Runs after the other GPU tests (pytest collects files in alphabetical order): the rate of
2nd-moment code flips over every code the session compared, and the report of their margins."""
import pytest

import parity_common as pc

pytestmark = pytest.mark.gpu


def test_flip_rate_over_all_compared_codes():
    counted, largest = pc.write_flip_report()
    print(f"\n2nd-moment codes compared: {pc.CODES_COMPARED[0]}; flips: {len(pc.FLIP_LOG)}, of them "
          f"{counted} in well-conditioned blocks (largest margin {largest:.3g}, bound {pc.FLIP_MARGIN:g})")
    for line in pc.NOTES:
        print(line)
    if pc.CODES_COMPARED[0] == 0:
        pytest.skip("no parity test ran in this session")
    assert largest < pc.FLIP_MARGIN
    assert counted <= max(1.0, pc.FLIP_RATE * pc.CODES_COMPARED[0])
