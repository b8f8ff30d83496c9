import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def legal_blocks():
    """The legal 4x4 block masks, found independently of the oracle: filter all
    65536 uint16 encodings (bit 4i+j = m_ij) for two ones per row and column,
    then sort by the 16-character row-major string with '0' < '1'."""
    def key(enc):
        return "".join("1" if (enc >> t) & 1 else "0" for t in range(16))

    out = []
    for enc in range(1 << 16):
        rows = [bin((enc >> (4 * i)) & 0xF).count("1") for i in range(4)]
        cols = [bin(enc & (0x1111 << j)).count("1") for j in range(4)]
        if rows == [2] * 4 and cols == [2] * 4:
            out.append(enc)
    out.sort(key=key)
    return out
