// Host-only entry points: status text and the pattern table.
#include "s24_common.h"

extern "C" const char *s24_strerror(int status)
{
    switch (status) {
    case S24_OK: return "ok";
    case S24_ERR_NULL: return "a required pointer is NULL";
    case S24_ERR_SHAPE: return "bad shape: negative size or not a multiple of the required granularity";
    case S24_ERR_DTYPE: return "unknown dtype or activation";
    case S24_ERR_ALIGN: return "pointer or leading dimension not aligned as required";
    case S24_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
    case S24_ERR_UNSUPPORTED: return "not implemented for these arguments";
    default: return "unknown status";
    }
}

// Sec. 5.1 step 1.  A legal block is four rows, each one of the six rows with
// two ones, whose columns also sum to two.  Rows compare as strings
// m_i0 m_i1 m_i2 m_i3, so in bit encoding (bit j = m_ij) the ascending row
// order is 1100b, 1010b, 0110b, 1001b, 0101b, 0011b; iterating the four rows
// as nested digits in that order yields the blocks in pattern-id order.
extern "C" int s24_pattern_table(uint16_t out[S24_NUM_PATTERNS])
{
    S24_REQUIRE(out != nullptr, S24_ERR_NULL);
    static const unsigned kRows[6] = {0xC, 0xA, 0x6, 0x9, 0x5, 0x3};
    int n = 0;
    for (int a = 0; a < 6; ++a)
        for (int b = 0; b < 6; ++b)
            for (int c = 0; c < 6; ++c)
                for (int d = 0; d < 6; ++d) {
                    unsigned rows[4] = {kRows[a], kRows[b], kRows[c], kRows[d]};
                    bool ok = true;
                    for (int j = 0; j < 4 && ok; ++j) {
                        int s = 0;
                        for (int i = 0; i < 4; ++i) s += (rows[i] >> j) & 1u;
                        ok = (s == 2);
                    }
                    if (!ok) continue;
                    if (n < S24_NUM_PATTERNS)
                        out[n] = (uint16_t)(rows[0] | rows[1] << 4 | rows[2] << 8 | rows[3] << 12);
                    ++n;
                }
    return n == S24_NUM_PATTERNS ? S24_OK : S24_ERR_UNSUPPORTED;
}
