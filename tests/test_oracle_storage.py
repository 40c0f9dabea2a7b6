"""Oracle storage accounting against the values the paper prints (tests/golden/equivalent_bits.txt)."""
import os

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "equivalent_bits.txt")


def _rows():
    with open(GOLD) as f:
        for line in f:
            line = line.split("#")[0].split()
            if line:
                yield int(line[0]), int(line[1]), int(line[2]), float(line[3])


def test_equivalent_bits_match_paper():
    rows = list(_rows())
    assert len(rows) == 4
    for s, s_n, d_h, bits in rows:
        assert oracle.equivalent_bits(d_h, s, s_n) == bits
        # ratio form printed in the same section: d_h / (2 s s_n)
        assert oracle.compression_ratio(d_h, s, s_n) == d_h / (2.0 * s * s_n)
        # fp16 coefficient + 16-bit index per pair
        assert oracle.code_bytes(s, s_n) * 8 == bits * d_h


def test_value_cache_setting_same_bits():
    # CSR-8: keys s=8,s_n=1 and values s=4,s_n=2 occupy the same space (Experiments Settings, "CSR").
    assert oracle.equivalent_bits(128, 8, 1) == oracle.equivalent_bits(128, 4, 2) == 2.0
