"""The 2^(j/64) table of the acceptance kernels' fp64 exponential holds the doubles nearest to the exact values."""
import os
import re
from decimal import Decimal, getcontext

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2604_09562_amd", "csrc", "accept_common.h")


def test_table_entries_are_correctly_rounded():
    src = open(HEADER).read()
    body = src[src.index("kExp2Sixtyfourths[64] = {"):]
    body = body[body.index("{") + 1:body.index("};")]
    vals = [float.fromhex(x) for x in re.findall(r"0x1\.[0-9a-f]+p[+-]\d+", body)]
    assert len(vals) == 64
    getcontext().prec = 60
    for j, v in enumerate(vals):
        exact = Decimal(2) ** (Decimal(j) / Decimal(64))
        assert v == float(exact), j                      # Decimal -> float rounds to nearest
        assert abs(Decimal(v) - exact) <= Decimal(v) * Decimal(2) ** -53
    assert vals[0] == 1.0 and vals[32] == float(Decimal(2).sqrt())
