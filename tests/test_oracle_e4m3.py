"""Pins for the oracle's e4m3 decode: a library conversion of all 256 codes and
the format's published anchor values (tests/golden/e4m3_anchors.txt)."""
import math
import os

import numpy as np
import torch


def test_all_codes_match_library_conversion(oracle):
    codes = torch.arange(256, dtype=torch.uint8)
    lib = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    for c in range(256):
        mine = oracle.e4m3_decode(c)
        if math.isnan(lib[c]):
            assert math.isnan(mine), c
        else:
            assert mine == lib[c], (c, mine, lib[c])
            assert math.copysign(1.0, mine) == math.copysign(1.0, lib[c])


def test_published_anchor_values(oracle):
    path = os.path.join(os.path.dirname(__file__), "golden", "e4m3_anchors.txt")
    n = 0
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        code, val = line.split()
        got = oracle.e4m3_decode(int(code, 16))
        if val == "nan":
            assert math.isnan(got)
        else:
            assert got == float(eval(val)), (code, got)
        n += 1
    assert n >= 8
