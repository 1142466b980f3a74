"""Reader of the text fixtures under tests/golden/: '#' starts a comment, 'case NAME' opens a
case, every other line is 'key value value ...' (values: numbers, or a/b for a quotient
formed in fp32)."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _num(tok):
    if "/" in tok:
        a, b = tok.split("/")
        return float(np.float32(a) / np.float32(b))
    return float(tok)


def load(name):
    cases, cur = {}, None
    for line in open(os.path.join(GOLDEN, name)):
        line = line.split("#", 1)[0].strip()
        if not line:
            continue
        key, *vals = line.split()
        if key == "case":
            cur = cases.setdefault(vals[0], {})
        else:
            nums = [_num(v) for v in vals]
            cur[key] = nums[0] if len(nums) == 1 and key in ("q", "p", "m", "q1", "q2") else nums
    return cases
