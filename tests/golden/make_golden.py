"""Writes tests/golden/uniform_bits.json from the CPU oracle only.

The values freeze the counter-based generator that supplies the draws of
Alg. 2 line 9 ("+1 with probability p_j"), so that an accidental change of the
mixing function is caught.  Run:  python tests/golden/make_golden.py
"""
import json
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
import oracle  # noqa: E402

cases = [(0, 0, 0), (0, 0, 1), (1, 0, 0), (0, 1, 0), (0x250207861001, 64 * 3 + 1, 511),
         (2**64 - 1, 2**40 + 7, 2**33 + 5), (42, 7, 1023), (42, 7, 1024)]
vals = [dict(seed=s, stream=t, ctr=c, bits=oracle.uniform_bits(s, t, c)) for s, t, c in cases]
out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "uniform_bits.json")
with open(out, "w") as f:
    json.dump(dict(source="oracle.uniform_bits (two rounds of the SplitMix64 mixer, top 24 bits)",
                   values=vals), f, indent=1)
print("wrote", out)
