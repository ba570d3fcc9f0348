"""Writes tests/golden/digest_known_answers.json from the CPU oracle alone.

The digest is a definition of this build (the paper defines no hash), so these
values pin later changes of the oracle, not the paper.  Run from the repo root:
    python tests/golden/make_digest_golden.py
"""
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402

CASES = [
    (1, 0, 0, 1), (2, 0, 0, 2), (17, 0, 0, 17), (17, 5, 3, 11), (9, 0, 0, 9), (18, 0, 0, 18),
    (1000, 0, 0, 1000), (4096, 7, 0, 4096), (65537, 12345, 0, 65537),
    (1000003, 0, 500000, 500256), (2**31 - 1, 0, 2**31 - 1 - 4096, 2**31 - 1),
    (2**31 - 1, 0, 0, 4096),
]

items = []
for p, root, a, b in CASES:
    dg, fl = oracle.digest(p, root, a, b, send_mode=1)
    items.append({"p": p, "root": root, "r_begin": a, "r_end": b,
                  "digest": f"{dg:016x}", "flags": fl})
with open(os.path.join(HERE, "digest_known_answers.json"), "w") as fh:
    json.dump({"source": "oracle.digest, send by Algorithm 6", "items": items}, fh, indent=1)
print(f"wrote {len(items)} items")
