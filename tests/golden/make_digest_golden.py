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

# The huge streamed instance in full: p = 2^31 - 1, root 0, every rank, in the 32 chunks of 2^26
# ranks the library is driven with (a few minutes of oracle time on eight cores; `--streamed`).
# The digest and the sums of the edge check of every chunk, and their XOR over the instance.
if "--streamed" in sys.argv:
    p, chunk = 2**31 - 1, 2**26
    chunks, whole, whole_fl, xr_all, xs_all = [], 0, 0, 0, 0
    for a in range(0, p, chunk):
        b = min(a + chunk, p)
        dg, fl = oracle.digest(p, 0, a, b, send_mode=1)
        xr, xs = oracle.edgecheck(p, 0, a, b, send_mode=1)
        chunks.append({"r_begin": a, "r_end": b, "digest": f"{dg:016x}", "flags": fl,
                       "edge_recv": f"{xr:016x}", "edge_send": f"{xs:016x}"})
        whole ^= dg
        whole_fl |= fl
        xr_all ^= xr
        xs_all ^= xs
        print(f"chunk {len(chunks)}/32 {dg:016x}", flush=True)
    with open(os.path.join(HERE, "streamed_chunk_digests.json"), "w") as fh:
        json.dump({"source": "oracle.digest and oracle.edgecheck, send by Algorithm 6",
                   "p": p, "root": 0, "chunk": chunk, "digest": f"{whole:016x}", "flags": whole_fl,
                   "edge_recv": f"{xr_all:016x}", "edge_send": f"{xs_all:016x}",
                   "chunks": chunks}, fh, indent=1)
    print(f"wrote 32 chunks, whole digest {whole:016x}")
