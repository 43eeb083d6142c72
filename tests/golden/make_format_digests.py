#!/usr/bin/env python3
"""Writes tests/golden/format_digests.txt: SHA-256 of the serialised form of a few seeded tensors, as the
reference codec (oracle/) produces it.  Calls only oracle/ and the input generators.  Re-run it only when the
serialised format is changed on purpose (the format version in the header changes with it)."""
import hashlib
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import oracle as zo                      # noqa: E402
from paper_2601_21198_amd import synth               # noqa: E402

CASES = [("gauss", 20000, 4096, 4096, 8), ("gauss", 3 * 16384 + 77, 16384, 4096, 8), ("wide", 9000, 4096, 1024, 12),
         ("uniform_u16", 5000, 4096, 2048, 8), ("rare_last", 4097, 2048, 512, 8), ("all_equal", 513, 512, 512, 8)]


def digests():
    for kind, n, C, W, max_len in CASES:
        w = synth.special_tensor(kind, n, seed=1)
        blob, _ = zo.encode_tensor(w, C, W, max_len)
        yield f"{kind} {n} {C} {W} {max_len} {zo.header(blob)['version']} {blob.size} {hashlib.sha256(blob.tobytes()).hexdigest()}"


if __name__ == "__main__":
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "format_digests.txt"), "w") as f:
        f.write("# kind n chunk_values stream_values max_len format_version blob_bytes sha256 -- written by make_format_digests.py (reference codec only)\n")
        for line in digests():
            f.write(line + "\n")
