#!/usr/bin/env python3
"""Writes tests/golden/datagen_fingerprints.txt: fingerprints of the synthetic inputs, so that a test can tell
that the recipe still yields the same arrays on any device.  Calls only `datagen`.

    python tests/golden/write_datagen_fingerprints.py [--device cuda] [--full]

Without --full only the small cases are written (they run anywhere in seconds); with --full also the edge
count and id sum of the five benchmark workloads at full size (needs a GPU with room for the largest).
Lines of workloads that are not regenerated are kept as they are.
"""
import argparse
import hashlib
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
import datagen  # noqa: E402

OUT = os.path.join(HERE, "datagen_fingerprints.txt")
SMALL = [("tiny", 1.0), ("mid", 0.05), ("wide", 0.002), ("large", 0.0002), ("share", 0.0001)]


def digest(*arrays) -> str:
    m = hashlib.sha256()
    for a in arrays:
        m.update(np.ascontiguousarray(a).tobytes())
    return m.hexdigest()[:16]


def small_spec(name: str, scale: float):
    spec = datagen.WORKLOADS[name]
    return spec if scale == 1.0 else datagen.scaled(spec, scale)


def id_sum(indices: np.ndarray) -> int:
    total = 0
    for lo in range(0, indices.size, 1 << 26):
        total += int(indices[lo:lo + (1 << 26)].sum(dtype=np.int64))
    return total


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--device", default="cpu")
    ap.add_argument("--full", action="store_true")
    args = ap.parse_args()
    lines = {}
    if os.path.exists(OUT):
        for line in open(OUT):
            if line.strip() and not line.startswith("#"):
                lines[line.split()[0]] = line.rstrip("\n")
    for name, scale in SMALL:
        spec = small_spec(name, scale)
        indptr, indices = datagen.make_graph(spec, device=args.device)
        feats = datagen.make_features(spec, device=args.device)
        tablet = datagen.make_tablet(spec, device=args.device)
        key = f"small:{name}@{scale:g}"
        lines[key] = f"{key} E={indices.size} graph={digest(indptr, indices)} features={digest(feats)} tablet={digest(tablet)}"
        print(lines[key], flush=True)
    if args.full:
        for name in ("tiny", "mid", "wide", "large", "share"):
            spec = datagen.WORKLOADS[name]
            indptr, indices = datagen.make_graph(spec, device=args.device)
            key = f"full:{name}"
            lines[key] = f"{key} E={indices.size} id_sum={id_sum(indices)} last_offset={int(indptr[-1])}"
            print(lines[key], flush=True)
            del indptr, indices
    with open(OUT, "w") as f:
        f.write("# Fingerprints of the synthetic inputs (written by write_datagen_fingerprints.py; not paper values).\n"
                "# small:<workload>@<scale>: first 16 hex digits of SHA-256 over the arrays' bytes.\n"
                "# full:<workload>: edge count, sum of all column ids, last row offset at full size.\n")
        for key in sorted(lines):
            f.write(lines[key] + "\n")


if __name__ == "__main__":
    main()
