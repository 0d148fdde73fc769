#!/usr/bin/env python3
"""Writes tests/golden/synth_digest.json: what the seeded workload generator produces for c0 .. c4.

The benchmark and the full-size parity tests run on these partitions; the digest pins them, so that a change to
the generator (or to numpy's random streams) shows up as a failed test instead of as a silently different
workload.  Calls only paper_2306_01381_amd.synth (which holds none of the method's arithmetic).
Run from the repository root:  python tests/golden/make_synth_digest.py
"""
import hashlib
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2306_01381_amd.synth import CONFIGS, make_partition  # noqa: E402

ARRAYS = ("rowptr", "col", "val", "feat", "send_idx", "peer_of_slot", "bits", "halo_idx")


def digest(p) -> dict:
    """Sizes, an order-sensitive column checksum and one SHA-256 per array of a partition."""
    col64 = p.col.astype(np.int64)
    weights = (np.arange(col64.shape[0], dtype=np.int64) % 65521) + 1
    out = {
        "n_rows": int(p.n_rows), "n_cols": int(p.n_cols), "nnz": int(p.nnz), "n_central": int(p.n_central),
        "n_send": int(p.send_idx.shape[0]),
        "col_sum": int(col64.sum()),
        "col_weighted_sum_mod_2_61": int((col64 * weights % (2 ** 61 - 1)).sum() % (2 ** 61 - 1)),
        "max_row": int(np.diff(p.rowptr).max()),
        "bits_count_2_4_8": [int((p.bits == b).sum()) for b in (2, 4, 8)],
    }
    for name in ARRAYS:
        out["sha256_" + name] = hashlib.sha256(np.ascontiguousarray(getattr(p, name)).tobytes()).hexdigest()
    return out


def main() -> None:
    result = {"numpy": np.__version__}
    for name in ("c0", "c1", "c2", "c3", "c4", "c1m"):
        result[name] = digest(make_partition(CONFIGS[name]))
        print(name, result[name]["nnz"], flush=True)
    with open(os.path.join(HERE, "synth_digest.json"), "w") as f:
        json.dump(result, f, indent=1, sort_keys=True)
        f.write("\n")


if __name__ == "__main__":
    main()
