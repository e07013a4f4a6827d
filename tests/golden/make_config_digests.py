#!/usr/bin/env python3
"""Writes tests/golden/config<N>_digests.txt from the CPU oracle ONLY (never from the HIP path).

For a full-size configuration the oracle's complete result is too large to store, so the file
holds one 64-bit BLAKE2b digest per block of 4096 consecutive rows, over the bytes of the
int32 neighbour indices followed by the bytes of the float32 squared distances of the block.
The GPU parity test hashes its own output the same way and compares block by block, which
checks every row of the full-size run bit for bit.

    python tests/golden/make_config_digests.py 3 4          # configurations to (re)compute
    python tests/golden/make_config_digests.py 5:0          # configuration 5, row split 0 only

Cost (pair evaluations): config 3 1e11, config 4 2.5e11 (d = 8), config 5 1e12 per row split.
"""
import hashlib
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
import oracle                                              # noqa: E402
from paper_2511_10442_amd import workloads as W             # noqa: E402

BLOCK = 4096


def block_digests(idx: np.ndarray, d2: np.ndarray, block: int = BLOCK):
    out = []
    for b in range(0, idx.shape[0], block):
        h = hashlib.blake2b(digest_size=8)
        h.update(np.ascontiguousarray(idx[b:b + block]).tobytes())
        h.update(np.ascontiguousarray(d2[b:b + block]).tobytes())
        out.append(h.hexdigest())
    return out


def main():
    threads = int(os.environ.get("ORACLE_THREADS", "0"))
    for spec in sys.argv[1:]:
        cfg, _, seg = spec.partition(":")
        cfg = int(cfg)
        w = W.CONFIGS[cfg]()
        t0 = time.time()
        if seg:
            s = int(seg)
            b, e = int(w.row_splits[s]), int(w.row_splits[s + 1])
            idx, d2 = oracle.knn(w.coords[b:e], np.array([0, e - b], dtype=np.int32), w.k, threads)
            idx = np.where(idx >= 0, idx + b, -1).astype(np.int32)
            name, first = "config%d_seg%d_digests.txt" % (cfg, s), b
        else:
            idx, d2 = oracle.knn(w.coords, w.row_splits, w.k, threads)
            name, first = "config%d_digests.txt" % cfg, 0
        dig = block_digests(idx, d2)
        path = os.path.join(ROOT, "tests", "golden", name)
        with open(path, "w") as f:
            f.write("# oracle digests: %s k=%d rows [%d, %d) block=%d blake2b-64(idx bytes + d2 bytes)\n"
                    % (w.name, w.k, first, first + idx.shape[0], BLOCK))
            f.write("# written by tests/golden/make_config_digests.py (CPU oracle only), %.0f s\n" % (time.time() - t0))
            for h in dig:
                f.write(h + "\n")
        print("wrote", path, len(dig), "blocks in %.0f s" % (time.time() - t0), flush=True)


if __name__ == "__main__":
    main()
