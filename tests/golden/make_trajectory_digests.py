#!/usr/bin/env python3
"""Writes tests/golden/trajectory_digests.json from the CPU oracle alone.

For every workload the oracle runs the whole seeded trajectory (mask of the current state,
the (draw mod popcount)-th allowed token, advance) for the stated number of steps and the
tokens and states of every 64-step block are hashed.  The GPU parity test regenerates the
trajectory with the HIP library's own masks and must reproduce every digest.

    python tests/golden/make_trajectory_digests.py [config ...]
"""
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import wg_synth as ws                    # noqa: E402
from oracle import oracle as O           # noqa: E402

OUT = os.path.join(ROOT, "tests", "golden", "trajectory_digests.json")
BLOCK = 64


def block_digests(tokens, states):
    out = []
    for lo in range(0, len(tokens), BLOCK):
        h = hashlib.sha256()
        h.update(np.ascontiguousarray(tokens[lo:lo + BLOCK], dtype="<i4").tobytes())
        h.update(np.ascontiguousarray(states[lo:lo + BLOCK], dtype="<u4").tobytes())
        out.append(h.hexdigest()[:16])
    return out


def main():
    which = [int(a) for a in sys.argv[1:]] or [2, 3, 4, 5]
    data = {}
    if os.path.exists(OUT):
        with open(OUT) as f:
            data = json.load(f)
    for idx in which:
        w = ws.make_workload(idx)
        ov = O.OracleVocab(w.vocab.bytes, w.vocab.offsets, w.vocab.eos_id)
        o = O.Oracle(w.texts, w.args, ov, restart=True)
        start = np.array([[o.start_state(int(t)), 0] for t in w.request_template], dtype=np.uint32)
        t0 = time.time()
        toks, sts, n_masks = o.trajectory(start, w.token_draws())
        data[str(idx)] = {"steps": w.steps, "B": w.B, "V": w.vocab.V, "block": BLOCK,
                          "distinct_masks": n_masks, "errors": int((sts[:, :, 0] == O.SID_ERROR).sum()),
                          "digests": block_digests(toks, sts)}
        print("config %d: %d steps, %d masks, %.1f s" % (idx, w.steps, n_masks, time.time() - t0), flush=True)
        with open(OUT, "w") as f:
            json.dump(data, f, indent=0, sort_keys=True)


if __name__ == "__main__":
    main()
