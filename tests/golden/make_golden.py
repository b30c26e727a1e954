"""Writes tests/golden/tiny512_oracle.json: what the CPU checker computes for the `tiny512`
workload (seeded weights and prompt, schedule {2: 700, 3: 500}).

The paper prints no worked values, so this is a regression fixture, not a paper value: it freezes
the checker's answer so that a later edit of its arithmetic shows up as a diff.  It calls only
`oracle/` and the seeded input generators; nothing here comes from the HIP path.

    python tests/golden/make_golden.py
"""
import hashlib
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import lazyllm_oracle as O                      # noqa: E402
from paper_2407_14057_amd import synth                      # noqa: E402


def compute():
    wl = synth.WORKLOADS["tiny512"]
    shape = wl.shape
    w = synth.weights_to_host_bits(synth.make_weights(shape, wl.weight_seed, "cpu"))
    inp = synth.make_workload_inputs(wl)
    res = O.prefill(shape.as_dict(), w, inp["token_ids"], list(wl.schedule), dtype=np.float64)
    out = {
        "workload": "tiny512",
        "citation": "Sec. 3.2 (progressive token pruning, Eq. 1); regression fixture, not a paper value",
        "n_per_layer": [int(p.shape[0]) for p in res.kept_pos],
        "kept_pos_sha256": [hashlib.sha256(p.astype(np.int64).tobytes()).hexdigest() for p in res.kept_pos],
        "kept_pos_layer3_head": [int(x) for x in res.kept_pos[3][:16]],
        "aux_counts": {str(l): int(p.shape[0]) for l, p in sorted(res.aux_pos.items())},
        "scores_layer1_first8": [float(x) for x in res.scores[1][:8]],
        "scores_layer3_last4": [float(x) for x in res.scores[3][-4:]],
        "logits_argmax": int(np.argmax(res.logits)),
        "logits_first8": [float(x) for x in res.logits[:8]],
        "logits_sum": float(res.logits.sum()),
    }
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny512_oracle.json")
    with open(path, "w") as f:
        json.dump(compute(), f, indent=1)
        f.write("\n")
    print("wrote", path)
