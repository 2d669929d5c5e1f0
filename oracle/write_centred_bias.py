"""Writes synth/centred_bias.json: the classifier biases of the centred workloads (7-10).

TEST INFRASTRUCTURE: uses the CPU oracle only.  For each centred workload the FP32 model is run
(oracle.forward, binary64) on the workload's first 64 images, the pooled feature entering the
classifier is averaged over those images, and the bias becomes  -W_fc . mean_feature  rounded to
binary32: the classifier's response to what all images have in common is removed, so predictions
spread over the classes.  Values are stored as hexadecimal floats (exact).

    python oracle/write_centred_bias.py            # rewrite the file
    python oracle/write_centred_bias.py --check 7  # recompute one workload and compare with the file
"""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

import oracle  # noqa: E402
import synth  # noqa: E402
from synth import data as synth_data  # noqa: E402


def compute(index):
    wl = synth.make_workload(index, n_images=synth_data.CENTRE_IMAGES, centred=False)
    desc, n = wl["desc"], wl["images"].shape[0]
    r = oracle.forward(desc, wl["weights"], wl["biases"], wl["images"], want_acts=True)
    elems = oracle.node_out_elems(desc)
    fc = desc[-1]
    src = int(fc[9])  # the classifier's input node
    off = sum(elems[:src])
    c, hw = int(fc[1]), int(fc[7]) * int(fc[8])
    pooled = r["acts"][:, off:off + elems[src]].reshape(n, hw, c).mean(axis=1)
    bias = -(wl["weights"][-1].astype(np.float64) @ pooled.mean(axis=0))
    return bias.astype(np.float32)


def main():
    path = synth_data._BIAS_FILE
    if len(sys.argv) >= 3 and sys.argv[1] == "--check":
        idx = int(sys.argv[2])
        ok = compute(idx).tobytes() == synth_data.centred_bias(idx).tobytes()
        print("workload", idx, "matches" if ok else "DIFFERS")
        sys.exit(0 if ok else 1)
    table = {}
    for idx in sorted(synth_data.CENTRED_OF):
        table[str(idx)] = [float(v).hex() for v in compute(idx)]
        print("workload", idx, [round(float(v), 4) for v in compute(idx)], flush=True)
    with open(path, "w") as f:
        json.dump(table, f, indent=1)
        f.write("\n")


if __name__ == "__main__":
    main()
