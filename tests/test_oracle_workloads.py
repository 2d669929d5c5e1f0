"""The centred workloads (7-10) give the agreement metric something to measure.

With the plain recipe the FP32 model predicts one class for every image and every candidate scheme
agrees with it everywhere; the centred workloads exist so that top-1, near-tie and agreement
checks carry information.  These tests run the oracle only.
"""
import os
import subprocess
import sys

import numpy as np

import oracle
import synth
from synth import data as synth_data

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_stored_bias_is_what_the_oracle_script_computes():
    # workload 7 (ResNet-20) is recomputed here; the others take minutes and are covered by the
    # script's own --check mode
    r = subprocess.run([sys.executable, os.path.join(ROOT, "oracle", "write_centred_bias.py"), "--check", "7"],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    for idx, base in synth_data.CENTRED_OF.items():
        b = synth_data.centred_bias(idx)
        assert b.shape == (10,) and b.dtype == np.float32 and np.isfinite(b).all()


def test_centred_workloads_differ_from_their_originals_only_in_seed_and_bias():
    for idx, base in synth_data.CENTRED_OF.items():
        a = synth.make_workload(idx, n_images=2)
        b = synth.make_workload(base, n_images=2)
        raw = synth.make_workload(idx, n_images=2, centred=False)
        assert a["name"] == b["name"] + "_centred" and a["index"] == idx
        np.testing.assert_array_equal(a["desc"], b["desc"])
        assert a["schemes"].shape == b["schemes"].shape
        assert not np.array_equal(a["weights"][0], b["weights"][0])  # own seed
        for l in range(len(a["weights"])):
            np.testing.assert_array_equal(a["weights"][l], raw["weights"][l])
        for l in range(len(a["biases"]) - 1):
            np.testing.assert_array_equal(a["biases"][l], raw["biases"][l])
        np.testing.assert_array_equal(a["biases"][-1], synth_data.centred_bias(idx))


def test_resnet20_centred_predictions_spread_and_schemes_flip_some():
    n = 64
    wl = synth.make_workload(7, n_images=n)
    L = wl["L"]
    rows = [wl["schemes"][[1, 11, 26, 27, 39]], np.full((1, L), 8, np.uint8), np.full((1, L), 32, np.uint8)]
    schemes = np.concatenate(rows)
    r = oracle.eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], schemes, want_logits=False)
    hist = np.bincount(r["top1_base"], minlength=10)
    assert (hist > 0).sum() >= 5, hist
    assert hist.max() <= n // 2, hist
    agree = r["agree"]
    assert agree[-1] == n                       # the all-FP32 scheme agrees with itself
    assert ((agree > 0) & (agree < n)).sum() >= 4, agree
    assert len(set(agree.tolist())) >= 4, agree  # agreement varies across schemes
    # the same model with the drawn classifier bias is the degenerate case this workload replaces
    raw = synth.make_workload(7, n_images=16, centred=False)
    r0 = oracle.forward(raw["desc"], raw["weights"], raw["biases"], raw["images"])
    assert len(set(r0["top1"].tolist())) == 1
