"""Comparison rules shared by the GPU parity tests (no arithmetic of the method itself)."""
import numpy as np

LOGIT_REL_TOL = 1e-3   # max relative error on logits
NEAR_TIE = 1e-5        # relative top-1 margin under which the GPU may pick the other class


def logits_rel_error(z_gpu, z_ref):
    """max |z_gpu - z_ref| / max(|z_ref|, 1e-2 * max_j |z_ref[.., j]|): the floor keeps logits that
    happen to be near zero from dominating."""
    z_ref = np.asarray(z_ref, dtype=np.float64)
    z_gpu = np.asarray(z_gpu, dtype=np.float64)
    floor = 1e-2 * np.abs(z_ref).max(axis=-1, keepdims=True)
    return float((np.abs(z_gpu - z_ref) / np.maximum(np.abs(z_ref), np.maximum(floor, 1e-30))).max())


def near_tied(z_ref):
    """bool [...]: the two largest reference logits are closer than NEAR_TIE * max|z|."""
    z = np.sort(np.asarray(z_ref, dtype=np.float64), axis=-1)
    margin = z[..., -1] - z[..., -2]
    return margin < NEAR_TIE * np.maximum(np.abs(z_ref).max(axis=-1), 1e-30)


def check_eval(gpu, ref, n_images):
    """gpu / ref: dicts with logits [S][N][C], top1 [S][N], agree [S], top1_base [N], logits_base (ref)."""
    err = logits_rel_error(gpu["logits"], ref["logits"])
    assert err <= LOGIT_REL_TOL, f"logit relative error {err:.3e}"
    tie_base = near_tied(ref["logits_base"])
    diff_base = gpu["top1_base"] != ref["top1_base"]
    assert not (diff_base & ~tie_base).any(), "base top-1 differs on a clear margin"
    tie = near_tied(ref["logits"])
    diff = gpu["top1"] != ref["top1"]
    assert not (diff & ~tie).any(), "top-1 differs on a clear margin"
    slack = (tie | tie_base[None, :]).sum(axis=1)
    assert (np.abs(gpu["agree"].astype(np.int64) - ref["agree"]) <= slack).all(), (gpu["agree"], ref["agree"])
    # the GPU's own count is consistent with its own top-1
    np.testing.assert_array_equal(gpu["agree"], (gpu["top1"] == gpu["top1_base"][None, :]).sum(axis=1))
    assert (gpu["agree"] <= n_images).all() and (gpu["agree"] >= 0).all()
    return err


def check_centred_sample(gpu, ref, idx, fc_bias):
    """Parity on a centred workload (classifier bias = minus the classifier's response to the mean feature).

    There every logit is a small difference z = r + b of the classifier's response r and a bias of about
    the same size (|r| is 15-20 times |z|), and fp32 rounding errors scale with r, not with z.  So:
      * the response r = z - b is held to the logit bar (1e-3 max relative error) - the quantity that
        bar bounds on the benchmark workloads, where the bias is negligible;
      * the GPU's top-1 must be exactly the argmax (lowest index on ties) of the GPU's own logits: the
        integer decision, taken in the kernel's precision;
      * against the oracle, top-1 may differ only where the oracle's margin is below twice the largest
        logit deviation seen in this comparison (each of two logits can move by that much), and such
        samples must stay rare; agreement counts may differ by the number of such samples.
    gpu: logits [S][N][C], top1 [S][N], top1_base [N], agree [S] (all images); ref: the oracle on images idx.
    Returns (relative error of the response, agreement counts on the sample, exempt fraction)."""
    b = np.asarray(fc_bias, dtype=np.float64)
    zg = np.asarray(gpu["logits"][:, idx], dtype=np.float64)
    zr = np.asarray(ref["logits"], dtype=np.float64)
    err = logits_rel_error(zg - b, zr - b)
    assert err <= LOGIT_REL_TOL, f"classifier response relative error {err:.3e}"
    # the kernel's own decision: first maximum of its fp32 logits
    np.testing.assert_array_equal(gpu["top1"], np.asarray(gpu["logits"]).argmax(axis=-1))
    dev = float(np.abs(zg - zr).max())
    srt = np.sort(zr, axis=-1)
    exempt = (srt[..., -1] - srt[..., -2]) <= 2.0 * dev
    sb = np.sort(np.asarray(ref["logits_base"], dtype=np.float64), axis=-1)
    exempt_base = (sb[..., -1] - sb[..., -2]) <= 2.0 * dev
    assert not ((gpu["top1"][:, idx] != ref["top1"]) & ~exempt).any(), "top-1 differs on a clear margin"
    assert not ((gpu["top1_base"][idx] != ref["top1_base"]) & ~exempt_base).any(), "base top-1 differs on a clear margin"
    frac = float((exempt | exempt_base[None, :]).mean())
    assert frac <= 0.05, f"{frac:.3f} of the samples lie within the logit deviation of a tie"
    agree_sample = (gpu["top1"][:, idx] == gpu["top1_base"][idx][None]).sum(axis=1)
    slack = (exempt | exempt_base[None, :]).sum(axis=1)
    assert (np.abs(agree_sample - ref["agree"]) <= slack).all(), (agree_sample, ref["agree"], slack)
    np.testing.assert_array_equal(gpu["agree"], (gpu["top1"] == gpu["top1_base"][None]).sum(axis=1))
    return err, agree_sample, frac
