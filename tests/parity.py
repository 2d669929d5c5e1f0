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
