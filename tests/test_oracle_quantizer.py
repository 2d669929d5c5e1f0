"""Pins for the oracle's weight quantizer (CPU only).

The paper's Problem Formulation fixes only the per-layer bit-width; the rule is
symmetric per-output-channel with codes in [-(2^(b-1)-1), 2^(b-1)-1].  These
tests pin it against hand-worked rows, exact-rational arithmetic and the
invariants the rule implies, so that a wrong rounding mode, a reciprocal
multiply, a dropped clamp or a per-tensor scale each fail at least one test.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

BITS = (16, 8, 6, 4, 2)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "quantizer_rows.txt")


def _rows(n, k, seed, scale=1.0):
    rng = np.random.Generator(np.random.PCG64(seed))
    return (rng.standard_normal((n, k)) * scale).astype(np.float32)


def _golden_rows():
    out = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        bits, row, scale, codes, deq = [f.strip() for f in line.split("|")]
        out.append((int(bits), np.array(row.split(), dtype=np.float32), np.float32(scale),
                    np.array(codes.split(), dtype=np.int32), np.array(deq.split(), dtype=np.float32)))
    return out


@pytest.mark.parametrize("bits,row,scale,codes,deq", _golden_rows())
def test_hand_worked_rows(bits, row, scale, codes, deq):
    w_dq, s, q = oracle.quantize_weights(row[None, :], bits)
    assert s[0] == scale
    np.testing.assert_array_equal(q[0], codes)
    np.testing.assert_array_equal(w_dq[0], deq)


def test_b32_is_bitwise_identity():
    w = _rows(7, 33, 1)
    w_dq, s, _ = oracle.quantize_weights(w, 32)
    assert w_dq.tobytes() == w.tobytes()
    assert np.all(s == 1.0)


@pytest.mark.parametrize("bits", BITS)
def test_code_range_and_extreme_code(bits):
    w = _rows(64, 144, 2)
    _, _, q = oracle.quantize_weights(w, bits)
    qmax = 2 ** (bits - 1) - 1
    assert np.abs(q).max() <= qmax
    # the element of largest magnitude maps to +-qmax in every non-zero channel
    np.testing.assert_array_equal(np.abs(q).max(axis=1), np.full(64, qmax))
    am = np.abs(w).argmax(axis=1)
    np.testing.assert_array_equal(q[np.arange(64), am], np.sign(w[np.arange(64), am]).astype(np.int32) * qmax)


@pytest.mark.parametrize("bits", BITS)
def test_scale_and_quotient_are_correctly_rounded_binary32(bits):
    """Exact rationals: s is the binary32 nearest to amax/qmax, codes are the
    half-even rounding of the binary32 nearest to w/s (a reciprocal multiply or a
    double-precision quotient differs on some of these elements)."""
    w = _rows(24, 96, 3 + bits)
    w_dq, s, q = oracle.quantize_weights(w, bits)
    qmax = 2 ** (bits - 1) - 1

    def nearest_f32(fr):
        # fp64 holds a quotient of two binary32 values to far more than 2*24+2 bits,
        # so rounding the fp64 quotient to binary32 equals rounding the exact quotient.
        return np.float32(fr.numerator / fr.denominator)

    for c in range(w.shape[0]):
        amax = max(abs(float(v)) for v in w[c])
        assert s[c] == nearest_f32(Fraction(amax) / qmax)
        for i in range(w.shape[1]):
            t = nearest_f32(Fraction(float(w[c, i])) / Fraction(float(s[c])))
            fl = int(np.floor(t))
            frac = Fraction(float(t)) - fl
            r = fl + (1 if frac > Fraction(1, 2) or (frac == Fraction(1, 2) and fl % 2 == 1) else 0)
            r = max(-qmax, min(qmax, r))
            assert q[c, i] == r
            assert w_dq[c, i] == np.float32(Fraction(r) * Fraction(float(s[c])))


@pytest.mark.parametrize("bits", BITS)
def test_idempotent(bits):
    w = _rows(128, 576, 5, scale=0.06)
    w1, s1, q1 = oracle.quantize_weights(w, bits)
    w2, s2, q2 = oracle.quantize_weights(w1, bits)
    np.testing.assert_array_equal(q1, q2)
    assert np.all(np.abs(s1.view(np.int32) - s2.view(np.int32)) <= 1)
    np.testing.assert_allclose(w2, w1, rtol=2e-7, atol=0)


def test_two_bits_is_ternary_with_half_amax_threshold():
    w = _rows(32, 288, 6)
    w_dq, s, q = oracle.quantize_weights(w, 2)
    amax = np.abs(w).max(axis=1, keepdims=True)
    assert set(np.unique(q)) <= {-1, 0, 1}
    np.testing.assert_array_equal(s, amax[:, 0])
    clear = np.abs(np.abs(w) - amax / 2) > 1e-6 * amax
    expect = np.where(np.abs(w) > amax / 2, np.sign(w), 0).astype(np.int32)
    np.testing.assert_array_equal(q[clear], expect[clear])
    np.testing.assert_array_equal(w_dq, q.astype(np.float32) * amax)


@pytest.mark.parametrize("bits", BITS)
def test_power_of_two_scaling_and_sign_symmetry(bits):
    w = _rows(16, 144, 7)
    w1, s1, q1 = oracle.quantize_weights(w, bits)
    for p in (-9, 4):
        wp, sp, qp = oracle.quantize_weights(w * np.float32(2.0 ** p), bits)
        np.testing.assert_array_equal(qp, q1)
        np.testing.assert_array_equal(sp, s1 * np.float32(2.0 ** p))
        np.testing.assert_array_equal(wp, w1 * np.float32(2.0 ** p))
    wn, sn, qn = oracle.quantize_weights(-w, bits)
    np.testing.assert_array_equal(qn, -q1)
    np.testing.assert_array_equal(sn, s1)
    np.testing.assert_array_equal(wn, -w1)


@pytest.mark.parametrize("bits", BITS)
def test_error_bound_half_step(bits):
    w = _rows(64, 64, 8)
    w_dq, s, _ = oracle.quantize_weights(w, bits)
    err = np.abs(w.astype(np.float64) - w_dq.astype(np.float64))
    # half a step, plus one binary32 rounding each of the quotient and of the product
    assert np.all(err <= 0.5 * s[:, None].astype(np.float64) + np.abs(w).astype(np.float64) * 2.0 ** -22)


def test_scales_are_per_output_channel_not_per_tensor():
    w = _rows(4, 32, 9)
    w[2] *= 100.0
    _, s, _ = oracle.quantize_weights(w, 8)
    np.testing.assert_array_equal(s, np.abs(w).max(axis=1) / np.float32(127))
    for c in range(4):
        _, sc, _ = oracle.quantize_weights(w[c:c + 1], 8)
        assert sc[0] == s[c]


def test_all_zero_channel_and_unsupported_bits():
    w = _rows(3, 9, 10)
    w[1] = 0.0
    w_dq, s, q = oracle.quantize_weights(w, 4)
    assert s[1] == 1.0 and not q[1].any() and not w_dq[1].any()
    for bad in (0, 1, 3, 5, 7, 12, 24, 33):
        with pytest.raises(oracle.OracleError) as e:
            oracle.quantize_weights(w, bad)
        assert e.value.code == 2


@pytest.mark.parametrize("bits", BITS)
def test_matches_vectorised_numpy_float32(bits):
    """Second implementation (numpy binary32 array ops) on layer-sized rows."""
    w = _rows(64, 576, 11, scale=0.059)
    w_dq, s, q = oracle.quantize_weights(w, bits)
    qmax = np.float32(2 ** (bits - 1) - 1)
    amax = np.abs(w).max(axis=1)
    s_np = (amax / qmax).astype(np.float32)
    t = (w / s_np[:, None]).astype(np.float32)
    q_np = np.clip(np.rint(t), -qmax, qmax).astype(np.int32)
    np.testing.assert_array_equal(s, s_np)
    np.testing.assert_array_equal(q, q_np)
    np.testing.assert_array_equal(w_dq, (q_np.astype(np.float32) * s_np[:, None]).astype(np.float32))


# ---------------------------------------------------------------- per-tensor variant

def test_per_tensor_hand_worked(oracle_lib):
    """Two rows, 4 bits: the tensor's largest magnitude (7) sets the one scale s = 1, so the second row,
    whose own scale would be 0.25, keeps only coarse codes: 1.75 -> 2, 0.4 -> 0."""
    w = np.array([[7.0, -3.5], [1.75, 0.4]], dtype=np.float32)
    dq, s, q = oracle_lib.quantize_weights(w, 4, per_tensor=True)
    np.testing.assert_array_equal(s, np.array([1.0, 1.0], dtype=np.float32))
    np.testing.assert_array_equal(q, np.array([[7, -4], [2, 0]], dtype=np.int32))
    np.testing.assert_array_equal(dq, np.array([[7.0, -4.0], [2.0, 0.0]], dtype=np.float32))
    _, s_c, q_c = oracle_lib.quantize_weights(w, 4)
    np.testing.assert_array_equal(s_c, np.array([1.0, 0.25], dtype=np.float32))
    np.testing.assert_array_equal(q_c[1], np.array([7, 2], dtype=np.int32))


@pytest.mark.parametrize("bits", [16, 8, 6, 4, 2])
def test_per_tensor_properties(oracle_lib, bits):
    rng = np.random.Generator(np.random.PCG64(900 + bits))
    w = (rng.standard_normal((24, 50)) * rng.uniform(0.1, 2.0, size=(24, 1))).astype(np.float32)
    dq, s, q = oracle_lib.quantize_weights(w, bits, per_tensor=True)
    qmax = 2 ** (bits - 1) - 1
    # one scale, set by the largest magnitude of the whole tensor, computed in binary32
    assert (s == s[0]).all()
    assert s[0] == np.float32(np.abs(w).max()) / np.float32(qmax)
    assert np.abs(q).max() == qmax and (np.abs(q) <= qmax).all()
    # the row holding the tensor maximum is quantized exactly as the per-channel rule would
    r = int(np.abs(w).max(axis=1).argmax())
    dq_c, s_c, q_c = oracle_lib.quantize_weights(w, bits)
    assert s_c[r] == s[0]
    np.testing.assert_array_equal(q[r], q_c[r])
    assert (s_c <= s[0]).all()
    # vectorised binary32 second implementation
    t = (w / s[0]).astype(np.float32)
    ref_q = np.clip(np.rint(t), -qmax, qmax).astype(np.int32)
    np.testing.assert_array_equal(q, ref_q)
    assert dq.tobytes() == (ref_q.astype(np.float32) * s[0]).astype(np.float32).tobytes()
    # a single row: both granularities coincide
    a = oracle_lib.quantize_weights(w[:1], bits, per_tensor=True)
    b = oracle_lib.quantize_weights(w[:1], bits)
    for x, y in zip(a, b):
        assert x.tobytes() == y.tobytes()
    # b = 32 is the identity in both
    dq32, s32, _ = oracle_lib.quantize_weights(w, 32, per_tensor=True)
    assert dq32.tobytes() == w.tobytes() and (s32 == 1.0).all()


def test_per_tensor_scoring_uses_one_scale_per_layer(oracle_lib):
    import synth
    wl = synth.make_workload(0, n_images=6)
    schemes = np.full((2, wl["L"]), 4, dtype=np.uint8)
    schemes[1] = 32
    r_t = oracle_lib.eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], schemes, per_tensor=True)
    # equals a plain forward pass on weights quantized per tensor by hand
    wq = []
    for node, w in zip(wl["nodes"], wl["weights"]):
        wq.append(oracle_lib.quantize_weights(w, 4, per_tensor=True)[0] if node["scheme_slot"] >= 0 else w)
    f = oracle_lib.forward(wl["desc"], wq, wl["biases"], wl["images"])
    np.testing.assert_array_equal(r_t["logits"][0], f["logits"])
    np.testing.assert_array_equal(r_t["logits"][1], r_t["logits_base"])
    r_c = oracle_lib.eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], schemes)
    assert not np.array_equal(r_t["logits"][0], r_c["logits"][0])
