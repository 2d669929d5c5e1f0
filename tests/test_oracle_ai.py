"""Pins for the oracle's analytic arithmetic-intensity model (CPU only).

The paper prints no formula, only results: uniform INT8 raises ResNet-20's
global AI by about 42 percent, and INT4-level schemes reach 51-52 percent
(tests/golden/paper_ai_gains.txt).  Those two numbers, hand-computed per-layer
values and the monotonicity the paper describes pin the formula.
"""
import os

import numpy as np
import pytest

import oracle
import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_ai_gains.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            name, lo, hi = [f.strip() for f in line.split("|")]
            out[name] = (float(lo), float(hi))
    return out


@pytest.fixture(scope="module")
def r20():
    return synth.desc_array(synth.resnet_cifar(3))


def _ai(desc, bits):
    L = int(desc[:, 12].max()) + 1
    scheme = np.full(L, bits, dtype=np.uint8) if np.isscalar(bits) else np.asarray(bits, dtype=np.uint8)
    return oracle.layer_ai(desc, scheme)[2]


def test_paper_gains_on_resnet20(r20):
    g = _golden()
    base = _ai(r20, 32)
    gain8 = _ai(r20, 8) / base - 1
    gain4 = _ai(r20, 4) / base - 1
    assert g["uniform_int8"][0] <= gain8 <= g["uniform_int8"][1]
    assert g["uniform_int4_at_least_aiq"][0] <= gain4 <= g["uniform_int4_at_least_aiq"][1]
    # uniform INT4 has the highest AI of any scheme over {32, 8, 4}
    rng = np.random.Generator(np.random.PCG64(1))
    for _ in range(50):
        mixed = rng.choice(np.array([32, 8, 4], dtype=np.uint8), size=20)
        assert _ai(r20, mixed) <= _ai(r20, 4)


def test_hand_computed_layers(r20):
    flops, byts, ai = oracle.layer_ai(r20, np.full(20, 32, dtype=np.uint8))
    # stem 3->16, 3x3, 32x32: 1024*16*27 multiply-adds; 432 weights; 3072 in + 16384 out elements
    assert flops[0] == 2 * 442_368 and byts[0] == 432 * 4 + 4 * (3072 + 16384)
    # first stage-1 conv 16->16 at 32x32
    assert flops[1] == 2 * 2_359_296 and byts[1] == 2304 * 4 + 4 * (16384 + 16384)
    # projection shortcut 16->32, 1x1, stride 2 (node 8): always 32-bit
    assert r20[8, 12] == -1
    assert flops[8] == 2 * 131_072 and byts[8] == 512 * 4 + 4 * (16384 + 8192)
    # classifier 64->10
    assert flops[-1] == 2 * 640 and byts[-1] == 640 * 4 + 4 * (64 + 10)
    assert flops.sum() == 2 * 40_813_184
    assert ai == pytest.approx(flops.sum() / byts.sum(), rel=1e-15)
    # INT4 weights: half a byte each, activations unchanged, shortcut still 4 bytes per weight
    f4, b4, _ = oracle.layer_ai(r20, np.full(20, 4, dtype=np.uint8))
    assert b4[1] == 2304 * 0.5 + 4 * (16384 + 16384)
    assert b4[8] == byts[8]
    np.testing.assert_array_equal(f4, flops)
    # batch scales FLOPs and activation bytes, not weight bytes
    fb, bb, _ = oracle.layer_ai(r20, np.full(20, 8, dtype=np.uint8), batch=16)
    assert fb[1] == 16 * flops[1] and bb[1] == 2304 * 1 + 16 * 4 * (16384 + 16384)


def test_depthwise_counts_one_input_channel_per_filter():
    desc = synth.desc_array(synth.mobilenetv2_32())
    flops, byts, _ = oracle.layer_ai(desc, np.full(53, 32, dtype=np.uint8))
    assert flops.sum() == 2 * 296_473_088
    dw = 1  # node 1: depthwise 32 channels at 32x32
    assert desc[dw, 0] == 1
    assert flops[dw] == 2 * 32 * 32 * 32 * 9 and byts[dw] == 32 * 9 * 4 + 4 * 2 * 32 * 32 * 32


def test_lowering_any_layer_raises_ai_and_wide_layers_gain_most(r20):
    base = _ai(r20, 32)
    gains = []
    for i in range(20):
        for b_hi, b_lo in ((32, 16), (16, 8), (8, 6), (6, 4), (4, 2)):
            hi = np.full(20, 32, dtype=np.uint8)
            lo = hi.copy()
            hi[i], lo[i] = b_hi, b_lo
            assert _ai(r20, lo) > _ai(r20, hi)
        s = np.full(20, 32, dtype=np.uint8)
        s[i] = 4
        gains.append(_ai(r20, s) - base)
    n_weights = []
    for d in r20:
        if d[12] >= 0:
            n_weights.append(int(d[1]) * int(d[2]) * (int(d[3]) * int(d[4]) if d[0] != 2 else 1))
    # the gain of quantizing one layer is ordered by its weight count: 64-channel convs lead,
    # the stem and the classifier trail
    order = np.argsort(gains)
    assert set(order[-5:]) == set(np.argsort(n_weights)[-5:])
    assert set(order[:2]) == {0, 19}


def test_invalid_inputs(r20):
    with pytest.raises(oracle.OracleError) as e:
        oracle.layer_ai(r20, np.full(20, 3, dtype=np.uint8))
    assert e.value.code == 2
    with pytest.raises(oracle.OracleError) as e:
        oracle.layer_ai(r20, np.full(19, 8, dtype=np.uint8))
    assert e.value.code == 3
    with pytest.raises(oracle.OracleError):
        oracle.layer_ai(r20, np.full(20, 8, dtype=np.uint8), batch=0)
