"""Pins for the oracle's activation fake-quantization variant (CPU only).

Reading (the paper gives a layer only a bit-width): a layer at b < 32 bits reads its input tensor
quantized to b bits with one symmetric scale per image, by the same rule as a weight row; the residual
input stays as it is; the classifier reads the pooled vector quantized.  These tests pin it against
hand-worked tensors, against the (separately pinned) weight quantizer applied to the tensor as one row,
against a layer-by-layer reconstruction from pinned pieces, and against the invariants the reading
implies - so that a per-batch scale, a quantized residual, a quantizer applied to the output instead
of the input, an unquantized classifier input or a wrong byte count each fail a test.
"""
import os

import numpy as np
import pytest

import oracle
import synth
from synth import graphs as G

BITS = (16, 8, 6, 4, 2)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "quantizer_rows.txt")


def _golden_rows():
    out = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        bits, row, scale, codes, deq = [f.strip() for f in line.split("|")]
        out.append((int(bits), np.array(row.split(), dtype=np.float32), np.array(deq.split(), dtype=np.float32)))
    return out


def _np_quantize(x, bits):
    """Independent binary32 statement of the rule, one scale for the whole array."""
    if bits == 32:
        return np.asarray(x, dtype=np.float64)
    x = np.asarray(x, dtype=np.float32)
    qmax = np.float32(2 ** (bits - 1) - 1)
    amax = np.abs(x).max() if x.size else np.float32(0)
    s = np.float32(amax / qmax) if amax > 0 else np.float32(1)
    q = np.clip(np.rint((x / s).astype(np.float32)), -qmax, qmax).astype(np.float32)
    return (q * s).astype(np.float32).astype(np.float64)


@pytest.mark.parametrize("bits,row,deq", _golden_rows())
def test_hand_worked_tensors(bits, row, deq):
    # the hand-worked rows of the weight quantizer, read as an activation tensor (ties go to the even code)
    np.testing.assert_array_equal(oracle.quantize_activations(row.reshape(-1, 1, 1), bits).ravel(), deq.astype(np.float64))


@pytest.mark.parametrize("bits", BITS + (32,))
def test_is_the_weight_rule_on_the_tensor_as_one_row(bits):
    rng = np.random.Generator(np.random.PCG64(bits))
    x = (rng.standard_normal((5, 7, 12)) * 3).astype(np.float32)
    got = oracle.quantize_activations(x, bits)
    w_dq, _, _ = oracle.quantize_weights(x.reshape(1, -1), bits)
    np.testing.assert_array_equal(got.ravel(), w_dq.ravel().astype(np.float64))
    np.testing.assert_array_equal(got, _np_quantize(x, bits))
    # an all-zero tensor stays zero; values are taken in binary32 (a double that is not a float is rounded first)
    assert not oracle.quantize_activations(np.zeros(9), bits).any()
    y = np.array([1.0 + 2.0 ** -30, -0.25, 0.5])
    if bits == 32:  # nothing happens at 32 bits, not even the rounding to binary32
        np.testing.assert_array_equal(oracle.quantize_activations(y, bits), y)
    else:
        np.testing.assert_array_equal(oracle.quantize_activations(y, bits), _np_quantize(y.astype(np.float32), bits))


def _small_net(res=True):
    nodes = [G._node(G.KIND_CONV, 3, 8, 3, 1, 6, -1, act=G.ACT_RELU, slot=0),
             G._node(G.KIND_CONV, 8, 8, 3, 1, 6, 0, act=G.ACT_RELU, slot=1),
             G._node(G.KIND_DEPTHWISE, 8, 8, 3, 1, 6, 1, act=G.ACT_RELU6, slot=2),
             G._node(G.KIND_CONV, 8, 8, 1, 1, 6, 2, residual=0 if res else -1, act=G.ACT_NONE, slot=3),
             G._node(G.KIND_CONV, 8, 12, 1, 2, 6, 3, act=G.ACT_NONE, slot=-1),   # never part of a scheme
             G._node(G.KIND_FC, 12, 5, 1, 1, 3, 4, slot=4)]
    rng = np.random.Generator(np.random.PCG64(17))
    w, b = synth.make_model(nodes, rng)
    images = (rng.standard_normal((3, 6, 6, 3)) * np.array([1.0, 4.0, 0.25])[:, None, None, None]).astype(np.float32)
    return nodes, synth.desc_array(nodes), w, b, images


def test_layer_by_layer_reconstruction_from_pinned_pieces():
    """Scoring with activation quantization equals: per node, quantize a copy of its input (numpy rule above),
    run the pinned single-layer routine on separately quantized weights, add the residual unquantized; for the
    classifier, pool, quantize the pooled vector, multiply."""
    nodes, desc, w, b, images = _small_net()
    scheme = np.array([[8, 4, 6, 2, 16], [32, 8, 32, 4, 8]], dtype=np.uint8)
    r = oracle.eval_schemes(desc, w, b, images, scheme, act_quant=True, want_acts=True)
    elems = oracle.node_out_elems(desc)
    offs = np.concatenate([[0], np.cumsum(elems)])
    for si in range(scheme.shape[0]):
        for n in range(images.shape[0]):
            outs = []
            for l, nd in enumerate(nodes):
                bits = int(scheme[si, nd["scheme_slot"]]) if nd["scheme_slot"] >= 0 else 32
                wq = oracle.quantize_weights(w[l], bits)[0]
                x = images[n].astype(np.float64) if nd["input"] < 0 else outs[nd["input"]]
                if nd["kind"] == G.KIND_FC:
                    pooled = x.reshape(-1, nd["cin"]).mean(axis=0)
                    y = _np_quantize(pooled, bits) @ wq.astype(np.float64).T + b[l]
                else:
                    xq = _np_quantize(x, bits).reshape(nd["hin"], nd["win"], nd["cin"])
                    res = outs[nd["residual"]].ravel() if nd["residual"] >= 0 else None
                    y, _ = oracle.conv_layer(desc[l], xq, wq, b[l], res)
                outs.append(np.asarray(y, dtype=np.float64))
                got = r["acts"][si, n, offs[l]:offs[l + 1]]
                np.testing.assert_allclose(got, outs[-1].ravel(), rtol=1e-12, atol=1e-12, err_msg=f"scheme {si} image {n} node {l}")
            np.testing.assert_allclose(r["logits"][si, n], outs[-1], rtol=1e-12, atol=1e-12)


def test_all_fp32_scheme_and_flag_off_leave_scoring_unchanged():
    nodes, desc, w, b, images = _small_net()
    L = 5
    schemes = np.array([[32] * L, [8, 8, 8, 8, 8]], dtype=np.uint8)
    on = oracle.eval_schemes(desc, w, b, images, schemes, act_quant=True)
    off = oracle.eval_schemes(desc, w, b, images, schemes, act_quant=False)
    np.testing.assert_array_equal(on["logits"][0], off["logits"][0])        # nothing to quantize at 32 bits
    np.testing.assert_array_equal(on["logits"][0], on["logits_base"])
    assert on["agree"][0] == images.shape[0]
    assert np.abs(on["logits"][1] - off["logits"][1]).max() > 1e-6          # at 8 bits the activations matter
    np.testing.assert_array_equal(on["logits_base"], off["logits_base"])    # the FP32 reference never changes


def test_scale_is_per_image_not_per_batch():
    nodes, desc, w, b, images = _small_net()
    schemes = np.array([[4, 4, 4, 4, 4]], dtype=np.uint8)
    whole = oracle.eval_schemes(desc, w, b, images, schemes, act_quant=True)["logits"]
    for n in range(images.shape[0]):
        one = oracle.eval_schemes(desc, w, b, images[n:n + 1], schemes, act_quant=True)["logits"]
        np.testing.assert_array_equal(whole[:, n], one[:, 0])
    # and the order of the images does not matter
    perm = oracle.eval_schemes(desc, w, b, images[::-1].copy(), schemes, act_quant=True)["logits"]
    np.testing.assert_array_equal(whole[:, ::-1], perm)


def test_power_of_two_input_scaling_commutes_with_the_first_layer():
    """x -> 4x scales the first layer's quantized input exactly by 4 (scales are relative to the tensor's own
    maximum), so a bias-free first layer's pre-activation output scales by 4 too."""
    nodes = [G._node(G.KIND_CONV, 3, 8, 3, 1, 6, -1, act=G.ACT_NONE, slot=0), G._node(G.KIND_FC, 8, 4, 1, 1, 6, 0, slot=1)]
    rng = np.random.Generator(np.random.PCG64(3))
    w, b = synth.make_model(nodes, rng)
    b[0][:] = 0
    desc = synth.desc_array(nodes)
    x = rng.standard_normal((2, 6, 6, 3)).astype(np.float32)
    sch = np.array([[4, 32]], dtype=np.uint8)
    a1 = oracle.eval_schemes(desc, w, b, x, sch, act_quant=True, want_acts=True)["acts"][0, :, :6 * 6 * 8]
    a4 = oracle.eval_schemes(desc, w, b, (4 * x).astype(np.float32), sch, act_quant=True, want_acts=True)["acts"][0, :, :6 * 6 * 8]
    np.testing.assert_allclose(a4, 4 * a1, rtol=1e-13, atol=0)


def test_residual_input_is_not_quantized_and_shortcuts_read_full_precision():
    nodes, desc, w, b, images = _small_net(res=True)
    # node 3 adds node 0's output: with 2-bit activations everywhere a quantized residual would be ternary
    sch = np.array([[32, 32, 32, 2, 32]], dtype=np.uint8)
    r = oracle.eval_schemes(desc, w, b, images, sch, act_quant=True, want_acts=True)
    elems = oracle.node_out_elems(desc)
    offs = np.concatenate([[0], np.cumsum(elems)])
    out0 = r["acts"][0, 0, offs[0]:offs[1]]
    out3 = r["acts"][0, 0, offs[3]:offs[4]]
    x2 = r["acts"][0, 0, offs[2]:offs[3]]
    wq = oracle.quantize_weights(w[3], 2)[0]
    conv_only, _ = oracle.conv_layer(desc[3], _np_quantize(x2, 2).reshape(6, 6, 8), wq, b[3], None)
    np.testing.assert_allclose(out3 - conv_only, out0, rtol=0, atol=1e-12)   # the residual arrived unquantized
    # node 4 is outside every scheme: its input (node 3's output) is read as it is
    y4, _ = oracle.conv_layer(desc[4], out3.reshape(6, 6, 8), w[4], b[4], None)
    np.testing.assert_allclose(r["acts"][0, 0, offs[4]:offs[5]], y4, rtol=1e-12, atol=1e-12)


def test_ai_model_with_activation_bits():
    nodes = synth.resnet_cifar(3)
    desc = synth.desc_array(nodes)
    L = synth.n_scheme_layers(nodes)
    q8 = np.full(L, 8, np.uint8)
    f0, b0, ai0 = oracle.layer_ai(desc, q8)
    f1, b1, ai1 = oracle.layer_ai(desc, q8, act_quant=True)
    np.testing.assert_array_equal(f0, f1)
    # a 16 -> 16 layer at 32x32, 8 bits: 2304 weight bytes + 16384 input bytes + 65536 output bytes
    assert b1[1] == 2304 + 16384 + 4 * 16384
    assert b0[1] == 2304 + 4 * 16384 + 4 * 16384
    # projection shortcuts are outside the scheme: counted in full either way
    sc = [i for i, nd in enumerate(nodes) if nd["scheme_slot"] < 0]
    assert sc and all(b0[i] == b1[i] for i in sc)
    assert ai1 > ai0
    # all-FP32: the flag changes nothing; lowering a layer raises AI more with the flag than without
    q32 = np.full(L, 32, np.uint8)
    assert oracle.layer_ai(desc, q32, act_quant=True)[2] == oracle.layer_ai(desc, q32)[2]
    for i in (0, 5, 19):
        q = q32.copy()
        q[i] = 4
        assert oracle.layer_ai(desc, q, act_quant=True)[2] > oracle.layer_ai(desc, q)[2] > oracle.layer_ai(desc, q32)[2]
    # batch: activations scale with it, weights do not
    _, bb, _ = oracle.layer_ai(desc, q8, batch=3, act_quant=True)
    assert bb[1] == 2304 + 3 * (16384 + 4 * 16384)
