"""Pins for the oracle's forward pass and agreement count (CPU only).

The oracle's loops are checked against things that are not the oracle: an
einsum over explicitly padded patches, a library matmul, torch's float64
conv2d on whole networks, closed-form multiply-add counts and structural
identities (delta kernels, stride subsampling, linearity).
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import synth
from synth import graphs as G


def _desc(kind, cin, cout, k, stride, hin, act=0):
    pad = 1 if k == 3 else 0
    return np.array([kind, cin, cout, k, k, stride, pad, hin, hin, -1, -1, act, 0], dtype=np.int32)


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


@pytest.mark.parametrize("stride", [1, 2])
@pytest.mark.parametrize("hin", [4, 5])
def test_conv3x3_against_einsum_over_padded_patches(stride, hin):
    rng = _rng(100 + stride + hin)
    cin, cout = 2, 3
    x = rng.standard_normal((hin, hin, cin))
    w = rng.standard_normal((cout, cin, 3, 3)).astype(np.float32)
    b = rng.standard_normal(cout).astype(np.float32)
    y, macs = oracle.conv_layer(_desc(0, cin, cout, 3, stride, hin), x, w.reshape(cout, -1), b)
    ho = (hin + 2 - 3) // stride + 1
    xp = np.zeros((hin + 2, hin + 2, cin))
    xp[1:-1, 1:-1] = x
    patches = np.empty((ho, ho, cin, 3, 3))
    for oy in range(ho):
        for ox in range(ho):
            patches[oy, ox] = xp[oy * stride:oy * stride + 3, ox * stride:ox * stride + 3].transpose(2, 0, 1)
    ref = np.einsum("yxcij,ocij->yxo", patches, w.astype(np.float64)) + b
    np.testing.assert_allclose(y.reshape(ho, ho, cout), ref, rtol=1e-13, atol=1e-13)
    assert macs == ho * ho * cout * cin * 9


def test_conv1x1_is_a_matrix_product():
    rng = _rng(7)
    hin, cin, cout = 6, 5, 4
    x = rng.standard_normal((hin, hin, cin))
    w = rng.standard_normal((cout, cin)).astype(np.float32)
    b = rng.standard_normal(cout).astype(np.float32)
    y, _ = oracle.conv_layer(_desc(0, cin, cout, 1, 1, hin), x, w, b)
    ref = x.reshape(-1, cin) @ w.astype(np.float64).T + b
    np.testing.assert_allclose(y.reshape(-1, cout), ref, rtol=1e-13, atol=1e-13)
    # stride 2 picks the even positions
    y2, _ = oracle.conv_layer(_desc(0, cin, cout, 1, 2, hin), x, w, b)
    np.testing.assert_allclose(y2.reshape(3, 3, cout), ref.reshape(hin, hin, cout)[::2, ::2], rtol=1e-13)


@pytest.mark.parametrize("stride", [1, 2])
def test_depthwise_equals_dense_conv_with_diagonal_filters(stride):
    rng = _rng(8)
    hin, c = 6, 4
    x = rng.standard_normal((hin, hin, c))
    wd = rng.standard_normal((c, 9)).astype(np.float32)
    b = rng.standard_normal(c).astype(np.float32)
    yd, macs = oracle.conv_layer(_desc(1, c, c, 3, stride, hin, act=2), x, wd, b)
    dense = np.zeros((c, c, 9), dtype=np.float32)
    for i in range(c):
        dense[i, i] = wd[i]
    yg, _ = oracle.conv_layer(_desc(0, c, c, 3, stride, hin, act=2), x, dense.reshape(c, -1), b)
    np.testing.assert_allclose(yd, yg, rtol=1e-14, atol=1e-14)
    ho = (hin - 1) // stride + 1
    assert macs == ho * ho * c * 9


def test_delta_kernels_copy_and_shift_the_input():
    rng = _rng(9)
    hin, c = 5, 3
    x = rng.standard_normal((hin, hin, c))
    zero_b = np.zeros(c, dtype=np.float32)
    for ky in range(3):
        for kx in range(3):
            w = np.zeros((c, c, 3, 3), dtype=np.float32)
            for i in range(c):
                w[i, i, ky, kx] = 1.0
            y, _ = oracle.conv_layer(_desc(0, c, c, 3, 1, hin), x, w.reshape(c, -1), zero_b)
            ref = np.zeros_like(x)
            for oy in range(hin):
                for ox in range(hin):
                    iy, ix = oy + ky - 1, ox + kx - 1
                    if 0 <= iy < hin and 0 <= ix < hin:
                        ref[oy, ox] = x[iy, ix]
            np.testing.assert_array_equal(y.reshape(hin, hin, c), ref)


def test_linear_in_weights_and_stride2_subsamples_stride1():
    rng = _rng(10)
    hin, cin, cout = 8, 3, 4
    x = rng.standard_normal((hin, hin, cin))
    w1 = rng.standard_normal((cout, cin * 9)).astype(np.float32)
    w2 = rng.standard_normal((cout, cin * 9)).astype(np.float32)
    wsum = (w1.astype(np.float64) + w2).astype(np.float32)
    z = np.zeros(cout, dtype=np.float32)
    d = _desc(0, cin, cout, 3, 1, hin)
    y1, _ = oracle.conv_layer(d, x, w1, z)
    y2, _ = oracle.conv_layer(d, x, w2, z)
    ys, _ = oracle.conv_layer(d, x, wsum, z)
    np.testing.assert_allclose(ys, y1 + y2, rtol=0, atol=1e-5)
    ystr, _ = oracle.conv_layer(_desc(0, cin, cout, 3, 2, hin), x, w1, z)
    np.testing.assert_array_equal(ystr.reshape(4, 4, cout), y1.reshape(hin, hin, cout)[::2, ::2])


def test_residual_is_added_before_the_activation():
    x = np.full((2, 2, 1), 1.0)
    w = np.array([[1.0]], dtype=np.float32)
    b = np.array([0.5], dtype=np.float32)
    res = np.array([-3.0, 1.0, 4.0, 10.0])
    d = _desc(0, 1, 1, 1, 1, 2, act=2)
    y, _ = oracle.conv_layer(d, x, w, b, res=res)
    np.testing.assert_array_equal(y, [0.0, 2.5, 5.5, 6.0])
    d[11] = 1
    y, _ = oracle.conv_layer(d, x, w, b, res=res)
    np.testing.assert_array_equal(y, [0.0, 2.5, 5.5, 11.5])


def _torch_forward(nodes, weights, biases, images):
    """Independent float64 forward with torch's library convolutions."""
    x0 = torch.from_numpy(images.astype(np.float64)).permute(0, 3, 1, 2)
    outs = []
    for node, w, b in zip(nodes, weights, biases):
        x = x0 if node["input"] < 0 else outs[node["input"]]
        wt = torch.from_numpy(w.astype(np.float64))
        bt = torch.from_numpy(b.astype(np.float64))
        if node["kind"] == G.KIND_FC:
            y = F.linear(x.mean(dim=(2, 3)), wt, bt)
        else:
            groups = node["cin"] if node["kind"] == G.KIND_DEPTHWISE else 1
            wt = wt.reshape(node["cout"], node["cin"] // groups, node["kh"], node["kw"])
            y = F.conv2d(x, wt, bt, stride=node["stride"], padding=node["pad"], groups=groups)
            if node["residual"] >= 0:
                y = y + outs[node["residual"]]
        if node["act"] == G.ACT_RELU:
            y = torch.relu(y)
        elif node["act"] == G.ACT_RELU6:
            y = torch.clamp(y, 0.0, 6.0)
        outs.append(y)
    return outs


@pytest.mark.parametrize("index,n", [(0, 6), (1, 3), (3, 2)])
def test_whole_networks_match_torch_float64(index, n):
    wl = synth.make_workload(index, n_images=n)
    r = oracle.forward(wl["desc"], wl["weights"], wl["biases"], wl["images"], want_acts=True)
    outs = _torch_forward(wl["nodes"], wl["weights"], wl["biases"], wl["images"])
    off = 0
    for node, o in zip(wl["nodes"], outs):
        ref = (o if node["kind"] == G.KIND_FC else o.permute(0, 2, 3, 1)).reshape(n, -1).numpy()
        got = r["acts"][:, off:off + ref.shape[1]]
        scale = max(np.abs(ref).max(), 1e-30)
        assert np.abs(got - ref).max() <= 1e-11 * scale, node["name"]
        off += ref.shape[1]
    np.testing.assert_array_equal(r["top1"], outs[-1].argmax(dim=1).numpy())


@pytest.mark.parametrize("index,macs", [(0, 12_501_632), (1, 40_813_184), (3, 296_473_088)])
def test_multiply_add_count_matches_closed_form(index, macs):
    """Counted in the innermost loop; closed form: sum over layers of Hout*Wout*Cout*(Cin/groups)*k*k."""
    wl = synth.make_workload(index, n_images=1)
    closed = 0
    for nd in wl["nodes"]:
        if nd["kind"] == G.KIND_FC:
            closed += nd["cin"] * nd["cout"]
        else:
            ho = (nd["hin"] + 2 * nd["pad"] - nd["kh"]) // nd["stride"] + 1
            cg = 1 if nd["kind"] == G.KIND_DEPTHWISE else nd["cin"]
            closed += ho * ho * nd["cout"] * cg * nd["kh"] * nd["kw"]
    assert closed == macs
    assert oracle.forward(wl["desc"], wl["weights"], wl["biases"], wl["images"])["macs_per_image"] == macs


def test_all_fp32_scheme_agrees_on_every_image_and_b32_logits_equal_base():
    wl = synth.make_workload(0, n_images=12)
    sch = np.full((2, wl["L"]), 32, dtype=np.uint8)
    r = oracle.eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], sch)
    np.testing.assert_array_equal(r["agree"], [12, 12])
    np.testing.assert_array_equal(r["logits"][0], r["logits_base"])
    np.testing.assert_array_equal(r["top1"][1], r["top1_base"])


def test_eval_schemes_equals_forward_on_separately_quantized_weights():
    wl = synth.make_workload(0, n_images=10)
    sch = np.array([[4, 8, 32, 2, 16, 6, 4, 8], [2] * 8], dtype=np.uint8)
    r = oracle.eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], sch)
    for s in range(2):
        wq = []
        for nd, w in zip(wl["nodes"], wl["weights"]):
            bits = 32 if nd["scheme_slot"] < 0 else int(sch[s, nd["scheme_slot"]])
            wq.append(oracle.quantize_weights(w, bits)[0])
        f = oracle.forward(wl["desc"], wq, wl["biases"], wl["images"])
        np.testing.assert_array_equal(r["logits"][s], f["logits"])
        np.testing.assert_array_equal(r["top1"][s], f["top1"])
        assert r["agree"][s] == int((f["top1"] == r["top1_base"]).sum())
    # two-bit weights everywhere must change some predictions of a random network
    assert r["agree"][1] < 10


def test_projection_shortcuts_are_never_quantized():
    wl = synth.make_workload(0, n_images=4)
    sc = [i for i, nd in enumerate(wl["nodes"]) if nd["scheme_slot"] < 0]
    assert len(sc) == 2 and all(wl["nodes"][i]["kh"] == 1 for i in sc)
    sch = np.full((1, wl["L"]), 2, dtype=np.uint8)
    r = oracle.eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], sch)
    wq = [oracle.quantize_weights(w, 2)[0] for w in wl["weights"]]
    f_all = oracle.forward(wl["desc"], wq, wl["biases"], wl["images"])
    for i in sc:
        wq[i] = wl["weights"][i]
    f_keep = oracle.forward(wl["desc"], wq, wl["biases"], wl["images"])
    np.testing.assert_array_equal(r["logits"][0], f_keep["logits"])
    assert np.abs(f_all["logits"] - f_keep["logits"]).max() > 0


def test_argmax_ties_go_to_the_lowest_index():
    wl = synth.make_workload(0, n_images=3)
    w = [a.copy() for a in wl["weights"]]
    b = [a.copy() for a in wl["biases"]]
    w[-1][:] = 0.0
    b[-1][:] = np.array([1, 3, 3, 0, 3, -1, 2, 3, 0, 1], dtype=np.float32)
    r = oracle.forward(wl["desc"], w, b, wl["images"])
    np.testing.assert_array_equal(r["top1"], [1, 1, 1])


def test_permuting_images_permutes_results():
    wl = synth.make_workload(0, n_images=9)
    sch = wl["schemes"]
    r = oracle.eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], sch)
    perm = _rng(3).permutation(9)
    rp = oracle.eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"][perm], sch)
    np.testing.assert_array_equal(rp["top1"][0], r["top1"][0][perm])
    np.testing.assert_array_equal(rp["logits"][0], r["logits"][0][perm])
    np.testing.assert_array_equal(rp["agree"], r["agree"])


def test_graph_checks_and_scheme_validation():
    wl = synth.make_workload(0, n_images=1)
    assert oracle.check_graph(wl["desc"]) == 0
    bad = wl["desc"].copy()
    bad[3, 1] += 1  # cin no longer matches its producer
    assert oracle.check_graph(bad) == 3
    with pytest.raises(oracle.OracleError) as e:
        oracle.eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"],
                            np.full((1, wl["L"]), 5, dtype=np.uint8))
    assert e.value.code == 2
    with pytest.raises(oracle.OracleError) as e:
        oracle.eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"],
                            np.full((1, wl["L"] + 1), 8, dtype=np.uint8))
    assert e.value.code == 3
