"""GPU parity of the activation fake-quantization variant (AIQ_MODEL_ACT_QUANT).

Rounding an activation to a code is a discontinuity: the GPU's fp32 activations and the oracle's fp64 ones
differ in the last bits, a value that sits on a rounding boundary gets neighbouring codes on the two sides,
and a deep network amplifies that (fp32 against fp64 of the same plain PyTorch model differ by up to 5e-2 on
ResNet-20 logits and by order 1 on MobileNetV2).  So an end-to-end logit tolerance does not exist for this
variant; what is unique is each layer's result given the tensors it actually read.  The tests therefore
  * compare every node's GPU output (aiq_forward_nodes) with the oracle's single-layer routines applied to
    the GPU's own input tensors of that node - activation codes are then decided on identical binary32
    values on both sides and must agree exactly, the rest is fp32 accumulation (1e-5 of the layer's range);
  * compare end to end where no rounding boundary can matter: all-FP32 schemes and 32-bit layers, and
    schemes with a single low-bit layer (bounded effect of an isolated flip), at the usual 1e-3;
  * check on deep networks that most samples still agree closely (median) and that counts are consistent.
"""
import numpy as np
import pytest

from parity import check_eval, logits_rel_error

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2512_14090_amd as aiq
    import oracle
    import synth
    aiq.load_library()
    return dict(torch=torch, aiq=aiq, oracle=oracle, synth=synth)


def _node_reference(oracle, nodes, desc, w, b, scheme, image, outs, l):
    """Oracle result of node l for one image from the tensors the GPU gave that node."""
    nd = nodes[l]
    bits = int(scheme[nd["scheme_slot"]]) if nd["scheme_slot"] >= 0 else 32
    wq = oracle.quantize_weights(w[l], bits)[0]
    x = image.astype(np.float64) if nd["input"] < 0 else outs[nd["input"]].astype(np.float64)
    if nd["kind"] == 2:
        pooled = x.reshape(-1, nd["cin"]).mean(axis=0)
        return oracle.quantize_activations(pooled, bits) @ wq.astype(np.float64).T + b[l].astype(np.float64)
    xq = oracle.quantize_activations(x, bits).reshape(nd["hin"], nd["win"], nd["cin"])
    res = outs[nd["residual"]].astype(np.float64).ravel() if nd["residual"] >= 0 else None
    return oracle.conv_layer(desc[l], xq, wq, b[l], res)[0]


def _check_nodes(env, nodes, desc, w, b, images, schemes, tol=2e-5):
    torch, aiq, oracle = env["torch"], env["aiq"], env["oracle"]
    m = aiq.Model(desc, w, b, act_quant=True)
    assert not m.lds_resident and m.lds_resident_blocks == 0
    img = torch.from_numpy(images).cuda()
    worst = 0.0
    for scheme in schemes:
        outs = m.forward_nodes(img, scheme)
        torch.cuda.synchronize()
        outs = [o.cpu().numpy() for o in outs]
        for n in range(images.shape[0]):
            per_image = [o[n] for o in outs]
            for l in range(len(nodes)):
                ref = _node_reference(oracle, nodes, desc, w, b, scheme, images[n], per_image, l)
                err = np.abs(per_image[l] - ref).max() / max(np.abs(ref).max(), 1e-30)
                assert err <= tol, f"node {l} ({nodes[l].get('name', '')}) image {n} scheme {scheme.tolist()}: {err:.3e}"
                worst = max(worst, err)
    m.close()
    return worst


def _schemes(L, rng, extra=()):
    rows = [np.full(L, 8, np.uint8), np.full(L, 4, np.uint8), np.full(L, 2, np.uint8), np.full(L, 32, np.uint8)]
    rows += [rng.choice(np.array([32, 16, 8, 6, 4, 2], np.uint8), size=L) for _ in range(3)]
    return rows + list(extra)


@pytest.mark.parametrize("index,n", [(0, 6), (1, 3), (3, 2), (5, 2), (6, 2)])
def test_every_node_against_the_oracle_on_the_gpu_s_own_inputs(env, index, n):
    wl = env["synth"].make_workload(index, n_images=n)
    rng = np.random.Generator(np.random.PCG64(60 + index))
    schemes = _schemes(wl["L"], rng)
    if index == 3:
        schemes = schemes[:1] + schemes[4:6]
    print(f"act-quant, node by node: {wl['name']} N={n} schemes={len(schemes)}", flush=True)
    worst = _check_nodes(env, wl["nodes"], wl["desc"], wl["weights"], wl["biases"], wl["images"], schemes)
    print("  worst node error %.3e of the node's range" % worst, flush=True)


def test_random_graphs_and_odd_shapes_node_by_node(env):
    """Layer kinds, strides, residual links and tensors whose size is not a multiple of four (scalar path of the
    activation quantizer), from the seeded random graphs of the scoring tests."""
    from test_gpu_eval import _random_graph
    synth = env["synth"]
    for seed in range(8):
        rng = np.random.Generator(np.random.PCG64(9000 + seed))
        nodes, ci, h = _random_graph(synth.graphs, rng)
        w, b = synth.make_model(nodes, rng)
        images = rng.standard_normal((3, h, h, ci)).astype(np.float32)
        L = len(nodes)
        print(f"act-quant random graph {seed}: {L} nodes, input {h}x{h}x{ci}", flush=True)
        _check_nodes(env, nodes, synth.desc_array(nodes), w, b, images, _schemes(L, rng)[:6])


def test_end_to_end_where_no_rounding_boundary_can_decide(env):
    """All-FP32 and 16-bit-free cases: a scheme with every layer at 32 bits reproduces plain scoring bit for bit;
    schemes with one low-bit layer stay within the usual logit bar (an isolated neighbouring code moves a logit
    by far less than 1e-3)."""
    torch, aiq, oracle = env["torch"], env["aiq"], env["oracle"]
    wl = env["synth"].make_workload(0, n_images=48)
    L = wl["L"]
    single = np.full((2 * L, L), 32, np.uint8)
    for i in range(L):
        single[2 * i, i] = 8
        single[2 * i + 1, i] = 4
    schemes = np.concatenate([np.full((1, L), 32, np.uint8), single])
    ref = oracle.eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], schemes, act_quant=True)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"], act_quant=True)
    plain = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=True)
    img = torch.from_numpy(wl["images"]).cuda()
    r = m.eval_schemes(img, schemes, chunk=20, want_logits=True, want_top1=True)
    p = plain.eval_schemes(img, schemes[:1], chunk=20, want_logits=True)
    torch.cuda.synchronize()
    gpu = {k: v.cpu().numpy() for k, v in r.items()}
    assert torch.equal(r["logits"][0], p["logits"][0]) and gpu["agree"][0] == 48
    err = check_eval(gpu, ref, 48)
    # activation quantization is really applied: the same schemes scored weight-only differ
    ref_w = oracle.eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], schemes)
    assert logits_rel_error(gpu["logits"][1:], ref_w["logits"][1:]) > 1e-3
    print("single-layer schemes end to end: max logit rel err %.3e" % err, flush=True)
    m.close()
    plain.close()


def test_deep_networks_agree_on_most_samples_and_counts_are_consistent(env):
    torch, aiq, oracle = env["torch"], env["aiq"], env["oracle"]
    wl = env["synth"].make_workload(7, n_images=48)
    L = wl["L"]
    schemes = np.stack([np.full(L, b, np.uint8) for b in (16, 8, 6, 4)])
    ref = oracle.eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], schemes, act_quant=True)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"], act_quant=True)
    img = torch.from_numpy(wl["images"]).cuda()
    r = m.eval_schemes(img, schemes, chunk=32, want_logits=True, want_top1=True)
    torch.cuda.synchronize()
    gpu = {k: v.cpu().numpy() for k, v in r.items()}
    b = wl["biases"][-1].astype(np.float64)
    zr, zg = ref["logits"] - b, gpu["logits"].astype(np.float64) - b
    e = np.abs(zg - zr).max(axis=-1) / np.abs(zr).max(axis=-1)
    print("uniform 16/8/6/4-bit ResNet-20, response error per sample: median %s, share within 1e-3 %s" %
          (np.median(e, axis=1), (e <= 1e-3).mean(axis=1)), flush=True)
    assert (np.median(e, axis=1) <= 1e-4).all()
    assert ((e <= 1e-3).mean(axis=1) >= 0.5).all()
    np.testing.assert_array_equal(gpu["top1"], gpu["logits"].argmax(axis=-1))
    np.testing.assert_array_equal(gpu["agree"], (gpu["top1"] == gpu["top1_base"][None]).sum(axis=1))
    np.testing.assert_array_equal(gpu["top1_base"], ref["top1_base"])
    # identical when run again and with another chunking
    r2 = m.eval_schemes(img, schemes, chunk=48, want_logits=True)
    torch.cuda.synchronize()
    assert torch.equal(r2["logits"], r["logits"])
    m.close()


def test_search_and_ai_model_with_activation_bits(env):
    torch, aiq, oracle = env["torch"], env["aiq"], env["oracle"]
    wl = env["synth"].make_workload(7, n_images=32)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"], act_quant=True)
    img = torch.from_numpy(wl["images"]).cuda()
    q, trace = m.search(wl["desc"], img, method="greedy", bits=(32, 8, 4), lam=0.9, max_iters=2, chunk=32)
    assert len(trace) >= 2
    # the trace's AI is the activation-aware one of the scheme reached
    assert trace[-1]["ai"] == oracle.layer_ai(wl["desc"], q, act_quant=True)[2]
    assert trace[-1]["ai"] > oracle.layer_ai(wl["desc"], q)[2]
    r = m.eval_schemes(img, q[None, :])
    torch.cuda.synchronize()
    assert int(r["agree"][0]) == trace[-1]["agree"]
    m.close()
