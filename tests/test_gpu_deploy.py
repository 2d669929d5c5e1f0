"""GPU parity: deployed inference (aiq_deploy_forward) against the oracle's forward pass of the same scheme.

The deployed path computes the scored function - the network with layer i's weights quantized to
scheme[i] bits - with the dense convolutions of at most 8 bits on the bf16 matrix pipe (integer codes
times three exact bf16 terms of every activation).  Bars are those of scheme scoring: logits within
1e-3 max relative error of the fp64 oracle, top-1 identical except where the oracle's two best logits
are nearly tied.
"""
import numpy as np
import pytest

from parity import LOGIT_REL_TOL, logits_rel_error, near_tied
from test_gpu_eval import _random_graph

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


def _code_layer_count(nodes, scheme):
    """Layers the deployment should run from integer codes: dense convolutions that read an activation
    (not the network input) and carry at most 8 bits."""
    return sum(1 for nd in nodes if nd["kind"] == 0 and nd["input"] >= 0 and nd["scheme_slot"] >= 0
               and scheme[nd["scheme_slot"]] <= 8)


def _deploy_all(env, wl, schemes, chunk, per_tensor=False, fp32_matrix=False, expect_codes=True):
    """Deploys every scheme in turn on one layer-by-layer model; returns logits [S][N][C], top1 [S][N]."""
    torch, aiq = env["torch"], env["aiq"]
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=True, per_tensor=per_tensor)
    img = torch.from_numpy(wl["images"]).cuda()
    logits, top1 = [], []
    for s in schemes:
        d = aiq.Deployed(m, s, fp32_matrix=fp32_matrix)
        if "nodes" in wl and expect_codes:
            assert d.code_layers == (0 if fp32_matrix else _code_layer_count(wl["nodes"], s)), (d.code_layers, s)
        r = d.forward(img, chunk=chunk, want_logits=True)
        torch.cuda.synchronize()
        logits.append(r["logits"].cpu().numpy())
        top1.append(r["top1"].cpu().numpy())
        d.close()
    m.close()
    return np.stack(logits), np.stack(top1)


def _check(logits, top1, ref):
    err = logits_rel_error(logits, ref["logits"])
    assert err <= LOGIT_REL_TOL, f"logit relative error {err:.3e}"
    diff = top1 != ref["top1"]
    assert not (diff & ~near_tied(ref["logits"])).any(), "top-1 differs on a clear margin"
    return err


def _schemes(L, seed):
    """Uniform 8 / 6 / 4 / 2 (every eligible layer on codes), all-FP32, the paper's {32, 8, 4} alphabet, all six."""
    rng = np.random.Generator(np.random.PCG64(seed))
    rows = [np.full((1, L), b, dtype=np.uint8) for b in (8, 6, 4, 2, 32)]
    rows.append(rng.choice(np.array([32, 8, 4], dtype=np.uint8), size=(2, L)))
    rows.append(rng.choice(np.array([32, 16, 8, 6, 4, 2], dtype=np.uint8), size=(2, L)))
    return np.ascontiguousarray(np.concatenate(rows, axis=0))


@pytest.mark.parametrize("index,n", [(5, 20), (1, 24), (6, 12), (0, 40)])
def test_conv_models(env, index, n):
    """PlainConvNet20 (64 channels), ResNet-20 (16/32/64, stride-2 3x3 and 1x1 projections, residuals),
    HeavyEarlyResNet20 and ResNet-8: several tiles per layer, 8x8 maps grouped four images to a workgroup."""
    wl = env["synth"].make_workload(index, n_images=n)
    schemes = _schemes(wl["L"], 100 + index)
    print("deploy %s: S=%d N=%d" % (wl["name"], len(schemes), n), flush=True)
    ref = env["oracle"].eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], schemes)
    logits, top1 = _deploy_all(env, wl, schemes, chunk=16)
    err = _check(logits, top1, ref)
    print("max logit rel err %.3e" % err, flush=True)


def test_mobilenetv2(env):
    """1x1 convolutions of 16..1280 channels (24 and 144 are not multiples of the tile sizes) around depthwise layers."""
    wl = env["synth"].make_workload(3, n_images=4)
    L = wl["L"]
    schemes = np.concatenate([wl["schemes"][:2], np.full((1, L), 8, np.uint8), np.full((1, L), 4, np.uint8)])
    print("deploy mobilenetv2: S=%d" % len(schemes), flush=True)
    ref = env["oracle"].eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], schemes)
    logits, top1 = _deploy_all(env, wl, schemes, chunk=3)
    _check(logits, top1, ref)


@pytest.mark.parametrize("n,chunk", [(37, 16), (5, 1), (3, 1024), (64, 64)])
def test_ragged_chunks(env, n, chunk):
    """N not a multiple of the chunk or of the images-per-workgroup grouping."""
    wl = env["synth"].make_workload(0, n_images=n)
    schemes = _schemes(wl["L"], 7)[[0, 2, 5]]
    print(f"deploy resnet8 ragged n={n} chunk={chunk}", flush=True)
    ref = env["oracle"].eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], schemes)
    logits, top1 = _deploy_all(env, wl, schemes, chunk=chunk)
    _check(logits, top1, ref)


@pytest.mark.parametrize("seed", list(range(12)))
def test_random_graphs(env, seed):
    """Seeded random layer graphs (odd map sizes, channel counts that are multiples of 4 only, both strides,
    residual links) with every layer at 8, 4 or 2 bits and with mixed widths."""
    synth, oracle = env["synth"], env["oracle"]
    rng = np.random.Generator(np.random.PCG64(9000 + seed))
    nodes, ci, h = _random_graph(synth.graphs, rng)
    L = len(nodes)
    w, b = synth.make_model(nodes, rng)
    n = 5
    images = rng.standard_normal((n, h, h, ci)).astype(np.float32)
    desc = synth.desc_array(nodes)
    schemes = np.concatenate([np.full((1, L), 8), np.full((1, L), 4), np.full((1, L), 2),
                              rng.choice([32, 16, 8, 6, 4, 2], size=(2, L))]).astype(np.uint8)
    print("deploy random graph %d: %s" % (seed, " ".join(
        "%s%d>%d/%d@%d%s" % ("cdf"[nd["kind"]], nd["cin"], nd["cout"], nd["stride"], nd["hin"],
                              "+r%d" % nd["residual"] if nd["residual"] >= 0 else "") for nd in nodes)), flush=True)
    ref = oracle.eval_schemes(desc, w, b, images, schemes)
    wl = dict(desc=desc, weights=w, biases=b, images=images, nodes=nodes)
    logits, top1 = _deploy_all(env, wl, schemes, chunk=2, expect_codes=False)
    _check(logits, top1, ref)


def test_per_tensor_scales(env):
    """One quantization scale per layer: the codes and the scale vector come from the per-tensor quantizer."""
    wl = env["synth"].make_workload(0, n_images=24)
    schemes = _schemes(wl["L"], 8)[[0, 2, 6]]
    ref = env["oracle"].eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], schemes, per_tensor=True)
    logits, top1 = _deploy_all(env, wl, schemes, chunk=24, per_tensor=True)
    _check(logits, top1, ref)


def test_fp32_matrix_flag_reproduces_scheme_scoring(env):
    """With every layer kept on the fp32 kernels the deployment runs the launches of aiq_eval_schemes for one
    scheme: bit-identical logits."""
    torch, aiq = env["torch"], env["aiq"]
    wl = env["synth"].make_workload(1, n_images=16)
    scheme = _schemes(wl["L"], 9)[5]
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=True)
    img = torch.from_numpy(wl["images"]).cuda()
    r = m.eval_schemes(img, scheme[None, :], chunk=16, want_logits=True, want_top1=True)
    d = aiq.Deployed(m, scheme, fp32_matrix=True)
    assert d.code_layers == 0
    o = d.forward(img, chunk=16, want_logits=True)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(o["logits"].cpu().numpy().view(np.uint32), r["logits"][0].cpu().numpy().view(np.uint32))
    np.testing.assert_array_equal(o["top1"].cpu().numpy(), r["top1"][0].cpu().numpy())
    d.close()
    m.close()


def test_full_size_sampled(env):
    """The configuration the deployment benchmark times (PlainConvNet20, 2048 images in one chunk, twelve of
    the 64-channel layers at 4 bits), checked on sampled images: every image's forward pass is independent."""
    torch, aiq = env["torch"], env["aiq"]
    wl = env["synth"].make_workload(5, n_images=2048)
    L = wl["L"]
    scheme = np.full(L, 32, np.uint8)
    scheme[8:20] = 4
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=True)
    d = aiq.Deployed(m, scheme)
    assert d.code_layers == 12
    r = d.forward(torch.from_numpy(wl["images"]).cuda(), chunk=2048, want_logits=True)
    torch.cuda.synchronize()
    sample = np.array([0, 1, 255, 256, 1000, 1023, 1024, 2047])
    ref = env["oracle"].eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"][sample], scheme[None, :])
    _check(r["logits"].cpu().numpy()[sample][None], r["top1"].cpu().numpy()[sample][None], ref)
    d.close()
    m.close()


def test_empty_and_errors(env):
    torch, aiq = env["torch"], env["aiq"]
    wl = env["synth"].make_workload(0, n_images=4)
    L = wl["L"]
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=True)
    d = aiq.Deployed(m, np.full(L, 8, np.uint8))
    r = d.forward(torch.empty((0, 32, 32, 3), dtype=torch.float32, device="cuda"))
    assert r["top1"].shape[0] == 0
    d.close()
    with pytest.raises(aiq.AiqError) as e:
        aiq.Deployed(m, np.full(L, 5, np.uint8))
    assert e.value.code == 2
    with pytest.raises(aiq.AiqError) as e:
        aiq.Deployed(m, np.full(L + 1, 8, np.uint8))
    assert e.value.code == 3
    m.close()


@pytest.mark.parametrize("index,n,chunk", [(0, 37, 16), (1, 24, 24), (3, 5, 3)])
def test_lds_resident_models_deploy_on_their_own_kernels(env, index, n, chunk):
    """A model that keeps its activations in LDS is deployed on those kernels: same bits as scoring the scheme,
    parity with the oracle, no integer-code layers."""
    torch, aiq, oracle = env["torch"], env["aiq"], env["oracle"]
    wl = env["synth"].make_workload(index, n_images=n)
    L = wl["L"]
    rng = np.random.Generator(np.random.PCG64(90 + index))
    schemes = [np.full(L, 8, np.uint8), rng.choice(np.array([32, 16, 8, 6, 4, 2], np.uint8), size=L), np.full(L, 32, np.uint8)]
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"])
    assert m.lds_resident or m.lds_resident_blocks > 0
    img = torch.from_numpy(wl["images"]).cuda()
    ref = oracle.eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], np.stack(schemes))
    scored = m.eval_schemes(img, np.stack(schemes), chunk=chunk, want_logits=True, want_top1=True)
    torch.cuda.synchronize()
    blocks = m.lds_resident_blocks
    for i, q in enumerate(schemes):
        # inverted-residual blocks whose 1x1 layers carry at most 8 bits run from integer codes (another
        # summation order); with the fp32-matrix flag every model runs the scoring kernels bit for bit
        d = aiq.Deployed(m, q, fp32_matrix=blocks > 0)
        assert d.code_layers == 0
        out = d.forward(img, chunk=chunk, want_logits=True)
        torch.cuda.synchronize()
        assert torch.equal(out["logits"].view(torch.int32), scored["logits"][i].view(torch.int32))
        assert torch.equal(out["top1"], scored["top1"][i])
        assert logits_rel_error(out["logits"].cpu().numpy(), ref["logits"][i]) <= 1e-3
        only_top1 = d.forward(img[:3], chunk=2)
        torch.cuda.synchronize()
        assert torch.equal(only_top1["top1"], scored["top1"][i][:3]) and only_top1["logits"] is None
        d.close()
    m.close()


def _block_code_layers(nodes, scheme):
    """Layers of inverted-residual blocks (1x1 expand, depthwise, 1x1 project with no other reader of the hidden
    tensors) that a deployment runs from integer codes: every expand or project layer of at most 8 bits; the block
    with 320 output channels (block input in LDS) only when both are."""
    n = 0
    for i in range(len(nodes) - 2):
        e, dw, pj = nodes[i], nodes[i + 1], nodes[i + 2]
        if e["kind"] == 0 and e["kh"] == 1 and e["input"] >= 0 and dw["kind"] == 1 and dw["input"] == i and \
                pj["kind"] == 0 and pj["kh"] == 1 and pj["input"] == i + 1:
            ec, pc = scheme[e["scheme_slot"]] <= 8, scheme[pj["scheme_slot"]] <= 8
            if pj["cout"] == 320 and not (ec and pc):
                continue
            n += int(ec) + int(pc)
    return n


def test_inverted_residual_blocks_from_integer_codes_one_by_one(env):
    """Each block shape of MobileNetV2-32 as a tiny network of its own, deployed: expand and project at 8 / 6 / 4 /
    2 bits run from integer codes inside the block kernel (the depthwise layer at any width); a wider expand or
    project layer keeps the fp32 MFMA inside the same kernel (the 320-channel block then runs on the fp32 block
    kernel).  Logits against the oracle's scoring of the same scheme."""
    synth, oracle, aiq, torch = env["synth"], env["oracle"], env["aiq"], env["torch"]
    shapes = [(16, 96, 24, 32, 1), (24, 144, 24, 32, 1), (24, 144, 32, 32, 1), (32, 192, 32, 32, 1),
              (32, 192, 64, 32, 2), (64, 384, 64, 16, 1), (64, 384, 96, 16, 1), (96, 576, 96, 16, 1),
              (96, 576, 160, 16, 2), (160, 960, 160, 8, 1), (160, 960, 320, 8, 1)]
    schemes = np.array([[32, 8, 8, 8, 32], [32, 8, 32, 8, 32], [8, 4, 16, 6, 8], [32, 2, 4, 2, 32], [32, 6, 2, 4, 4],
                        [32, 16, 8, 8, 32], [32, 8, 8, 32, 32], [32, 4, 32, 16, 8], [16, 32, 6, 2, 32], [32, 32, 8, 16, 32]],
                       dtype=np.uint8)
    on_codes = [2, 2, 2, 2, 2, 1, 1, 1, 1, 0]
    worst = 0.0
    for k, (cin, hid, cout, h, stride) in enumerate(shapes):
        res = stride == 1 and cin == cout
        G = synth.graphs
        nodes = [G._node(G.KIND_CONV, 4, cin, 1, 1, h, -1, act=G.ACT_NONE, slot=0, name="in"),
                 G._node(G.KIND_CONV, cin, hid, 1, 1, h, 0, act=G.ACT_RELU6, slot=1, name="expand"),
                 G._node(G.KIND_DEPTHWISE, hid, hid, 3, stride, h, 1, act=G.ACT_RELU6, slot=2, name="dw"),
                 G._node(G.KIND_CONV, hid, cout, 1, 1, h // stride, 2, residual=0 if res else -1, act=G.ACT_NONE,
                         slot=3, name="project"),
                 G._node(G.KIND_FC, cout, 10, 1, 1, h // stride, 3, act=G.ACT_NONE, slot=4, name="fc")]
        rng = np.random.Generator(np.random.PCG64(700 + k))
        w, b = synth.make_model(nodes, rng)
        n = 5  # an odd count: the 8x8 shapes take two images per workgroup
        images = rng.standard_normal((n, h, h, 4)).astype(np.float32)
        desc = synth.desc_array(nodes)
        print(f"block {cin}->{hid}->{cout} h{h} s{stride} res={res}", flush=True)
        ref = oracle.eval_schemes(desc, w, b, images, schemes)
        m = aiq.Model(desc, w, b)
        assert m.lds_resident_blocks == 1
        img = torch.from_numpy(images).cuda()
        for i, q in enumerate(schemes):
            d = aiq.Deployed(m, q)
            expect = on_codes[i] if (cout != 320 or on_codes[i] != 1) else 0
            assert d.code_layers == expect, (d.code_layers, q)
            out = d.forward(img, chunk=3, want_logits=True)
            torch.cuda.synchronize()
            err = logits_rel_error(out["logits"].cpu().numpy(), ref["logits"][i])
            assert err <= LOGIT_REL_TOL, f"scheme {q}: logit relative error {err:.3e}"
            diff = out["top1"].cpu().numpy() != ref["top1"][i]
            assert not (diff & ~near_tied(ref["logits"][i])).any()
            worst = max(worst, err)
            d.close()
        m.close()
    print("worst logit rel err %.3e" % worst, flush=True)


@pytest.mark.parametrize("n,chunk", [(9, 4), (24, 24)])
def test_mobilenetv2_blocks_from_integer_codes(env, n, chunk):
    """MobileNetV2 deployed on its block kernels: blocks whose 1x1 layers carry at most 8 bits from integer codes,
    the others (and stem, first block, last layer, classifier) on the fp32 kernels; against the oracle."""
    torch, aiq, oracle = env["torch"], env["aiq"], env["oracle"]
    wl = env["synth"].make_workload(3, n_images=n)
    L = wl["L"]
    rng = np.random.Generator(np.random.PCG64(123))
    mixed = rng.choice(np.array([32, 16, 8, 6, 4, 2], np.uint8), size=L)
    low = rng.choice(np.array([8, 6, 4], np.uint8), size=L)
    schemes = [np.full(L, 8, np.uint8), mixed, low, wl["schemes"][0]]
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"])
    assert m.lds_resident_blocks == 16
    img = torch.from_numpy(wl["images"]).cuda()
    ref = oracle.eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], np.stack(schemes))
    for i, q in enumerate(schemes):
        d = aiq.Deployed(m, q)
        last_conv = wl["nodes"][-2]  # the 1x1 layer whose epilogue forms the classifier's pooling
        assert d.code_layers == _block_code_layers(wl["nodes"], q) + (1 if q[last_conv["scheme_slot"]] <= 8 else 0), (d.code_layers, q)
        out = d.forward(img, chunk=chunk, want_logits=True)
        torch.cuda.synchronize()
        err = _check(out["logits"].cpu().numpy(), out["top1"].cpu().numpy(), dict(logits=ref["logits"][i], top1=ref["top1"][i]))
        print("scheme %d: %d layers on codes, logit rel err %.3e" % (i, d.code_layers, err), flush=True)
        if i == 0:
            assert d.code_layers == 33
        d.close()
    m.close()


def test_last_1x1_layer_with_pooling_from_integer_codes(env):
    """A 1x1 layer on 8x8 pixels that only the classifier reads writes the mean of its outputs; deployed at 8 bits or
    less it runs from integer codes.  Channel counts that leave partial 32-channel steps, partial tiles of 16 output
    channels and both tile groupings (five tiles at a time when the tile count is a multiple of five, else two)."""
    synth, oracle, aiq, torch = env["synth"], env["oracle"], env["aiq"], env["torch"]
    G = synth.graphs
    cases = [(320, 1280, G.ACT_RELU6), (24, 36, G.ACT_RELU), (40, 80, G.ACT_NONE), (96, 100, G.ACT_RELU6), (8, 16, G.ACT_RELU6),
             (416, 64, G.ACT_RELU6), (20, 32, G.ACT_RELU6)]  # the last one stays on the fp32 kernel: 20 % 8 != 0
    schemes = np.array([[32, 8, 32], [8, 4, 8], [32, 2, 4], [32, 6, 32], [32, 16, 32]], dtype=np.uint8)
    worst = 0.0
    for k, (cin, cout, act) in enumerate(cases):
        nodes = [G._node(G.KIND_CONV, 4, cin, 1, 1, 8, -1, act=G.ACT_RELU, slot=0, name="in"),
                 G._node(G.KIND_CONV, cin, cout, 1, 1, 8, 0, act=act, slot=1, name="last"),
                 G._node(G.KIND_FC, cout, 10, 1, 1, 8, 1, act=G.ACT_NONE, slot=2, name="fc")]
        rng = np.random.Generator(np.random.PCG64(900 + k))
        w, b = synth.make_model(nodes, rng)
        n = 7
        images = rng.standard_normal((n, 8, 8, 4)).astype(np.float32)
        desc = synth.desc_array(nodes)
        ref = oracle.eval_schemes(desc, w, b, images, schemes)
        m = aiq.Model(desc, w, b)
        img = torch.from_numpy(images).cuda()
        for i, q in enumerate(schemes):
            d = aiq.Deployed(m, q)
            assert d.code_layers == (1 if q[1] <= 8 and cin % 8 == 0 else 0), (d.code_layers, q)
            out = d.forward(img, chunk=4, want_logits=True)
            torch.cuda.synchronize()
            err = logits_rel_error(out["logits"].cpu().numpy(), ref["logits"][i])
            assert err <= LOGIT_REL_TOL, f"{cin}->{cout} scheme {q}: logit relative error {err:.3e}"
            diff = out["top1"].cpu().numpy() != ref["top1"][i]
            assert not (diff & ~near_tied(ref["logits"][i])).any()
            worst = max(worst, err)
            d.close()
        m.close()
        print(f"{cin}->{cout}: ok", flush=True)
    print("worst logit rel err %.3e" % worst, flush=True)


@pytest.mark.parametrize("index", [3, 8])
def test_mobilenetv2_full_size_sampled_from_integer_codes(env, index):
    """The configuration the deployment benchmark times on MobileNetV2 (2048 images in one chunk, every layer at 8
    bits: 33 layers from integer codes inside the block kernels; and a mixed scheme), on sampled images including
    the first and last of the launch; on the model with the centred classifier also the agreement with FP32."""
    torch, aiq, oracle = env["torch"], env["aiq"], env["oracle"]
    wl = env["synth"].make_workload(index, n_images=2048)
    L = wl["L"]
    rng = np.random.Generator(np.random.PCG64(77))
    mixed = rng.choice(np.array([32, 8, 4], np.uint8), size=L)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"])
    img = torch.from_numpy(wl["images"]).cuda()
    sample = np.array([0, 1, 2, 255, 256, 511, 512, 1000, 1023, 1024, 1025, 2046, 2047])
    for q, layers in ((np.full(L, 8, np.uint8), 33), (mixed, None)):
        d = aiq.Deployed(m, q)
        if layers is not None:
            assert d.code_layers == layers
        r = d.forward(img, chunk=2048, want_logits=True)
        torch.cuda.synchronize()
        ref = oracle.eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"][sample], q[None, :])
        if index == 8:
            # centred classifier: every logit is a small difference of the classifier's response and a bias of about
            # the same size, so the response (logit minus bias) is what the 1e-3 bar is applied to (parity.py), and
            # the integer decision must be the argmax of the GPU's own logits
            b = np.asarray(wl["biases"][-1], np.float64)
            zg = r["logits"].cpu().numpy().astype(np.float64)
            err = logits_rel_error(zg[sample][None] - b, ref["logits"] - b)
            assert err <= LOGIT_REL_TOL, err
            np.testing.assert_array_equal(r["top1"].cpu().numpy(), zg.argmax(axis=1))
        else:
            err = _check(r["logits"].cpu().numpy()[sample][None], r["top1"].cpu().numpy()[sample][None], ref)
        print("workload %d: %d layers on codes, sampled error %.3e" % (index, d.code_layers, err), flush=True)
        d.close()
    m.close()


def test_per_tensor_scales_on_block_kernels(env):
    """One quantization scale per layer on a model deployed on its block kernels: the codes and the (constant)
    scale vectors of the blocks' 1x1 layers and of the pooled last layer come from the per-tensor quantizer."""
    torch, aiq, oracle = env["torch"], env["aiq"], env["oracle"]
    wl = env["synth"].make_workload(3, n_images=10)
    L = wl["L"]
    rng = np.random.Generator(np.random.PCG64(31))
    schemes = np.stack([np.full(L, 8, np.uint8), rng.choice(np.array([32, 8, 6, 4], np.uint8), size=L)])
    ref = oracle.eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], schemes, per_tensor=True)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"], per_tensor=True)
    assert m.lds_resident_blocks == 16
    img = torch.from_numpy(wl["images"]).cuda()
    for i, q in enumerate(schemes):
        d = aiq.Deployed(m, q)
        assert d.code_layers > 0
        out = d.forward(img, chunk=6, want_logits=True)
        torch.cuda.synchronize()
        err = _check(out["logits"].cpu().numpy()[None], out["top1"].cpu().numpy()[None],
                     dict(logits=ref["logits"][i][None], top1=ref["top1"][i][None]))
        print("scheme %d: %d layers on codes, logit rel err %.3e" % (i, d.code_layers, err), flush=True)
        d.close()
    m.close()
