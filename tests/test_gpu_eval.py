"""GPU parity: aiq_eval_schemes against the oracle on the benchmark workloads.

Bars: logits within 1e-3 max relative error, top-1 identical except where the
oracle's two best logits are nearly tied (relative margin < 1e-5), agreement
counts equal up to the number of such near-ties.
"""
import numpy as np
import pytest

from parity import check_centred_sample, check_eval, logits_rel_error, near_tied

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


PATHS = [pytest.param(False, id="lds_resident"), pytest.param(True, id="layerwise")]


def _run_gpu(env, wl, schemes, chunk, top1_base=None, model=None, layerwise=False, expect_resident=None):
    torch, aiq = env["torch"], env["aiq"]
    m = model or aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=layerwise)
    if expect_resident is not None:
        assert m.lds_resident == expect_resident
    img = torch.from_numpy(wl["images"]).cuda()
    r = m.eval_schemes(img, schemes, chunk=chunk, want_logits=True, want_top1=True, top1_base=top1_base)
    torch.cuda.synchronize()
    out = {k: (None if v is None else v.cpu().numpy()) for k, v in r.items()}
    if model is None:
        m.close()
    return out


def _extra_schemes(wl, seed):
    """The workload's schemes plus: all-FP32, every uniform width, and random mixes of all six widths."""
    L = wl["L"]
    rng = np.random.Generator(np.random.PCG64(seed))
    rows = [wl["schemes"], np.full((1, L), 32, dtype=np.uint8)]
    rows += [np.full((1, L), b, dtype=np.uint8) for b in (16, 8, 6, 4, 2)]
    rows.append(rng.choice(np.array([32, 16, 8, 6, 4, 2], dtype=np.uint8), size=(3, L)))
    return np.ascontiguousarray(np.concatenate(rows, axis=0))


_ORACLE_CACHE = {}


def _oracle_sample(env, key, wl, idx, schemes):
    """Oracle scoring of `schemes` on images `idx` of a workload, computed once per test session
    (the two kernel paths are checked against the same reference)."""
    if key not in _ORACLE_CACHE:
        _ORACLE_CACHE[key] = env["oracle"].eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"][idx],
                                                        schemes)
    return _ORACLE_CACHE[key]


def _check_sample(gpu, ref, idx):
    """Logits, top-1 and the agreement count restricted to the sampled images `idx`, against the oracle."""
    err = logits_rel_error(gpu["logits"][:, idx], ref["logits"])
    assert err <= 1e-3, err
    tie, tie_base = near_tied(ref["logits"]), near_tied(ref["logits_base"])
    assert not ((gpu["top1"][:, idx] != ref["top1"]) & ~tie).any()
    assert not ((gpu["top1_base"][idx] != ref["top1_base"]) & ~tie_base).any()
    agree_sample = (gpu["top1"][:, idx] == gpu["top1_base"][idx][None]).sum(axis=1)
    slack = (tie | tie_base[None, :]).sum(axis=1)
    assert (np.abs(agree_sample - ref["agree"]) <= slack).all(), (agree_sample, ref["agree"])
    np.testing.assert_array_equal(gpu["agree"], (gpu["top1"] == gpu["top1_base"][None]).sum(axis=1))
    return err, agree_sample


@pytest.mark.parametrize("layerwise", PATHS)
def test_resnet8_full_workload(env, layerwise):
    """Workload 0 at full size: 256 images, the seeded scheme plus uniform and mixed extras."""
    wl = env["synth"].make_workload(0)
    schemes = _extra_schemes(wl, 5)
    print("resnet8 full: S=%d N=%d" % (schemes.shape[0], wl["images"].shape[0]), flush=True)
    ref = env["oracle"].eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], schemes)
    gpu = _run_gpu(env, wl, schemes, chunk=1024, layerwise=layerwise, expect_resident=not layerwise)
    err = check_eval(gpu, ref, 256)
    print("max logit rel err %.3e agree gpu %s" % (err, gpu["agree"]), flush=True)
    # the all-FP32 scheme (row 1) reproduces the base pass exactly
    assert gpu["agree"][1] == 256


@pytest.mark.parametrize("layerwise", PATHS)
@pytest.mark.parametrize("n,chunk", [(37, 16), (5, 1), (64, 64), (3, 1024)])
def test_resnet8_ragged_chunks(env, n, chunk, layerwise):
    """N not a multiple of the chunk, of the images-per-workgroup grouping, or of anything else."""
    wl = env["synth"].make_workload(0, n_images=n)
    schemes = _extra_schemes(wl, 6)[:4]
    print(f"resnet8 ragged n={n} chunk={chunk}", flush=True)
    ref = env["oracle"].eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], schemes)
    gpu = _run_gpu(env, wl, schemes, chunk=chunk, layerwise=layerwise)
    check_eval(gpu, ref, n)


@pytest.mark.parametrize("layerwise", PATHS)
def test_resnet20_workload1(env, layerwise):
    """Workload 1 (ResNet-20, one scheme over {32,16,8,4}) on its first 96 images, chunked 64 + 32."""
    wl = env["synth"].make_workload(1, n_images=96)
    schemes = _extra_schemes(wl, 7)
    print("resnet20: S=%d N=96" % schemes.shape[0], flush=True)
    ref = env["oracle"].eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], schemes)
    gpu = _run_gpu(env, wl, schemes, chunk=64, layerwise=layerwise, expect_resident=not layerwise)
    err = check_eval(gpu, ref, 96)
    print("max logit rel err %.3e" % err, flush=True)


@pytest.mark.parametrize("layerwise", [pytest.param(False, id="lds_resident_blocks"), pytest.param(True, id="layerwise")])
def test_mobilenetv2_workload3(env, layerwise):
    """Workload 3 (MobileNetV2-32, 10 random layers at 4 bits) on 7 images, 5 of its schemes + extras;
    chunks of 5 and 2 images (odd counts: the 8x8 blocks take two images per workgroup)."""
    aiq = env["aiq"]
    wl = env["synth"].make_workload(3, n_images=7, n_schemes=5)
    schemes = np.concatenate([wl["schemes"], np.full((1, wl["L"]), 32, np.uint8), np.full((1, wl["L"]), 8, np.uint8),
                              np.full((1, wl["L"]), 2, np.uint8)])
    print("mobilenetv2: S=%d N=7 layerwise=%s" % (schemes.shape[0], layerwise), flush=True)
    ref = env["oracle"].eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], schemes)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=layerwise)
    assert not m.lds_resident
    # every inverted-residual block with an expand layer (16 of 17) keeps its hidden tensor in LDS
    assert m.lds_resident_blocks == (0 if layerwise else 16)
    gpu = _run_gpu(env, wl, schemes, chunk=5, model=m)
    m.close()
    err = check_eval(gpu, ref, 7)
    print("max logit rel err %.3e" % err, flush=True)


def test_mobilenetv2_full_size_sampled(env):
    """Workload 3 in the benchmark's launch configuration (16 schemes x 512 images, one chunk); the
    oracle recomputes every scheme on a sample of images, the agreement identity covers the rest."""
    wl = env["synth"].make_workload(3)
    print("mobilenetv2 full size", flush=True)
    gpu = _run_gpu(env, wl, wl["schemes"], chunk=1024)
    rng = np.random.Generator(np.random.PCG64(4))
    idx = np.unique(np.concatenate([[0, 1, 255, 256, 510, 511], rng.choice(512, 20, replace=False)]))[:26]
    assert len(idx) >= 24
    ref = _oracle_sample(env, "w3", wl, idx, wl["schemes"])
    err, _ = _check_sample(gpu, ref, idx)
    print("sampled (%d images) max logit rel err %.3e; agree %s" % (len(idx), err, gpu["agree"]), flush=True)


@pytest.mark.parametrize("layerwise", [pytest.param(False, id="lds_resident_blocks"), pytest.param(True, id="layerwise")])
def test_mobilenetv2_centred_full_size_sampled(env, layerwise):
    """Workload 8: MobileNetV2 with the centred classifier at the benchmark's size (16 schemes x 512 images):
    the FP32 predictions cover the classes and ten layers at 4 bits change most of them, so top-1 and the
    agreement counts are compared with the oracle where they are not trivially N."""
    wl = env["synth"].make_workload(8)
    print("mobilenetv2 centred full size, layerwise=%s" % layerwise, flush=True)
    gpu = _run_gpu(env, wl, wl["schemes"], chunk=1024, layerwise=layerwise)
    idx = np.concatenate([np.arange(0, 12), np.arange(500, 512)])
    ref = _oracle_sample(env, "w8", wl, idx, wl["schemes"])
    err, agree_sample, frac = check_centred_sample(gpu, ref, idx, wl["biases"][-1])
    assert len(set(np.bincount(gpu["top1_base"], minlength=10).nonzero()[0])) >= 5
    assert gpu["agree"].max() < 512 and len(set(gpu["agree"].tolist())) >= 4, gpu["agree"]
    print("sampled max response rel err %.3e; %.4f of the samples within the deviation of a tie; agree %s; on the sample %s "
          "(oracle %s)" % (err, frac, gpu["agree"], agree_sample, ref["agree"]), flush=True)


def test_inverted_residual_blocks_one_by_one(env):
    """Each block shape of MobileNetV2-32 as a tiny network of its own (stem-like 1x1 feeding the
    block is not needed: the block reads the network input), LDS-resident against layer by layer
    and against the oracle, with every bit-width on each of the three layers."""
    synth, oracle, aiq, torch = env["synth"], env["oracle"], env["aiq"], env["torch"]
    shapes = [(16, 96, 24, 32, 1), (24, 144, 24, 32, 1), (24, 144, 32, 32, 1), (32, 192, 32, 32, 1),
              (32, 192, 64, 32, 2), (64, 384, 64, 16, 1), (64, 384, 96, 16, 1), (96, 576, 96, 16, 1),
              (96, 576, 160, 16, 2), (160, 960, 160, 8, 1), (160, 960, 320, 8, 1)]
    for k, (cin, hid, cout, h, stride) in enumerate(shapes):
        res = stride == 1 and cin == cout
        G = synth.graphs
        nodes = [G._node(G.KIND_CONV, 4, cin, 1, 1, h, -1, act=G.ACT_NONE, slot=0, name="in"),
                 G._node(G.KIND_CONV, cin, hid, 1, 1, h, 0, act=G.ACT_RELU6, slot=1, name="expand"),
                 G._node(G.KIND_DEPTHWISE, hid, hid, 3, stride, h, 1, act=G.ACT_RELU6, slot=2, name="dw"),
                 G._node(G.KIND_CONV, hid, cout, 1, 1, h // stride, 2, residual=0 if res else -1, act=G.ACT_NONE,
                         slot=3, name="project"),
                 G._node(G.KIND_FC, cout, 10, 1, 1, h // stride, 3, act=G.ACT_NONE, slot=4, name="fc")]
        rng = np.random.Generator(np.random.PCG64(300 + k))
        w, b = synth.make_model(nodes, rng)
        n = 5
        images = rng.standard_normal((n, h, h, 4)).astype(np.float32)
        desc = synth.desc_array(nodes)
        schemes = np.array([[32, 32, 32, 32, 32], [32, 8, 4, 2, 32], [32, 2, 16, 6, 8], [8, 4, 8, 4, 4]], dtype=np.uint8)
        print(f"block {cin}->{hid}->{cout} h{h} s{stride} res={res}", flush=True)
        ref = oracle.eval_schemes(desc, w, b, images, schemes)
        wl = dict(desc=desc, weights=w, biases=b, images=images)
        m = aiq.Model(desc, w, b)
        assert m.lds_resident_blocks == 1
        gpu = _run_gpu(env, wl, schemes, chunk=3, model=m)
        m.close()
        err = check_eval(gpu, ref, n)
        print("  max logit rel err %.3e" % err, flush=True)


def test_depthwise_layers_outside_blocks(env):
    """Stand-alone depthwise kernel: widths that are multiples of 4, of 2 only, and odd; both strides;
    channel counts from 8 to 200; every bit-width on the depthwise layer."""
    synth, oracle, aiq = env["synth"], env["oracle"], env["aiq"]
    G = synth.graphs
    cases = [(32, 32, 1), (12, 24, 1), (10, 8, 1), (7, 200, 1), (5, 16, 1), (32, 48, 2), (12, 16, 2), (14, 40, 2),
             (9, 8, 2), (6, 96, 2)]
    for k, (h, c, stride) in enumerate(cases):
        ho = (h + 2 - 3) // stride + 1
        nodes = [G._node(G.KIND_CONV, 4, c, 1, 1, h, -1, act=G.ACT_RELU, slot=0, name="in"),
                 G._node(G.KIND_DEPTHWISE, c, c, 3, stride, h, 0, act=G.ACT_RELU6, slot=1, name="dw"),
                 G._node(G.KIND_DEPTHWISE, c, c, 3, 1, ho, 1, act=G.ACT_NONE, slot=2, name="dw2"),
                 G._node(G.KIND_FC, c, 10, 1, 1, ho, 2, act=G.ACT_NONE, slot=3, name="fc")]
        rng = np.random.Generator(np.random.PCG64(500 + k))
        w, b = synth.make_model(nodes, rng)
        n = 6
        images = rng.standard_normal((n, h, h, 4)).astype(np.float32)
        desc = synth.desc_array(nodes)
        schemes = np.array([[32, 32, 32, 32], [32, 8, 4, 32], [8, 2, 16, 6], [4, 6, 2, 8]], dtype=np.uint8)
        print(f"depthwise h={h} c={c} stride={stride}", flush=True)
        ref = oracle.eval_schemes(desc, w, b, images, schemes)
        gpu = _run_gpu(env, dict(desc=desc, weights=w, biases=b, images=images), schemes, chunk=4)
        err = check_eval(gpu, ref, n)
        print("  max logit rel err %.3e" % err, flush=True)


def test_stem_dense_and_pooled_layers_on_odd_shapes(env):
    """Layer-by-layer kernels on shapes the workloads do not have: stems with 1, 2, 3 and 4 input channels
    and 16 to 72 output channels on images of 5 to 32 pixels (several images per workgroup, ragged last
    group, widths that are not a multiple of 16); dense 3x3 layers with 20 to 112 input channels (one, two and
    three staging passes, a last pass of three channel blocks), both strides, with a residual; and an 8x8
    1x1 layer read only by the classifier, whose average pool is formed inside that layer."""
    synth, oracle, aiq = env["synth"], env["oracle"], env["aiq"]
    G = synth.graphs
    cases = [  # image channels, image size, stem width, mid width, stride of the second conv, last 1x1 width
        (3, 32, 64, 64, 1, 0), (1, 16, 16, 20, 2, 0), (2, 5, 24, 24, 1, 0), (4, 9, 72, 112, 2, 0),
        (3, 16, 40, 48, 2, 96), (4, 8, 112, 64, 1, 1280), (3, 8, 16, 16, 1, 44)]
    for k, (ci, h, c1, c2, stride, cl) in enumerate(cases):
        ho = (h + 2 - 3) // stride + 1
        nodes = [G._node(G.KIND_CONV, ci, c1, 3, 1, h, -1, act=G.ACT_RELU, slot=0, name="stem"),
                 G._node(G.KIND_CONV, c1, c2, 3, stride, h, 0, act=G.ACT_RELU6, slot=1, name="c2"),
                 G._node(G.KIND_CONV, c2, c2, 3, 1, ho, 1, residual=1, act=G.ACT_RELU, slot=2, name="c3")]
        if cl:
            nodes.append(G._node(G.KIND_CONV, c2, cl, 1, 1, ho, 2, act=G.ACT_RELU6, slot=3, name="last"))
        nodes.append(G._node(G.KIND_FC, cl or c2, 10, 1, 1, ho, len(nodes) - 1, act=G.ACT_NONE, slot=len(nodes), name="fc"))
        L = len(nodes)
        rng = np.random.Generator(np.random.PCG64(700 + k))
        w, b = synth.make_model(nodes, rng)
        n = 7
        images = rng.standard_normal((n, h, h, ci)).astype(np.float32)
        desc = synth.desc_array(nodes)
        schemes = np.concatenate([np.full((1, L), 32), rng.choice([32, 16, 8, 6, 4, 2], size=(3, L))]).astype(np.uint8)
        print(f"odd shapes: {ci}x{h}x{h} -> {c1} -> {c2} (stride {stride}) -> {cl or '-'}", flush=True)
        ref = oracle.eval_schemes(desc, w, b, images, schemes)
        gpu = _run_gpu(env, dict(desc=desc, weights=w, biases=b, images=images), schemes, chunk=3)
        err = check_eval(gpu, ref, n)
        print("  max logit rel err %.3e" % err, flush=True)


def _random_graph(G, rng):
    """A seeded chain of 4 to 7 layers with optional residual links: 3x3 / 1x1 convolutions and depthwise
    layers of both strides on square maps of 6 to 20 pixels, channel counts that are multiples of 4."""
    ci = int(rng.choice([1, 3, 4]))
    h = int(rng.integers(6, 21))
    widths = [8, 12, 16, 24, 40, 64, 100]
    c = int(rng.choice(widths))
    nodes = [G._node(G.KIND_CONV, ci, c, 3, 1, h, -1, act=int(rng.integers(0, 3)), slot=0, name="stem")]
    shapes = [(c, h)]  # output (channels, size) of every node
    for i in range(int(rng.integers(3, 7))):
        c_in, h_in = shapes[-1]
        kind = str(rng.choice(["c3", "c3", "c1", "dw", "c3s2", "dws2", "c1s2"]))
        stride = 2 if kind.endswith("s2") and h_in >= 4 else 1
        k = 1 if kind.startswith("c1") else 3
        h_out = (h_in + 2 * (k // 2) - k) // stride + 1
        if kind.startswith("dw"):
            nodes.append(G._node(G.KIND_DEPTHWISE, c_in, c_in, 3, stride, h_in, len(nodes) - 1, act=int(rng.integers(0, 3)),
                                 slot=len(nodes), name=f"dw{i}"))
            shapes.append((c_in, h_out))
            continue
        c_out = int(rng.choice(widths))
        # a residual link to any earlier output of the same shape (choose the width to match one half of the time)
        cands = [j for j, (cj, hj) in enumerate(shapes) if hj == h_out]
        res = -1
        if cands and rng.random() < 0.5:
            res = int(rng.choice(cands))
            c_out = shapes[res][0]
        nodes.append(G._node(G.KIND_CONV, c_in, c_out, k, stride, h_in, len(nodes) - 1, residual=res,
                             act=int(rng.integers(0, 3)), slot=len(nodes), name=f"c{i}"))
        shapes.append((c_out, h_out))
    c_last, h_last = shapes[-1]
    nodes.append(G._node(G.KIND_FC, c_last, int(rng.choice([2, 10, 37])), 1, 1, h_last, len(nodes) - 1, act=G.ACT_NONE,
                         slot=len(nodes), name="fc"))
    return nodes, ci, h


@pytest.mark.parametrize("seed", list(range(12)))
def test_random_graphs(env, seed):
    """Seeded random layer graphs against the oracle, in the default mode and with the layer-by-layer kernels
    forced, and the shared-prefix entry point against the plain one on the same graph."""
    synth, oracle, aiq, torch = env["synth"], env["oracle"], env["aiq"], env["torch"]
    rng = np.random.Generator(np.random.PCG64(9000 + seed))
    nodes, ci, h = _random_graph(synth.graphs, rng)
    L = len(nodes)
    w, b = synth.make_model(nodes, rng)
    n = 5
    images = rng.standard_normal((n, h, h, ci)).astype(np.float32)
    desc = synth.desc_array(nodes)
    schemes = np.concatenate([np.full((1, L), 32), rng.choice([32, 16, 8, 6, 4, 2], size=(4, L))]).astype(np.uint8)
    print("random graph %d: %s" % (seed, " ".join(
        "%s%d>%d/%d@%d%s" % ("cdf"[nd["kind"]], nd["cin"], nd["cout"], nd["stride"], nd["hin"],
                              "+r%d" % nd["residual"] if nd["residual"] >= 0 else "") for nd in nodes)), flush=True)
    ref = oracle.eval_schemes(desc, w, b, images, schemes)
    wl = dict(desc=desc, weights=w, biases=b, images=images)
    for layerwise in (False, True):
        gpu = _run_gpu(env, wl, schemes, chunk=2, layerwise=layerwise)
        check_eval(gpu, ref, n)
    m = aiq.Model(desc, w, b)
    img = torch.from_numpy(images).cuda()
    outs = []
    for r in (None, schemes[1]):
        o = m.eval_schemes(img, schemes, chunk=3, want_logits=True, want_top1=True, ref_scheme=r)
        torch.cuda.synchronize()
        outs.append({k: v.cpu().numpy() for k, v in o.items()})
    m.close()
    for k in ("agree", "top1_base", "top1"):
        np.testing.assert_array_equal(outs[0][k], outs[1][k], err_msg=k)
    np.testing.assert_array_equal(outs[0]["logits"].view(np.uint32), outs[1]["logits"].view(np.uint32))


@pytest.mark.parametrize("case", ["resnet8", "resnet8_layerwise", "mobilenetv2"])
def test_per_tensor_scales(env, case):
    """Scheme scoring with one quantization scale per layer (per-tensor variant) against the oracle's."""
    aiq = env["aiq"]
    if case == "mobilenetv2":
        wl = env["synth"].make_workload(3, n_images=4, n_schemes=3)
        schemes = np.concatenate([wl["schemes"], np.full((1, wl["L"]), 8, np.uint8), np.full((1, wl["L"]), 4, np.uint8)])
    else:
        wl = env["synth"].make_workload(0, n_images=24)
        schemes = _extra_schemes(wl, 11)
    n = wl["images"].shape[0]
    print(f"per-tensor scales: {case}", flush=True)
    ref = env["oracle"].eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], schemes, per_tensor=True)
    ref_c = env["oracle"].eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], schemes)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=case.endswith("layerwise"), per_tensor=True)
    gpu = _run_gpu(env, wl, schemes, chunk=16, model=m)
    m.close()
    check_eval(gpu, ref, n)
    # and it is not the per-channel result
    assert logits_rel_error(gpu["logits"], ref_c["logits"]) > 1e-3


def test_variant_models(env):
    """PlainConvNet20 and HeavyEarlyResNet20 descriptors (64-channel layers at 32x32, stride-1 projection)."""
    synth, oracle = env["synth"], env["oracle"]
    for name, nodes in (("plain", synth.plain_convnet20()), ("heavy", synth.heavy_early_resnet20())):
        rng = np.random.Generator(np.random.PCG64(99))
        w, b = synth.make_model(nodes, rng)
        images = synth.make_images(5, rng)
        L = synth.n_scheme_layers(nodes)
        wl = dict(desc=synth.desc_array(nodes), weights=w, biases=b, images=images, L=L,
                  schemes=rng.choice(np.array([32, 8, 4], dtype=np.uint8), size=(2, L)))
        print(f"variant {name}: L={L}", flush=True)
        ref = oracle.eval_schemes(wl["desc"], w, b, images, wl["schemes"])
        gpu = _run_gpu(env, wl, wl["schemes"], chunk=4, expect_resident=False)
        check_eval(gpu, ref, 5)


@pytest.mark.parametrize("layerwise", PATHS)
def test_greedy_step_full_size_sampled(env, layerwise):
    """Workload 2 in the benchmark's launch configuration (40 schemes x 1024 images, one chunk);
    the oracle recomputes every scheme on a sample of images, properties cover the rest."""
    torch = env["torch"]
    wl = env["synth"].make_workload(2)
    print("greedy step full size", flush=True)
    gpu = _run_gpu(env, wl, wl["schemes"], chunk=1024, layerwise=layerwise)
    rng = np.random.Generator(np.random.PCG64(3))
    idx = np.unique(np.concatenate([[0, 1, 1022, 1023], rng.choice(1024, 126, replace=False)]))
    assert len(idx) >= 128
    ref = _oracle_sample(env, "w2", wl, idx, wl["schemes"])
    err, _ = _check_sample(gpu, ref, idx)
    print("sampled (%d images) max logit rel err %.3e; agree %s" % (len(idx), err, gpu["agree"]), flush=True)


@pytest.mark.parametrize("layerwise", PATHS)
def test_greedy_step_centred_full_size(env, layerwise):
    """Workload 7: the greedy step of workload 2 on a ResNet-20 whose classifier is centred, at the
    benchmark's size (40 schemes x 1024 images, one chunk).  The FP32 predictions cover all classes, 8-bit
    single-layer moves flip a few per cent of them and 4-bit moves up to four fifths, so the argmax, the
    near-tie rule and the agreement counts are checked where their outcome is not trivial: every scheme on
    256 images (the first and the last 128 of the grid) against the oracle, by the rule for centred
    workloads (parity.check_centred_sample)."""
    wl = env["synth"].make_workload(7)
    print("greedy step, centred classifier, full size, layerwise=%s" % layerwise, flush=True)
    gpu = _run_gpu(env, wl, wl["schemes"], chunk=1024, layerwise=layerwise)
    idx = np.concatenate([np.arange(0, 128), np.arange(896, 1024)])
    ref = _oracle_sample(env, "w7", wl, idx, wl["schemes"])
    err, agree_sample, frac = check_centred_sample(gpu, ref, idx, wl["biases"][-1])
    hist = np.bincount(gpu["top1_base"], minlength=10)
    assert (hist > 0).sum() >= 8 and hist.max() < 512, hist
    agree = gpu["agree"]
    assert agree.max() < 1024 and agree.min() > 0 and len(set(agree.tolist())) >= 20, agree
    # single-layer 8-bit moves keep more predictions than the 4-bit move of the same layer
    assert (agree[0::2] > agree[1::2]).all(), agree
    # the oracle's counts on the sample vary as well (they were compared above, near-tie slack included)
    assert len(set(ref["agree"].tolist())) >= 20 and ref["agree"].max() < 256
    print("max response rel err %.3e; %.4f of the samples within the deviation of a tie; agree %s; on the sample %s" %
          (err, frac, agree.tolist(), agree_sample.tolist()), flush=True)


def test_resnet20_workload1_full_size_sampled(env):
    """Workload 1 at full size (1 scheme over {32,16,8,4} x 1024 images, one chunk); oracle on a sample."""
    wl = env["synth"].make_workload(1)
    print("workload 1 full size", flush=True)
    gpu = _run_gpu(env, wl, wl["schemes"], chunk=1024)
    rng = np.random.Generator(np.random.PCG64(6))
    idx = np.unique(np.concatenate([[0, 1, 2, 511, 512, 1000, 1022, 1023], rng.choice(1024, 64, replace=False)]))
    ref = env["oracle"].eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"][idx], wl["schemes"])
    _check_sample(gpu, ref, idx)


def test_cd_sweep_full_size_sampled(env):
    """Workload 4 in the benchmark's launch configuration: 64 schemes over all six widths x 10 000
    images in chunks of 1024 (9 full chunks and one of 784), agreement counts only - plus one call
    with logits for the oracle to check on images around every chunk boundary."""
    torch, aiq = env["torch"], env["aiq"]
    wl = env["synth"].make_workload(4)
    print("workload 4 full size", flush=True)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"])
    img = torch.from_numpy(wl["images"]).cuda()
    r = m.eval_schemes(img, wl["schemes"], chunk=1024)
    torch.cuda.synchronize()
    agree = r["agree"].cpu().numpy()
    assert r["logits"] is None and agree.shape == (64,)
    full = m.eval_schemes(img, wl["schemes"], chunk=1024, want_logits=True, want_top1=True, top1_base=r["top1_base"])
    torch.cuda.synchronize()
    top1, top1_base = full["top1"].cpu().numpy(), full["top1_base"].cpu().numpy()
    np.testing.assert_array_equal(agree, (top1 == top1_base[None]).sum(axis=1))
    np.testing.assert_array_equal(agree, full["agree"].cpu().numpy())
    # both sides of every chunk boundary, the ends of the grid, and 64 images in between
    bounds = np.arange(1024, 10000, 1024)
    rng = np.random.Generator(np.random.PCG64(5))
    idx = np.unique(np.concatenate([[0, 1, 9998, 9999], bounds - 1, bounds, bounds + 1, rng.choice(10000, 64, replace=False)]))
    assert len(idx) >= 64 + 27
    ref = env["oracle"].eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"][idx], wl["schemes"])
    logits = full["logits"][:, torch.from_numpy(idx).cuda()].cpu().numpy()
    assert logits_rel_error(logits, ref["logits"]) <= 1e-3
    tie, tie_base = near_tied(ref["logits"]), near_tied(ref["logits_base"])
    assert not ((top1[:, idx] != ref["top1"]) & ~tie).any()
    assert not ((top1_base[idx] != ref["top1_base"]) & ~tie_base).any()
    agree_sample = (top1[:, idx] == top1_base[idx][None]).sum(axis=1)
    assert (np.abs(agree_sample - ref["agree"]) <= (tie | tie_base[None]).sum(axis=1)).all()
    # schemes made only of 32- and 16-bit layers barely change a prediction; 2-bit layers change many
    sch = wl["schemes"]
    assert agree.max() <= 10000 and agree.min() >= 0
    m.close()
    print("agree min/max", agree.min(), agree.max(), flush=True)


def test_cd_sweep_chunk_remainder_sampled(env):
    """Workload 4's chunking (chunks of 1024 with a ragged last chunk) on 2100 images and 6 of its
    schemes; the oracle checks images on both sides of every chunk boundary and in the tail."""
    wl = env["synth"].make_workload(4, n_images=2100, n_schemes=6)
    print("cd sweep chunks", flush=True)
    gpu = _run_gpu(env, wl, wl["schemes"], chunk=1024)
    idx = np.array([0, 1, 1022, 1023, 1024, 1025, 2046, 2047, 2048, 2049, 2098, 2099])
    ref = env["oracle"].eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"][idx], wl["schemes"])
    assert logits_rel_error(gpu["logits"][:, idx], ref["logits"]) <= 1e-3
    assert not ((gpu["top1"][:, idx] != ref["top1"]) & ~near_tied(ref["logits"])).any()
    np.testing.assert_array_equal(gpu["agree"], (gpu["top1"] == gpu["top1_base"][None]).sum(axis=1))


@pytest.mark.parametrize("layerwise", PATHS)
def test_base_reuse_optional_outputs_and_determinism(env, layerwise):
    torch, aiq = env["torch"], env["aiq"]
    wl = env["synth"].make_workload(0, n_images=50)
    schemes = _extra_schemes(wl, 8)[:5]
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=layerwise)
    img = torch.from_numpy(wl["images"]).cuda()
    a = m.eval_schemes(img, schemes, chunk=32, want_logits=True, want_top1=True)
    torch.cuda.synchronize()
    a = {k: v.clone() for k, v in a.items()}
    # same call again: identical bits (no float atomics, no order dependence)
    b = m.eval_schemes(img, schemes, chunk=32, want_logits=True, want_top1=True)
    torch.cuda.synchronize()
    for k in a:
        assert torch.equal(a[k], b[k]), k
    # reuse the base top-1, drop the optional outputs, different chunking
    c = m.eval_schemes(img, schemes, chunk=7, top1_base=a["top1_base"])
    torch.cuda.synchronize()
    assert c["logits"] is None and c["top1"] is None
    assert torch.equal(c["agree"], a["agree"])
    # a different chunk size changes nothing in the logits
    d = m.eval_schemes(img, schemes, chunk=50, want_logits=True)
    torch.cuda.synchronize()
    assert torch.equal(d["logits"], a["logits"])
    m.close()


@pytest.mark.parametrize("layerwise", PATHS)
def test_empty_inputs_and_error_paths(env, layerwise):
    torch, aiq = env["torch"], env["aiq"]
    wl = env["synth"].make_workload(0, n_images=4)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=layerwise)
    img = torch.from_numpy(wl["images"]).cuda()
    r = m.eval_schemes(img, np.zeros((0, wl["L"]), dtype=np.uint8), want_top1=True)
    torch.cuda.synchronize()
    assert r["agree"].numel() == 0 and r["top1_base"].numel() == 4
    r = m.eval_schemes(img[:0], wl["schemes"])
    torch.cuda.synchronize()
    assert r["agree"].cpu().tolist() == [0]
    bad = wl["schemes"].copy()
    bad[0, 3] = 5
    with pytest.raises(aiq.AiqError) as e:
        m.eval_schemes(img, bad)
    assert e.value.code == 2
    with pytest.raises(aiq.AiqError) as e:
        m.eval_schemes(img, np.full((1, wl["L"] + 1), 8, dtype=np.uint8))
    assert e.value.code == 3
    m.close()
