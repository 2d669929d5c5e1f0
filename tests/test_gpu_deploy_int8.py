"""Deployed inference of the activation variant on the INT8 matrix pipe (conv_i8_kernel) against the oracle.

The function is the activation variant's: a layer at b <= 8 bits reads its input quantized to b bits with one
scale per image and weights quantized to b bits per output channel.  Rounding activations to codes is a
discontinuity, so - as for the scoring path of this variant - every node is compared with the oracle's
single-layer routines applied to the tensors the GPU actually gave that node: the codes are decided on
identical binary32 values on both sides, the integer sum is exact, and what is left is the fp32 rounding of
the final scaling (the oracle multiplies every weight and activation by its scale first, in fp64).  Which
nodes ran from int8 codes is asserted, so the test cannot pass on the fp32 kernels alone."""
import numpy as np
import pytest

from test_gpu_act_quant import _node_reference

pytestmark = pytest.mark.gpu

TOL = 2e-5  # of the node's largest magnitude, as for the scoring path of the variant


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2512_14090_amd as aiq
    import oracle
    import synth
    aiq.load_library()
    return dict(torch=torch, aiq=aiq, oracle=oracle, synth=synth)


def _eligible(nodes, scheme):
    """Nodes the library should run from int8 codes: dense convolutions of at most 8 bits that read another
    node's output with a multiple of 16 channels."""
    n = 0
    for nd in nodes:
        if nd["kind"] != 0 or nd["input"] < 0 or nd["scheme_slot"] < 0:
            continue
        if int(scheme[nd["scheme_slot"]]) <= 8 and nd["cin"] % 16 == 0 and nd["cout"] % 4 == 0:
            n += 1
    return n


def _check(env, nodes, desc, w, b, images, schemes, want_code_layers=True):
    torch, aiq, oracle = env["torch"], env["aiq"], env["oracle"]
    m = aiq.Model(desc, w, b, act_quant=True)
    img = torch.from_numpy(images).cuda()
    worst = 0.0
    for scheme in schemes:
        scheme = np.ascontiguousarray(scheme, dtype=np.uint8)
        dep = aiq.Deployed(m, scheme)
        expect = _eligible(nodes, scheme)
        if want_code_layers:
            assert dep.code_layers == expect, (dep.code_layers, expect, scheme.tolist())
        outs = dep.forward_nodes(img)
        torch.cuda.synchronize()
        outs = [o.cpu().numpy() for o in outs]
        for n in range(images.shape[0]):
            per_image = [o[n] for o in outs]
            for l in range(len(nodes)):
                ref = _node_reference(oracle, nodes, desc, w, b, scheme, images[n], per_image, l)
                err = np.abs(per_image[l] - ref).max() / max(np.abs(ref).max(), 1e-30)
                assert err <= TOL, f"node {l} ({nodes[l].get('name', '')}) image {n} scheme {scheme.tolist()}: {err:.3e}"
                worst = max(worst, err)
        # the chunked forward gives the same logits as the node-by-node one
        r = dep.forward(img, chunk=max(1, images.shape[0] // 2), want_logits=True)
        torch.cuda.synchronize()
        assert np.array_equal(r["logits"].cpu().numpy(), outs[-1])
        dep.close()
    m.close()
    return worst


def _schemes(L, rng):
    rows = [np.full(L, 8, np.uint8), np.full(L, 4, np.uint8), np.full(L, 2, np.uint8)]
    return rows + [rng.choice(np.array([32, 16, 8, 6, 4, 2], np.uint8), size=L) for _ in range(3)]


@pytest.mark.parametrize("index,n", [(0, 5), (1, 3), (5, 3), (6, 3), (3, 2)])
def test_model_families_node_by_node(env, index, n):
    wl = env["synth"].make_workload(index, n_images=n)
    rng = np.random.Generator(np.random.PCG64(800 + index))
    schemes = _schemes(wl["L"], rng)
    if index == 3:
        schemes = [schemes[0], schemes[3]]
    print(f"int8 deployment, node by node: {wl['name']} N={n} schemes={len(schemes)}", flush=True)
    worst = _check(env, wl["nodes"], wl["desc"], wl["weights"], wl["biases"], wl["images"], schemes)
    print("  worst node error %.3e of the node's range; int8 layers at 8 bits: %d"
          % (worst, _eligible(wl["nodes"], schemes[0])), flush=True)


def _wide_graph(G, rng):
    """A seeded chain whose layers have multiples of 16 input channels, so that most of them run from int8
    codes: 3x3 / 1x1, both strides, odd map sizes, output widths that do not fill a tile of 32, maps small
    enough for several images per workgroup, residual links."""
    ci = int(rng.choice([3, 4]))
    h = int(rng.choice([5, 8, 13, 16, 19, 32]))
    widths = [16, 32, 48, 64, 80, 96, 144]
    c = int(rng.choice(widths))
    nodes = [G._node(G.KIND_CONV, ci, c, 3, 1, h, -1, act=int(rng.integers(0, 3)), slot=0, name="stem")]
    shapes = [(c, h)]
    for i in range(int(rng.integers(3, 7))):
        c_in, h_in = shapes[-1]
        kind = str(rng.choice(["c3", "c3", "c1", "c3s2", "c1s2"]))
        stride = 2 if kind.endswith("s2") and h_in >= 4 else 1
        k = 1 if kind.startswith("c1") else 3
        h_out = (h_in + 2 * (k // 2) - k) // stride + 1
        c_out = int(rng.choice(widths + [24, 40, 200]))
        if i < 5 and c_out % 16:  # keep the chain on multiples of 16 except possibly at its end
            c_out = int(rng.choice(widths))
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


@pytest.mark.parametrize("seed", list(range(10)))
def test_wide_random_graphs_node_by_node(env, seed):
    synth = env["synth"]
    rng = np.random.Generator(np.random.PCG64(9300 + seed))
    nodes, ci, h = _wide_graph(synth.graphs, rng)
    w, b = synth.make_model(nodes, rng)
    n = 9 if h <= 8 else 3  # small maps: several images per workgroup and a ragged last group
    images = rng.standard_normal((n, h, h, ci)).astype(np.float32)
    L = len(nodes)
    shapes = [(nd["cin"], nd["cout"], nd["kh"], nd["stride"], nd["hin"]) for nd in nodes]
    print(f"int8 random graph {seed}: input {h}x{h}x{ci}, N={n}, layers (cin, cout, k, stride, hin): {shapes}", flush=True)
    worst = _check(env, nodes, synth.desc_array(nodes), w, b, images, _schemes(L, rng)[:5])
    print("  worst node error %.3e of the node's range" % worst, flush=True)


def test_narrow_random_graphs_fall_back_where_the_shape_does_not_fit(env):
    """The graphs of the scoring tests (channel counts of any multiple of 4, depthwise layers): layers the int8
    kernel does not take run on the scoring kernels, the rest from codes; every node is checked."""
    from test_gpu_eval import _random_graph
    synth = env["synth"]
    for seed in range(6):
        rng = np.random.Generator(np.random.PCG64(9000 + seed))
        nodes, ci, h = _random_graph(synth.graphs, rng)
        w, b = synth.make_model(nodes, rng)
        images = rng.standard_normal((3, h, h, ci)).astype(np.float32)
        print(f"int8 narrow random graph {seed}: {len(nodes)} nodes, input {h}x{h}x{ci}", flush=True)
        _check(env, nodes, synth.desc_array(nodes), w, b, images, _schemes(len(nodes), rng)[:4])


def test_many_images_so_that_workgroups_walk_several_regions(env):
    """At benchmark-like batch sizes a workgroup of the int8 kernel keeps its weight codes for up to eight consecutive
    regions and fetches the next region's activations ahead; the last workgroup's share is ragged and the last
    group of small images incomplete.  2049 images through ResNet-8 (16 / 32 / 64 channels at 32 / 16 / 8 pixels);
    every node of sampled images - the first and last regions of workgroups, the tail - against the oracle on the
    GPU's own input tensors."""
    torch, aiq, oracle = env["torch"], env["aiq"], env["oracle"]
    N = 2049
    wl = env["synth"].make_workload(0, n_images=N)
    nodes, desc, w, b = wl["nodes"], wl["desc"], wl["weights"], wl["biases"]
    m = aiq.Model(desc, w, b, act_quant=True)
    img = torch.from_numpy(wl["images"]).cuda()
    sample = [0, 1, 2, 3, 7, 8, 511, 512, 1023, 1024, 1025, 2040, 2043, 2044, 2046, 2047, 2048]
    worst = 0.0
    for scheme in (np.full(wl["L"], 8, np.uint8), np.full(wl["L"], 4, np.uint8)):
        dep = aiq.Deployed(m, scheme)
        assert dep.code_layers == _eligible(nodes, scheme) > 0
        print(f"int8 deployment, {N} images, scheme of {int(scheme[0])} bits: {dep.code_layers} layers on int8 codes", flush=True)
        outs = dep.forward_nodes(img)
        torch.cuda.synchronize()
        idx = torch.tensor(sample, device="cuda")
        outs = [o.index_select(0, idx).cpu().numpy() for o in outs]
        for k, n in enumerate(sample):
            per_image = [o[k] for o in outs]
            for l in range(len(nodes)):
                ref = _node_reference(oracle, nodes, desc, w, b, scheme, wl["images"][n], per_image, l)
                err = np.abs(per_image[l] - ref).max() / max(np.abs(ref).max(), 1e-30)
                assert err <= TOL, f"node {l} image {n} scheme {scheme.tolist()}: {err:.3e}"
                worst = max(worst, err)
        # the chunked forward (chunks of 1000 + a remainder of 49) gives the same logits
        r = dep.forward(img, chunk=1000, want_logits=True)
        torch.cuda.synchronize()
        assert np.array_equal(r["logits"].index_select(0, idx).cpu().numpy(), outs[-1])
        dep.close()
    print("  worst node error %.3e of the node's range" % worst, flush=True)
    m.close()
