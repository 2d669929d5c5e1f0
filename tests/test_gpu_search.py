"""GPU parity: the host search drivers (greedy, coordinate descent) driving the GPU scorer
against the oracle's search loops driving the oracle's forward pass."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2512_14090_amd as aiq
    import oracle
    import synth
    from oracle import search
    aiq.load_library()
    return dict(torch=torch, aiq=aiq, oracle=oracle, synth=synth, search=search)


def _compare(trace_gpu, trace_ref):
    assert [(t["layer"], t["bits"]) for t in trace_gpu] == [(t["layer"], t["bits"]) for t in trace_ref]
    for g, r in zip(trace_gpu, trace_ref):
        assert g["loss"] == pytest.approx(r["loss"], rel=1e-12, abs=1e-12)


@pytest.mark.parametrize("layerwise", [False, True])
@pytest.mark.parametrize("method,kwargs", [("greedy", {}), ("greedy", {"only_fp32_layers": True}),
                                            ("greedy", {"bits": (32, 16, 8, 6, 4, 2), "max_iters": 4}), ("cd", {})])
def test_search_matches_oracle_on_resnet8(env, method, kwargs, layerwise):
    torch, aiq, search = env["torch"], env["aiq"], env["search"]
    wl = env["synth"].make_workload(0, n_images=64)
    bits = kwargs.get("bits", (32, 8, 4))
    lam = 0.9
    print(f"search {method} {kwargs} layerwise={layerwise}", flush=True)
    ai_fn, accloss_many = search.model_callbacks(wl["desc"], wl["weights"], wl["biases"], wl["images"])
    if method == "greedy":
        q_ref, t_ref = search.greedy(wl["L"], bits, lam, ai_fn, accloss_many, max_iters=kwargs.get("max_iters"),
                                     only_fp32_layers=kwargs.get("only_fp32_layers", False))
    else:
        q_ref, t_ref = search.coordinate_descent(wl["L"], bits, lam, ai_fn, accloss_many)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=layerwise)
    img = torch.from_numpy(wl["images"]).cuda()
    q, trace = m.search(wl["desc"], img, method=method, bits=bits, lam=lam, chunk=48,
                        max_iters=kwargs.get("max_iters", 0), only_fp32_layers=kwargs.get("only_fp32_layers", False))
    np.testing.assert_array_equal(q, q_ref)
    _compare(trace, t_ref)
    # the reported agreement of the final scheme is what a direct scoring gives
    r = m.eval_schemes(img, q[None, :])
    torch.cuda.synchronize()
    if len(trace) > 1:
        assert int(r["agree"][0]) == trace[-1]["agree"]
    assert trace[0]["agree"] == 64 and trace[0]["layer"] == -1
    m.close()


_REF_SEARCH = {}


@pytest.mark.parametrize("layerwise", [False, True])
@pytest.mark.parametrize("method", ["greedy", "cd"])
def test_search_on_resnet20_with_accuracy_loss_on_the_path(env, method, layerwise):
    """ResNet-20 with the centred classifier (workload 7, 64 images): single-layer moves cost accuracy, so the
    loss trades AI against AccLoss > 0 and the searches have real decisions to take.  Three greedy iterations
    and one coordinate-descent sweep, move for move against the oracle's loops on the oracle's forward pass,
    with and without the shared forward prefix, LDS-resident and layer by layer."""
    torch, aiq, search = env["torch"], env["aiq"], env["search"]
    wl = env["synth"].make_workload(7, n_images=64)
    bits, lam, n = (32, 8, 4), 0.9, 64
    print(f"resnet20 centred search {method} layerwise={layerwise}", flush=True)
    if method not in _REF_SEARCH:
        ai_fn, accloss_many = search.model_callbacks(wl["desc"], wl["weights"], wl["biases"], wl["images"])
        if method == "greedy":
            _REF_SEARCH[method] = search.greedy(wl["L"], bits, lam, ai_fn, accloss_many, max_iters=3)
        else:
            _REF_SEARCH[method] = search.coordinate_descent(wl["L"], bits, lam, ai_fn, accloss_many, max_passes=1)
    q_ref, t_ref = _REF_SEARCH[method]
    # the path is not the degenerate one: moves were accepted, and accepted moves cost agreement
    assert len(t_ref) >= 3
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=layerwise)
    img = torch.from_numpy(wl["images"]).cuda()
    for share in (False, True):
        q, trace = m.search(wl["desc"], img, method=method, bits=bits, lam=lam, chunk=64,
                            max_iters=3 if method == "greedy" else 1, share_prefix=share)
        np.testing.assert_array_equal(q, q_ref)
        _compare(trace, t_ref)
        assert trace[0]["agree"] == n
        assert min(t["agree"] for t in trace[1:]) < n, [t["agree"] for t in trace]
    m.close()


@pytest.mark.parametrize("builder", ["plain", "heavy", "resnet8"])
def test_layer_sensitivity_table(env, builder):
    """Single-layer 8-bit / 4-bit agreement counts (the sensitivity columns of the paper's Table 1) for the
    two variant models (workloads 9 and 10: centred classifier, so the counts are not all N) and ResNet-8,
    against the oracle scoring the same single-layer schemes."""
    torch, aiq, oracle, synth = env["torch"], env["aiq"], env["oracle"], env["synth"]
    import sys, os
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    from parity import near_tied
    if builder == "resnet8":
        nodes = synth.resnet_cifar(1)
        rng = np.random.Generator(np.random.PCG64(41))
        w, b = synth.make_model(nodes, rng)
        n = 40
        images = synth.make_images(n, rng)
        desc = synth.desc_array(nodes)
        L = synth.n_scheme_layers(nodes)
    else:
        n = 12 if builder == "plain" else 16
        wl = synth.make_workload(9 if builder == "plain" else 10, n_images=n)
        w, b, images, desc, L = wl["weights"], wl["biases"], wl["images"], wl["desc"], wl["L"]
    bits = (8, 4)
    print(f"sensitivity {builder}: L={L} N={n}", flush=True)
    m = aiq.Model(desc, w, b)
    got = m.layer_sensitivity(torch.from_numpy(images).cuda(), bits=bits, chunk=7)
    m.close()
    schemes = np.full((L * len(bits), L), 32, dtype=np.uint8)
    for i in range(L):
        for k, bb in enumerate(bits):
            schemes[i * len(bits) + k, i] = bb
    ref = oracle.eval_schemes(desc, w, b, images, schemes)
    slack = (near_tied(ref["logits"]) | near_tied(ref["logits_base"])[None, :]).sum(axis=1)
    assert got.shape == (L, len(bits))
    assert (np.abs(got.reshape(-1).astype(np.int64) - ref["agree"]) <= slack).all(), (got.reshape(-1), ref["agree"])
    assert (got <= n).all() and (got >= 0).all()
    if builder != "resnet8":
        assert (got < n).sum() >= L // 2, got  # sensitivities that are not identically zero


def test_search_argument_errors(env):
    torch, aiq = env["torch"], env["aiq"]
    wl = env["synth"].make_workload(0, n_images=8)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"])
    img = torch.from_numpy(wl["images"]).cuda()
    for bad_bits, code in (((8, 4), 1), ((32, 4, 8), 1), ((32, 5), 2), ((32, 8, 8), 1)):
        with pytest.raises(aiq.AiqError) as e:
            m.search(wl["desc"], img, bits=bad_bits)
        assert e.value.code == code, bad_bits
    with pytest.raises(aiq.AiqError) as e:
        m.search(wl["desc"], img, lam=1.5)
    assert e.value.code == 1
    other = wl["desc"].copy()
    other[2, 11] = 0
    with pytest.raises(aiq.AiqError) as e:
        m.search(other, img)
    assert e.value.code == 3
    m.close()
