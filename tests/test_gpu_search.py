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
