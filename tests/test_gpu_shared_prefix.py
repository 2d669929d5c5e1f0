"""GPU: scoring with a shared forward prefix (aiq_eval_schemes_shared).

The contract is exact: every output equals, bit for bit, what aiq_eval_schemes returns for
the same schemes.  The tests therefore compare the two entry points element by element,
on candidate batches with the structure of the search steps (one layer changed against a
reference scheme) and on batches that have nothing to do with the reference; one case is
also checked against the oracle so that the pair cannot be wrong together.
"""
import numpy as np
import pytest

from parity import check_eval

pytestmark = pytest.mark.gpu

ALPHABET = np.array([32, 16, 8, 6, 4, 2], dtype=np.uint8)


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2512_14090_amd as aiq
    import oracle
    import synth
    aiq.load_library()
    return dict(torch=torch, aiq=aiq, oracle=oracle, synth=synth)


def _single_layer_moves(ref, widths):
    """Every scheme that differs from ref in exactly one layer, taking the given widths."""
    rows = []
    for i in range(ref.shape[0]):
        for b in widths:
            if b != ref[i]:
                q = ref.copy()
                q[i] = b
                rows.append(q)
    return np.ascontiguousarray(np.stack(rows))


def _both(env, m, img, schemes, ref, chunk, top1_base=None):
    torch = env["torch"]
    outs = []
    for r in (None, ref):
        tb = None if top1_base is None else top1_base.clone()
        o = m.eval_schemes(img, schemes, chunk=chunk, want_logits=True, want_top1=True, top1_base=tb, ref_scheme=r)
        torch.cuda.synchronize()
        outs.append({k: v.cpu().numpy() for k, v in o.items()})
    return outs


def _assert_identical(plain, shared):
    for k in ("agree", "top1_base", "top1"):
        np.testing.assert_array_equal(plain[k], shared[k], err_msg=k)
    # logits compared as bit patterns: equal floats, and no NaN slipping through
    np.testing.assert_array_equal(plain["logits"].view(np.uint32), shared["logits"].view(np.uint32))


@pytest.mark.parametrize("blocks,n,chunk", [(1, 70, 32), (3, 150, 64), (3, 33, 1024)])
def test_single_layer_moves_from_fp32(env, blocks, n, chunk):
    """The first greedy step / the sensitivity sweep: reference all-FP32, the FP32 pass requested."""
    torch, aiq, synth = env["torch"], env["aiq"], env["synth"]
    wl = synth.make_workload(0 if blocks == 1 else 2, n_images=n)
    L = wl["L"]
    ref = np.full(L, 32, dtype=np.uint8)
    schemes = _single_layer_moves(ref, (8, 4))
    print(f"shared prefix, fp32 reference: blocks={blocks} S={schemes.shape[0]} N={n} chunk={chunk}", flush=True)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"])
    assert m.lds_resident and m.shares_prefix
    img = torch.from_numpy(wl["images"]).cuda()
    plain, shared = _both(env, m, img, schemes, ref, chunk)
    m.close()
    _assert_identical(plain, shared)


@pytest.mark.parametrize("base_valid", [False, True])
def test_moves_from_a_mixed_reference(env, base_valid):
    """A later search step: the reference is a mixed scheme; the batch also holds the reference itself,
    schemes unrelated to it and one that differs in the first layer only."""
    torch, aiq, synth = env["torch"], env["aiq"], env["synth"]
    wl = synth.make_workload(1, n_images=97)
    L = wl["L"]
    rng = np.random.Generator(np.random.PCG64(77))
    ref = rng.choice(ALPHABET, size=L).astype(np.uint8)
    first = ref.copy()
    first[0] = 2 if ref[0] != 2 else 4
    schemes = np.concatenate([_single_layer_moves(ref, (16, 4)), ref[None, :], first[None, :],
                              rng.choice(ALPHABET, size=(3, L)).astype(np.uint8)])
    schemes = np.ascontiguousarray(schemes[rng.permutation(schemes.shape[0])])
    print(f"shared prefix, mixed reference {ref.tolist()}: S={schemes.shape[0]} base_valid={base_valid}", flush=True)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"])
    img = torch.from_numpy(wl["images"]).cuda()
    tb = None
    if base_valid:
        r0 = m.eval_schemes(img, schemes[:0], chunk=40)
        torch.cuda.synchronize()
        tb = r0["top1_base"]
    plain, shared = _both(env, m, img, schemes, ref, 40, top1_base=tb)
    m.close()
    _assert_identical(plain, shared)


def test_shared_against_oracle(env):
    """The shared path on its own against the oracle, to the bars of the plain path."""
    torch, aiq, oracle, synth = env["torch"], env["aiq"], env["oracle"], env["synth"]
    wl = synth.make_workload(0, n_images=48)
    L = wl["L"]
    ref = np.full(L, 32, dtype=np.uint8)
    ref[2] = 8
    schemes = _single_layer_moves(ref, (32, 4))
    print(f"shared prefix vs oracle: S={schemes.shape[0]}", flush=True)
    want = oracle.eval_schemes(wl["desc"], wl["weights"], wl["biases"], wl["images"], schemes)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"])
    img = torch.from_numpy(wl["images"]).cuda()
    o = m.eval_schemes(img, schemes, chunk=20, want_logits=True, want_top1=True, ref_scheme=ref)
    torch.cuda.synchronize()
    m.close()
    check_eval({k: v.cpu().numpy() for k, v in o.items()}, want, 48)


def test_empty_batches_and_errors(env):
    torch, aiq, synth = env["torch"], env["aiq"], env["synth"]
    wl = synth.make_workload(0, n_images=9)
    L = wl["L"]
    ref = np.full(L, 32, dtype=np.uint8)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"])
    img = torch.from_numpy(wl["images"]).cuda()
    # no schemes: only the FP32 pass runs
    a = m.eval_schemes(img, np.zeros((0, L), dtype=np.uint8), chunk=4)
    b = m.eval_schemes(img, np.zeros((0, L), dtype=np.uint8), chunk=4, ref_scheme=ref)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(a["top1_base"].cpu().numpy(), b["top1_base"].cpu().numpy())
    # no images
    c = m.eval_schemes(img[:0], _single_layer_moves(ref, (4,)), ref_scheme=ref)
    torch.cuda.synchronize()
    assert int(c["agree"].sum()) == 0
    bad = ref.copy()
    bad[1] = 7
    with pytest.raises(aiq.AiqError) as e:
        m.eval_schemes(img, ref[None, :], ref_scheme=bad)
    assert e.value.code == 2
    m.close()


def _variant_workload(synth, builder, n):
    nodes = {"plain": synth.plain_convnet20, "heavy": synth.heavy_early_resnet20,
             "mobilenet": synth.mobilenetv2_32}[builder]()
    rng = np.random.Generator(np.random.PCG64(53))
    w, b = synth.make_model(nodes, rng)
    return dict(desc=synth.desc_array(nodes), weights=w, biases=b, images=synth.make_images(n, rng),
                L=synth.n_scheme_layers(nodes))


@pytest.mark.parametrize("builder,n,chunk,layerwise", [
    ("resnet8", 21, 8, True), ("plain", 10, 4, False), ("heavy", 11, 16, False), ("heavy", 11, 16, True),
    ("mobilenet", 9, 4, False), ("mobilenet", 9, 4, True)])
def test_layer_by_layer_models(env, builder, n, chunk, layerwise):
    """Models that run layer by layer or through the inverted-residual block kernel: rows sorted by
    the node they leave the reference at, each node launched for the rows that have left it."""
    torch, aiq, synth = env["torch"], env["aiq"], env["synth"]
    if builder == "resnet8":
        wl = synth.make_workload(0, n_images=n)
    else:
        wl = _variant_workload(synth, builder, n)
    L = wl["L"]
    rng = np.random.Generator(np.random.PCG64(91))
    ref = np.full(L, 32, dtype=np.uint8)
    ref[rng.choice(L, 3, replace=False)] = (8, 4, 16)
    moves = _single_layer_moves(ref, (32, 4))
    moves = moves[rng.choice(moves.shape[0], min(12, moves.shape[0]), replace=False)]
    schemes = np.ascontiguousarray(np.concatenate([moves, ref[None, :],
                                                   rng.choice(ALPHABET, size=(2, L)).astype(np.uint8)]))
    print(f"shared prefix, {builder} layerwise={layerwise}: S={schemes.shape[0]} N={n} chunk={chunk}", flush=True)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=layerwise)
    assert m.shares_prefix and not m.lds_resident
    img = torch.from_numpy(wl["images"]).cuda()
    plain, shared = _both(env, m, img, schemes, ref, chunk)
    _assert_identical(plain, shared)
    # and with the FP32 pass as the reference
    ref32 = np.full(L, 32, dtype=np.uint8)
    plain, shared = _both(env, m, img, schemes, ref32, chunk)
    m.close()
    _assert_identical(plain, shared)


SEARCHES = [("greedy", (32, 8, 4)), ("cd", (32, 8, 4)), ("cd", (32, 16, 8, 6, 4, 2)), ("greedy", (32, 16, 4))]
SEARCH_CASES = [(mth, b, 1, 64, 48, False) for mth, b in SEARCHES] + [(mth, b, 1, 64, 64, False) for mth, b in SEARCHES] + \
               [(mth, b, 1, 30, 30, True) for mth, b in SEARCHES] + [(mth, b, 3, 40, 1024, False) for mth, b in SEARCHES[:2]]


@pytest.mark.parametrize("method,bits,blocks,n,chunk,layerwise", SEARCH_CASES)
def test_search_is_unchanged_by_sharing(env, method, bits, blocks, n, chunk, layerwise):
    """Whole searches with and without the shared prefix: same scheme, same trace.  When all images fit in one
    chunk the reference pass of a step continues from the checkpoints the previous steps left in the workspace
    (the LDS-resident path), so consecutive steps with changing and unchanged references are covered."""
    torch, aiq, synth = env["torch"], env["aiq"], env["synth"]
    wl = synth.make_workload(0 if blocks == 1 else 1, n_images=n)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=layerwise)
    img = torch.from_numpy(wl["images"]).cuda()
    print(f"search {method} {bits} blocks={blocks} n={n} chunk={chunk} layerwise={layerwise}", flush=True)
    q0, t0 = m.search(wl["desc"], img, method=method, bits=bits, chunk=chunk, share_prefix=False)
    q1, t1 = m.search(wl["desc"], img, method=method, bits=bits, chunk=chunk, share_prefix=True)
    # a second shared search on the same model and workspace starts from a clean cache
    q2, t2 = m.search(wl["desc"], img, method=method, bits=bits, chunk=chunk, share_prefix=True)
    m.close()
    np.testing.assert_array_equal(q0, q1)
    np.testing.assert_array_equal(q0, q2)
    assert t0 == t1 == t2


@pytest.mark.parametrize("method,layerwise", [("cd", False), ("greedy", True)])
def test_search_on_mobilenet_is_unchanged_by_sharing(env, method, layerwise):
    """The same on a model of inverted-residual blocks (block kernel and layer by layer): the reference pass of a
    step recomputes only the nodes between the previous step's layer and this one's."""
    torch, aiq, synth = env["torch"], env["aiq"], env["synth"]
    wl = _variant_workload(synth, "mobilenet", 6)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=layerwise)
    img = torch.from_numpy(wl["images"]).cuda()
    kw = dict(method=method, bits=(32, 8, 2), chunk=8, max_iters=3 if method == "greedy" else 1)
    print(f"mobilenet search {method} layerwise={layerwise}", flush=True)
    q0, t0 = m.search(wl["desc"], img, share_prefix=False, **kw)
    q1, t1 = m.search(wl["desc"], img, share_prefix=True, **kw)
    m.close()
    np.testing.assert_array_equal(q0, q1)
    assert t0 == t1
