"""The entry point that allocates nothing (aiq_eval_schemes_noalloc) against aiq_eval_schemes.

Same kernels, so every output must be bit for bit the same.  Two calls in a row share the library's
one fixed workspace; the second is smaller (fewer schemes, fewer images, another chunking) and must
not see anything the first left behind.  No device memory is allocated between the two calls' set-up
and their results (torch's allocator statistics are the witness for the binding's side)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2512_14090_amd as aiq
    import synth
    aiq.load_library()
    return dict(torch=torch, aiq=aiq, synth=synth)


def _outs(torch, S, N, classes, fill):
    return dict(top1_base=torch.full((N,), fill, dtype=torch.int32, device="cuda"),
                agree=torch.full((S,), fill, dtype=torch.int32, device="cuda"),
                logits=torch.full((S, N, classes), float(fill), dtype=torch.float32, device="cuda"),
                top1=torch.full((S, N), fill, dtype=torch.int32, device="cuda"))


@pytest.mark.parametrize("index", [0, 7])
def test_noalloc_matches_eval_schemes_on_two_calls_in_a_row(env, index):
    torch, aiq = env["torch"], env["aiq"]
    wl = env["synth"].make_workload(index, n_images=200)
    L = wl["L"]
    rng = np.random.Generator(np.random.PCG64(77 + index))
    big = np.ascontiguousarray(np.concatenate([rng.choice(np.array([32, 16, 8, 6, 4, 2], np.uint8), size=(9, L)),
                                               np.full((1, L), 32, np.uint8)]))
    small = np.ascontiguousarray(big[[3, 9, 0]])
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"])
    assert m.lds_resident
    img = torch.from_numpy(wl["images"]).cuda()
    calls = [(big, img, 64), (small, img[:37], 16)]
    want = []
    for sch, im, chunk in calls:
        r = m.eval_schemes(im, sch, chunk=chunk, want_logits=True, want_top1=True)
        torch.cuda.synchronize()
        want.append({k: v.clone() for k, v in r.items()})
    outs = [_outs(torch, sch.shape[0], im.shape[0], m.classes, -9) for sch, im, _ in calls]
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    for (sch, im, chunk), out in zip(calls, outs):
        need, have = m.noalloc_workspace_bytes(sch.shape[0], min(chunk, im.shape[0]))
        assert need <= have == 2 << 20
        print(f"noalloc call: workload {index}, S={sch.shape[0]} N={im.shape[0]} chunk={chunk}, needs {need} of {have} bytes",
              flush=True)
        m.eval_schemes_noalloc(im, sch, out, chunk=chunk)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
    for w, out in zip(want, outs):
        for k in ("agree", "top1_base", "top1"):
            assert torch.equal(w[k], out[k]), k
        assert torch.equal(w["logits"].view(torch.int32), out["logits"].view(torch.int32))
    # with the base pass handed in, and only the agreement counts asked for
    out = dict(top1_base=want[1]["top1_base"].clone(), agree=torch.full((3,), -9, dtype=torch.int32, device="cuda"))
    m.eval_schemes_noalloc(img[:37], small, out, chunk=37, base_valid=True)
    torch.cuda.synchronize()
    assert torch.equal(out["agree"], want[1]["agree"])
    assert int(out["agree"][1]) == 37  # the all-FP32 scheme
    m.close()


def test_noalloc_refuses_what_does_not_fit(env):
    torch, aiq = env["torch"], env["aiq"]
    wl = env["synth"].make_workload(0, n_images=8)
    img = torch.from_numpy(wl["images"]).cuda()
    sch = wl["schemes"]
    # a model that runs layer by layer needs activation buffers far beyond the fixed array
    lw = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=True)
    need, have = lw.noalloc_workspace_bytes(1, 8)
    assert need > have
    out = _outs(torch, 1, 8, lw.classes, -9)
    with pytest.raises(aiq.AiqError) as e:
        lw.eval_schemes_noalloc(img, sch, out, chunk=8)
    assert e.value.code == 4
    lw.close()
    # an LDS-resident model with too many schemes x images per chunk
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"])
    many = np.full((600, wl["L"]), 8, np.uint8)
    big_img = torch.zeros((1024, 32, 32, 3), device="cuda")
    out2 = dict(top1_base=torch.full((1024,), -9, dtype=torch.int32, device="cuda"),
                agree=torch.full((600,), -9, dtype=torch.int32, device="cuda"))
    with pytest.raises(aiq.AiqError) as e:
        m.eval_schemes_noalloc(big_img, many, out2, chunk=1024)
    assert e.value.code == 4
    torch.cuda.synchronize()
    assert (out2["agree"] == -9).all() and (out2["top1_base"] == -9).all() and (out["agree"] == -9).all()
    # the same schemes in smaller chunks fit
    m.eval_schemes_noalloc(big_img, many, out2, chunk=512)
    torch.cuda.synchronize()
    assert (out2["agree"] >= 0).all()
    with pytest.raises(aiq.AiqError) as e:
        bad = sch.copy()
        bad[0, 0] = 3
        m.eval_schemes_noalloc(img, bad, _outs(torch, 1, 8, m.classes, -9), chunk=8)
    assert e.value.code == 2
    m.close()
