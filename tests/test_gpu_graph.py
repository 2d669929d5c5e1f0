"""A scoring call captured into a HIP graph and replayed.

aiq_eval_schemes_noalloc launches kernels only (host tables travel as kernel arguments, nothing is
allocated, copied or waited for), so a caller may record it once and replay it.  The replays must give
what the eager call gives, bit for bit, every time: also after other work has used the library's fixed
workspace in between, and with new images written into the same input tensor (the schemes are part of
the recording, the images are read at replay time)."""
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


def _same(torch, want, got):
    for k in ("agree", "top1_base", "top1"):
        assert torch.equal(want[k], got[k]), k
    assert torch.equal(want["logits"].view(torch.int32), got["logits"].view(torch.int32))


@pytest.mark.parametrize("index", [7, 0])
def test_captured_scoring_call_replays_bit_for_bit(env, index):
    torch, aiq = env["torch"], env["aiq"]
    N, chunk = 96, 48
    wl = env["synth"].make_workload(index, n_images=2 * N)
    L = wl["L"]
    rng = np.random.Generator(np.random.PCG64(400 + index))
    sch = np.ascontiguousarray(np.concatenate([rng.choice(np.array([32, 16, 8, 6, 4, 2], np.uint8), size=(5, L)),
                                               np.full((1, L), 4, np.uint8)]))
    other_sch = np.ascontiguousarray(rng.choice(np.array([32, 8, 2], np.uint8), size=(3, L)))
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"])
    assert m.lds_resident
    all_img = torch.from_numpy(wl["images"]).cuda()
    img = all_img[:N].clone()  # the tensor the recording reads
    want = []
    for part in (all_img[:N], all_img[N:]):
        r = m.eval_schemes(part, sch, chunk=chunk, want_logits=True, want_top1=True)
        torch.cuda.synchronize()
        want.append({k: v.clone() for k, v in r.items()})
    assert len(set(want[0]["agree"].tolist())) > 1 or index == 0  # workload 7: the schemes do not all agree alike

    out = _outs(torch, sch.shape[0], N, m.classes, -9)
    m.eval_schemes_noalloc(img, sch, out, chunk=chunk)  # eager: also does the library's first-use set-up
    torch.cuda.synchronize()
    _same(torch, want[0], out)

    print(f"capturing: workload {index}, S={sch.shape[0]} N={N} chunk={chunk}", flush=True)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        m.eval_schemes_noalloc(img, sch, out, chunk=chunk)  # the capturing stream is the current one here
    torch.cuda.synchronize()

    other = _outs(torch, other_sch.shape[0], 33, m.classes, -9)
    for rep in range(4):
        # eager work between the replays: outputs cleared, the fixed workspace used by another call,
        # and from the third replay on other images in the recorded input tensor
        for v in out.values():
            v.fill_(-7)
        m.eval_schemes_noalloc(all_img[5:38], other_sch, other, chunk=33)
        which = 0 if rep < 2 else 1
        img.copy_(all_img[:N] if which == 0 else all_img[N:])
        torch.cuda.synchronize()
        print(f"replay {rep}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        _same(torch, want[which], out)
    del graph
    m.close()


@pytest.mark.parametrize("index,layerwise,act_quant", [(3, False, False), (5, True, False), (5, False, True)])
def test_captured_deployed_forward_replays_bit_for_bit(env, index, layerwise, act_quant):
    """aiq_deploy_forward launches kernels only once its workspace exists (the binding allocates it on the first
    call), so a serving loop may record a forward and replay it: MobileNetV2 on its block kernels from integer codes,
    PlainConvNet20 layer by layer on bf16 codes, and its activation variant on int8 codes (whose per-image maxima are
    cleared by a fill kernel inside the recording).  Replays with other eager work between them and with new images
    in the recorded input tensor give what the eager call gives."""
    torch, aiq = env["torch"], env["aiq"]
    N = 24
    wl = env["synth"].make_workload(index, n_images=2 * N)
    L = wl["L"]
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=layerwise, act_quant=act_quant)
    d = aiq.Deployed(m, np.full(L, 8, np.uint8))
    assert d.code_layers > 0
    all_img = torch.from_numpy(wl["images"]).cuda()
    img = all_img[:N].clone()
    want = []
    for part in (all_img[:N], all_img[N:]):
        r = d.forward(part, chunk=N, want_logits=True)
        torch.cuda.synchronize()
        want.append({k: r[k].clone() for k in ("logits", "top1")})
    out = {"logits": torch.full((N, m.classes), -9.0, device="cuda"), "top1": torch.full((N,), -9, dtype=torch.int32, device="cuda")}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    print(f"capturing: deployed workload {index}, layerwise={layerwise}, act_quant={act_quant}, N={N}", flush=True)
    with torch.cuda.graph(graph, stream=side):
        d.forward(img, chunk=N, want_logits=True, out=out, stream=side)
    torch.cuda.synchronize()
    for rep in range(4):
        for v in out.values():
            v.fill_(-7)
        d.forward(all_img[3:20], chunk=17)  # eager work on the same deployment (its workspace) between the replays
        which = 0 if rep < 2 else 1
        img.copy_(all_img[:N] if which == 0 else all_img[N:])
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out["top1"], want[which]["top1"]), rep
        assert torch.equal(out["logits"].view(torch.int32), want[which]["logits"].view(torch.int32)), rep
    d.close()
    m.close()
