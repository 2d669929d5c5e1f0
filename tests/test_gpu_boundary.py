"""GPU checks of the C boundary's workspace contract: every entry point that takes a workspace refuses
one that is too small (AIQ_WORKSPACE_TOO_SMALL) or not 256-byte aligned (AIQ_INVALID_ARG) before any
device work, leaving its outputs untouched; a scheme axis too long for one grid is refused the same way;
host scheme tables may be reused as soon as a call returns."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

OK, INVALID_ARG, TOO_SMALL = 0, 1, 4


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2512_14090_amd as aiq
    import synth
    from paper_2512_14090_amd import binding
    return dict(torch=torch, aiq=aiq, synth=synth, binding=binding, lib=aiq.load_library())


def _stream(torch):
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


@pytest.mark.parametrize("layerwise", [False, True])
def test_eval_entry_points_refuse_bad_workspaces(env, layerwise):
    torch, aiq, lib = env["torch"], env["aiq"], env["lib"]
    wl = env["synth"].make_workload(0, n_images=6)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=layerwise)
    img = torch.from_numpy(wl["images"]).cuda()
    L, S, N, chunk = wl["L"], 3, 6, 4
    sch = np.ascontiguousarray(np.stack([np.full(L, b, np.uint8) for b in (8, 4, 32)]))
    ref = np.full(L, 32, np.uint8)
    top1_base = torch.full((N,), -7, dtype=torch.int32, device="cuda")
    agree = torch.full((S,), -7, dtype=torch.int32, device="cuda")
    for shared in (False, True):
        need = m.workspace_bytes(S, chunk, shared=shared)
        ws = torch.empty(need + 512, dtype=torch.uint8, device="cuda")
        base = (ws.data_ptr() + 255) // 256 * 256

        def call(ptr, nbytes, n_schemes=S, schemes=sch):
            if shared:
                return lib.aiq_eval_schemes_shared(m._h, img.data_ptr(), N, schemes.ctypes.data, n_schemes, ref.ctypes.data,
                                                   chunk, top1_base.data_ptr(), 0, None, None, agree.data_ptr(),
                                                   C.c_void_p(ptr), C.c_size_t(nbytes), _stream(torch))
            return lib.aiq_eval_schemes(m._h, img.data_ptr(), N, schemes.ctypes.data, n_schemes, chunk,
                                        top1_base.data_ptr(), 0, None, None, agree.data_ptr(), C.c_void_p(ptr),
                                        C.c_size_t(nbytes), _stream(torch))

        assert call(base, need - 1) == TOO_SMALL
        assert call(base, 0) == TOO_SMALL
        assert call(base + 4, need) == INVALID_ARG       # misaligned
        assert call(base + 128, need) == INVALID_ARG
        # a scheme axis that does not fit one grid: refused before anything is launched
        big = np.full((65535, L), 32, np.uint8)
        assert call(base, need, n_schemes=65535, schemes=big) == INVALID_ARG
        torch.cuda.synchronize()
        assert (top1_base == -7).all() and (agree == -7).all(), "outputs touched by a refused call"
        assert call(base, need) == OK
        torch.cuda.synchronize()
        assert (agree >= 0).all() and int(agree[2]) == N
        top1_base.fill_(-7)
        agree.fill_(-7)
    m.close()


def test_host_scheme_table_may_be_reused_at_once(env):
    """The scheme table is taken when the call is made: overwriting it right after the call returns, while
    the device is still busy, changes nothing - whether it lives in pageable or in pinned host memory."""
    torch, aiq, lib = env["torch"], env["aiq"], env["lib"]
    wl = env["synth"].make_workload(7, n_images=256)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"])
    img = torch.from_numpy(wl["images"]).cuda()
    L, S, N = wl["L"], wl["schemes"].shape[0], 256
    want = m.eval_schemes(img, wl["schemes"])["agree"].cpu().numpy()
    need = m.workspace_bytes(S, N, shared=True)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    ref = np.full(L, 32, np.uint8)
    for pinned in (False, True):
        host = torch.empty((S, L), dtype=torch.uint8, pin_memory=pinned)
        for shared in (False, True):
            host.copy_(torch.from_numpy(wl["schemes"]))
            top1_base = torch.empty(N, dtype=torch.int32, device="cuda")
            agree = torch.empty(S, dtype=torch.int32, device="cuda")
            if shared:
                rc = lib.aiq_eval_schemes_shared(m._h, img.data_ptr(), N, host.data_ptr(), S, ref.ctypes.data, N,
                                                 top1_base.data_ptr(), 0, None, None, agree.data_ptr(), ws.data_ptr(),
                                                 C.c_size_t(need), _stream(torch))
            else:
                rc = lib.aiq_eval_schemes(m._h, img.data_ptr(), N, host.data_ptr(), S, N, top1_base.data_ptr(), 0, None,
                                          None, agree.data_ptr(), ws.data_ptr(), C.c_size_t(need), _stream(torch))
            host.fill_(2)  # at once, the device has barely started
            assert rc == OK
            torch.cuda.synchronize()
            np.testing.assert_array_equal(agree.cpu().numpy(), want)
    m.close()


def test_search_and_sensitivity_refuse_bad_workspaces(env):
    torch, aiq, lib, binding = env["torch"], env["aiq"], env["lib"], env["binding"]
    wl = env["synth"].make_workload(0, n_images=6)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"])
    img = torch.from_numpy(wl["images"]).cuda()
    d = np.ascontiguousarray(wl["desc"], dtype=np.int32)
    L, N, chunk = wl["L"], 6, 6
    p = binding._SearchParams()
    p.lam, p.n_bits, p.batch, p.max_iters, p.only_fp32_layers, p.share_prefix = 0.9, 3, 1, 1, 0, 1
    for i, b in enumerate((32, 8, 4)):
        p.bits[i] = b
    need = C.c_size_t(0)
    assert lib.aiq_search_workspace_bytes(m._h, N, chunk, 3, C.byref(need)) == OK
    ws = torch.empty(need.value + 512, dtype=torch.uint8, device="cuda")
    base = (ws.data_ptr() + 255) // 256 * 256
    scheme = np.full(L, 99, np.uint8)
    trace = (binding._SearchStep * 8)()
    n_trace = C.c_int32(-5)
    for fn in (lib.aiq_search_greedy, lib.aiq_search_coordinate_descent):
        def call(ptr, nbytes):
            return fn(m._h, d.ctypes.data, d.shape[0], img.data_ptr(), N, chunk, C.byref(p), C.c_void_p(ptr),
                      C.c_size_t(nbytes), _stream(torch), scheme.ctypes.data, trace, 8, C.byref(n_trace))
        assert call(base, need.value - 1) == TOO_SMALL
        assert call(base + 64, need.value) == INVALID_ARG
        assert (scheme == 99).all() and n_trace.value == -5
        assert call(base, need.value) == OK
        assert n_trace.value >= 1 and set(scheme.tolist()) <= {32, 8, 4}
        scheme[:] = 99
        n_trace.value = -5
    bits = np.array([8, 4], np.uint8)
    assert lib.aiq_sensitivity_workspace_bytes(m._h, N, chunk, 2, C.byref(need)) == OK
    out = np.full((L, 2), -3, np.int32)

    def sens(ptr, nbytes):
        return lib.aiq_layer_sensitivity(m._h, img.data_ptr(), N, chunk, bits.ctypes.data, 2, C.c_void_p(ptr),
                                         C.c_size_t(nbytes), _stream(torch), out.ctypes.data)
    ws = torch.empty(need.value + 512, dtype=torch.uint8, device="cuda")
    base = (ws.data_ptr() + 255) // 256 * 256
    assert sens(base, need.value - 1) == TOO_SMALL
    assert sens(base + 8, need.value) == INVALID_ARG
    assert (out == -3).all()
    assert sens(base, need.value) == OK and (out >= 0).all() and (out <= N).all()
    m.close()


def test_deploy_forward_refuses_bad_workspaces(env):
    torch, aiq, lib = env["torch"], env["aiq"], env["lib"]
    wl = env["synth"].make_workload(0, n_images=5)
    m = aiq.Model(wl["desc"], wl["weights"], wl["biases"], layerwise=True)
    dep = aiq.Deployed(m, np.full(wl["L"], 8, np.uint8))
    img = torch.from_numpy(wl["images"]).cuda()
    N, chunk = 5, 3
    need = dep.workspace_bytes(chunk)
    ws = torch.empty(need + 512, dtype=torch.uint8, device="cuda")
    base = (ws.data_ptr() + 255) // 256 * 256
    top1 = torch.full((N,), -7, dtype=torch.int32, device="cuda")

    def call(ptr, nbytes):
        return lib.aiq_deploy_forward(dep._h, img.data_ptr(), N, chunk, None, top1.data_ptr(), C.c_void_p(ptr),
                                      C.c_size_t(nbytes), _stream(torch))
    assert call(base, need - 1) == TOO_SMALL
    assert call(base + 16, need) == INVALID_ARG
    torch.cuda.synchronize()
    assert (top1 == -7).all()
    assert call(base, need) == OK
    torch.cuda.synchronize()
    assert ((top1 >= 0) & (top1 < 10)).all()
    dep.close()
    m.close()
