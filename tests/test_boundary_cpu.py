"""CPU checks of the C boundary: the library loads, exports every symbol include/aiq.h declares,
and the host-only entry points validate and compute (no device work here)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def aiq():
    import paper_2512_14090_amd as m
    m.load_library()
    return m


def test_every_declared_symbol_is_exported(aiq):
    header = open(os.path.join(ROOT, "include", "aiq.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(aiq_[a-z0-9_]+)\s*\(", header))
    assert declared, "no declarations found"
    lib = C.CDLL(aiq.library_path())
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} declared in aiq.h but not exported"
    assert declared == set(aiq.EXPORTED_SYMBOLS)


def test_status_strings(aiq):
    lib = aiq.load_library()
    seen = {lib.aiq_status_str(i) for i in range(7)}
    assert len(seen) == 7 and all(s for s in seen)
    assert lib.aiq_status_str(99)


@pytest.mark.parametrize("builder", [lambda: synth.resnet_cifar(1), lambda: synth.resnet_cifar(3),
                                     synth.mobilenetv2_32, synth.plain_convnet20, synth.heavy_early_resnet20])
def test_layer_ai_matches_oracle(aiq, builder):
    nodes = builder()
    desc = synth.desc_array(nodes)
    L = synth.n_scheme_layers(nodes)
    rng = np.random.Generator(np.random.PCG64(4))
    for batch in (1, 7):
        for _ in range(4):
            scheme = rng.choice(np.array(synth.BITS_ALPHABET, dtype=np.uint8), size=L)
            f, b, ai = aiq.layer_ai(desc, scheme, batch)
            rf, rb, rai = oracle.layer_ai(desc, scheme, batch)
            np.testing.assert_array_equal(f, rf)
            np.testing.assert_array_equal(b, rb)
            assert ai == rai
            # the variant that counts input activations at the layer's width
            f, b, ai = aiq.layer_ai(desc, scheme, batch, act_quant=True)
            rf, rb, rai = oracle.layer_ai(desc, scheme, batch, act_quant=True)
            np.testing.assert_array_equal(f, rf)
            np.testing.assert_array_equal(b, rb)
            assert ai == rai


def test_layer_ai_errors_leave_outputs_untouched(aiq):
    desc = synth.desc_array(synth.resnet_cifar(1))
    lib = aiq.load_library()
    flops = np.full(desc.shape[0], -1.0)
    ai = C.c_double(-1.0)

    def call(scheme, L, batch=1, n=desc.shape[0]):
        s = np.asarray(scheme, dtype=np.uint8)
        return lib.aiq_layer_ai(desc.ctypes.data, n, s.ctypes.data, L, batch, flops.ctypes.data, None, C.byref(ai))

    assert call([8] * 8, 8, batch=0) == 1
    assert call([8] * 8, 8, n=0) == 1
    assert call([8] * 7 + [5], 8) == 2
    assert call([8] * 7, 7) == 3
    assert ai.value == -1.0 and (flops == -1.0).all()
    assert lib.aiq_layer_ai(None, 3, None, 0, 1, None, None, C.byref(ai)) == 1
    assert call([8] * 8, 8) == 0 and ai.value > 0


def test_host_validation_precedes_device_work(aiq):
    lib = aiq.load_library()
    # quantize: bad sizes / bits / null pointers are rejected without touching the device
    assert lib.aiq_quantize_weights(None, -1, 4, 8, None, None, None, None) == 1
    assert lib.aiq_quantize_weights(None, 4, 4, 7, None, None, None, None) == 2
    assert lib.aiq_quantize_weights(None, 4, 4, 8, None, None, None, None) == 1
    assert lib.aiq_quantize_weights(None, 0, 4, 8, None, None, None, None) == 0
    # model creation: graph errors are reported before any allocation
    wl = synth.make_workload(0, n_images=1)
    n = wl["desc"].shape[0]
    wp = (C.c_void_p * n)(*[w.ctypes.data for w in wl["weights"]])
    bp = (C.c_void_p * n)(*[b.ctypes.data for b in wl["biases"]])
    h = C.c_void_p(None)
    bad = wl["desc"].copy()
    bad[3, 1] += 4  # cin disagrees with the producer
    assert lib.aiq_model_create(bad.ctypes.data, n, wp, bp, C.byref(h)) == 3 and not h
    bad = wl["desc"].copy()
    bad[2, 3] = bad[2, 4] = 5  # 5x5 kernel
    assert lib.aiq_model_create(bad.ctypes.data, n, wp, bp, C.byref(h)) == 6 and not h
    bad = wl["desc"].copy()
    bad[4, 12] = bad[5, 12]  # duplicate scheme slot
    assert lib.aiq_model_create(bad.ctypes.data, n, wp, bp, C.byref(h)) == 3 and not h
    assert lib.aiq_model_create(None, n, wp, bp, C.byref(h)) == 1
    assert lib.aiq_eval_workspace_bytes(None, 1, 1, None) == 1
    assert lib.aiq_eval_schemes(None, None, 1, None, 1, 1, None, 0, None, None, None, None, 0, None) == 1
    assert lib.aiq_model_scheme_layers(None) == -1 and lib.aiq_model_classes(None) == -1
    # the shared-prefix entry points validate the same way
    assert lib.aiq_model_shares_prefix(None) == -1
    assert lib.aiq_eval_shared_workspace_bytes(None, 1, 1, None) == 1
    ref = np.full(8, 32, dtype=np.uint8)
    assert lib.aiq_eval_schemes_shared(None, None, 1, None, 1, ref.ctypes.data, 1, None, 0, None, None, None, None, 0,
                                       None) == 1
    assert lib.aiq_search_workspace_bytes(None, 1, 1, 3, None) == 1
    assert lib.aiq_sensitivity_workspace_bytes(None, 1, 1, 2, None) == 1
    lib.aiq_model_destroy(None)
    # deployment: the same for its entry points
    d = C.c_void_p(None)
    assert lib.aiq_deploy_create(None, ref.ctypes.data, 0, C.byref(d)) == 1 and not d
    assert lib.aiq_deploy_workspace_bytes(None, 1, None) == 1
    assert lib.aiq_deploy_forward(None, None, 1, 1, None, None, None, 0, None) == 1
    assert lib.aiq_deploy_code_layers(None) == -1
    lib.aiq_deploy_destroy(None)


def test_descriptor_layout_matches_the_header():
    header = open(os.path.join(ROOT, "include", "aiq.h")).read()
    body = re.search(r"typedef struct \{(.*?)\} aiq_layer_desc;", header, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = [f.strip() for decl in re.findall(r"int32_t ([^;]+);", body) for f in decl.split(",")]
    assert tuple(fields) == synth.DESC_FIELDS
