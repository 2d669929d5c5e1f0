"""ctypes front end of the CPU oracle (oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's CPU-baseline leg.  It never imports the HIP package and the HIP
package never imports it.  ``build()`` compiles liboracle.so with gcc; the
wrappers below only marshal numpy arrays.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force=False):
    """gcc -O2, no fast-math, no FMA contraction, OpenMP over (scheme, image)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-shared",
               "-fPIC", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.oracle_num_threads.restype = C.c_int
    return _lib


def num_threads():
    return int(lib().oracle_num_threads())


def _p(a, t):
    return None if a is None else a.ctypes.data_as(C.POINTER(t))


def _ptr_array(arrs):
    arr = (C.POINTER(C.c_float) * len(arrs))()
    for i, a in enumerate(arrs):
        assert a.dtype == np.float32 and a.flags.c_contiguous
        arr[i] = a.ctypes.data_as(C.POINTER(C.c_float))
    return arr


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"oracle status {code}")
        self.code = code


def _check(rc):
    if rc != 0:
        raise OracleError(rc)


def quantize_weights(w, bits, want_codes=True, per_tensor=False):
    """w fp32 [cout][k] -> (w_dq fp32 [cout][k], scales fp32 [cout], codes int32 [cout][k] or None).

    per_tensor: one scale for the whole matrix instead of one per output channel (row)."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    cout, k = w.shape
    w_dq = np.empty_like(w)
    scales = np.empty(cout, dtype=np.float32)
    codes = np.zeros((cout, k), dtype=np.int32) if want_codes else None
    fn = lib().oracle_quantize_weights_per_tensor if per_tensor else lib().oracle_quantize_weights
    _check(fn(_p(w, C.c_float), cout, k, int(bits), _p(w_dq, C.c_float), _p(scales, C.c_float), _p(codes, C.c_int32)))
    return w_dq, scales, codes


def quantize_activations(x, bits):
    """Activation fake-quantization of one tensor (any shape, one scale for all of it): returns fp64 array."""
    y = np.ascontiguousarray(x, dtype=np.float64).copy()
    _check(lib().oracle_quantize_activations(_p(y, C.c_double), C.c_int64(y.size), int(bits)))
    return y


def layer_ai(desc, scheme, batch=1, act_quant=False):
    """Returns (flops[n_layers], bytes[n_layers], global_ai).  act_quant: input activations counted at the
    layer's width as well."""
    desc = np.ascontiguousarray(desc, dtype=np.int32)
    n = desc.shape[0]
    scheme = None if scheme is None else np.ascontiguousarray(scheme, dtype=np.uint8)
    flops = np.empty(n, dtype=np.float64)
    byts = np.empty(n, dtype=np.float64)
    ai = C.c_double(0.0)
    _check(lib().oracle_layer_ai_ex(_p(desc, C.c_int32), n, _p(scheme, C.c_uint8),
                                    0 if scheme is None else scheme.shape[0], int(batch), 1 if act_quant else 0,
                                    _p(flops, C.c_double), _p(byts, C.c_double), C.byref(ai)))
    return flops, byts, ai.value


def check_graph(desc, hin=32, win=32, cin=3):
    desc = np.ascontiguousarray(desc, dtype=np.int32)
    return int(lib().oracle_check_graph(_p(desc, C.c_int32), desc.shape[0], hin, win, cin))


def node_out_elems(desc):
    out = []
    for d in np.asarray(desc):
        kind, cin, cout, kh, kw, st, pad, hin, win = [int(v) for v in d[:9]]
        if kind == 2:
            out.append(cout)
        else:
            out.append(((hin + 2 * pad - kh) // st + 1) * ((win + 2 * pad - kw) // st + 1) * cout)
    return out


def forward(desc, weights, biases, images, want_acts=False):
    """fp64 forward with the weights as given.  Returns dict(logits, top1, acts, macs_per_image)."""
    desc = np.ascontiguousarray(desc, dtype=np.int32)
    images = np.ascontiguousarray(images, dtype=np.float32)
    n_layers, N = desc.shape[0], images.shape[0]
    ncls = int(desc[-1, 2])
    logits = np.empty((N, ncls), dtype=np.float64)
    top1 = np.empty(N, dtype=np.int32)
    acts = np.empty((N, sum(node_out_elems(desc))), dtype=np.float64) if want_acts else None
    macs = C.c_int64(0)
    _check(lib().oracle_forward(_p(desc, C.c_int32), n_layers, _ptr_array(weights), _ptr_array(biases),
                                _p(images, C.c_float), N, _p(logits, C.c_double), _p(top1, C.c_int32),
                                _p(acts, C.c_double), C.byref(macs)))
    return dict(logits=logits, top1=top1, acts=acts, macs_per_image=macs.value)


def eval_schemes(desc, weights, biases, images, schemes, want_logits=True, per_tensor=False, act_quant=False,
                 want_acts=False):
    """Score schemes uint8 [S][L].  Returns dict(logits_base, top1_base, logits, top1, agree[, acts]).
    act_quant: a layer at b bits also reads its input activations at b bits.
    want_acts: every node's output under every scheme, fp64 [S][N][sum of node outputs]."""
    desc = np.ascontiguousarray(desc, dtype=np.int32)
    images = np.ascontiguousarray(images, dtype=np.float32)
    schemes = np.ascontiguousarray(schemes, dtype=np.uint8)
    n_layers, N = desc.shape[0], images.shape[0]
    S, L = schemes.shape
    ncls = int(desc[-1, 2])
    logits_base = np.empty((N, ncls), dtype=np.float64)
    top1_base = np.empty(N, dtype=np.int32)
    logits = np.empty((S, N, ncls), dtype=np.float64) if want_logits else None
    top1 = np.empty((S, N), dtype=np.int32)
    agree = np.empty(S, dtype=np.int32)
    acts = np.empty((S, N, sum(node_out_elems(desc))), dtype=np.float64) if want_acts else None
    _check(lib().oracle_eval_schemes_aq(_p(desc, C.c_int32), n_layers, _ptr_array(weights), _ptr_array(biases),
                                        _p(images, C.c_float), N, _p(schemes, C.c_uint8), S, L,
                                        1 if per_tensor else 0, 1 if act_quant else 0,
                                        _p(logits_base, C.c_double), _p(top1_base, C.c_int32),
                                        _p(logits, C.c_double), _p(top1, C.c_int32), _p(agree, C.c_int32),
                                        _p(acts, C.c_double)))
    return dict(logits_base=logits_base, top1_base=top1_base, logits=logits, top1=top1, agree=agree, acts=acts)


def conv_layer(desc_row, x, w, bias, res=None):
    """One layer on one image: x fp64 [hin][win][cin] -> (y flat fp64, multiply-add count)."""
    d = np.ascontiguousarray(desc_row, dtype=np.int32)
    x = np.ascontiguousarray(x, dtype=np.float64)
    w = np.ascontiguousarray(w, dtype=np.float32)
    bias = np.ascontiguousarray(bias, dtype=np.float32)
    n_out = node_out_elems(d[None, :])[0]
    y = np.empty(n_out, dtype=np.float64)
    res = None if res is None else np.ascontiguousarray(res, dtype=np.float64)
    macs = C.c_int64(0)
    _check(lib().oracle_conv_layer(_p(d, C.c_int32), _p(x, C.c_double), _p(w, C.c_float), _p(bias, C.c_float),
                                   _p(res, C.c_double), _p(y, C.c_double), C.byref(macs)))
    return y, macs.value
