"""ctypes binding of libaiq.so: the same entry points as include/aiq.h, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libaiq.so")
_lib = None

EXPORTED_SYMBOLS = (
    "aiq_status_str", "aiq_last_hip_error", "aiq_layer_ai", "aiq_layer_ai_ex", "aiq_model_nodes", "aiq_node_output_elems",
    "aiq_forward_nodes", "aiq_quantize_weights", "aiq_quantize_weights_ex", "aiq_model_create",
    "aiq_model_create_ex", "aiq_model_is_lds_resident", "aiq_model_lds_resident_blocks", "aiq_model_destroy", "aiq_model_scheme_layers", "aiq_model_classes", "aiq_eval_workspace_bytes",
    "aiq_eval_schemes", "aiq_eval_schemes_noalloc", "aiq_eval_noalloc_workspace_bytes", "aiq_model_shares_prefix", "aiq_eval_shared_workspace_bytes", "aiq_eval_schemes_shared",
    "aiq_profile_enable", "aiq_profile_read", "aiq_search_workspace_bytes",
    "aiq_search_greedy", "aiq_search_coordinate_descent", "aiq_sensitivity_workspace_bytes", "aiq_layer_sensitivity",
    "aiq_deploy_create", "aiq_deploy_destroy", "aiq_deploy_code_layers", "aiq_deploy_workspace_bytes",
    "aiq_deploy_forward", "aiq_deploy_forward_nodes",
)
K_QUANTIZE, K_CONV, K_DEPTHWISE, K_HEAD, K_AGREE, K_FUSED, K_MBCONV, K_CONV_CODES = range(8)
MODEL_LAYERWISE = 1
MODEL_PER_TENSOR = 2
MODEL_ACT_QUANT = 4
DEPLOY_FP32_MATRIX = 1
_DESC_INTS = 13


class _SearchParams(C.Structure):
    _fields_ = [("lam", C.c_double), ("n_bits", C.c_int32), ("bits", C.c_uint8 * 8), ("batch", C.c_int32),
                ("max_iters", C.c_int32), ("only_fp32_layers", C.c_int32), ("share_prefix", C.c_int32)]


class _SearchStep(C.Structure):
    _fields_ = [("layer", C.c_int32), ("bits", C.c_int32), ("agree", C.c_int32), ("sweep", C.c_int32),
                ("loss", C.c_double), ("ai", C.c_double)]


class AiqError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"{what}: {code}")
        self.code = code


def library_path():
    return _LIB_PATH


def library_is_stale():
    """True if a source or header is newer than the built library (or nothing is built)."""
    from . import build as _build
    return _build.stale()


def load_library():
    """Loads the built library; builds it first only if nothing is built.  A library older than its
    sources is loaded as it is, with a warning (building is a step of its own: __graft_entry__.build());
    AIQ_REQUIRE_FRESH=1 in the environment turns the warning into an error."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build as _build
        _build.build(force=True)
    elif library_is_stale():
        msg = f"{_LIB_PATH} is older than its sources: rebuild with paper_2512_14090_amd.build.build()"
        if os.environ.get("AIQ_REQUIRE_FRESH") == "1":
            raise RuntimeError(msg)
        import warnings
        warnings.warn(msg, RuntimeWarning, stacklevel=2)
    lib = C.CDLL(_LIB_PATH)
    lib.aiq_status_str.restype = C.c_char_p
    lib.aiq_status_str.argtypes = [C.c_int32]
    lib.aiq_last_hip_error.restype = C.c_int32
    lib.aiq_layer_ai.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                 C.POINTER(C.c_double)]
    lib.aiq_layer_ai_ex.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                    C.c_void_p, C.POINTER(C.c_double)]
    lib.aiq_model_nodes.argtypes = [C.c_void_p]
    lib.aiq_node_output_elems.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_size_t)]
    lib.aiq_forward_nodes.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t,
                                      C.c_void_p]
    lib.aiq_quantize_weights.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                         C.c_void_p, C.c_void_p]
    lib.aiq_quantize_weights_ex.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.aiq_model_create.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p)]
    lib.aiq_model_create_ex.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_uint32,
                                        C.POINTER(C.c_void_p)]
    lib.aiq_model_is_lds_resident.argtypes = [C.c_void_p]
    lib.aiq_model_lds_resident_blocks.argtypes = [C.c_void_p]
    lib.aiq_model_destroy.argtypes = [C.c_void_p]
    lib.aiq_model_destroy.restype = None
    lib.aiq_model_scheme_layers.argtypes = [C.c_void_p]
    lib.aiq_model_classes.argtypes = [C.c_void_p]
    lib.aiq_eval_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]
    lib.aiq_eval_schemes.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32,
                                     C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_size_t, C.c_void_p]
    lib.aiq_eval_schemes_noalloc.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32,
                                             C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.aiq_eval_noalloc_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_size_t),
                                                     C.POINTER(C.c_size_t)]
    lib.aiq_model_shares_prefix.argtypes = [C.c_void_p]
    lib.aiq_eval_shared_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]
    lib.aiq_eval_schemes_shared.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p,
                                            C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_size_t, C.c_void_p]
    lib.aiq_profile_enable.argtypes = [C.c_void_p, C.c_int32]
    lib.aiq_profile_read.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int64), C.POINTER(C.c_double),
                                     C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.aiq_search_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]
    for fn in (lib.aiq_search_greedy, lib.aiq_search_coordinate_descent):
        fn.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32,
                       C.POINTER(_SearchParams), C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p,
                       C.POINTER(_SearchStep), C.c_int32, C.POINTER(C.c_int32)]
    lib.aiq_sensitivity_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]
    lib.aiq_layer_sensitivity.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32,
                                          C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    lib.aiq_deploy_create.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.POINTER(C.c_void_p)]
    lib.aiq_deploy_destroy.argtypes = [C.c_void_p]
    lib.aiq_deploy_destroy.restype = None
    lib.aiq_deploy_code_layers.argtypes = [C.c_void_p]
    lib.aiq_deploy_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_size_t)]
    lib.aiq_deploy_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_size_t, C.c_void_p]
    lib.aiq_deploy_forward_nodes.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t,
                                             C.c_void_p]
    for name in EXPORTED_SYMBOLS:
        getattr(lib, name)
    _lib = lib
    return lib


def _check(st, what):
    if st != 0:
        lib = load_library()
        msg = lib.aiq_status_str(st).decode()
        if st == 5:
            msg += f" (hipError {lib.aiq_last_hip_error()})"
        raise AiqError(st, f"{what}: {msg}")


def _desc(desc):
    d = np.ascontiguousarray(desc, dtype=np.int32)
    if d.ndim != 2 or d.shape[1] != _DESC_INTS:
        raise ValueError("layer descriptors must be int32 [n_layers][13]")
    return d


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def layer_ai(desc, scheme, batch=1, act_quant=False):
    """aiq_layer_ai / aiq_layer_ai_ex: returns (flops[n_layers], bytes[n_layers], global_ai).  Host only."""
    d = _desc(desc)
    sch = None if scheme is None else np.ascontiguousarray(scheme, dtype=np.uint8)
    flops = np.empty(d.shape[0], dtype=np.float64)
    byts = np.empty(d.shape[0], dtype=np.float64)
    ai = C.c_double(0.0)
    if act_quant:
        st = load_library().aiq_layer_ai_ex(d.ctypes.data, d.shape[0], None if sch is None else sch.ctypes.data,
                                            0 if sch is None else sch.shape[0], int(batch), 1, flops.ctypes.data,
                                            byts.ctypes.data, C.byref(ai))
    else:
        st = load_library().aiq_layer_ai(d.ctypes.data, d.shape[0], None if sch is None else sch.ctypes.data,
                                         0 if sch is None else sch.shape[0], int(batch), flops.ctypes.data,
                                         byts.ctypes.data, C.byref(ai))
    _check(st, "aiq_layer_ai")
    return flops, byts, ai.value


def quantize_weights(w, bits, want_codes=True, stream=None, per_tensor=False):
    """aiq_quantize_weights[_ex] on a CUDA fp32 tensor [cout][k]; returns (w_dq, scales, codes|None) tensors."""
    import torch
    if not (w.is_cuda and w.dtype == torch.float32 and w.dim() == 2 and w.is_contiguous()):
        raise ValueError("w must be a contiguous CUDA float32 matrix")
    cout, k = w.shape
    w_dq = torch.empty_like(w)
    scales = torch.empty(cout, dtype=torch.float32, device=w.device)
    codes = torch.zeros((cout, k), dtype=torch.int32, device=w.device) if want_codes else None
    if per_tensor:
        scratch = torch.empty(1, dtype=torch.int32, device=w.device)
        st = load_library().aiq_quantize_weights_ex(w.data_ptr(), cout, k, int(bits), 1, w_dq.data_ptr(),
                                                    scales.data_ptr(), None if codes is None else codes.data_ptr(),
                                                    scratch.data_ptr(), _stream_ptr(stream))
        _check(st, "aiq_quantize_weights_ex")
        return w_dq, scales, codes
    st = load_library().aiq_quantize_weights(w.data_ptr(), cout, k, int(bits), w_dq.data_ptr(), scales.data_ptr(),
                                             None if codes is None else codes.data_ptr(), _stream_ptr(stream))
    _check(st, "aiq_quantize_weights")
    return w_dq, scales, codes


class Model:
    """Owns an aiq_model handle.  desc: int32 [n][13]; weights / biases: lists of fp32 numpy arrays."""

    def __init__(self, desc, weights, biases, layerwise=False, per_tensor=False, act_quant=False):
        self._h = C.c_void_p(None)
        self._lib = load_library()
        d = _desc(desc)
        n = d.shape[0]
        if len(weights) != n or len(biases) != n:
            raise ValueError("one weight and one bias array per layer")
        ws = [np.ascontiguousarray(w, dtype=np.float32) for w in weights]
        bs = [np.ascontiguousarray(b, dtype=np.float32) for b in biases]
        wp = (C.c_void_p * n)(*[w.ctypes.data for w in ws])
        bp = (C.c_void_p * n)(*[b.ctypes.data for b in bs])
        h = C.c_void_p(None)
        flags = ((MODEL_LAYERWISE if layerwise else 0) | (MODEL_PER_TENSOR if per_tensor else 0) |
                 (MODEL_ACT_QUANT if act_quant else 0))
        _check(self._lib.aiq_model_create_ex(d.ctypes.data, n, wp, bp, flags, C.byref(h)), "aiq_model_create_ex")
        self._h = h
        self.lds_resident = bool(self._lib.aiq_model_is_lds_resident(h))
        self.lds_resident_blocks = int(self._lib.aiq_model_lds_resident_blocks(h))
        self.shares_prefix = bool(self._lib.aiq_model_shares_prefix(h))
        self.L = int(self._lib.aiq_model_scheme_layers(h))
        self.classes = int(self._lib.aiq_model_classes(h))
        self._workspace = None
        self._ws_streams = []

    def close(self):
        if self._h:
            self._lib.aiq_model_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def workspace_bytes(self, S, chunk, shared=False):
        out = C.c_size_t(0)
        if shared:
            _check(self._lib.aiq_eval_shared_workspace_bytes(self._h, int(S), int(chunk), C.byref(out)),
                   "aiq_eval_shared_workspace_bytes")
        else:
            _check(self._lib.aiq_eval_workspace_bytes(self._h, int(S), int(chunk), C.byref(out)),
                   "aiq_eval_workspace_bytes")
        return out.value

    def _get_workspace(self, nbytes, device, stream=None):
        """The model's workspace tensor, regrown when too small.  Work enqueued earlier, possibly on another
        stream than the allocator knows of, may still be using the old one: every stream that has used it is
        drained before it is released."""
        import torch
        if self._workspace is None or self._workspace.numel() < nbytes or self._workspace.device != device:
            if self._workspace is not None:
                for st in self._ws_streams:
                    st.synchronize()
            self._ws_streams = []
            self._workspace = None
            self._workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
        st = stream if hasattr(stream, "synchronize") else torch.cuda.current_stream(device)
        if all(st != u for u in self._ws_streams):
            self._ws_streams.append(st)
        return self._workspace

    def eval_schemes(self, images, schemes, chunk=1024, top1_base=None, want_logits=False, want_top1=False,
                     out=None, stream=None, ref_scheme=None):
        """aiq_eval_schemes, or aiq_eval_schemes_shared when ref_scheme (uint8 [L], host) is given.

        images: CUDA fp32 [N][H][W][C]; schemes: uint8 [S][L] (host).
        top1_base: CUDA int32 [N] from an earlier call (then the FP32 pass is skipped), or None.
        out: optional dict of preallocated CUDA tensors (top1_base, logits, top1, agree) to reuse.
        Returns dict(agree, top1_base, logits|None, top1|None); all CUDA tensors, not synchronised.
        """
        import torch
        if not (images.is_cuda and images.dtype == torch.float32 and images.is_contiguous()):
            raise ValueError("images must be a contiguous CUDA float32 tensor")
        sch = np.ascontiguousarray(schemes, dtype=np.uint8)
        if sch.ndim != 2 or sch.shape[1] != self.L:
            raise AiqError(3, "aiq_eval_schemes: scheme length differs from the model's L")
        S, N = sch.shape[0], images.shape[0]
        dev = images.device
        out = out or {}
        base_valid = 1 if top1_base is not None else 0
        if top1_base is None:
            top1_base = out.get("top1_base")
            if top1_base is None:
                top1_base = torch.empty(max(N, 1), dtype=torch.int32, device=dev)
        agree = out.get("agree")
        if agree is None:
            agree = torch.empty(max(S, 1), dtype=torch.int32, device=dev)
        logits = top1 = None
        if want_logits:
            logits = out.get("logits")
            if logits is None:
                logits = torch.empty((S, N, self.classes), dtype=torch.float32, device=dev)
        if want_top1:
            top1 = out.get("top1")
            if top1 is None:
                top1 = torch.empty((S, N), dtype=torch.int32, device=dev)
        chunk = max(1, min(int(chunk), max(N, 1)))
        nbytes = self.workspace_bytes(S, chunk, shared=ref_scheme is not None)
        ws = self._get_workspace(nbytes, dev, stream)
        lg = None if logits is None else logits.data_ptr()
        t1 = None if top1 is None else top1.data_ptr()
        if ref_scheme is None:
            st = self._lib.aiq_eval_schemes(self._h, images.data_ptr(), N, sch.ctypes.data, S, chunk,
                                            top1_base.data_ptr(), base_valid, lg, t1, agree.data_ptr(),
                                            ws.data_ptr(), ws.numel(), _stream_ptr(stream))
            _check(st, "aiq_eval_schemes")
        else:
            ref = np.ascontiguousarray(ref_scheme, dtype=np.uint8)
            if ref.shape != (self.L,):
                raise AiqError(3, "aiq_eval_schemes_shared: reference scheme length differs from the model's L")
            st = self._lib.aiq_eval_schemes_shared(self._h, images.data_ptr(), N, sch.ctypes.data, S,
                                                   ref.ctypes.data, chunk, top1_base.data_ptr(), base_valid, lg, t1,
                                                   agree.data_ptr(), ws.data_ptr(), ws.numel(), _stream_ptr(stream))
            _check(st, "aiq_eval_schemes_shared")
        return dict(agree=agree[:S], top1_base=top1_base[:N], logits=logits, top1=top1)

    def forward_nodes(self, images, scheme, stream=None):
        """aiq_forward_nodes: one scheme (uint8 [L]) on images, every node's output.  Returns a list of CUDA fp32
        tensors [N][elems] in node order (the last holds the logits), not synchronised."""
        import torch
        sch = np.ascontiguousarray(scheme, dtype=np.uint8)
        if sch.shape != (self.L,):
            raise AiqError(3, "aiq_forward_nodes: scheme length differs from the model's L")
        N, dev = images.shape[0], images.device
        n_nodes = int(self._lib.aiq_model_nodes(self._h))
        outs = []
        for l in range(n_nodes):
            e = C.c_size_t(0)
            _check(self._lib.aiq_node_output_elems(self._h, l, C.byref(e)), "aiq_node_output_elems")
            outs.append(torch.empty((max(N, 1), e.value), dtype=torch.float32, device=dev))
        ptrs = (C.c_void_p * n_nodes)(*[t.data_ptr() for t in outs])
        ws = self._get_workspace(self.workspace_bytes(1, max(N, 1)), dev, stream)
        _check(self._lib.aiq_forward_nodes(self._h, images.data_ptr(), N, sch.ctypes.data, ptrs, ws.data_ptr(),
                                           ws.numel(), _stream_ptr(stream)), "aiq_forward_nodes")
        return [t[:N] for t in outs]

    def noalloc_workspace_bytes(self, S, chunk):
        """aiq_eval_noalloc_workspace_bytes: (bytes a call would need, bytes the library's fixed array holds)."""
        need, have = C.c_size_t(0), C.c_size_t(0)
        _check(self._lib.aiq_eval_noalloc_workspace_bytes(self._h, int(S), int(chunk), C.byref(need), C.byref(have)),
               "aiq_eval_noalloc_workspace_bytes")
        return need.value, have.value

    def eval_schemes_noalloc(self, images, schemes, out, chunk=1024, base_valid=False, stream=None):
        """aiq_eval_schemes_noalloc: scoring without any device allocation.  out: dict of CUDA tensors the caller
        has allocated - top1_base int32 [N] and agree int32 [S] (required), logits fp32 [S][N][classes] and top1
        int32 [S][N] (optional).  Nothing is allocated here either.  Returns out."""
        sch = np.ascontiguousarray(schemes, dtype=np.uint8)
        if sch.ndim != 2 or sch.shape[1] != self.L:
            raise AiqError(3, "aiq_eval_schemes_noalloc: scheme length differs from the model's L")
        S, N = sch.shape[0], images.shape[0]
        lg, t1 = out.get("logits"), out.get("top1")
        st = self._lib.aiq_eval_schemes_noalloc(self._h, images.data_ptr(), N, sch.ctypes.data, S, int(chunk),
                                                out["top1_base"].data_ptr(), 1 if base_valid else 0,
                                                None if lg is None else lg.data_ptr(),
                                                None if t1 is None else t1.data_ptr(), out["agree"].data_ptr(),
                                                _stream_ptr(stream))
        _check(st, "aiq_eval_schemes_noalloc")
        return out

    def search(self, desc, images, method="greedy", bits=(32, 8, 4), lam=0.9, batch=1, max_iters=0,
               only_fp32_layers=False, chunk=1024, stream=None, share_prefix=True):
        """aiq_search_greedy / aiq_search_coordinate_descent.  Returns (scheme uint8[L], trace list of dicts)."""
        import torch
        d = _desc(desc)
        p = _SearchParams()
        p.lam, p.n_bits, p.batch, p.max_iters = float(lam), len(bits), int(batch), int(max_iters)
        p.only_fp32_layers = 1 if only_fp32_layers else 0
        p.share_prefix = 1 if share_prefix else 0
        for i, b in enumerate(bits):
            p.bits[i] = int(b)
        N = images.shape[0]
        chunk = max(1, min(int(chunk), max(N, 1)))
        need = C.c_size_t(0)
        _check(self._lib.aiq_search_workspace_bytes(self._h, N, chunk, len(bits), C.byref(need)),
               "aiq_search_workspace_bytes")
        ws = self._get_workspace(need.value, images.device, stream)
        scheme = np.zeros(self.L, dtype=np.uint8)
        cap = 4096
        trace = (_SearchStep * cap)()
        n = C.c_int32(0)
        fn = {"greedy": self._lib.aiq_search_greedy, "cd": self._lib.aiq_search_coordinate_descent}[method]
        st = fn(self._h, d.ctypes.data, d.shape[0], images.data_ptr(), N, chunk, C.byref(p), ws.data_ptr(),
                ws.numel(), _stream_ptr(stream), scheme.ctypes.data, trace, cap, C.byref(n))
        _check(st, "aiq_search_" + method)
        steps = [dict(layer=t.layer, bits=t.bits, agree=t.agree, sweep=t.sweep, loss=t.loss, ai=t.ai)
                 for t in trace[:min(n.value, cap)]]
        return scheme, steps

    def layer_sensitivity(self, images, bits=(8, 4), chunk=1024, stream=None):
        """aiq_layer_sensitivity.  Returns int32 [L][len(bits)] agreement counts of the single-layer schemes."""
        b = np.ascontiguousarray(bits, dtype=np.uint8)
        N = images.shape[0]
        chunk = max(1, min(int(chunk), max(N, 1)))
        need = C.c_size_t(0)
        _check(self._lib.aiq_sensitivity_workspace_bytes(self._h, N, chunk, len(b), C.byref(need)),
               "aiq_sensitivity_workspace_bytes")
        ws = self._get_workspace(need.value, images.device, stream)
        out = np.zeros((self.L, len(b)), dtype=np.int32)
        _check(self._lib.aiq_layer_sensitivity(self._h, images.data_ptr(), N, chunk, b.ctypes.data, len(b),
                                               ws.data_ptr(), ws.numel(), _stream_ptr(stream), out.ctypes.data),
               "aiq_layer_sensitivity")
        return out

    def profile_enable(self, on=True):
        _check(self._lib.aiq_profile_enable(self._h, 1 if on else 0), "aiq_profile_enable")

    def profile_read(self, cls):
        n, ms, fl, by = C.c_int64(0), C.c_double(0), C.c_double(0), C.c_double(0)
        _check(self._lib.aiq_profile_read(self._h, int(cls), C.byref(n), C.byref(ms), C.byref(fl), C.byref(by)),
               "aiq_profile_read")
        return dict(launches=n.value, total_ms=ms.value, flops=fl.value, bytes=by.value)


class Deployed:
    """Owns an aiq_deployed handle: one scheme of a layer-by-layer Model, ready for inference."""

    def __init__(self, model, scheme, fp32_matrix=False):
        self._h = C.c_void_p(None)
        self._lib = load_library()
        self._model = model  # the deployment reads the model's weights and banks: keep it alive
        sch = np.ascontiguousarray(scheme, dtype=np.uint8)
        if sch.shape != (model.L,):
            raise AiqError(3, "aiq_deploy_create: scheme length differs from the model's L")
        h = C.c_void_p(None)
        _check(self._lib.aiq_deploy_create(model._h, sch.ctypes.data, DEPLOY_FP32_MATRIX if fp32_matrix else 0,
                                           C.byref(h)), "aiq_deploy_create")
        self._h = h
        self.code_layers = int(self._lib.aiq_deploy_code_layers(h))
        self._workspace = None

    def close(self):
        if self._h:
            self._lib.aiq_deploy_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def workspace_bytes(self, chunk):
        out = C.c_size_t(0)
        _check(self._lib.aiq_deploy_workspace_bytes(self._h, int(chunk), C.byref(out)), "aiq_deploy_workspace_bytes")
        return out.value

    def forward(self, images, chunk=1024, want_logits=False, out=None, stream=None):
        """aiq_deploy_forward.  images: CUDA fp32 [N][H][W][C].  Returns dict(top1, logits|None), not synchronised."""
        import torch
        if not (images.is_cuda and images.dtype == torch.float32 and images.is_contiguous()):
            raise ValueError("images must be a contiguous CUDA float32 tensor")
        N, dev = images.shape[0], images.device
        out = out or {}
        top1 = out.get("top1")
        if top1 is None:
            top1 = torch.empty(max(N, 1), dtype=torch.int32, device=dev)
        logits = None
        if want_logits:
            logits = out.get("logits")
            if logits is None:
                logits = torch.empty((N, self._model.classes), dtype=torch.float32, device=dev)
        chunk = max(1, min(int(chunk), max(N, 1)))
        ws = self._get_workspace(self.workspace_bytes(chunk), dev)
        _check(self._lib.aiq_deploy_forward(self._h, images.data_ptr(), N, chunk,
                                            None if logits is None else logits.data_ptr(), top1.data_ptr(),
                                            ws.data_ptr(), ws.numel(), _stream_ptr(stream)), "aiq_deploy_forward")
        return dict(top1=top1[:N], logits=logits)

    def _get_workspace(self, nbytes, dev):
        import torch
        if self._workspace is None or self._workspace.numel() < nbytes or self._workspace.device != dev:
            if self._workspace is not None:
                torch.cuda.synchronize(dev)  # earlier forwards, on whatever stream, may still use the old one
            self._workspace = None
            self._workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
        return self._workspace

    def forward_nodes(self, images, stream=None):
        """aiq_deploy_forward_nodes: every node's output of the deployed scheme.  Returns a list of CUDA fp32
        tensors [N][elems] in node order (the last holds the logits), not synchronised."""
        import torch
        N, dev = images.shape[0], images.device
        lib, mh = self._lib, self._model._h
        n_nodes = int(lib.aiq_model_nodes(mh))
        outs = []
        for l in range(n_nodes):
            e = C.c_size_t(0)
            _check(lib.aiq_node_output_elems(mh, l, C.byref(e)), "aiq_node_output_elems")
            outs.append(torch.empty((max(N, 1), e.value), dtype=torch.float32, device=dev))
        ptrs = (C.c_void_p * n_nodes)(*[t.data_ptr() for t in outs])
        ws = self._get_workspace(self.workspace_bytes(max(N, 1)), dev)
        _check(lib.aiq_deploy_forward_nodes(self._h, images.data_ptr(), N, ptrs, ws.data_ptr(), ws.numel(),
                                            _stream_ptr(stream)), "aiq_deploy_forward_nodes")
        return [t[:N] for t in outs]
