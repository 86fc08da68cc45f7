"""Thin Python binding of libminikv.so: argument marshalling only.

Every function here has the name and the argument order of its C entry point in include/minikv.h and
forwards device pointers of torch tensors (torch is used for device memory and streams, nothing else).
There is no CPU fallback: if the HIP library is missing, loading raises.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libminikv.so")

BUF_NAMES = ("Kc", "Ks", "Kz", "Vc", "Vs", "Vz", "q_len", "Rk", "Rv", "r_len")
_BUF_DTYPE = dict(Kc=torch.int32, Vc=torch.int32, q_len=torch.int32, r_len=torch.int32,
                  Ks=torch.float16, Kz=torch.float16, Vs=torch.float16, Vz=torch.float16,
                  Rk=torch.float16, Rv=torch.float16)


class MinikvShape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "Hq", "Hkv", "D", "G", "Tcap", "Rcap")]


class MinikvCache(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in BUF_NAMES]


class MinikvPtShape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "Hq", "Hkv", "D", "G", "bits", "Tcap")]


PT_BUF_NAMES = ("Kc", "Ks", "Kz", "Vc", "Vs", "Vz", "q_len")


class MinikvPtCache(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in PT_BUF_NAMES]


class MinikvError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, lib().minikv_strerror(status).decode(), status))


_lib = None


def lib():
    """Load libminikv.so (built in-tree by `python -m paper_2411_18077_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libminikv.so is not built: run `python -m paper_2411_18077_amd.build` "
                              "(there is no fallback path)")
        l = C.CDLL(LIB_PATH)
        l.minikv_abi_version.restype = C.c_int
        l.minikv_strerror.restype = C.c_char_p
        l.minikv_strerror.argtypes = [C.c_int]
        l.minikv_strvariant.restype = C.c_char_p
        l.minikv_strvariant.argtypes = [C.c_int]
        l.minikv_set_variant.restype = C.c_int
        l.minikv_set_variant.argtypes = [C.c_int]
        l.minikv_diag_decode_weights.restype = C.c_int
        l.minikv_diag_decode_weights.argtypes = [C.c_int]
        l.minikv_diag_select_path.restype = C.c_int
        l.minikv_diag_select_path.argtypes = [C.c_int]
        l.minikv_buffer_bytes.restype = C.c_size_t
        l.minikv_buffer_bytes.argtypes = [C.POINTER(MinikvShape), C.c_int]
        l.minikv_cache_bytes.restype = C.c_size_t
        l.minikv_cache_bytes.argtypes = [C.POINTER(MinikvShape), C.c_int]
        l.minikv_workspace_bytes.restype = C.c_size_t
        l.minikv_workspace_bytes.argtypes = [C.POINTER(MinikvShape)]
        P = C.c_void_p
        l.kv_quantize_pack.restype = C.c_int
        l.kv_quantize_pack.argtypes = [C.POINTER(MinikvShape), P, P, C.c_int64, P, C.c_int64, P, C.c_int32,
                                       C.POINTER(MinikvCache), P]
        l.kv_append_residual.restype = C.c_int
        l.kv_append_residual.argtypes = [C.POINTER(MinikvShape), P, P, C.POINTER(MinikvCache), P]
        l.kv_flush_residual.restype = C.c_int
        l.kv_flush_residual.argtypes = [C.POINTER(MinikvShape), C.POINTER(MinikvCache), P]
        l.minikv_decode_attn.restype = C.c_int
        l.minikv_decode_attn.argtypes = [C.POINTER(MinikvShape), P, C.POINTER(MinikvCache), C.c_float, P, P,
                                         C.c_size_t, P]
        l.minikv_decode_step.restype = C.c_int
        l.minikv_decode_step.argtypes = [C.POINTER(MinikvShape), P, P, P, C.POINTER(MinikvCache), P, C.c_float, P, P,
                                         C.c_size_t, P]
        l.minikv_decode_attn_static.restype = C.c_int
        l.minikv_decode_attn_static.argtypes = [C.POINTER(MinikvShape), P, C.POINTER(MinikvCache), C.c_float, P, P]
        l.minikv_static_workspace_units.restype = C.c_size_t
        l.minikv_static_workspace_units.argtypes = []
        l.minikv_pt_cache_bytes.restype = C.c_size_t
        l.minikv_pt_cache_bytes.argtypes = [C.POINTER(MinikvPtShape), C.c_int]
        l.minikv_pt_workspace_bytes.restype = C.c_size_t
        l.minikv_pt_workspace_bytes.argtypes = [C.POINTER(MinikvPtShape)]
        l.kv_quantize_pack_pt.restype = C.c_int
        l.kv_quantize_pack_pt.argtypes = [C.POINTER(MinikvPtShape), P, P, C.c_int64, P, C.c_int64, P, C.c_int32,
                                          C.POINTER(MinikvPtCache), P]
        l.minikv_decode_attn_pt.restype = C.c_int
        l.minikv_decode_attn_pt.argtypes = [C.POINTER(MinikvPtShape), P, C.POINTER(MinikvPtCache), C.c_float, P, P,
                                            C.c_size_t, P]
        l.selective_flash_attn.restype = C.c_int
        l.selective_flash_attn.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int64, P, P, P, C.c_float, P, P, P, P,
                                           C.c_size_t, P]
        l.selective_flash_attn_workspace_bytes.restype = C.c_size_t
        l.selective_flash_attn_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int64]
        l.minikv_diag_redo_count.restype = C.c_int
        l.minikv_diag_redo_count.argtypes = [C.POINTER(MinikvShape), P, C.POINTER(C.c_int32)]
        l.minikv_stream_read_probe.restype = C.c_int
        l.minikv_stream_read_probe.argtypes = [P, C.c_size_t, P, P]
        l.kv_select_workspace_bytes.restype = C.c_size_t
        l.kv_select_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int64]
        l.kv_select_hh_rw.restype = C.c_int
        l.kv_select_hh_rw.argtypes = [C.c_int32, C.c_int32, C.c_int64, P, P, P, P, C.c_int64, P, P, C.c_size_t, P]
        l.kv_pyramid_budget.restype = C.c_int
        l.kv_pyramid_budget.argtypes = [C.c_int32, C.c_double, C.c_int32, C.c_int32, C.POINTER(C.c_double)]
        _lib = l
    return _lib


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _check(rc, where):
    if rc != 0:
        raise MinikvError(rc, where)


def make_shape(B, Hq, Hkv, D, G, Tcap, Rcap):
    return MinikvShape(B, Hq, Hkv, D, G, Tcap, Rcap)


def buffer_bytes(shape, which):
    return int(lib().minikv_buffer_bytes(C.byref(shape), which))


def cache_bytes(shape, which):
    return int(lib().minikv_cache_bytes(C.byref(shape), which))


def workspace_bytes(shape):
    return int(lib().minikv_workspace_bytes(C.byref(shape)))


class Cache:
    """Caller-owned device buffers of one cache (torch tensors), sized by minikv_cache_bytes."""

    def __init__(self, shape, device="cuda", fill=None):
        self.shape = shape
        self.t = {}
        for i, name in enumerate(BUF_NAMES):
            nbytes = cache_bytes(shape, i)
            dt = _BUF_DTYPE[name]
            n = max(nbytes // dt.itemsize, 1)         # Rcap == 0: a 1-element placeholder
            self.t[name] = torch.zeros(n, dtype=dt, device=device)
        self.workspace = torch.zeros(max(workspace_bytes(shape), 16), dtype=torch.uint8, device=device)   # zeroed once

    def __getattr__(self, name):
        t = self.__dict__.get("t", {})
        if name in t:
            return t[name]
        raise AttributeError(name)

    def c(self):
        return MinikvCache(*(self.t[n].data_ptr() for n in BUF_NAMES))

    def nbytes(self):
        return sum(v.numel() * v.element_size() for v in self.t.values())

    def swap_r_len(self, other):
        """After minikv_decode_step: `other` (the array it wrote) becomes the cache's r_len; returns the old one."""
        old = self.t["r_len"]
        self.t["r_len"] = other
        return old


def kv_quantize_pack(shape, K, V, L, idx, idx_stride, n_tok, max_tok, cache, stream=None):
    cc = cache.c()
    _check(lib().kv_quantize_pack(C.byref(shape), _ptr(K), _ptr(V), int(L), _ptr(idx), int(idx_stride),
                                  _ptr(n_tok), int(max_tok), C.byref(cc), _stream(stream)), "kv_quantize_pack")


def kv_append_residual(shape, k_new, v_new, cache, stream=None):
    cc = cache.c()
    _check(lib().kv_append_residual(C.byref(shape), _ptr(k_new), _ptr(v_new), C.byref(cc), _stream(stream)),
           "kv_append_residual")


def kv_flush_residual(shape, cache, stream=None):
    cc = cache.c()
    _check(lib().kv_flush_residual(C.byref(shape), C.byref(cc), _stream(stream)), "kv_flush_residual")


def minikv_decode_attn(shape, q, cache, sm_scale, out, workspace=None, stream=None):
    cc = cache.c()
    ws = cache.workspace if workspace is None else workspace
    _check(lib().minikv_decode_attn(C.byref(shape), _ptr(q), C.byref(cc), float(sm_scale), _ptr(out), _ptr(ws),
                                    ws.numel() * ws.element_size(), _stream(stream)), "minikv_decode_attn")


def minikv_decode_attn_static(shape, q, cache, sm_scale, out, stream=None):
    cc = cache.c()
    _check(lib().minikv_decode_attn_static(C.byref(shape), _ptr(q), C.byref(cc), float(sm_scale), _ptr(out),
                                           _stream(stream)), "minikv_decode_attn_static")


def selective_flash_attn_workspace_bytes(B, Hkv, L):
    return int(lib().selective_flash_attn_workspace_bytes(int(B), int(Hkv), int(L)))


def selective_flash_attn(B, Hq, Hkv, L, Q, K, V, sm_scale, X_O, lse, A_cumul, workspace, stream=None):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().selective_flash_attn(int(B), int(Hq), int(Hkv), int(L), _ptr(Q), _ptr(K), _ptr(V), float(sm_scale),
                                      _ptr(X_O), _ptr(lse), _ptr(A_cumul), _ptr(workspace), nbytes, _stream(stream)),
           "selective_flash_attn")


def kv_select_workspace_bytes(units, rep, L):
    return int(lib().kv_select_workspace_bytes(int(units), int(rep), int(L)))


def kv_select_hh_rw(units, rep, L, A_cumul, n_hh, n_rw, idx, idx_stride, n_tok, workspace=None, stream=None):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().kv_select_hh_rw(int(units), int(rep), int(L), _ptr(A_cumul), _ptr(n_hh), _ptr(n_rw), _ptr(idx),
                                 int(idx_stride), _ptr(n_tok), _ptr(workspace), nbytes, _stream(stream)),
           "kv_select_hh_rw")


def kv_pyramid_budget(n_layers, x, d, bottom_heavy):
    out = (C.c_double * max(int(n_layers), 1))()
    _check(lib().kv_pyramid_budget(int(n_layers), float(x), int(d), int(bottom_heavy), out), "kv_pyramid_budget")
    return list(out)[: int(n_layers)]


def minikv_stream_read_probe(src, sums, stream=None):
    _check(lib().minikv_stream_read_probe(_ptr(src), src.numel() * src.element_size(), _ptr(sums), _stream(stream)),
           "minikv_stream_read_probe")


def minikv_diag_redo_count(shape, workspace):
    n = C.c_int32(0)
    _check(lib().minikv_diag_redo_count(C.byref(shape), _ptr(workspace), C.byref(n)), "minikv_diag_redo_count")
    return int(n.value)


def minikv_decode_step(shape, q, k_new, v_new, cache, r_len_next, sm_scale, out, stream=None):
    """Append + attend in one launch; afterwards r_len_next holds the residual lengths (the caller swaps it with
    cache.r_len: see Cache.swap_r_len)."""
    cc = cache.c()
    _check(lib().minikv_decode_step(C.byref(shape), _ptr(q), _ptr(k_new), _ptr(v_new), C.byref(cc), _ptr(r_len_next),
                                    float(sm_scale), _ptr(out), _ptr(cache.workspace),
                                    cache.workspace.numel() * cache.workspace.element_size(), _stream(stream)),
           "minikv_decode_step")


def minikv_diag_decode_weights(mode):
    _check(lib().minikv_diag_decode_weights(int(mode)), "minikv_diag_decode_weights")


def minikv_diag_select_path(path):
    _check(lib().minikv_diag_select_path(int(path)), "minikv_diag_select_path")


def minikv_set_variant(v):
    _check(lib().minikv_set_variant(int(v)), "minikv_set_variant")


# ---------------------------------------------------------------------------------------------------------
# per-token quantized variant

def make_pt_shape(B, Hq, Hkv, D, G, bits, Tcap):
    return MinikvPtShape(B, Hq, Hkv, D, G, bits, Tcap)


class PtCache:
    """Caller-owned device buffers of one per-token quantized cache, sized by minikv_pt_cache_bytes."""

    def __init__(self, shape, device="cuda"):
        self.shape = shape
        self.t = {}
        for name in PT_BUF_NAMES:
            nbytes = int(lib().minikv_pt_cache_bytes(C.byref(shape), BUF_NAMES.index(name)))
            dt = _BUF_DTYPE[name]
            self.t[name] = torch.zeros(max(nbytes // dt.itemsize, 1), dtype=dt, device=device)
        self.workspace = torch.empty(max(int(lib().minikv_pt_workspace_bytes(C.byref(shape))), 16), dtype=torch.uint8,
                                     device=device)

    def __getattr__(self, name):
        t = self.__dict__.get("t", {})
        if name in t:
            return t[name]
        raise AttributeError(name)

    def c(self):
        return MinikvPtCache(*(self.t[n].data_ptr() for n in PT_BUF_NAMES))

    def nbytes(self):
        return sum(v.numel() * v.element_size() for v in self.t.values())


def kv_quantize_pack_pt(shape, K, V, L, idx, idx_stride, n_tok, max_tok, cache, stream=None):
    cc = cache.c()
    _check(lib().kv_quantize_pack_pt(C.byref(shape), _ptr(K), _ptr(V), int(L), _ptr(idx), int(idx_stride),
                                     _ptr(n_tok), int(max_tok), C.byref(cc), _stream(stream)), "kv_quantize_pack_pt")


def minikv_decode_attn_pt(shape, q, cache, sm_scale, out, stream=None):
    cc = cache.c()
    ws = cache.workspace
    _check(lib().minikv_decode_attn_pt(C.byref(shape), _ptr(q), C.byref(cc), float(sm_scale), _ptr(out), _ptr(ws),
                                       ws.numel(), _stream(stream)), "minikv_decode_attn_pt")
