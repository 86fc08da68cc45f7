"""ctypes view of the CPU oracle (oracle/minikv_ref.c).  Test infrastructure, not the product.

Everything here takes and returns numpy arrays in host memory; fp16 travels as numpy float16 whose
buffer is handed to C as raw binary16 bit patterns.  Nothing in this file does arithmetic of the
method: it allocates buffers and forwards pointers.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


class _Shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "Hq", "Hkv", "D", "G", "Tcap", "Rcap")]


class _Cache(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("Kc", "Ks", "Kz", "Vc", "Vs", "Vz", "q_len", "Rk", "Rv", "r_len")]


def lib():
    global _lib
    if _lib is None:
        path = _build.build()
        _lib = C.CDLL(path)
        _lib.ref_f16_to_f32.restype = C.c_float
        _lib.ref_f16_to_f32.argtypes = [C.c_uint16]
        _lib.ref_f32_to_f16.restype = C.c_uint16
        _lib.ref_f32_to_f16.argtypes = [C.c_float]
        _lib.ref_f64_to_f16.restype = C.c_uint16
        _lib.ref_f64_to_f16.argtypes = [C.c_double]
        _lib.ref_group_bytes.restype = C.c_size_t
        _lib.ref_group_bytes.argtypes = [C.c_int]
        for name in ("ref_check_shape", "kv_quantize_pack_ref", "kv_append_residual_ref",
                     "kv_flush_residual_ref", "minikv_decode_attn_ref", "ref_unpack_codes", "ref_dequant",
                     "ref_k_meta_pos", "kv_select_hh_rw_ref", "kv_pyramid_budget_ref",
                     "selective_flash_attn_ref", "selective_flash_attn_rows_ref", "ref_pt_check_shape", "kv_quantize_pack_pt_ref",
                     "minikv_decode_attn_pt_ref", "ref_pt_unpack_codes"):
            getattr(_lib, name).restype = C.c_int
        _lib.ref_pt_token_bytes.restype = C.c_size_t
        _lib.ref_pt_token_bytes.argtypes = [C.c_int, C.c_int, C.c_int]
    return _lib


def _p(a):
    return None if a is None else C.c_void_p(a.ctypes.data)


class RefShape:
    def __init__(self, B, Hq, Hkv, D, G, Tcap, Rcap):
        self.B, self.Hq, self.Hkv, self.D, self.G, self.Tcap, self.Rcap = B, Hq, Hkv, D, G, Tcap, Rcap

    @property
    def units(self):
        return self.B * self.Hkv

    def c(self):
        return _Shape(self.B, self.Hq, self.Hkv, self.D, self.G, self.Tcap, self.Rcap)

    def check(self):
        return lib().ref_check_shape(C.byref(self.c()))


class RefCache:
    """Host buffers of one cache, zero-initialised, in the storage order minikv_ref.h documents."""

    def __init__(self, s: RefShape):
        U, D, G, T, R = s.units, s.D, s.G, s.Tcap, s.Rcap
        self.shape = s
        self.Kc = np.zeros((U, T // 128 * 1024), np.uint32)
        self.Ks = np.zeros((U, T // G, D), np.float16)
        self.Kz = np.zeros((U, T // G, D), np.float16)
        self.Vc = np.zeros((U, T // 64 * 4 * D), np.uint32)
        self.Vs = np.zeros((U, T, D // G), np.float16)
        self.Vz = np.zeros((U, T, D // G), np.float16)
        self.q_len = np.zeros((U,), np.int32)
        self.Rk = np.zeros((U, max(R, 1), D), np.float16)
        self.Rv = np.zeros((U, max(R, 1), D), np.float16)
        self.r_len = np.zeros((U,), np.int32)

    def c(self):
        return _Cache(*(a.ctypes.data for a in (self.Kc, self.Ks, self.Kz, self.Vc, self.Vs, self.Vz,
                                                self.q_len, self.Rk, self.Rv, self.r_len)))


def _f16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float16, a.dtype
    return a


def quantize_pack(cache: RefCache, K, V, n_tok, idx=None):
    """K, V: float16 [U, L, D]; n_tok int32 [U]; idx int32 [U, stride] or None."""
    s = cache.shape
    K, V = _f16(K), _f16(V)
    L = K.shape[1]
    n_tok = np.ascontiguousarray(n_tok, np.int32)
    stride = 0
    if idx is not None:
        idx = np.ascontiguousarray(idx, np.int32)
        stride = idx.shape[1]
    cc = cache.c()
    return lib().kv_quantize_pack_ref(C.byref(s.c()), _p(K), _p(V), C.c_int64(L), _p(idx),
                                      C.c_int64(stride), _p(n_tok), C.byref(cc))


def append_residual(cache: RefCache, k_new, v_new):
    cc = cache.c()
    return lib().kv_append_residual_ref(C.byref(cache.shape.c()), _p(_f16(k_new)), _p(_f16(v_new)), C.byref(cc))


def flush_residual(cache: RefCache):
    cc = cache.c()
    return lib().kv_flush_residual_ref(C.byref(cache.shape.c()), C.byref(cc))


def decode_attn(cache: RefCache, q, sm_scale, want_f64=False, want_probs=False):
    """q float16 [B, Hq, D] -> (out float16 [B,Hq,D], out float64 or None, probs or None)."""
    s = cache.shape
    q = _f16(q)
    out16 = np.zeros((s.B, s.Hq, s.D), np.float16)
    out64 = np.zeros((s.B, s.Hq, s.D), np.float64) if want_f64 else None
    probs = np.zeros((s.B, s.Hq, s.Tcap + s.Rcap), np.float64) if want_probs else None
    cc = cache.c()
    rc = lib().minikv_decode_attn_ref(C.byref(s.c()), _p(q), C.byref(cc), C.c_float(sm_scale),
                                      _p(out16), _p(out64), _p(probs))
    if rc:
        raise RuntimeError("minikv_decode_attn_ref failed: %d" % rc)
    return out16, out64, probs


def selective_flash_attn(Q, K, V, sm_scale):
    """Q float16 [B, Hq, L, D]; K, V float16 [B, Hkv, L, D] -> (X_O float16, X_O float64, lse float64 [B, Hq, L],
    A_cumul float64 [B, Hq, L])."""
    Q, K, V = _f16(Q), _f16(K), _f16(V)
    B, Hq, L, D = Q.shape
    Hkv = K.shape[1]
    assert K.shape == (B, Hkv, L, D) and V.shape == K.shape
    xo16 = np.zeros((B, Hq, L, D), np.float16)
    xo64 = np.zeros((B, Hq, L, D), np.float64)
    lse = np.zeros((B, Hq, L), np.float64)
    acc = np.zeros((B, Hq, L), np.float64)
    rc = lib().selective_flash_attn_ref(C.c_int32(B), C.c_int32(Hq), C.c_int32(Hkv), C.c_int64(L), C.c_int32(D),
                                        _p(Q), _p(K), _p(V), C.c_float(sm_scale), _p(xo16), _p(xo64), _p(lse),
                                        _p(acc))
    if rc:
        raise RuntimeError("selective_flash_attn_ref failed: %d" % rc)
    return xo16, xo64, lse, acc


def selective_flash_attn_rows(Q, K, V, sm_scale, rows, tail=0):
    """Q, K, V float16 [L, D] of one head; rows: query positions -> (X_O float64 [n, D], lse float64 [n],
    weights of the last `tail` keys float64 [n, tail])."""
    Q, K, V = _f16(Q), _f16(K), _f16(V)
    L, D = Q.shape
    rows = np.ascontiguousarray(rows, np.int64)
    n = rows.shape[0]
    xo = np.zeros((n, D), np.float64)
    lse = np.zeros((n,), np.float64)
    pt = np.zeros((n, max(tail, 1)), np.float64)
    rc = lib().selective_flash_attn_rows_ref(C.c_int64(L), C.c_int32(D), _p(Q), _p(K), _p(V), C.c_float(sm_scale),
                                             _p(rows), C.c_int32(n), _p(xo), _p(lse), _p(pt) if tail else None,
                                             C.c_int32(tail))
    if rc:
        raise RuntimeError("selective_flash_attn_rows_ref failed: %d" % rc)
    return xo, lse, pt[:, :tail]


def select_hh_rw(A_cumul, n_hh, n_rw, rep=1, idx_stride=None):
    """A_cumul float32 [U*rep, L]; n_hh, n_rw int32 [U] -> (idx int32 [U, idx_stride] filled with -1 beyond
    n_tok, n_tok int32 [U])."""
    A = np.ascontiguousarray(A_cumul)
    assert A.dtype == np.float32 and A.ndim == 2 and A.shape[0] % rep == 0
    U, L = A.shape[0] // rep, A.shape[1]
    n_hh = np.ascontiguousarray(n_hh, np.int32)
    n_rw = np.ascontiguousarray(n_rw, np.int32)
    assert n_hh.shape == (U,) and n_rw.shape == (U,)
    if idx_stride is None:
        idx_stride = L
    idx = np.full((U, idx_stride), -1, np.int32)
    n_tok = np.full(U, -1, np.int32)
    rc = lib().kv_select_hh_rw_ref(C.c_int32(U), C.c_int32(rep), C.c_int64(L), _p(A), _p(n_hh), _p(n_rw),
                                   _p(idx), C.c_int64(idx_stride), _p(n_tok))
    if rc:
        raise RuntimeError("kv_select_hh_rw_ref failed: %d" % rc)
    return idx, n_tok


def pyramid_budget(n_layers, x, d=7, bottom_heavy=True):
    out = np.zeros(max(n_layers, 1), np.float64)
    rc = lib().kv_pyramid_budget_ref(C.c_int32(n_layers), C.c_double(x), C.c_int32(d),
                                     C.c_int32(1 if bottom_heavy else 0), _p(out))
    if rc:
        raise RuntimeError("kv_pyramid_budget_ref failed: %d" % rc)
    return out


def unpack_codes(cache: RefCache, unit):
    s = cache.shape
    T = int(cache.q_len[unit])
    kc = np.zeros((max(T, 1), s.D), np.uint8)
    vc = np.zeros((max(T, 1), s.D), np.uint8)
    cc = cache.c()
    rc = lib().ref_unpack_codes(C.byref(s.c()), C.byref(cc), C.c_int(unit), _p(kc), _p(vc))
    assert rc == 0
    return kc[:T], vc[:T]


def dequant(cache: RefCache, unit):
    s = cache.shape
    T = int(cache.q_len[unit])
    kh = np.zeros((max(T, 1), s.D), np.float64)
    vh = np.zeros((max(T, 1), s.D), np.float64)
    cc = cache.c()
    rc = lib().ref_dequant(C.byref(s.c()), C.byref(cc), C.c_int(unit), _p(kh), _p(vh))
    assert rc == 0
    return kh[:T], vh[:T]


def k_meta_perm(G, D=128):
    """perm[c] = position of channel c inside a stored K scale / zero row; natural = stored[..., perm]."""
    l = lib()
    return np.array([l.ref_k_meta_pos(C.c_int(G), C.c_int(c)) for c in range(D)], dtype=np.int64)


def group_bytes(G):
    return int(lib().ref_group_bytes(G))


def f32_to_f16_bits(x):
    return int(lib().ref_f32_to_f16(C.c_float(x)))


def f64_to_f16_bits(x):
    return int(lib().ref_f64_to_f16(C.c_double(x)))


def f16_bits_to_f32(h):
    return float(lib().ref_f16_to_f32(C.c_uint16(h)))


# ---------------------------------------------------------------------------------------------------------
# per-token quantized cache (oracle/minikv_pt_ref.c)

class _PtShape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "Hq", "Hkv", "D", "G", "bits", "Tcap")]


class _PtCache(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("Kc", "Ks", "Kz", "Vc", "Vs", "Vz", "q_len")]


class RefPtShape:
    def __init__(self, B, Hq, Hkv, D, G, bits, Tcap):
        self.B, self.Hq, self.Hkv, self.D, self.G, self.bits, self.Tcap = B, Hq, Hkv, D, G, bits, Tcap

    @property
    def units(self):
        return self.B * self.Hkv

    def c(self):
        return _PtShape(self.B, self.Hq, self.Hkv, self.D, self.G, self.bits, self.Tcap)

    def check(self):
        return lib().ref_pt_check_shape(C.byref(self.c()))


class RefPtCache:
    """Host buffers of one per-token quantized cache, zero-initialised (storage order: minikv_pt_ref.h)."""

    def __init__(self, s: RefPtShape):
        U, D, G, T, b = s.units, s.D, s.G, s.Tcap, s.bits
        self.shape = s
        self.Kc = np.zeros((U, T * D * b // 32), np.uint32)
        self.Vc = np.zeros((U, T * D * b // 32), np.uint32)
        self.Ks = np.zeros((U, T, D // G), np.float16)
        self.Kz = np.zeros((U, T, D // G), np.float16)
        self.Vs = np.zeros((U, T, D // G), np.float16)
        self.Vz = np.zeros((U, T, D // G), np.float16)
        self.q_len = np.zeros((U,), np.int32)

    def c(self):
        return _PtCache(*(a.ctypes.data for a in (self.Kc, self.Ks, self.Kz, self.Vc, self.Vs, self.Vz, self.q_len)))


def pt_token_bytes(D, G, bits):
    return int(lib().ref_pt_token_bytes(D, G, bits))


def quantize_pack_pt(cache: RefPtCache, K, V, n_tok, idx=None):
    s = cache.shape
    K, V = _f16(K), _f16(V)
    n_tok = np.ascontiguousarray(n_tok, np.int32)
    stride = 0
    if idx is not None:
        idx = np.ascontiguousarray(idx, np.int32)
        stride = idx.shape[1]
    cc = cache.c()
    return lib().kv_quantize_pack_pt_ref(C.byref(s.c()), _p(K), _p(V), C.c_int64(K.shape[1]), _p(idx),
                                         C.c_int64(stride), _p(n_tok), C.byref(cc))


def decode_attn_pt(cache: RefPtCache, q, sm_scale):
    """q float16 [B, Hq, D] -> (out float16, out float64)."""
    s = cache.shape
    q = _f16(q)
    out16 = np.zeros((s.B, s.Hq, s.D), np.float16)
    out64 = np.zeros((s.B, s.Hq, s.D), np.float64)
    cc = cache.c()
    rc = lib().minikv_decode_attn_pt_ref(C.byref(s.c()), _p(q), C.byref(cc), C.c_float(sm_scale), _p(out16), _p(out64))
    assert rc == 0
    return out16, out64


def unpack_codes_pt(cache: RefPtCache, unit):
    s = cache.shape
    T = int(cache.q_len[unit])
    kc = np.zeros((max(T, 1), s.D), np.uint8)
    vc = np.zeros((max(T, 1), s.D), np.uint8)
    cc = cache.c()
    assert lib().ref_pt_unpack_codes(C.byref(s.c()), C.byref(cc), int(unit), _p(kc), _p(vc)) == 0
    return kc[:T], vc[:T]
