"""Plumbing shared by the GPU parity tests: run the same seeded inputs through libminikv (device) and
through the CPU oracle (host) and hand back both caches.  No arithmetic of the method lives here."""
import math

import numpy as np
import torch

from oracle import ref
from paper_2411_18077_amd import api
from paper_2411_18077_amd import workloads as W

RAW = ("Kc", "Ks", "Kz", "Vc", "Vs", "Vz", "q_len", "Rk", "Rv", "r_len")


def shapes_for(w, Tcap):
    return (api.make_shape(w.B, w.Hq, w.Hkv, w.D, w.G, Tcap, w.Rcap),
            ref.RefShape(w.B, w.Hq, w.Hkv, w.D, w.G, Tcap, w.Rcap))


def to_np(t):
    return t.detach().cpu().numpy()


def gpu_build_cache(inp, shape, r_len=None):
    """Prefill-quantize the retained rows of inp on the GPU; optionally preload the residual."""
    w = inp.w
    cache = api.Cache(shape, device=inp.K.device)
    n_max = int(inp.n_tok.max())
    api.kv_quantize_pack(shape, inp.K, inp.V, w.L, inp.idx, inp.idx.shape[1], inp.n_tok, n_max, cache)
    if r_len is not None and w.Rcap:
        cache.Rk.view(w.units, w.Rcap, w.D).copy_(inp.Rk)
        cache.Rv.view(w.units, w.Rcap, w.D).copy_(inp.Rv)
        cache.r_len.copy_(torch.as_tensor(r_len, dtype=torch.int32).to(cache.r_len.device).expand(w.units))
    torch.cuda.synchronize()
    return cache


def ref_build_cache(inp, rshape, r_len=None, units=None):
    """The same through the oracle.  `units`: optional list of unit indices; then the oracle cache holds
    only those units (as a batch of len(units) single-head sequences)."""
    w = inp.w
    if units is None:
        K, V, idx, n_tok = to_np(inp.K), to_np(inp.V), to_np(inp.idx), to_np(inp.n_tok)
        Rk, Rv = to_np(inp.Rk), to_np(inp.Rv)
    else:
        sel = torch.as_tensor(units, device=inp.K.device)
        K, V, idx, n_tok = (to_np(x[sel]) for x in (inp.K, inp.V, inp.idx, inp.n_tok))
        Rk, Rv = to_np(inp.Rk[sel]), to_np(inp.Rv[sel])
    c = ref.RefCache(rshape)
    rc = ref.quantize_pack(c, K, V, n_tok, idx)
    assert rc == 0
    if r_len is not None and w.Rcap:
        c.Rk[:] = Rk
        c.Rv[:] = Rv
        c.r_len[:] = np.broadcast_to(np.asarray(r_len, np.int32), c.r_len.shape)
    return c


def assert_cache_bit_exact(gpu_cache, ref_cache, unit_map=None, what=RAW):
    """Raw buffers equal byte for byte.  unit_map[i] = GPU unit held at oracle unit i (None: identity)."""
    U = gpu_cache.shape.B * gpu_cache.shape.Hkv
    for name in what:
        g = to_np(gpu_cache.t[name])
        r = getattr(ref_cache, name)
        g = g[: (g.size // U) * U].reshape(U, -1)
        if unit_map is not None:
            g = g[np.asarray(unit_map)]
        r = r.reshape(r.shape[0], -1)
        if r.shape[1] == 0 or g.shape[1] != r.shape[1]:
            assert gpu_cache.shape.Rcap == 0 and name in ("Rk", "Rv"), (name, g.shape, r.shape)
            continue
        gb = np.ascontiguousarray(g).view(np.uint8)
        rb = np.ascontiguousarray(r).view(np.uint8)
        if not np.array_equal(gb, rb):
            bad = np.argwhere(gb != rb)
            raise AssertionError("%s differs at %d bytes, first (unit, byte) = %s" % (name, len(bad), bad[0]))


def sm_scale(D=128):
    return 1.0 / math.sqrt(D)
