"""The allocation-free decode entry point (minikv_decode_attn_static: the split-K workspace is a device array
of the library) against minikv_decode_attn with a caller-provided workspace, through the raw C ABI: two calls in
a row, the second with a smaller input, then a shape too large for the array."""
import ctypes as C
import math

import numpy as np
import pytest
import torch

from paper_2411_18077_amd import workloads as W

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _case(api, gpu_common, w, r_len):
    inp = W.make_inputs(w, "cuda")
    shape, _ = gpu_common.shapes_for(w, inp.Tcap)
    cache = gpu_common.gpu_build_cache(inp, shape, r_len=r_len)
    return inp, shape, cache


def _both(api, inp, shape, cache, w):
    """(static entry point, workspace entry point) outputs, both through ctypes on the current stream."""
    l = api.lib()
    sm = 1.0 / math.sqrt(w.D)
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    cc = cache.c()
    out_s = torch.full((w.B, w.Hq, w.D), float("nan"), dtype=torch.float16, device="cuda")
    out_w = torch.full_like(out_s, float("nan"))
    rc = l.minikv_decode_attn_static(C.byref(shape), C.c_void_p(inp.q.data_ptr()), C.byref(cc), C.c_float(sm),
                                     C.c_void_p(out_s.data_ptr()), st)
    assert rc == 0, rc
    ws = cache.workspace
    rc = l.minikv_decode_attn(C.byref(shape), C.c_void_p(inp.q.data_ptr()), C.byref(cc), C.c_float(sm),
                              C.c_void_p(out_w.data_ptr()), C.c_void_p(ws.data_ptr()), ws.numel(), st)
    assert rc == 0, rc
    torch.cuda.synchronize()
    return out_s.float().cpu().numpy(), out_w.float().cpu().numpy()


def test_static_workspace_entry_point_matches_the_workspace_one():
    import gpu_common
    from oracle import ref
    from paper_2411_18077_amd import api
    assert torch.cuda.is_available()
    # first call: grouped-query shape whose units are each served by many waves (partials and tickets in use)
    big = W.Workload("na_big", B=2, Hq=16, Hkv=4, L=8192, keep=0.5, G=32, Rcap=64, seed=901, n_outlier=3, outlier_scale=8.0)
    inp, shape, cache = _case(api, gpu_common, big, big.Rcap)
    got_s, got_w = _both(api, inp, shape, cache, big)
    assert np.isfinite(got_s).all()
    assert np.max(np.abs(got_s - got_w)) <= TOL
    _, rs = gpu_common.shapes_for(big, inp.Tcap)
    want, _, _ = ref.decode_attn(gpu_common.ref_build_cache(inp, rs, r_len=big.Rcap), gpu_common.to_np(inp.q), 1.0 / math.sqrt(big.D))
    assert np.max(np.abs(got_s - want.astype(np.float32))) <= TOL
    # second call, right after: a smaller input of another shape (more heads per unit, another group size)
    small = W.Workload("na_small", B=1, Hq=8, Hkv=1, L=1536, keep=0.5, G=64, Rcap=64, seed=902)
    inp2, shape2, cache2 = _case(api, gpu_common, small, 17)
    got_s2, got_w2 = _both(api, inp2, shape2, cache2, small)
    assert np.isfinite(got_s2).all()
    assert np.max(np.abs(got_s2 - got_w2)) <= TOL
    # and the first one again (the array keeps what the second call left)
    got_s3, _ = _both(api, inp, shape, cache, big)
    assert np.max(np.abs(got_s3 - got_w)) <= TOL
