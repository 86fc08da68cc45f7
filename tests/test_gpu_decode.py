"""GPU parity for minikv_decode_attn against the oracle (Algorithm 1 lines 17-19; eq. (1)):
max-abs <= 2e-3 on the fp16 outputs, fp32 accumulation on the GPU, fp64 in the oracle."""
import numpy as np
import pytest
import torch

from paper_2411_18077_amd import workloads as W

pytestmark = pytest.mark.gpu
TOL = 2e-3

import os

VARIANTS = [int(v) for v in os.environ.get("MINIKV_TEST_VARIANTS", "1,3").split(",")]


@pytest.fixture(scope="module")
def g():
    import gpu_common
    assert torch.cuda.is_available()
    return gpu_common


def run_both(g, w, r_len, variant, Tcap=None, seed_offset=0, mutate=None):
    from paper_2411_18077_amd import api
    from oracle import ref
    inp = W.make_inputs(w, "cuda", seed_offset=seed_offset)
    if mutate:
        mutate(inp)
    s, rs = g.shapes_for(w, Tcap or inp.Tcap)
    gc = g.gpu_build_cache(inp, s, r_len=r_len)
    rc = g.ref_build_cache(inp, rs, r_len=r_len)
    out = torch.full((w.B, w.Hq, w.D), float("nan"), dtype=torch.float16, device="cuda")
    api.minikv_set_variant(variant)
    try:
        api.minikv_decode_attn(s, inp.q, gc, g.sm_scale(), out)
        torch.cuda.synchronize()
    finally:
        api.minikv_set_variant(0)
    want, _, _ = ref.decode_attn(rc, g.to_np(inp.q), g.sm_scale())
    got = g.to_np(out).astype(np.float64)
    assert np.isfinite(got).all()
    return got, want.astype(np.float64)


def tiny(G=32, **kw):
    base = dict(name="t", B=2, Hq=4, Hkv=2, L=1536, keep=0.5, G=G, Rcap=max(G, 32), seed=70 + G,
                n_outlier=3, outlier_scale=8.0)
    base.update(kw)
    return W.Workload(**base)


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("G,Hq,Hkv", [(32, 4, 4), (32, 8, 2), (16, 2, 2), (64, 8, 1), (128, 4, 2), (32, 2, 1)])
def test_decode_matches_oracle(g, variant, G, Hq, Hkv):
    w = tiny(G, Hq=Hq, Hkv=Hkv)
    got, want = run_both(g, w, r_len=w.Rcap, variant=variant)
    assert np.max(np.abs(got - want)) <= TOL


@pytest.mark.parametrize("variant", VARIANTS)
@pytest.mark.parametrize("r", [0, 1, 31, 32])
def test_residual_lengths(g, variant, r):
    w = tiny(32, Rcap=32)
    got, want = run_both(g, w, r_len=r, variant=variant)
    assert np.max(np.abs(got - want)) <= TOL


@pytest.mark.parametrize("variant", VARIANTS)
def test_ragged_units_including_empty_ones(g, variant):
    """Per-unit lengths from 1 group to the full context, one unit with only residual tokens, one with
    nothing at all (zeros)."""
    w = tiny(64, B=3, Hq=4, Hkv=2, L=2048, keep=None, keep_range=(0.03, 1.0), Rcap=64, dist="student_t4",
             n_outlier=0)

    def mutate(inp):
        inp.n_tok[1] = 0
        inp.n_tok[4] = 0

    r_len = [64, 5, 0, 64, 0, 17]
    got, want = run_both(g, w, r_len=r_len, variant=variant, mutate=mutate)
    assert np.max(np.abs(got - want)) <= TOL
    assert not got.reshape(3, 2, 2, 128)[2, 0].any()          # unit 4: no tokens at all -> zeros


@pytest.mark.parametrize("variant", VARIANTS)
def test_peaked_attention_with_outlier_channels(g, variant):
    """Few tokens, the query aligned with one key, x10 outlier channels: the case that stresses 2e-3."""
    w = tiny(32, B=1, Hq=4, Hkv=1, L=128, keep=1.0, Rcap=32, n_outlier=4, outlier_scale=10.0)

    def mutate(inp):
        inp.q[0, 0] = inp.K[0, 17] * 0.5
        inp.q[0, 1] = inp.K[0, 99] * 0.25
        inp.q[0, 2] = inp.Rk[0, 3]

    got, want = run_both(g, w, r_len=8, variant=variant, mutate=mutate)
    assert np.max(np.abs(got - want)) <= TOL


@pytest.mark.parametrize("variant", VARIANTS)
def test_cfg1_full(g, variant):
    w = W.WORKLOADS[0]
    got, want = run_both(g, w, r_len=w.Rcap, variant=variant)
    assert np.max(np.abs(got - want)) <= TOL
