"""GPU parity over whole decode loops (Algorithm 1, Decoding procedure: append, flush every n_r steps,
attend) and for units that are served by very many waves.  Outputs against the oracle at 2e-3, caches
bit-exact."""
import numpy as np
import pytest
import torch

from paper_2411_18077_amd import workloads as W

pytestmark = pytest.mark.gpu
TOL = 2e-3


@pytest.fixture(scope="module")
def g():
    import gpu_common
    assert torch.cuda.is_available()
    return gpu_common


def small(G=32, **kw):
    base = dict(name="loop", B=2, Hq=8, Hkv=2, L=512, keep=0.5, G=G, Rcap=32, seed=311, n_outlier=2,
                outlier_scale=6.0)
    base.update(kw)
    return W.Workload(**base)


def test_generation_loop_attends_every_step(g):
    """2*n_r + 3 steps of append -> flush -> attend on both sides: the residual runs through 1..n_r-1, is
    compressed twice, and every step's output is compared (Algorithm 1 lines 9-19)."""
    from paper_2411_18077_amd import api
    from oracle import ref
    w = small()
    inp = W.make_inputs(w, "cuda")
    Tcap = 512
    s, rs = g.shapes_for(w, Tcap)
    gc = g.gpu_build_cache(inp, s)
    rc = g.ref_build_cache(inp, rs)
    gen = torch.Generator(device="cuda"); gen.manual_seed(5)
    out = torch.empty(w.B, w.Hq, w.D, dtype=torch.float16, device="cuda")
    worst = 0.0
    for i in range(2 * w.Rcap + 3):
        k = torch.randn(w.units, w.D, generator=gen, device="cuda").to(torch.float16)
        v = torch.randn(w.units, w.D, generator=gen, device="cuda").to(torch.float16)
        q = torch.randn(w.B, w.Hq, w.D, generator=gen, device="cuda").to(torch.float16)
        api.kv_append_residual(s, k, v, gc)
        api.kv_flush_residual(s, gc)
        api.minikv_decode_attn(s, q, gc, g.sm_scale(), out)
        assert ref.append_residual(rc, g.to_np(k), g.to_np(v)) == 0
        assert ref.flush_residual(rc) == 0
        want, _, _ = ref.decode_attn(rc, g.to_np(q), g.sm_scale())
        got = g.to_np(out).astype(np.float64)
        assert np.isfinite(got).all()
        worst = max(worst, float(np.max(np.abs(got - want))))
        assert worst <= TOL, "step %d" % i
    torch.cuda.synchronize()
    assert gc.q_len.cpu().tolist() == rc.q_len.tolist() and gc.r_len.cpu().tolist() == rc.r_len.tolist()
    g.assert_cache_bit_exact(gc, rc, what=("Kc", "Ks", "Kz", "Vc", "Vs", "Vz"))


def test_one_step_captured_in_a_graph_and_replayed(g):
    """append + flush + attend captured once in a HIP graph and replayed with new inputs in the static
    buffers; eager work and synchronisations between the replays; every replay against the oracle."""
    from paper_2411_18077_amd import api
    from oracle import ref
    w = small(seed=312)
    inp = W.make_inputs(w, "cuda")
    s, rs = g.shapes_for(w, 512)
    gc = g.gpu_build_cache(inp, s)
    rc = g.ref_build_cache(inp, rs)
    k = torch.zeros(w.units, w.D, dtype=torch.float16, device="cuda")
    v = torch.zeros_like(k)
    q = torch.zeros(w.B, w.Hq, w.D, dtype=torch.float16, device="cuda")
    out = torch.zeros_like(q)
    ws = gc.workspace                                       # allocated (and zeroed) outside the capture
    assert ws is not None
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    gen = torch.Generator(device="cuda"); gen.manual_seed(6)

    def fresh():
        k.copy_(torch.randn(w.units, w.D, generator=gen, device="cuda").to(torch.float16))
        v.copy_(torch.randn(w.units, w.D, generator=gen, device="cuda").to(torch.float16))
        q.copy_(torch.randn(w.B, w.Hq, w.D, generator=gen, device="cuda").to(torch.float16))

    def oracle_step():
        assert ref.append_residual(rc, g.to_np(k), g.to_np(v)) == 0
        assert ref.flush_residual(rc) == 0
        want, _, _ = ref.decode_attn(rc, g.to_np(q), g.sm_scale())
        return want

    # one eager step first (also warms everything up), then capture
    fresh()
    api.kv_append_residual(s, k, v, gc); api.kv_flush_residual(s, gc)
    api.minikv_decode_attn(s, q, gc, g.sm_scale(), out, workspace=ws)
    torch.cuda.synchronize()
    assert np.max(np.abs(g.to_np(out).astype(np.float64) - oracle_step())) <= TOL
    with torch.cuda.graph(graph, stream=side):
        api.kv_append_residual(s, k, v, gc)
        api.kv_flush_residual(s, gc)
        api.minikv_decode_attn(s, q, gc, g.sm_scale(), out, workspace=ws)
    for i in range(w.Rcap + 4):                             # crosses a flush
        fresh()
        graph.replay()
        torch.cuda.synchronize()
        got = g.to_np(out).astype(np.float64)
        want = oracle_step()
        assert np.max(np.abs(got - want)) <= TOL, "replay %d" % i
        (k.float().sum() + q.float().sum()).item()          # unrelated eager work between replays
    torch.cuda.synchronize()
    assert gc.q_len.cpu().tolist() == rc.q_len.tolist() and gc.r_len.cpu().tolist() == rc.r_len.tolist()
    g.assert_cache_bit_exact(gc, rc, what=("Kc", "Ks", "Kz", "Vc", "Vs", "Vz"))


def test_generation_of_1024_tokens_replaying_one_captured_step(g):
    """The paper's generation length (1024 new tokens): one captured step (append, flush, attend) replayed
    1024 times on a small shape with G = 16 and n_r = 64, i.e. 16 flushes; the oracle follows every step
    (its state must match at the end, bit for bit) and its attention output is compared on every 7th step
    and around every flush."""
    from paper_2411_18077_amd import api
    from oracle import ref
    steps = 1024
    w = small(G=16, B=1, Hq=4, Hkv=2, L=256, Rcap=64, seed=314)
    inp = W.make_inputs(w, "cuda")
    Tcap = 128 + steps + 128                                # kept prompt tokens + everything generated, in tiles of 128
    s, rs = g.shapes_for(w, Tcap)
    gc = g.gpu_build_cache(inp, s)
    rc = g.ref_build_cache(inp, rs)
    gen = torch.Generator(device="cuda"); gen.manual_seed(8)
    ks = torch.randn(steps, w.units, w.D, generator=gen, device="cuda").to(torch.float16)
    vs = torch.randn(steps, w.units, w.D, generator=gen, device="cuda").to(torch.float16)
    qs = torch.randn(steps, w.B, w.Hq, w.D, generator=gen, device="cuda").to(torch.float16)
    ks_h, vs_h, qs_h = g.to_np(ks), g.to_np(vs), g.to_np(qs)
    k = torch.zeros(w.units, w.D, dtype=torch.float16, device="cuda"); v = torch.zeros_like(k)
    q = torch.zeros(w.B, w.Hq, w.D, dtype=torch.float16, device="cuda"); out = torch.zeros_like(q)
    ws = gc.workspace
    side = torch.cuda.Stream(); side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()

    def step_eager():
        api.kv_append_residual(s, k, v, gc); api.kv_flush_residual(s, gc)
        api.minikv_decode_attn(s, q, gc, g.sm_scale(), out, workspace=ws)

    k.copy_(ks[0]); v.copy_(vs[0]); q.copy_(qs[0])
    step_eager()                                            # step 0 eagerly (warm-up), then capture
    torch.cuda.synchronize()
    assert ref.append_residual(rc, ks_h[0], vs_h[0]) == 0 and ref.flush_residual(rc) == 0
    with torch.cuda.graph(graph, stream=side):
        step_eager()
    worst, checked = 0.0, 0
    for i in range(1, steps):
        k.copy_(ks[i]); v.copy_(vs[i]); q.copy_(qs[i])
        graph.replay()
        assert ref.append_residual(rc, ks_h[i], vs_h[i]) == 0 and ref.flush_residual(rc) == 0
        if i % 7 == 0 or (i + 1) % w.Rcap <= 1:
            torch.cuda.synchronize()
            want, _, _ = ref.decode_attn(rc, qs_h[i], g.sm_scale())
            worst = max(worst, float(np.max(np.abs(g.to_np(out).astype(np.float64) - want))))
            checked += 1
            assert worst <= TOL, "step %d" % i
    torch.cuda.synchronize()
    assert checked > 150
    assert gc.q_len.cpu().tolist() == rc.q_len.tolist() == [128 + steps // w.Rcap * w.Rcap] * w.units
    assert gc.r_len.cpu().tolist() == rc.r_len.tolist()
    g.assert_cache_bit_exact(gc, rc, what=("Kc", "Ks", "Kz", "Vc", "Vs", "Vz"))


@pytest.mark.parametrize("L,Hq", [(32768, 4), (262144, 4), (262144, 8)])
def test_one_unit_served_by_many_waves(g, L, Hq):
    """A single (batch, KV head) with a very long cache: hundreds of waves share the unit, so the split-K
    merge runs in two levels (and, at 262144 tokens, the second level in more than one round); with 8
    query heads the unit has two head sets."""
    from paper_2411_18077_amd import api
    from oracle import ref
    w = small(B=1, Hq=Hq, Hkv=1, L=L, keep=1.0, Rcap=64, seed=313 + Hq, n_outlier=0)
    inp = W.make_inputs(w, "cuda")
    s, rs = g.shapes_for(w, inp.Tcap)
    gc = g.gpu_build_cache(inp, s, r_len=w.Rcap - 3)
    rc = g.ref_build_cache(inp, rs, r_len=w.Rcap - 3)
    g.assert_cache_bit_exact(gc, rc, what=("Kc", "Ks", "Kz", "Vc", "Vs", "Vz"))
    out = torch.full((w.B, w.Hq, w.D), float("nan"), dtype=torch.float16, device="cuda")
    for _ in range(2):                                      # twice: the ticket counters must be back at zero
        out.fill_(float("nan"))
        api.minikv_decode_attn(s, inp.q, gc, g.sm_scale(), out)
        torch.cuda.synchronize()
        want, _, _ = ref.decode_attn(rc, g.to_np(inp.q), g.sm_scale())
        got = g.to_np(out).astype(np.float64)
        assert np.isfinite(got).all()
        assert np.max(np.abs(got - want)) <= TOL
