"""GPU parity of the token selection (Section 3.1.2, Algorithm 1 line 3) against the oracle: kept positions
and counts bit-exact, nothing written beyond the count; then the selected positions carried through
kv_quantize_pack and one decode step (Algorithm 1 lines 3-5, 17-19)."""
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


@pytest.fixture(autouse=True, params=[0, 1, 2], ids=["by-shape", "one-workgroup-per-unit", "chunked"])
def select_path(request):
    """Every test runs with the kernels chosen by shape and with each of the two sets forced."""
    from paper_2411_18077_amd import api
    api.minikv_diag_select_path(request.param)
    yield request.param
    api.minikv_diag_select_path(0)


def run_gpu(A, n_hh, n_rw, rep, idx_stride):
    """A: cuda float32 [U*rep, L].  Returns (idx [U, idx_stride] with -1 where nothing was written, n_tok)."""
    from paper_2411_18077_amd import api
    U, L = A.shape[0] // rep, A.shape[1]
    hh = torch.as_tensor(np.asarray(n_hh, np.int32), device="cuda")
    rw = torch.as_tensor(np.asarray(n_rw, np.int32), device="cuda")
    idx = torch.full((U, idx_stride), -1, dtype=torch.int32, device="cuda")
    n_tok = torch.full((U,), -1, dtype=torch.int32, device="cuda")
    nws = api.kv_select_workspace_bytes(U, rep, L)
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda").fill_(0xA5) if nws else None   # no initial state needed
    api.kv_select_hh_rw(U, rep, L, A, hh, rw, idx, idx_stride, n_tok, ws)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), n_tok.cpu().numpy()


def check(g, A, n_hh, n_rw, rep=1, idx_stride=None):
    from oracle import ref
    L = A.shape[1]
    stride = L if idx_stride is None else idx_stride
    got_idx, got_n = run_gpu(A, n_hh, n_rw, rep, stride)
    want_idx, want_n = ref.select_hh_rw(g.to_np(A), n_hh, n_rw, rep=rep, idx_stride=stride)
    assert np.array_equal(got_n, want_n)
    assert np.array_equal(got_idx, want_idx)


@pytest.mark.parametrize("kind", ["attention", "ties", "signed"])
@pytest.mark.parametrize("L,k,n_rw", [(1000, 250, 250), (257, 64, 32), (4097, 1024, 1023), (9000, 33, 4500),
                                      (5, 2, 1), (64, 1, 0), (300, 0, 7), (32768, 8192, 8192)])
def test_selection_bit_exact(g, kind, L, k, n_rw):
    U = 7
    A = W.make_scores(U, L, seed=21 + L, device="cuda", kind=kind)
    check(g, A, np.full(U, k), np.full(U, n_rw))


@pytest.mark.parametrize("L", [32769, 40000, 70001])
def test_prompts_longer_than_the_on_chip_key_cache(g, L):
    """Beyond 32768 tokens the keys no longer fit in LDS and every pass reads them from memory."""
    U = 3
    for kind in ("attention", "ties"):
        A = W.make_scores(U, L, seed=5 + L, device="cuda", kind=kind)
        check(g, A, [L // 4, 1, L - 100], [L // 4, L // 2, 100])


@pytest.mark.parametrize("L", [40000, 200000])
def test_scores_tied_en_masse(g, L):
    """More equal or near-equal scores than the on-chip candidate list holds (16384): constant scores, eight
    levels, and attention-like scores squeezed into one binade take the general path of the kernel."""
    flat = torch.full((2, L), 3.5, device="cuda")
    check(g, flat, [L // 3, 17], [L // 4, 0], idx_stride=L)
    ties = W.make_scores(2, L, seed=L, device="cuda", kind="ties")
    check(g, ties, [L // 3, L // 2], [L // 4, 5], idx_stride=L)
    narrow = (1.0 + W.make_scores(4, L, seed=L + 1, device="cuda", kind="attention").clamp_(max=1.0) * 2.0 ** -12).contiguous()
    check(g, narrow, np.full(2, L // 5), np.full(2, L // 5), rep=2, idx_stride=L)


def test_million_token_prompt(g):
    L = (1 << 20) + 5
    A = W.make_scores(4, L, seed=3, device="cuda", kind="attention")
    check(g, A, [L // 4, 1000], [L // 8, L // 2], rep=2, idx_stride=L // 2 + 1000)


def test_ragged_degenerate_and_invalid_budgets(g):
    L = 777
    A = W.make_scores(12, L, seed=6, device="cuda", kind="ties")
    n_hh = np.array([0, 1, 100, 333, 777, 0, -1, 10, 700, 10, 400, 776], np.int32)
    n_rw = np.array([0, 776, 50, 444, 0, 777, 5, -2, 100, 778, 200, 0], np.int32)
    check(g, A, n_hh, n_rw)
    check(g, A, n_hh, n_rw, idx_stride=512)                  # several units no longer fit their row


def test_constant_and_monotone_scores(g):
    L = 5000
    flat = torch.full((2, L), 0.25, device="cuda")
    check(g, flat, [1200, 1], [600, 0])
    inc = torch.arange(L, dtype=torch.float32, device="cuda").repeat(2, 1).contiguous()
    check(g, inc, [1200, 4999], [600, 0])
    check(g, inc.flip(1).contiguous(), [1200, 4999], [600, 1])
    zeros = torch.zeros(1, L, device="cuda"); zeros[0, 1::2] = -0.0
    check(g, zeros, [7], [3])


@pytest.mark.parametrize("rep,L", [(4, 1000), (2, 4099), (8, 333), (4, 40000), (3, 5000), (5, 777), (16, 130)])
def test_query_heads_of_a_group_are_summed(g, rep, L):
    U = 5
    A = W.make_scores(U * rep, L, seed=31 + rep, device="cuda", kind="attention")
    check(g, A, np.full(U, L // 4), np.full(U, L // 5), rep=rep)
    T = W.make_scores(U * rep, L, seed=32 + rep, device="cuda", kind="ties")
    check(g, T, np.full(U, L // 3), np.full(U, 0), rep=rep)


def test_random_shapes_and_budgets(g):
    """Seeded sweep: 40 random (units, heads per unit, prompt length, kind) with random budgets per unit, a
    few of them out of range, and rows narrower than the prompt."""
    rng = np.random.default_rng(2024)
    for case in range(40):
        U = int(rng.integers(1, 7))
        rep = int(rng.choice([1, 1, 2, 3, 4, 6, 8]))
        L = int(rng.choice([rng.integers(1, 200), rng.integers(200, 6000), rng.integers(30000, 36000)]))
        kind = str(rng.choice(["attention", "ties", "signed"]))
        A = W.make_scores(U * rep, L, seed=1000 + case, device="cuda", kind=kind)
        n_rw = rng.integers(0, L + 1, U)
        n_hh = np.array([rng.integers(0, L - w + 1) for w in n_rw])
        if case % 5 == 0:
            n_hh[0] = L + 1                                  # out of range: that unit keeps nothing
        stride = int(rng.choice([L, max(1, L // 2), L + 3]))
        check(g, A, n_hh.astype(np.int32), n_rw.astype(np.int32), rep=rep, idx_stride=stride)


@pytest.mark.parametrize("U,rep,L", [(9, 4, 9000), (13, 1, 20000), (21, 2, 40000), (8, 3, 12289)])
def test_unit_counts_that_do_not_fill_a_group_of_eight(g, U, rep, L):
    """The several-workgroups-per-unit kernels number their workgroups in groups of eight units (one die each);
    the last group is partly empty here.  Budgets differ from unit to unit; one unit is out of range, one keeps
    only the window, one keeps every candidate."""
    rng = np.random.default_rng(77 + U)
    A = W.make_scores(U * rep, L, seed=300 + U, device="cuda", kind="attention" if U % 2 else "ties")
    n_rw = rng.integers(0, L // 2, U)
    n_hh = np.array([rng.integers(1, L - w) for w in n_rw])
    n_hh[1] = L + 5                                          # out of range
    n_hh[2] = 0                                              # window only
    n_hh[3] = L - n_rw[3]                                    # every candidate
    check(g, A, n_hh.astype(np.int32), n_rw.astype(np.int32), rep=rep)


def test_empty_prompt_and_no_units(g):
    from paper_2411_18077_amd import api
    A = torch.zeros(2, 0, device="cuda")
    got_idx, got_n = run_gpu(A, [0, 0], [0, 0], 1, 4)
    assert got_n.tolist() == [0, 0] and (got_idx == -1).all()
    got_idx, got_n = run_gpu(A, [1, 0], [0, 1], 1, 4)        # budgets beyond an empty prompt
    assert got_n.tolist() == [0, 0]
    api.kv_select_hh_rw(0, 1, 16, None, None, None, None, 16, None)   # nothing to do


def test_second_call_on_other_inputs(g):
    """The launch keeps no state: a smaller problem right after a larger one, same buffers' worth of LDS."""
    A = W.make_scores(4, 20000, seed=1, device="cuda", kind="attention")
    check(g, A, np.full(4, 5000), np.full(4, 5000))
    B = W.make_scores(4, 300, seed=2, device="cuda", kind="ties")
    check(g, B, np.full(4, 75), np.full(4, 75))


@pytest.mark.parametrize("name,U,rep,L", [("32k, 32 query / 8 KV heads, batch 16", 128, 4, 32768),
                                          ("128k, 32 query / 8 KV heads, batch 1", 8, 4, 131072),
                                          ("16k, 32 heads, batch 32", 1024, 1, 16384)])
def test_full_size_prompts(g, name, U, rep, L):
    """The shapes of the benchmark configurations, 20 % heavy hitters + 20 % recent window, every unit."""
    gen = np.random.default_rng(L)
    A = W.make_scores(U * rep, L, seed=77, device="cuda", kind="attention")
    n_hh = (gen.integers(L // 8, L // 4, U) // 32 * 32).astype(np.int32)
    n_rw = np.full(U, L // 5 // 32 * 32, np.int32)
    check(g, A, n_hh, n_rw, rep=rep, idx_stride=L // 2)


def test_selected_tokens_through_quantize_and_decode(g):
    """Algorithm 1 lines 3-5 then 17-19 on both sides: select from scores, gather + quantize + pack the
    selected rows, append one token, attend."""
    from paper_2411_18077_amd import api
    from oracle import ref
    w = W.Workload(name="sel", B=2, Hq=8, Hkv=2, L=1024, keep=0.5, G=32, Rcap=32, seed=411, n_outlier=2,
                   outlier_scale=6.0)
    inp = W.make_inputs(w, "cuda")
    U, rep = w.units, w.Hq // w.Hkv
    A = W.make_scores(U * rep, w.L, seed=412, device="cuda", kind="attention")
    n_hh = np.array([256, 128, 320, 0], np.int32)
    n_rw = np.array([256, 384, 32, 512], np.int32)
    stride = 512
    idx = torch.zeros(U, stride, dtype=torch.int32, device="cuda")
    n_tok = torch.zeros(U, dtype=torch.int32, device="cuda")
    ws = torch.empty(api.kv_select_workspace_bytes(U, rep, w.L), dtype=torch.uint8, device="cuda")
    api.kv_select_hh_rw(U, rep, w.L, A, torch.as_tensor(n_hh, device="cuda"), torch.as_tensor(n_rw, device="cuda"),
                        idx, stride, n_tok, ws)
    s, rs = g.shapes_for(w, 640)
    gc = api.Cache(s)
    api.kv_quantize_pack(s, inp.K, inp.V, w.L, idx, stride, n_tok, 512, gc)
    api.kv_append_residual(s, inp.Rk[:, 0].contiguous(), inp.Rv[:, 0].contiguous(), gc)
    out = torch.empty(w.B, w.Hq, w.D, dtype=torch.float16, device="cuda")
    api.minikv_decode_attn(s, inp.q, gc, g.sm_scale(), out)
    torch.cuda.synchronize()

    ridx, rn = ref.select_hh_rw(g.to_np(A), n_hh, n_rw, rep=rep, idx_stride=stride)
    assert np.array_equal(g.to_np(n_tok), rn)
    rc = ref.RefCache(rs)
    assert ref.quantize_pack(rc, g.to_np(inp.K), g.to_np(inp.V), rn, np.maximum(ridx, 0)) == 0
    assert ref.append_residual(rc, g.to_np(inp.Rk[:, 0]), g.to_np(inp.Rv[:, 0])) == 0
    g.assert_cache_bit_exact(gc, rc, what=("Kc", "Ks", "Kz", "Vc", "Vs", "Vz", "q_len", "r_len"))
    want, _, _ = ref.decode_attn(rc, g.to_np(inp.q), g.sm_scale())
    assert np.max(np.abs(g.to_np(out).astype(np.float64) - want)) <= TOL
