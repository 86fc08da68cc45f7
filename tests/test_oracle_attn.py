"""Pins for the oracle's decode attention (Algorithm 1 lines 9-19; Appendix A eq. (1)).

The independent check is a numpy fp64 brute force that never touches packed words: it re-derives the
dequantized cache from the source tensors with vectorised numpy and evaluates softmax(q K^T / sqrt d) V
with library routines.  Further pins are special cases with textbook answers.
"""
import numpy as np
import pytest
from scipy.special import softmax

from helpers import ref_cache_from


def _rand16(shape, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(shape) * scale).astype(np.float16)


def np_dequantized(X, G, axis):
    """fp64 x_hat of a [L, D] fp16 matrix, groups of G along `axis`, via numpy only (binary32 decisions)."""
    L, D = X.shape
    x = X.astype(np.float32)
    g = x.reshape(L // G, G, D) if axis == 0 else x.reshape(L, D // G, G)
    ax = 1 if axis == 0 else 2
    mn = g.min(axis=ax, keepdims=True)
    mx = g.max(axis=ax, keepdims=True)
    s = ((mx - mn) / np.float32(3)).astype(np.float16).astype(np.float32)
    with np.errstate(divide="ignore"):
        inv = np.where(s == 0, np.float32(0), np.float32(1) / s).astype(np.float32)
    code = np.clip(np.rint(((g - mn).astype(np.float32) * inv).astype(np.float32)), 0, 3)
    return (code.astype(np.float64) * s.astype(np.float64) + mn.astype(np.float64)).reshape(L, D)


def brute_force(q, Khat, Vhat, Rk, Rv, sm_scale):
    """Textbook single-query attention over [K_hat; R_K], [V_hat; R_V] in fp64."""
    Kall = np.concatenate([Khat, Rk.astype(np.float64)], axis=0)
    Vall = np.concatenate([Vhat, Rv.astype(np.float64)], axis=0)
    p = softmax(np.float64(np.float32(sm_scale)) * (Kall @ q.astype(np.float64)))
    return p @ Vall, p


@pytest.mark.parametrize("G,Hq,Hkv,T,r", [(16, 2, 2, 64, 5), (32, 4, 2, 128, 8), (32, 4, 1, 96, 0), (64, 2, 2, 64, 1)])
def test_matches_fp64_brute_force(ref, G, Hq, Hkv, T, r):
    B, D = 2, 128
    U = B * Hkv
    Rcap = max(G, 16)
    K = _rand16((U, T, D), 1); V = _rand16((U, T, D), 2)
    K[:, :, [3, 77]] *= 10
    c = ref_cache_from(ref, K, V, G, Hq=Hq, B=B, Rcap=Rcap)
    Rk = _rand16((U, Rcap, D), 3); Rv = _rand16((U, Rcap, D), 4)
    c.Rk[:] = Rk; c.Rv[:] = Rv; c.r_len[:] = r
    q = _rand16((B, Hq, D), 5)
    sm = 1.0 / np.sqrt(D)
    out16, out64, probs = ref.decode_attn(c, q, sm, want_f64=True, want_probs=True)
    rep = Hq // Hkv
    for b in range(B):
        for h in range(Hq):
            u = b * Hkv + h // rep
            want, p = brute_force(q[b, h], np_dequantized(K[u], G, 0), np_dequantized(V[u], G, 1),
                                  Rk[u, :r], Rv[u, :r], sm)
            assert np.max(np.abs(out64[b, h] - want)) <= 1e-9
            assert np.max(np.abs(probs[b, h, : T + r] - p)) <= 1e-12
            assert abs(probs[b, h].sum() - 1.0) <= 1e-12             # attention rows sum to 1
            assert np.all(probs[b, h, T + r:] == 0)
            assert np.array_equal(out16[b, h], want.astype(np.float16)) or \
                np.max(np.abs(out16[b, h].astype(np.float64) - want)) <= 2.0 ** -11 * np.max(np.abs(want))
    # and the oracle's own layout-free view agrees with the numpy re-derivation bit for bit
    for u in range(U):
        kh, vh = ref.dequant(c, u)
        assert np.array_equal(kh, np_dequantized(K[u], G, 0)) and np.array_equal(vh, np_dequantized(V[u], G, 1))


def test_empty_quantized_part_is_textbook_fp16_attention(ref):
    B, H, D, G, Rcap, r = 1, 2, 128, 32, 32, 7
    s = ref.RefShape(B, H, H, D, G, 128, Rcap); c = ref.RefCache(s)
    c.Rk[:] = _rand16((H, Rcap, D), 1); c.Rv[:] = _rand16((H, Rcap, D), 2); c.r_len[:] = r
    q = _rand16((B, H, D), 3)
    _, out64, _ = ref.decode_attn(c, q, 0.125, want_f64=True)
    for h in range(H):
        p = softmax(0.125 * (c.Rk[h, :r].astype(np.float64) @ q[0, h].astype(np.float64)))
        assert np.max(np.abs(out64[0, h] - p @ c.Rv[h, :r].astype(np.float64))) <= 1e-12


def test_empty_unit_gives_zeros(ref):
    s = ref.RefShape(1, 2, 2, 128, 32, 128, 32); c = ref.RefCache(s)
    out16, out64, _ = ref.decode_attn(c, _rand16((1, 2, 128), 1), 1.0, want_f64=True)
    assert not out16.view(np.uint16).any() and not out64.any()


def test_equal_keys_give_the_mean_value(ref):
    """All key rows equal => uniform weights => output is the mean of the dequantized values."""
    G, T, D = 32, 64, 128
    K = np.tile(_rand16((1, 1, D), 1), (1, T, 1)); V = _rand16((1, T, D), 2)
    c = ref_cache_from(ref, K, V, G)
    _, out64, probs = ref.decode_attn(c, _rand16((1, 1, D), 3), 0.3, want_f64=True, want_probs=True)
    assert np.allclose(probs[0, 0, :T], 1.0 / T, rtol=0, atol=1e-15)
    _, vh = ref.dequant(c, 0)
    assert np.max(np.abs(out64[0, 0] - vh.mean(axis=0))) <= 1e-12


def test_lattice_cache_equals_exact_attention_on_the_original(ref):
    """On lossless lattice data the whole pipeline is eq. (1) on the ORIGINAL fp16 K, V."""
    G, T, D = 16, 128, 128
    rng = np.random.default_rng(9)
    lk = rng.integers(0, 4, (1, T, D)); lv = rng.integers(0, 4, (1, T, D))
    lk[:, 0::G] = 0; lk[:, 1::G] = 3; lv[:, :, 0::G] = 0; lv[:, :, 1::G] = 3
    K = (lk * 0.25 - 0.5).astype(np.float16); V = (lv * 0.5 - 1.0).astype(np.float16)
    c = ref_cache_from(ref, K, V, G)
    q = _rand16((1, 1, D), 4)
    _, out64, _ = ref.decode_attn(c, q, 1 / np.sqrt(D), want_f64=True)
    p = softmax(np.float64(np.float32(1 / np.sqrt(D))) * (K[0].astype(np.float64) @ q[0, 0].astype(np.float64)))
    assert np.max(np.abs(out64[0, 0] - p @ V[0].astype(np.float64))) <= 1e-12


def test_gqa_equals_mha_on_replicated_kv_and_units_permute(ref):
    B, Hq, Hkv, D, G, T, Rcap = 2, 4, 2, 128, 32, 96, 32
    U = B * Hkv
    K = _rand16((U, T, D), 1); V = _rand16((U, T, D), 2)
    Rk = _rand16((U, Rcap, D), 3); Rv = _rand16((U, Rcap, D), 4)
    q = _rand16((B, Hq, D), 5)
    r_len = np.array([3, 0, 32, 9], np.int32)
    gqa = ref_cache_from(ref, K, V, G, Hq=Hq, B=B, Rcap=Rcap)
    gqa.Rk[:] = Rk; gqa.Rv[:] = Rv; gqa.r_len[:] = r_len
    a, _, _ = ref.decode_attn(gqa, q, 0.1)
    rep = np.repeat(np.arange(U).reshape(B, Hkv), Hq // Hkv, axis=1).reshape(-1)     # unit of each (b, hq)
    mha = ref_cache_from(ref, K[rep], V[rep], G, Hq=Hq, B=B, Rcap=Rcap)
    mha.Rk[:] = Rk[rep]; mha.Rv[:] = Rv[rep]; mha.r_len[:] = r_len[rep]
    b, _, _ = ref.decode_attn(mha, q, 0.1)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
    # permuting the batch entries permutes the outputs
    perm = np.array([1, 0])
    pu = (perm[:, None] * Hkv + np.arange(Hkv)).reshape(-1)
    pc = ref_cache_from(ref, K[pu], V[pu], G, Hq=Hq, B=B, Rcap=Rcap)
    pc.Rk[:] = Rk[pu]; pc.Rv[:] = Rv[pu]; pc.r_len[:] = r_len[pu]
    d, _, _ = ref.decode_attn(pc, q[perm], 0.1)
    assert np.array_equal(d.view(np.uint16), a[perm].view(np.uint16))


def test_decode_loop_state_machine(ref):
    """Algorithm 1 lines 9-15 over 2*n_r + 3 steps: append, flush exactly when the residual is full,
    and the flushed tokens are quantized as their own groups appended after the prefill tokens."""
    B, H, D, G, Rcap, T0 = 1, 2, 128, 16, 32, 64
    K = _rand16((H, T0, D), 1); V = _rand16((H, T0, D), 2)
    c = ref_cache_from(ref, K, V, G, B=B, Rcap=Rcap, Tcap=256)
    steps = 2 * Rcap + 3
    newk = _rand16((steps, H, D), 3); newv = _rand16((steps, H, D), 4)
    for i in range(steps):
        assert ref.append_residual(c, newk[i], newv[i]) == 0
        assert ref.flush_residual(c) == 0
        assert np.all(c.r_len == (i + 1) % Rcap) and np.all(c.q_len == T0 + (i + 1) // Rcap * Rcap)
    # same cache as quantizing prefill, then each full residual block, in three separate calls
    d = ref_cache_from(ref, K, V, G, B=B, Rcap=Rcap, Tcap=256)
    for blk in range(2):
        kb = np.ascontiguousarray(newk[blk * Rcap:(blk + 1) * Rcap].transpose(1, 0, 2))
        vb = np.ascontiguousarray(newv[blk * Rcap:(blk + 1) * Rcap].transpose(1, 0, 2))
        assert ref.quantize_pack(d, kb, vb, np.full((H,), Rcap, np.int32)) == 0
    for name in ("Kc", "Ks", "Kz", "Vc", "Vs", "Vz", "q_len"):
        assert np.array_equal(getattr(c, name).view(np.uint8), getattr(d, name).view(np.uint8)), name
    assert np.array_equal(c.Rk[:, :3], newk[2 * Rcap:].transpose(1, 0, 2))
    # a full residual refuses further tokens (caller must flush): fill without flushing
    for i in range(Rcap):
        ref.append_residual(c, newk[i], newv[i])
    before = c.Rk.copy()
    assert np.all(c.r_len == Rcap)
    ref.append_residual(c, newk[0], newv[0])
    assert np.all(c.r_len == Rcap) and np.array_equal(before, c.Rk)
    # the new token attends to itself: the residual rows take part in the softmax
    q = _rand16((B, H, D), 6)
    _, _, probs = ref.decode_attn(c, q, 0.1, want_probs=True)
    T = int(c.q_len[0])
    assert np.all(probs[0, :, T:T + Rcap] > 0) and abs(probs[0, 0].sum() - 1) < 1e-12
