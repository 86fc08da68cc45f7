"""Pins of the oracle's prefill attention with cumulative attention scores (Section 3.2, Algorithm 1 line 2,
eq. (1) on the causal part): a numpy matmul + softmax written independently, closed forms for equal keys,
invariants of a row-stochastic lower-triangular matrix, and the grouped-query head mapping."""
import math

import numpy as np
import pytest

from oracle import ref


def draw(B, Hq, Hkv, L, D, seed, scale=1.0):
    g = np.random.default_rng(seed)
    Q = (g.standard_normal((B, Hq, L, D)) * scale).astype(np.float16)
    K = (g.standard_normal((B, Hkv, L, D)) * scale).astype(np.float16)
    V = g.standard_normal((B, Hkv, L, D)).astype(np.float16)
    return Q, K, V


def numpy_attention(Q, K, V, sm_scale):
    """The textbook form with the whole matrix in memory (what the kernel exists to avoid)."""
    B, Hq, L, D = Q.shape
    rep = Hq // K.shape[1]
    Kr = np.repeat(K.astype(np.float64), rep, axis=1)
    Vr = np.repeat(V.astype(np.float64), rep, axis=1)
    S = np.einsum("bhid,bhjd->bhij", Q.astype(np.float64), Kr) * np.float64(np.float32(sm_scale))
    S = np.where(np.tril(np.ones((L, L), bool)), S, -np.inf)
    m = S.max(-1, keepdims=True)
    E = np.exp(S - m)
    P = E / E.sum(-1, keepdims=True)
    return P @ Vr, (m + np.log(E.sum(-1, keepdims=True)))[..., 0], P.sum(-2), P


@pytest.mark.parametrize("B,Hq,Hkv,L,D,scale", [(2, 4, 4, 97, 128, 1.0), (1, 8, 2, 64, 128, 1.0), (1, 2, 1, 33, 16, 3.0),
                                                 (1, 1, 1, 1, 128, 1.0)])
def test_matches_a_library_matmul_and_softmax(B, Hq, Hkv, L, D, scale):
    Q, K, V = draw(B, Hq, Hkv, L, D, seed=L + Hq, scale=scale)
    sm = 1.0 / math.sqrt(D)
    xo16, xo64, lse, acc = ref.selective_flash_attn(Q, K, V, sm)
    O, LSE, A, _ = numpy_attention(Q, K, V, sm)
    assert np.max(np.abs(xo64 - O)) <= 1e-12
    assert np.max(np.abs(lse - LSE)) <= 1e-12
    assert np.max(np.abs(acc - A)) <= 1e-12
    assert np.array_equal(xo16, O.astype(np.float16)) or np.max(np.abs(xo16.astype(np.float64) - O)) <= 1e-3


def test_invariants_of_a_causal_row_stochastic_matrix():
    Q, K, V = draw(1, 3, 3, 200, 128, seed=4, scale=1.5)
    _, xo64, lse, acc = ref.selective_flash_attn(Q, K, V, 0.1)
    L = 200
    assert np.allclose(acc.sum(-1), L, rtol=0, atol=1e-9)               # every row sums to one
    assert (acc > 0).all() and (acc[..., 0] >= 1.0).all()                # token 0 holds all of row 0
    assert np.allclose(xo64[:, :, 0], V[:, :, 0].astype(np.float64))     # the first token sees only itself
    # the last column has one entry: the last row's weight on its own key
    qk = (Q[0, :, -1].astype(np.float64) * K[0, :, -1].astype(np.float64)).sum(-1) * np.float64(np.float32(0.1))
    assert np.allclose(acc[0, :, -1], np.exp(qk - lse[0, :, -1]), rtol=1e-12)


def test_equal_keys_give_harmonic_column_sums():
    """All keys equal: every visible key gets 1/(i+1), so A_cumul[j] = H_L - H_j, lse_i = s_i + log(i+1) and
    X_O[i] is the running mean of V."""
    L, D = 150, 128
    g = np.random.default_rng(2)
    Q = g.standard_normal((1, 2, L, D)).astype(np.float16)
    K = np.broadcast_to(g.standard_normal((1, 2, 1, D)).astype(np.float16), (1, 2, L, D)).copy()
    V = g.standard_normal((1, 2, L, D)).astype(np.float16)
    _, xo64, lse, acc = ref.selective_flash_attn(Q, K, V, 0.25)
    H = np.concatenate([[0.0], np.cumsum(1.0 / np.arange(1, L + 1))])
    assert np.allclose(acc, (H[L] - H[:L])[None, None], rtol=0, atol=1e-10)
    s = (Q.astype(np.float64) * K.astype(np.float64)).sum(-1) * 0.25
    assert np.allclose(lse, s + np.log(np.arange(1, L + 1)), rtol=0, atol=1e-10)
    means = np.cumsum(V.astype(np.float64), axis=2) / np.arange(1, L + 1)[None, None, :, None]
    assert np.allclose(xo64, means, rtol=0, atol=1e-10)


def test_one_dominant_key_takes_the_column_mass():
    """A key far more aligned with every query than the rest: from its position on, it takes (almost) all of
    each row, so its column sum is about the number of rows that see it."""
    L, D, j0 = 64, 128, 10
    Q = np.zeros((1, 1, L, D), np.float16); Q[..., 0] = 8.0
    K = np.zeros((1, 1, L, D), np.float16); K[0, 0, j0, 0] = 8.0
    V = np.random.default_rng(3).standard_normal((1, 1, L, D)).astype(np.float16)
    _, xo64, _, acc = ref.selective_flash_attn(Q, K, V, 1.0)
    assert abs(acc[0, 0, j0] - (L - j0)) < 1e-20 * L + 1e-9
    assert np.allclose(xo64[0, 0, j0:], V[0, 0, j0].astype(np.float64), atol=1e-9)


def test_grouped_query_heads_read_their_kv_head():
    Q, K, V = draw(2, 8, 2, 40, 128, seed=9)
    a = ref.selective_flash_attn(Q, K, V, 0.09)
    b = ref.selective_flash_attn(Q, np.repeat(K, 4, axis=1), np.repeat(V, 4, axis=1), 0.09)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_a_transposed_operand_or_a_missing_mask_would_show():
    """Planted mistakes in the independent numpy form (not in the oracle) must move it away from the oracle."""
    Q, K, V = draw(1, 1, 1, 48, 128, seed=12)
    sm = 1.0 / math.sqrt(128)
    _, xo64, lse, acc = ref.selective_flash_attn(Q, K, V, sm)
    O, LSE, A, P = numpy_attention(Q, K, V, sm)
    assert np.max(np.abs(acc - P.sum(-1))) > 1e-3            # row sums instead of column sums
    S = np.einsum("bhid,bhjd->bhij", Q.astype(np.float64), K.astype(np.float64)) * sm
    full = np.exp(S - S.max(-1, keepdims=True)); full /= full.sum(-1, keepdims=True)
    assert np.max(np.abs(acc - full.sum(-2))) > 1e-3         # no causal mask


def test_rows_view_equals_the_full_oracle_and_numpy(ref):
    """selective_flash_attn_rows (the per-row form used at full size) against the full oracle and against a
    numpy softmax: outputs, lse, and the cumulative score of late columns rebuilt from the rows' tail weights."""
    from scipy.special import softmax, logsumexp
    rng = np.random.default_rng(17)
    L, D, tail = 150, 128, 40
    Q = rng.standard_normal((L, D)).astype(np.float16)
    K = rng.standard_normal((L, D)).astype(np.float16)
    V = rng.standard_normal((L, D)).astype(np.float16)
    sm = 0.11
    _, xo64, lse64, acc64 = ref.selective_flash_attn(Q[None, None], K[None, None], V[None, None], sm)
    rows = np.array([0, 1, 63, 64, 127, 128, 149], np.int64)
    xo, lse, _ = ref.selective_flash_attn_rows(Q, K, V, sm, rows)
    assert np.max(np.abs(xo - xo64[0, 0, rows])) <= 1e-12 and np.max(np.abs(lse - lse64[0, 0, rows])) <= 1e-12
    for r, i in enumerate(rows):
        s = float(np.float32(sm)) * (K[: i + 1].astype(np.float64) @ Q[i].astype(np.float64))
        assert abs(lse[r] - logsumexp(s)) <= 1e-12
        assert np.max(np.abs(xo[r] - softmax(s) @ V[: i + 1].astype(np.float64))) <= 1e-12
    # the last `tail` columns only receive weight from the last `tail` rows
    late = np.arange(L - tail, L, dtype=np.int64)
    _, _, pt = ref.selective_flash_attn_rows(Q, K, V, sm, late, tail=tail)
    assert np.max(np.abs(pt.sum(axis=0) - acc64[0, 0, L - tail:])) <= 1e-12
    assert np.all(np.triu(pt, 1) == 0)                     # a row gives nothing to the keys after it
