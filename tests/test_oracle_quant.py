"""Pins for the oracle's quantizer (Section 3.1.1 / 3.3: asymmetric 2-bit, fp16 scale and zero-point).

None of these re-types the oracle's formula: they check what the mathematics fixes -- the half-step
round-trip bound, the end codes of every non-degenerate group, lossless lattices with codes known in
closed form, an fp64 arg-min over the four levels with ties listed explicitly, and hand-worked ties.
"""
import numpy as np
import pytest

from helpers import ref_cache_from, k_meta_natural


def _rand(U, L, D, seed, scale=1.0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((U, L, D)) * scale).astype(np.float16)


@pytest.mark.parametrize("G", [16, 32, 64, 128])
def test_round_trip_half_step_and_end_codes(ref, G):
    U, L, D = 2, 256, 128
    K = _rand(U, L, D, 10 + G)
    V = _rand(U, L, D, 20 + G)
    K[:, :, 5] *= 10                                   # an outlier channel
    c = ref_cache_from(ref, K, V, G)
    for u in range(U):
        kc, vc = ref.unpack_codes(c, u)
        kh, vh = ref.dequant(c, u)
        ks = np.repeat(k_meta_natural(ref, c.Ks[u, : L // G], G).astype(np.float64), G, axis=0)          # [L, D]
        vs = np.repeat(c.Vs[u, :L].astype(np.float64), G, axis=1)                # [L, D]
        # |x - x_hat| <= (stored step)/2, up to the three binary32 roundings inside the code decision
        assert np.all(np.abs(K[u].astype(np.float64) - kh) <= ks * 0.5 * (1 + 2.0 ** -18))
        assert np.all(np.abs(V[u].astype(np.float64) - vh) <= vs * 0.5 * (1 + 2.0 ** -18))
        assert kc.max() <= 3 and vc.max() <= 3
        # every group with a non-zero step holds a 0 (its minimum, reproduced exactly) and a 3 (its maximum)
        kg = kc.reshape(L // G, G, D)
        assert np.all(kg.min(axis=1) == 0) and np.all(kg.max(axis=1) == 3)
        vg = vc.reshape(L, D // G, G)
        assert np.all(vg.min(axis=2) == 0) and np.all(vg.max(axis=2) == 3)
        # zero-point is the group minimum itself
        assert np.array_equal(k_meta_natural(ref, c.Kz[u, : L // G], G), K[u].reshape(L // G, G, D).min(axis=1))
        assert np.array_equal(c.Vz[u, :L], V[u].reshape(L, D // G, G).min(axis=2))
        xmin = K[u].reshape(L // G, G, D).astype(np.float64)
        at_min = xmin == xmin.min(axis=1, keepdims=True)
        assert np.all(kh.reshape(L // G, G, D)[at_min] == xmin[at_min])


@pytest.mark.parametrize("G", [16, 32])
def test_lattice_is_lossless_with_known_codes(ref, G):
    """Data on {z, z+s, z+2s, z+3s} with s a power of two: range/3 == s exactly, codes are the levels."""
    U, L, D = 1, 128, 128
    rng = np.random.default_rng(5)
    lev_k = rng.integers(0, 4, (U, L, D))
    lev_v = rng.integers(0, 4, (U, L, D))
    lev_k[:, 0::G, :] = 0; lev_k[:, 1::G, :] = 3           # each K group (G tokens of a channel) spans 0..3
    lev_v[:, :, 0::G] = 0; lev_v[:, :, 1::G] = 3           # each V group (G channels of a token) spans 0..3
    s_k = 2.0 ** rng.integers(-6, 3, (U, L // G, 1, D)); z_k = s_k * rng.integers(-20, 20, (U, L // G, 1, D))
    s_v = 2.0 ** rng.integers(-6, 3, (U, L, D // G, 1)); z_v = s_v * rng.integers(-20, 20, (U, L, D // G, 1))
    K = (lev_k.reshape(U, L // G, G, D) * s_k + z_k).reshape(U, L, D)
    V = (lev_v.reshape(U, L, D // G, G) * s_v + z_v).reshape(U, L, D)
    K16, V16 = K.astype(np.float16), V.astype(np.float16)
    assert np.array_equal(K16.astype(np.float64), K) and np.array_equal(V16.astype(np.float64), V)
    c = ref_cache_from(ref, K16, V16, G)
    kc, vc = ref.unpack_codes(c, 0)
    kh, vh = ref.dequant(c, 0)
    assert np.array_equal(kc, lev_k[0]) and np.array_equal(vc, lev_v[0])
    assert np.array_equal(kh, K[0]) and np.array_equal(vh, V[0])
    assert np.array_equal(k_meta_natural(ref, c.Ks[0, : L // G], G).astype(np.float64), s_k[0, :, 0, :])
    assert np.array_equal(c.Vz[0, :L].astype(np.float64), z_v[0, :, :, 0])


def test_codes_are_the_nearest_level_in_fp64(ref):
    """Brute force: code == argmin_k |x - (z + k s)| in fp64 with the STORED s, z; exact ties listed."""
    G, U, L, D = 32, 2, 128, 128
    K = _rand(U, L, D, 77, 1.5)
    V = _rand(U, L, D, 78, 0.7)
    c = ref_cache_from(ref, K, V, G)
    n_ties = 0
    for u in range(U):
        kc, vc = ref.unpack_codes(c, u)
        for x, codes, s, z in (
            (K[u], kc, np.repeat(k_meta_natural(ref, c.Ks[u, : L // G], G), G, axis=0),
             np.repeat(k_meta_natural(ref, c.Kz[u, : L // G], G), G, axis=0)),
            (V[u], vc, np.repeat(c.Vs[u, :L], G, axis=1), np.repeat(c.Vz[u, :L], G, axis=1)),
        ):
            x, s, z = x.astype(np.float64), s.astype(np.float64), z.astype(np.float64)
            dist = np.abs(x[..., None] - (z[..., None] + np.arange(4) * s[..., None]))     # [L, D, 4]
            best = dist.min(axis=-1)
            mine = np.take_along_axis(dist, codes[..., None].astype(np.int64), axis=-1)[..., 0]
            # the chosen level is a nearest level (allowing the 2^-20 slack of the binary32 decision)
            assert np.all(mine <= best + s * 2.0 ** -20)
            n_ties += int(np.sum(np.sum(dist <= best[..., None] + s[..., None] * 2.0 ** -20, axis=-1) > 1))
    assert n_ties < 50          # ties are rare on continuous data; they are pinned by hand below


def test_hand_worked_ties_round_half_to_even(ref):
    """z = 0, s = 1 (group holds 0 and 3): 0.5 -> 0, 1.5 -> 2, 2.5 -> 2; also 0.25 -> 0, 2.75 -> 3."""
    G, D = 16, 128
    vals = [0.0, 3.0, 0.5, 1.5, 2.5, 0.25, 2.75, 1.0, 2.0, 0.75, 1.25, 0.0, 0.0, 0.0, 0.0, 0.0]
    want = [0, 3, 0, 2, 2, 0, 3, 1, 2, 1, 1, 0, 0, 0, 0, 0]
    K = np.zeros((1, 128, D), np.float16)
    V = np.zeros((1, 128, D), np.float16)
    K[0, :16, :] = np.array(vals, np.float16)[:, None]          # K groups run along tokens
    V[0, :, :16] = np.array(vals, np.float16)[None, :]          # V groups run along channels
    c = ref_cache_from(ref, K, V, G)
    kc, vc = ref.unpack_codes(c, 0)
    assert kc[:16, 3].tolist() == want
    assert vc[7, :16].tolist() == want
    assert float(k_meta_natural(ref, c.Ks[0, 0], G)[3]) == 1.0 and float(k_meta_natural(ref, c.Kz[0, 0], G)[3]) == 0.0


def test_degenerate_group_and_negative_zero(ref):
    """max == min: scale 0, codes 0, x_hat == x; a zero-point of -0.0 is stored as +0.0."""
    G, D = 16, 128
    K = np.full((1, 128, D), 2.5, np.float16)
    V = np.full((1, 128, D), -0.0, np.float16)
    c = ref_cache_from(ref, K, V, G)
    kc, vc = ref.unpack_codes(c, 0)
    kh, vh = ref.dequant(c, 0)
    assert not kc.any() and not vc.any()
    assert np.all(c.Ks[0] == 0) and np.all(kh == 2.5) and np.all(vh == 0)
    assert not c.Vz.view(np.uint16).any()
    assert not c.Vc.any() and not c.Kc.any()


def test_gather_takes_rows_in_ascending_order(ref):
    """Retained rows idx[u, :] of the source are what gets quantized (Algorithm 1 line 3 -> 4)."""
    G, U, L, D = 16, 2, 256, 128
    K = _rand(U, L, D, 1); V = _rand(U, L, D, 2)
    rng = np.random.default_rng(0)
    idx = np.stack([np.sort(rng.permutation(L)[:64]) for _ in range(U)]).astype(np.int32)
    a = ref_cache_from(ref, K, V, G, idx=idx)
    Kg = np.stack([K[u, idx[u]] for u in range(U)]); Vg = np.stack([V[u, idx[u]] for u in range(U)])
    b = ref_cache_from(ref, Kg, Vg, G)
    for name in ("Kc", "Ks", "Kz", "Vc", "Vs", "Vz", "q_len"):
        assert np.array_equal(getattr(a, name).view(np.uint8), getattr(b, name).view(np.uint8)), name
    bad = idx.copy(); bad[0, 3], bad[0, 4] = bad[0, 4], bad[0, 3]       # not ascending -> refused
    s = ref.RefShape(1, U, U, D, G, 128, 0); c = ref.RefCache(s)
    assert ref.quantize_pack(c, K, V, np.full((U,), 64, np.int32), bad) != 0
    assert ref.quantize_pack(c, K, V, np.full((U,), 40, np.int32), idx) != 0    # not a multiple of G


@pytest.mark.parametrize("G", [16, 32])
def test_keys_with_outlier_channels_quantize_better_per_channel_than_per_token(ref, G):
    """Section 3.1.1 / the appendix on per-token key quantization: keys have a few large-magnitude CHANNELS, so
    grouping a channel over tokens (the K path) keeps the outliers in groups of their own, while grouping a
    token over channels (the V path, fed here with the same keys) lets one outlier set the step of its whole
    group.  The same data through both paths of the oracle: the per-channel error is several times smaller."""
    U, L, D = 2, 512, 128
    K = _rand(U, L, D, 77 + G)
    outliers = [3, 40, 41, 100]
    K[:, :, outliers] *= 12
    c = ref_cache_from(ref, K, K.copy(), G)               # V := K, so Vhat is K quantized per token
    for u in range(U):
        per_channel, per_token = ref.dequant(c, u)
        x = K[u].astype(np.float64)
        # the ordinary channels that share a channel group with an outlier pay for it under per-token grouping
        groups = sorted({o // G for o in outliers})
        victims = np.setdiff1d(np.concatenate([np.arange(gr * G, (gr + 1) * G) for gr in groups]), outliers)
        e_ch = np.sqrt(np.mean((per_channel[:, victims] - x[:, victims]) ** 2))
        e_tok = np.sqrt(np.mean((per_token[:, victims] - x[:, victims]) ** 2))
        assert e_tok > 3 * e_ch, (e_ch, e_tok)
        # channel groups without an outlier are unaffected: there the two groupings err alike
        clean = np.arange(64, 96) if G == 32 else np.arange(64, 80)
        r = np.sqrt(np.mean((per_token[:, clean] - x[:, clean]) ** 2)) / np.sqrt(np.mean((per_channel[:, clean] - x[:, clean]) ** 2))
        assert 0.5 < r < 2.0
