"""Pins for the per-token quantized cache of the oracle (oracle/minikv_pt_ref.c): the token-wise
quantization of the paper's appendix (8 / 4 / 2 bits, keys and values alike) and its 4-bit baseline.

What the checks rest on, none of which re-types the oracle's own formula: the half-step round-trip bound
and the end codes that any min/max quantizer must show; lattices whose codes are known in closed form;
words packed by hand; the compression factor the appendix on KV cache sizes prints; the 2-bit per-token
codes against the VALUE path of the first oracle file (another piece of code with the same grouping); an
fp64 attention computed in numpy from a re-quantization that never touches packed words; and the ordering
of errors on keys with outlier channels that motivates per-channel key quantization (Section 3.1.1).
"""
import os

import numpy as np
import pytest

from helpers import ref_cache_from

ROOT = os.path.dirname(os.path.abspath(__file__))


def _rand(U, L, D, seed, scale=1.0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((U, L, D)) * scale).astype(np.float16)


def _pt_cache(ref, K, V, G, bits, Hq=None, B=1, idx=None, n_tok=None):
    U, L, D = K.shape
    Hkv = U // B
    n = L if idx is None else idx.shape[1]
    if n_tok is None:
        n_tok = np.full((U,), n, np.int32)
    Tcap = max(64, (int(np.max(n_tok)) + 63) // 64 * 64)
    s = ref.RefPtShape(B, Hq or Hkv, Hkv, D, G, bits, Tcap)
    assert s.check() == 0
    c = ref.RefPtCache(s)
    assert ref.quantize_pack_pt(c, K, V, n_tok, idx) == 0
    return c


def _np_quantize(x, G, bits):
    """Per-token min/max quantization in numpy float64/float32, written independently: returns codes,
    scale, zero with x [..., D]."""
    lev = (1 << bits) - 1
    g = x.reshape(*x.shape[:-1], x.shape[-1] // G, G).astype(np.float32)
    mn, mx = g.min(-1, keepdims=True), g.max(-1, keepdims=True)
    zero = mn.astype(np.float16)
    zero = np.where(zero == 0, np.float16(0), zero)                 # -0 -> +0
    scale = ((mx - mn) / np.float32(lev)).astype(np.float16)
    sf = scale.astype(np.float32)
    with np.errstate(divide="ignore"):
        inv = np.where(sf == 0, np.float32(0), np.float32(1) / sf).astype(np.float32)
    u = ((g - zero.astype(np.float32)).astype(np.float32) * inv).astype(np.float32)
    codes = np.clip(np.rint(u), 0, lev).astype(np.int64)
    return codes.reshape(x.shape), scale[..., 0], zero[..., 0]


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("G", [32, 64, 128])
def test_round_trip_half_step_and_end_codes(ref, G, bits):
    U, L, D = 2, 64, 128
    K, V = _rand(U, L, D, 100 + G + bits), _rand(U, L, D, 200 + G + bits, 3.0)
    K[:, :, 7] *= 12
    c = _pt_cache(ref, K, V, G, bits)
    lev = (1 << bits) - 1
    for u in range(U):
        kc, vc = ref.unpack_codes_pt(c, u)
        for x, codes, sc, zp in ((K[u], kc, c.Ks[u, :L], c.Kz[u, :L]), (V[u], vc, c.Vs[u, :L], c.Vz[u, :L])):
            assert codes.max() <= lev
            s = np.repeat(sc.astype(np.float64), G, axis=1)
            z = np.repeat(zp.astype(np.float64), G, axis=1)
            xhat = codes * s + z
            assert np.all(np.abs(x.astype(np.float64) - xhat) <= s * 0.5 * (1 + 2.0 ** -18) + s * lev * 2.0 ** -11)
            grp = codes.reshape(L, D // G, G)
            assert np.all(grp.min(axis=2) == 0) and np.all(grp.max(axis=2) == lev)
            assert np.array_equal(zp, x.reshape(L, D // G, G).min(axis=2))       # zero-point = group minimum
    # (the last term of the bound: with 2^bits - 1 steps the fp16 rounding of the scale can move the top level
    #  by up to levels * 2^-11 * scale away from the maximum, which the clamp then absorbs)


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_lattice_is_lossless_with_known_codes(ref, bits):
    U, L, D, G = 1, 32, 128, 32
    lev = (1 << bits) - 1
    rng = np.random.default_rng(7 + bits)
    lv = rng.integers(0, lev + 1, (U, L, D))
    lv[:, :, 0::G] = 0; lv[:, :, 1::G] = lev                   # every group spans all levels
    s = 2.0 ** rng.integers(-5, 2, (U, L, D // G, 1)); z = s * rng.integers(-9, 9, (U, L, D // G, 1))
    X = (lv.reshape(U, L, D // G, G) * s + z).reshape(U, L, D).astype(np.float16)
    # range / levels is exact here only when levels divides the range exactly in binary: s * lev / lev = s
    c = _pt_cache(ref, X, X, G, bits)
    kc, vc = ref.unpack_codes_pt(c, 0)
    assert np.array_equal(kc, lv[0]) and np.array_equal(vc, lv[0])
    assert np.array_equal(c.Ks[0, :L].astype(np.float64), s[0, :, :, 0])
    assert np.array_equal(c.Kz[0, :L].astype(np.float64), z[0, :, :, 0])


def test_words_packed_by_hand(ref):
    """Code i of a word sits at bits [bits*i, bits*i + bits): K words run along the channels of a token, V
    words along the tokens of a channel."""
    U, L, D, G = 1, 16, 128, 128
    # 4 bits: channel c of every token at level c % 16 -> every K word is 0x76543210 or 0xFEDCBA98
    X = np.tile((np.arange(D) % 16).astype(np.float16), (U, L, 1))
    c = _pt_cache(ref, X, X, G, 4)
    kw = c.Kc[0, : L * D * 4 // 32].reshape(L, D // 8)
    assert np.all(kw[:, 0::2] == 0x76543210) and np.all(kw[:, 1::2] == 0xFEDCBA98)
    # V words hold 8 consecutive tokens of one channel, all at that channel's level: nibble repeated 8 times
    vw = c.Vc[0, : L * D * 4 // 32].reshape(L // 8, D)
    assert np.array_equal(vw[0], (np.arange(D) % 16).astype(np.uint32) * 0x11111111)
    # 2 bits: token t at level t % 4 in every channel (one group per token spans 0..3 only across tokens, so
    # put the spread inside each token as well: channels 0 and 1 are pinned to 0 and 3)
    Y = np.zeros((U, L, D), np.float16)
    Y[:, :, :] = (np.arange(L) % 4)[None, :, None]
    Y[:, :, 0] = 0; Y[:, :, 1] = 3
    c = _pt_cache(ref, Y, Y, G, 2)
    vw = c.Vc[0, : L * D * 2 // 32].reshape(L // 16, D)
    assert vw[0, 5] == 0xE4E4E4E4                            # tokens 0..15 at levels 0,1,2,3,0,1,2,3,...
    assert vw[0, 1] == 0xFFFFFFFF and vw[0, 0] == 0
    kw = c.Kc[0, : L * D * 2 // 32].reshape(L, D // 16)
    assert kw[2, 3] == 0xAAAAAAAA and kw[2, 0] == (0xAAAAAAAA & ~0xF) | (3 << 2)   # token 2: level 2 everywhere but c0, c1
    # 8 bits: one byte per code
    Z = np.tile((np.arange(D) * 2 % 256).astype(np.float16), (U, L, 1))
    Z[:, :, 0] = 0; Z[:, :, 1] = 255
    c = _pt_cache(ref, Z, Z, G, 8)
    kc, _ = ref.unpack_codes_pt(c, 0)
    assert np.array_equal(kc[0], Z[0, 0].astype(np.int64))
    assert c.Kc[0, 1] == (8 | (10 << 8) | (12 << 16) | (14 << 24))      # channels 4..7 of token 0


def test_compression_factor_printed_in_the_appendix(ref):
    vals = {}
    for line in open(os.path.join(ROOT, "golden", "appendix_I_sizes.txt")):
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = [x.strip() for x in line.split("=")]
            vals[k] = float(v)
    d, bits = int(vals["qhitter_head_dim"]), int(vals["qhitter_bits"])
    per_token = ref.pt_token_bytes(d, d, bits)               # one group per head, as in the appendix
    assert per_token == d * bits // 8 + 4
    assert round(d * 2 / per_token, 2) == vals["qhitter_compression"]
    # and MiniKV's own 8 bytes per 16 scalars is the G = 16, 2-bit case of the same arithmetic
    assert ref.pt_token_bytes(128, 32, 2) == 128 * 2 // 8 + 4 * 4


@pytest.mark.parametrize("G", [32, 64, 128])
def test_two_bit_per_token_codes_equal_the_value_path_of_the_first_oracle_file(ref, G):
    """minikv_ref.c quantizes VALUES per token over channel groups of G: the same grouping, other code."""
    U, L, D = 2, 128, 128
    X = _rand(U, L, D, 31 + G, 2.0)
    main = ref_cache_from(ref, X, X, G)
    pt = _pt_cache(ref, X, X, G, 2)
    for u in range(U):
        _, vmain = ref.unpack_codes(main, u)
        kpt, vpt = ref.unpack_codes_pt(pt, u)
        assert np.array_equal(vmain, kpt) and np.array_equal(vmain, vpt)
        assert np.array_equal(main.Vs[u, :L], pt.Ks[u, :L]) and np.array_equal(main.Vz[u, :L], pt.Vz[u, :L])


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_codes_equal_a_numpy_requantization_with_gather(ref, bits):
    U, L, D, G = 2, 96, 128, 64
    K, V = _rand(U, L, D, 51 + bits), _rand(U, L, D, 52 + bits)
    rng = np.random.default_rng(3)
    idx = np.stack([np.sort(rng.choice(L, 48, replace=False)) for _ in range(U)]).astype(np.int32)
    c = _pt_cache(ref, K, V, G, bits, idx=idx)
    for u in range(U):
        kc, vc = ref.unpack_codes_pt(c, u)
        wk, sk, zk = _np_quantize(K[u][idx[u]], G, bits)
        wv, sv, zv = _np_quantize(V[u][idx[u]], G, bits)
        assert np.array_equal(kc, wk) and np.array_equal(vc, wv)
        assert np.array_equal(c.Ks[u, :48], sk) and np.array_equal(c.Vz[u, :48], zv)


def _np_attention(q, Khat, Vhat, sm):
    from scipy.special import softmax
    p = softmax(sm * (Khat @ q), axis=0)
    return p @ Vhat, p


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_attention_equals_fp64_brute_force_and_rows_sum_to_one(ref, bits):
    B, Hq, Hkv, L, D, G = 2, 4, 2, 80, 128, 32
    K, V = _rand(B * Hkv, L, D, 61), _rand(B * Hkv, L, D, 62)
    q = _rand(B, Hq, D, 63)
    n_tok = np.array([80, 48, 0, 16], np.int32)
    c = _pt_cache(ref, K, V, G, bits, Hq=Hq, B=B, n_tok=n_tok)
    out16, out64 = ref.decode_attn_pt(c, q, 0.11)
    for b in range(B):
        for h in range(Hq):
            u = b * Hkv + h // (Hq // Hkv)
            n = n_tok[u]
            if n == 0:
                assert not out64[b, h].any()
                continue
            wk, sk, zk = _np_quantize(K[u, :n], G, bits)
            wv, sv, zv = _np_quantize(V[u, :n], G, bits)
            Kh = wk * np.repeat(sk.astype(np.float64), G, 1) + np.repeat(zk.astype(np.float64), G, 1)
            Vh = wv * np.repeat(sv.astype(np.float64), G, 1) + np.repeat(zv.astype(np.float64), G, 1)
            want, p = _np_attention(q[b, h].astype(np.float64), Kh, Vh, float(np.float32(0.11)))
            assert abs(p.sum() - 1) <= 1e-12
            assert np.max(np.abs(out64[b, h] - want)) <= 1e-9
            assert np.array_equal(out16[b, h], want.astype(np.float16)) or np.max(np.abs(out16[b, h].astype(np.float64) - want)) <= 2.0 ** -11 * np.abs(want).max()


def test_eight_bits_is_close_to_unquantized_attention_and_equal_keys_give_the_mean(ref):
    B, Hq, Hkv, L, D, G = 1, 2, 2, 64, 128, 128
    K, V = _rand(Hkv, L, D, 71), _rand(Hkv, L, D, 72)
    q = _rand(B, Hq, D, 73)
    c = _pt_cache(ref, K, V, G, 8, Hq=Hq, B=B)
    _, out64 = ref.decode_attn_pt(c, q, 0.09)
    for h in range(Hq):
        want, _ = _np_attention(q[0, h].astype(np.float64), K[h].astype(np.float64), V[h].astype(np.float64), float(np.float32(0.09)))
        assert np.max(np.abs(out64[0, h] - want)) <= 0.02          # 255 levels over a range of ~7: step 0.03
    K2 = np.repeat(K[:, :1], L, axis=1)                            # all keys equal -> uniform weights
    c = _pt_cache(ref, K2, V, G, 8, Hq=Hq, B=B)
    _, out64 = ref.decode_attn_pt(c, q, 0.09)
    kc, vc = ref.unpack_codes_pt(c, 0)
    vh = vc * np.repeat(c.Vs[0, :L].astype(np.float64), G, 1) + np.repeat(c.Vz[0, :L].astype(np.float64), G, 1)
    assert np.max(np.abs(out64[0, 0] - vh.mean(axis=0))) <= 1e-12


def test_outlier_channels_break_two_bit_per_token_keys_but_not_per_channel_keys(ref):
    """The reason for MiniKV's per-channel key quantization (Section 3.1.1) and the failure the appendix on
    token-wise quantization reports: with a few large-magnitude key CHANNELS, 2-bit per-token codes lose the
    ordinary channels (the group range is set by the outliers), 4 and 8 bits per token keep them, and 2 bits
    per channel keep them as well.  Measured on the attention output against unquantized fp64 attention."""
    B, Hq, Hkv, L, D = 1, 4, 4, 256, 128
    rng = np.random.default_rng(81)
    K = rng.standard_normal((Hkv, L, D))
    K[:, :, [3, 40, 77, 101]] *= 12.0                              # outlier channels, every token
    K = K.astype(np.float16)
    V = _rand(Hkv, L, D, 82)
    q = _rand(B, Hq, D, 83)
    q[:, :, [3, 40, 77, 101]] *= np.float16(0.2)                   # their score share stays moderate
    sm = 0.088
    exact = np.stack([_np_attention(q[0, h].astype(np.float64), K[h].astype(np.float64), V[h].astype(np.float64), float(np.float32(sm)))[0]
                      for h in range(Hq)])
    err = {}
    for bits in (2, 4, 8):
        c = _pt_cache(ref, K, V, 128, bits, Hq=Hq, B=B)
        err["pt%d" % bits] = float(np.abs(ref.decode_attn_pt(c, q, sm)[1][0] - exact).max())
    main = ref_cache_from(ref, K, V, 32, Hq=Hq, B=B)
    err["per_channel2"] = float(np.abs(ref.decode_attn(main, q, sm, want_f64=True)[1][0] - exact).max())
    assert err["pt8"] < err["pt4"] < err["pt2"]
    assert err["per_channel2"] < 0.5 * err["pt2"]
    assert err["pt2"] > 4 * err["pt4"]


def test_rule_violations_touch_nothing(ref):
    K = _rand(1, 64, 128, 1)
    s = ref.RefPtShape(1, 1, 1, 128, 32, 4, 64)
    c = ref.RefPtCache(s)
    assert ref.quantize_pack_pt(c, K, K, np.array([24], np.int32)) == -1          # not a multiple of 16
    assert ref.quantize_pack_pt(c, K, K, np.array([128], np.int32)) == -1         # beyond the capacity
    assert not c.Kc.any() and c.q_len[0] == 0
    for bad in (dict(G=16), dict(bits=3), dict(Tcap=100), dict(D=64)):
        kw = dict(B=1, Hq=1, Hkv=1, D=128, G=32, bits=4, Tcap=64); kw.update(bad)
        assert ref.RefPtShape(**kw).check() == -1
