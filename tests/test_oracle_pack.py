"""Pins for the bit-packing (Section 3.3: 16 two-bit codes per 32-bit word) and the size arithmetic of
Appendix I.  Expected words are worked out by hand from the documented storage order:
  K word = 16 channels of one token; channel i of the word sits at bit 16*(i%2) + 2*(i//2).
  V word = 16 tokens of one channel; token p of the block sits at bit 16*(p%2) + 2*(p//2).
"""
import numpy as np

from helpers import ref_cache_from, k_word_index, v_word_index


def _golden():
    import os
    out = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "appendix_I_sizes.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = [x.strip() for x in line.split("=")]
                out[k] = float(v)
    return out


def test_hand_derived_k_words(ref):
    G, L, D = 16, 128, 128
    codes = np.zeros((L, D), np.int64)
    codes[1::G] = 3                                    # every K group (per channel) spans 0..3
    codes[0, 0:16] = np.arange(16) % 4                 # word 0 of token 0: codes i mod 4
    codes[0, 16:32] = 3                                # word 1 of token 0: all 3
    codes[0, 32 + 5] = 2                               # word 2 of token 0: only channel 5 -> 2
    codes[3, 64 + 14] = 1                              # token 3, word 4: channel 14 -> 1
    K = codes.astype(np.float16)[None]
    V = np.zeros((1, L, D), np.float16)
    c = ref_cache_from(ref, K, V, G)
    Kc = c.Kc[0]
    # even channels 0,2,..,14 carry 0,2,0,2,.. -> low half 0x8888; odd channels carry 1,3,1,3,.. -> 0xDDDD
    assert Kc[0] == 0xDDDD8888
    assert Kc[1] == 0xFFFFFFFF
    assert Kc[2] == 0x00200000                         # channel 5 is odd, pair 2: bit 16 + 4
    # token 3 = pair-lane 1, second token of the pair; word 4 is the first word of the upper half
    assert Kc[((2 * 1 + 1) * 64 + 1) * 4 + 0] == 0x00004000       # channel 14 even, pair 7: bit 14
    # token 1 (all codes 3) fills its 8 words: chunks 2 and 3 of pair-lane 0
    assert all(Kc[(ch * 64 + 0) * 4 + w] == 0xFFFFFFFF for ch in (2, 3) for w in range(4))
    # every word is accounted for: unpack(pack(codes)) == codes
    kc, _ = ref.unpack_codes(c, 0)
    assert np.array_equal(kc, codes)


def test_hand_derived_v_words(ref):
    G, L, D = 16, 128, 128
    codes = np.zeros((L, D), np.int64)
    codes[:, 1::G] = 3                                 # every V group (per token) spans 0..3
    codes[0:16, 0] = np.arange(16) % 4                 # block 0 of channel 0: token p -> p mod 4
    codes[16 + 5, 2] = 2                               # block 1 of channel 2: only token 5 -> 2
    codes[64 + 47, 127] = 1                            # second tile, block 2, token 15 of block, channel 127
    V = codes.astype(np.float16)[None]
    K = np.zeros((1, L, D), np.float16)
    c = ref_cache_from(ref, K, V, G)
    Vc = c.Vc[0]
    assert Vc[0 * 4 + 0] == 0xDDDD8888
    assert Vc[1 * 4 + 0] == 0xFFFFFFFF and Vc[1 * 4 + 3] == 0xFFFFFFFF     # channel 1 is all 3
    assert Vc[2 * 4 + 1] == 0x00200000
    assert Vc[4 * D + 127 * 4 + 2] == 0x40000000                            # odd token, pair 7: bit 16+14
    _, vc = ref.unpack_codes(c, 0)
    assert np.array_equal(vc, codes)


def test_pack_unpack_random_and_slot_formula(ref):
    G, U, L, D = 32, 3, 384, 128
    rng = np.random.default_rng(11)
    ck = rng.integers(0, 4, (U, L, D)); cv = rng.integers(0, 4, (U, L, D))
    ck[:, 0::G] = 0; ck[:, 1::G] = 3; cv[:, :, 0::G] = 0; cv[:, :, 1::G] = 3
    c = ref_cache_from(ref, ck.astype(np.float16), cv.astype(np.float16), G)
    for u in range(U):
        kc, vc = ref.unpack_codes(c, u)
        assert np.array_equal(kc, ck[u]) and np.array_equal(vc, cv[u])
    # sampled slots against the documented index formula, restated by hand in helpers.py
    for _ in range(500):
        u, t, ch = rng.integers(U), rng.integers(L), rng.integers(D)
        w, bit = k_word_index(t, ch)
        assert (int(c.Kc[u, w]) >> bit) & 3 == ck[u, t, ch]
        w, bit = v_word_index(t, ch)
        assert (int(c.Vc[u, w]) >> bit) & 3 == cv[u, t, ch]
    # each storage position is used exactly once: the number of set bit-pairs equals the non-zero codes
    def nonzero_pairs(a):
        a = a.astype(np.uint64)
        return sum(int(np.count_nonzero((a >> np.uint64(s)) & np.uint64(3))) for s in range(0, 32, 2))
    assert nonzero_pairs(c.Kc) == np.count_nonzero(ck) and nonzero_pairs(c.Vc) == np.count_nonzero(cv)


def test_appendix_I_size_arithmetic(ref):
    """A group of 16 two-bit codes with fp16 scale and zero-point takes 8 bytes; with prompt 4096,
    generation 512 and a 50 % budget a LLaMA2-7B cache is 0.33 GB against 2.4 GB in fp16 (86 % less)."""
    g = _golden()
    assert ref.group_bytes(int(g["group_size"])) == g["bytes_per_group"] == 8
    assert ref.group_bytes(32) == 12 and ref.group_bytes(64) == 20
    layers, hidden, lp, lg = (int(g[k]) for k in ("model_layers", "model_hidden", "prompt_len", "gen_len"))
    full = 2 * (layers * hidden) * (lp + lg) * 2
    scalars_per_token = 2 * layers * hidden                       # K and V
    minikv = scalars_per_token // 16 * ref.group_bytes(16) * int(g["budget_total"] * lp + lg)
    assert round(full / 1e9, 1) == g["full_cache_GB"]
    assert int(minikv / 1e7) / 100 == g["minikv_cache_GB"]        # the paper truncates 0.3355 to 0.33
    assert minikv == layers * hidden * (lp // 2 + lg)             # the paper's closed form
    assert round(100 * (1 - minikv / full)) == g["reduction_percent"]
    # the buffers the oracle allocates hold exactly 64 + 8*D/G bytes per token and head
    for G in (16, 32, 64, 128):
        s = ref.RefShape(1, 1, 1, 128, G, 256, 0); c = ref.RefCache(s)
        per_tok = sum(a.nbytes for a in (c.Kc, c.Ks, c.Kz, c.Vc, c.Vs, c.Vz)) / 256
        assert per_tok == 64 + 8 * 128 // G == 2 * (128 // G) * ref.group_bytes(G)
