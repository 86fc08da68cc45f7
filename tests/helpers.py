"""Small conveniences for the oracle tests (buffer plumbing only)."""
import numpy as np


def ref_cache_from(ref, K, V, G, Hq=None, B=1, Rcap=0, idx=None, n_tok=None, Tcap=None):
    """Quantize K, V (float16 [U, L, D]) through the oracle into a fresh cache; returns the cache."""
    U, L, D = K.shape
    Hkv = U // B
    Hq = Hq or Hkv
    if n_tok is None:
        n_tok = np.full((U,), L if idx is None else idx.shape[1], np.int32)
    if Tcap is None:
        Tcap = (int(np.max(n_tok)) + Rcap + 127) // 128 * 128
        Tcap = max(Tcap, 128)
    s = ref.RefShape(B, Hq, Hkv, D, G, Tcap, Rcap)
    assert s.check() == 0
    c = ref.RefCache(s)
    rc = ref.quantize_pack(c, K, V, n_tok, idx)
    assert rc == 0
    return c


def k_word_index(t, c):
    """Hand-written restatement of the documented K storage order, used only by the packing pins."""
    tile, tau, w = t // 128, t % 128, c // 16
    return tile * 1024 + ((2 * (tau % 2) + w // 4) * 64 + tau // 2) * 4 + w % 4, 16 * (c % 2) + 2 * ((c % 16) // 2)


def v_word_index(t, c, D=128):
    tile, tau = t // 64, t % 64
    return tile * 4 * D + c * 4 + tau // 16, 16 * (tau % 2) + 2 * ((tau % 16) // 2)


def k_meta_pos(G, c):
    """Hand-written restatement of the documented position of channel c in a K scale / zero row."""
    nb, q = G // 8, c // 4
    return ((q % nb) * (32 // nb) + q // nb) * 4 + c % 4


def k_meta_natural(ref, a, G):
    """K scale / zero rows [.., D] re-ordered to natural channel order."""
    perm = np.array([k_meta_pos(G, c) for c in range(a.shape[-1])])
    assert np.array_equal(perm, ref.k_meta_perm(G))
    assert sorted(perm.tolist()) == list(range(a.shape[-1]))
    return a[..., perm]
