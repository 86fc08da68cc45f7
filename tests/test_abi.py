"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and its host-side
argument validation returns the documented status codes before anything is launched."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def api():
    from paper_2411_18077_amd import api as _api
    if not os.path.exists(_api.LIB_PATH):
        from paper_2411_18077_amd import build
        build.build(verbose=False)
    return _api


def test_exports_every_declared_symbol(api):
    text = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("minikv.h", "minikv_diag.h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(minikv_\w+|kv_\w+|selective_flash_attn\w*)\s*\(", text)
    names = sorted(set(names))
    assert {"kv_quantize_pack", "kv_append_residual", "kv_flush_residual", "minikv_decode_attn",
            "minikv_workspace_bytes", "minikv_buffer_bytes", "minikv_cache_bytes", "minikv_abi_version", "kv_select_hh_rw",
            "minikv_set_variant", "minikv_stream_read_probe", "minikv_diag_redo_count", "minikv_diag_decode_weights",
            "kv_select_workspace_bytes", "kv_pyramid_budget", "selective_flash_attn",
            "selective_flash_attn_workspace_bytes"} <= set(names)
    l = api.lib()
    for n in names:
        assert hasattr(l, n), n
    assert l.minikv_abi_version() == 1


def test_buffer_sizes_follow_the_documented_layout(api):
    s = api.make_shape(2, 8, 4, 128, 32, 256, 64)
    U = 8
    want = [U * 2 * 1024 * 4, U * 8 * 128 * 2, U * 8 * 128 * 2, U * 4 * 4 * 128 * 4, U * 256 * 4 * 2, U * 256 * 4 * 2,
            U * 4, U * 64 * 128 * 2, U * 64 * 128 * 2, U * 4]
    assert [api.buffer_bytes(s, i) for i in range(10)] == want
    # 64 + 8*D/G bytes per token
    assert sum(want[:6]) == U * 256 * (64 + 8 * 128 // 32)
    assert [api.cache_bytes(s, i) for i in range(10)] == want
    assert api.workspace_bytes(s) >= 2 * 8 * 2 * 132 * 4
    assert api.buffer_bytes(api.make_shape(1, 1, 1, 64, 32, 128, 0), 0) == 0


@pytest.mark.parametrize("bad,status", [
    (dict(D=64), -2), (dict(G=8), -2), (dict(Tcap=100), -1), (dict(Rcap=40), -1), (dict(Hq=6, Hkv=4), -1),
    (dict(Hq=32, Hkv=2), -2), (dict(B=0), -1),
])
def test_shape_rules_are_checked_on_the_host(api, bad, status):
    kw = dict(B=1, Hq=4, Hkv=4, D=128, G=32, Tcap=256, Rcap=32)
    kw.update(bad)
    s = api.make_shape(**kw)
    cache = api.MinikvCache(*([0x1000] * 10))
    rc = api.lib().minikv_decode_attn(C.byref(s), C.c_void_p(0x1000), C.byref(cache), 1.0, C.c_void_p(0x1000),
                                      C.c_void_p(0x1000), 1 << 30, None)
    assert rc == status
    assert api.lib().minikv_strerror(rc)


def test_pointer_and_workspace_checks(api):
    s = api.make_shape(1, 4, 4, 128, 32, 256, 32)
    l = api.lib()
    good = api.MinikvCache(*([0x1000] * 10))
    P = C.c_void_p
    assert l.minikv_decode_attn(C.byref(s), P(0x1000), C.byref(good), 1.0, P(0x1000), P(0x1000), 16, None) == -3
    assert l.minikv_decode_attn(C.byref(s), None, C.byref(good), 1.0, P(0x1000), P(0x1000), 1 << 30, None) == -1
    assert l.minikv_decode_attn(C.byref(s), P(0x1008), C.byref(good), 1.0, P(0x1000), P(0x1000), 1 << 30, None) == -1
    assert l.minikv_decode_attn(C.byref(s), P(0x1000), C.byref(good), float("nan"), P(0x1000), P(0x1000), 1 << 30, None) == -1
    bad = api.MinikvCache(*([0x1000] * 3 + [0] + [0x1000] * 6))
    assert l.minikv_decode_attn(C.byref(s), P(0x1000), C.byref(bad), 1.0, P(0x1000), P(0x1000), 1 << 30, None) == -1
    assert l.kv_append_residual(C.byref(s), None, P(0x1000), C.byref(good), None) == -1
    assert l.kv_quantize_pack(C.byref(s), P(0x1000), P(0x1000), 64, None, 0, P(0x1000), 48, C.byref(good), None) == -1
    assert l.kv_quantize_pack(C.byref(s), P(0x1000), P(0x1000), 64, None, 0, P(0x1000), 512, C.byref(good), None) == -1
    assert l.kv_quantize_pack(C.byref(s), P(0x1000), P(0x1000), 64, P(0x1000), 16, P(0x1000), 32, C.byref(good), None) == -1
    assert l.kv_quantize_pack(C.byref(s), P(0x1000), P(0x1000), 64, None, 0, P(0x1000), 0, C.byref(good), None) == 0
    assert l.minikv_set_variant(99) == -1 and l.minikv_set_variant(2) == -1 and l.minikv_set_variant(4) == -1
    assert l.minikv_set_variant(0) == 0
    assert l.minikv_diag_decode_weights(3) == -1 and l.minikv_diag_decode_weights(-1) == -1
    assert l.minikv_diag_decode_weights(2) == 0 and l.minikv_diag_decode_weights(0) == 0
    assert b"workspace" in l.minikv_strerror(-3)


def test_selection_arguments_are_checked_on_the_host(api):
    l, P = api.lib(), C.c_void_p
    ok = [P(0x1000)] * 5                                     # A_cumul, n_hh, n_rw, idx (stride follows), n_tok
    call = lambda units, rep, L, A, hh, rw, idx, stride, ntok, ws, wsb: l.kv_select_hh_rw(
        units, rep, L, A, hh, rw, idx, stride, ntok, ws, wsb, None)
    assert call(0, 1, 64, None, None, None, None, 64, None, None, 0) == 0            # no units: nothing to do
    assert call(-1, 1, 64, *ok[:4], 64, ok[4], None, 0) == -1
    assert call(4, 0, 64, *ok[:4], 64, ok[4], None, 0) == -1                         # rep < 1
    assert call(4, 1, -1, *ok[:4], 64, ok[4], None, 0) == -1
    assert call(4, 1, (1 << 30) + 1, *ok[:4], 64, ok[4], None, 0) == -1
    assert call(4, 1, 64, None, *ok[1:4], 64, ok[4], None, 0) == -1                  # null scores
    assert call(4, 1, 64, P(0x1002), *ok[1:4], 64, ok[4], None, 0) == -1             # misaligned scores
    assert call(4, 1, 64, ok[0], None, *ok[2:4], 64, ok[4], None, 0) == -1
    assert call(4, 1, 64, *ok[:4], -1, ok[4], None, 0) == -1
    need4, need1 = api.kv_select_workspace_bytes(4, 4, 64), api.kv_select_workspace_bytes(4, 1, 64)
    assert call(4, 4, 64, *ok[:4], 64, ok[4], None, 0) == -1                         # a workspace is needed
    assert call(4, 1, 64, *ok[:4], 64, ok[4], None, 0) == -1
    assert call(4, 4, 64, *ok[:4], 64, ok[4], P(0x1000), need4 - 1) == -3
    assert call(4, 1, 64, *ok[:4], 64, ok[4], P(0x1000), need1 - 1) == -3
    assert call(4, 1, 64, *ok[:4], 64, ok[4], P(0x1004), need1) == -1                # workspace not 16-byte aligned
    # summed-score keys (several heads only) + per 4096-token chunk: candidate list, histogram, counts + unit histogram
    assert need4 - need1 == 4 * 64 * 4 and need1 == 4 * (4096 + 1024 + 4 + 2048) * 4
    assert api.kv_select_workspace_bytes(0, 4, 64) == 0 and api.kv_select_workspace_bytes(4, 4, 0) == 0
    # prompts beyond 1024 chunks take the one-workgroup-per-unit kernel, which keeps only the keys
    assert api.kv_select_workspace_bytes(2, 4, 4096 * 1024 + 1) == 2 * (4096 * 1024 + 1) * 4
    assert api.kv_select_workspace_bytes(2, 1, 4096 * 1024 + 1) == 0


def test_pyramid_budget_is_host_arithmetic_and_matches_the_oracle(api):
    """The one entry point that runs entirely on the host: compared with the oracle here, without a GPU."""
    from oracle import ref
    for n_layers, x, d in [(32, 1024.0, 7), (32, 8192.0, 7), (2, 10.0, 7), (40, 333.0, 3), (1, 77.0, 7), (5, 0.0, 2)]:
        for bottom_heavy in (1, 0):
            got = api.kv_pyramid_budget(n_layers, x, d, bottom_heavy)
            want = ref.pyramid_budget(n_layers, x, d, bool(bottom_heavy))
            assert len(got) == n_layers
            assert max(abs(a - b) for a, b in zip(got, want)) <= 1e-12 * max(x, 1.0)
    # values worked by hand (end layers x/d and 2x - x/d, straight line between, mean x)
    assert api.kv_pyramid_budget(3, 7.0, 7, 1) == [13.0, 7.0, 1.0]
    assert api.kv_pyramid_budget(3, 7.0, 7, 0) == [1.0, 7.0, 13.0]
    assert api.kv_pyramid_budget(5, 8.0, 2, 1) == [12.0, 10.0, 8.0, 6.0, 4.0]
    for bad in [(0, 1.0, 7, 1), (4, -1.0, 7, 1), (4, float("nan"), 7, 1), (4, 1.0, 0, 1)]:
        with pytest.raises(api.MinikvError):
            api.kv_pyramid_budget(*bad)


def test_prefill_arguments_are_checked_on_the_host(api):
    l, P = api.lib(), C.c_void_p
    p = P(0x1000)
    nws = api.selective_flash_attn_workspace_bytes(2, 2, 100)
    assert nws == 2 * 2 * 128 * 128 * 2                      # V transposed, 100 keys padded to 128
    assert api.selective_flash_attn_workspace_bytes(0, 2, 100) == 0
    call = lambda B, Hq, Hkv, L, sm, ws=p, wsb=nws, Q=p, acc=p: l.selective_flash_attn(
        B, Hq, Hkv, L, Q, p, p, sm, p, p, acc, ws, wsb, None)
    assert call(0, 4, 2, 100, 0.1) == -1
    assert call(2, 5, 2, 100, 0.1) == -1                     # Hq not a multiple of Hkv
    assert call(2, 4, 2, 0, 0.1) == -1                       # empty prompt
    assert call(2, 4, 2, 100, 0.0) == -1 and call(2, 4, 2, 100, -1.0) == -1      # scale must be positive
    assert call(2, 4, 2, 100, float("nan")) == -1 and call(2, 4, 2, 100, float("inf")) == -1
    assert call(2, 4, 2, 100, 0.1, Q=P(0x1008)) == -1        # misaligned
    assert call(2, 4, 2, 100, 0.1, acc=P(0x1004)) == -1
    assert call(2, 4, 2, 100, 0.1, ws=None) == -1
    assert call(2, 4, 2, 100, 0.1, wsb=nws - 1) == -3


def test_static_workspace_entry_point_refuses_what_does_not_fit(api):
    """Host-side checks of minikv_decode_attn_static: nothing is launched and no device is touched."""
    l = api.lib()
    cap = int(l.minikv_static_workspace_units())
    assert cap == 2048
    P = C.c_void_p
    cache = api.MinikvCache(*([0x1000] * 10))
    too_many = api.make_shape(cap + 1, 4, 1, 128, 32, 256, 32)           # cap + 1 units
    assert l.minikv_decode_attn_static(C.byref(too_many), P(0x1000), C.byref(cache), C.c_float(1.0), P(0x1000), None) == -3
    two_sets = api.make_shape(cap // 2 + 1, 8, 1, 128, 32, 256, 32)      # two sets of four heads per unit
    assert l.minikv_decode_attn_static(C.byref(two_sets), P(0x1000), C.byref(cache), C.c_float(1.0), P(0x1000), None) == -3
    bad = api.make_shape(1, 4, 1, 64, 32, 256, 32)
    assert l.minikv_decode_attn_static(C.byref(bad), P(0x1000), C.byref(cache), C.c_float(1.0), P(0x1000), None) == -2
    assert l.minikv_decode_attn_static(C.byref(api.make_shape(1, 4, 1, 128, 32, 256, 32)), None, C.byref(cache),
                                       C.c_float(1.0), P(0x1000), None) == -1


def test_per_token_variant_sizes_and_host_checks(api):
    """minikv_pt_cache_bytes follows the documented layout (the appendix's 4-bit case: 68 bytes per token, head and
    tensor against 256 in fp16) and the entry points refuse bad arguments before anything is launched."""
    l, P = api.lib(), C.c_void_p
    s = api.make_pt_shape(2, 8, 2, 128, 128, 4, 256)
    U = 4
    sizes = [int(l.minikv_pt_cache_bytes(C.byref(s), i)) for i in range(10)]
    assert sizes[:7] == [U * 256 * 64, U * 256 * 2, U * 256 * 2, U * 256 * 64, U * 256 * 2, U * 256 * 2, U * 4]
    assert sizes[7:] == [0, 0, 0]
    assert (sizes[0] + sizes[1] + sizes[2]) == U * 256 * 68 and round(256 / 68, 2) == 3.76
    assert int(l.minikv_pt_workspace_bytes(C.byref(s))) >= 2 * 8 * 132 * 4
    cache = api.MinikvPtCache(*([0x1000] * 7))
    good = (P(0x1000), P(0x1000), 64, None, 0, P(0x1000))
    for bad, status in ((dict(bits=3), -2), (dict(G=16), -2), (dict(Tcap=100), -1), (dict(Hq=7), -1), (dict(Hq=32, Hkv=2), -2),
                        (dict(D=64), -2)):
        kw = dict(B=2, Hq=8, Hkv=2, D=128, G=128, bits=4, Tcap=256); kw.update(bad)
        sb = api.make_pt_shape(**kw)
        assert l.kv_quantize_pack_pt(C.byref(sb), *good, 64, C.byref(cache), None) == status
        assert int(l.minikv_pt_cache_bytes(C.byref(sb), 0)) == 0
    assert l.kv_quantize_pack_pt(C.byref(s), *good, 24, C.byref(cache), None) == -1          # bound not a multiple of 16
    assert l.kv_quantize_pack_pt(C.byref(s), *good, 128, C.byref(cache), None) == -1         # bound beyond L
    assert l.kv_quantize_pack_pt(C.byref(s), *good, 0, C.byref(cache), None) == 0            # nothing to do
    assert l.kv_quantize_pack_pt(C.byref(s), None, P(0x1000), 64, None, 0, P(0x1000), 64, C.byref(cache), None) == -1
    assert l.minikv_decode_attn_pt(C.byref(s), P(0x1000), C.byref(cache), 1.0, P(0x1000), P(0x1000), 16, None) == -3
    assert l.minikv_decode_attn_pt(C.byref(s), P(0x1000), C.byref(cache), float("inf"), P(0x1000), P(0x1000), 1 << 30, None) == -1
    assert l.minikv_decode_attn_pt(C.byref(s), P(0x1004), C.byref(cache), 1.0, P(0x1000), P(0x1000), 1 << 30, None) == -1
