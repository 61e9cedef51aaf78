"""The C-ABI boundary without a GPU: every function include/vlcache.h declares is exported by the
built library, and host-side validation rejects bad calls before anything is enqueued."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def V():
    lib = os.path.join(ROOT, "paper_2410_23317_amd", "libvlcache.so")
    if not os.path.exists(lib):
        import __graft_entry__
        __graft_entry__.build()
    import paper_2410_23317_amd as V
    return V


def declared_functions():
    text = open(os.path.join(ROOT, "include", "vlcache.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vlc_[a-z_]+)\s*\(", text)))


def test_header_declares_the_five_calls():
    names = declared_functions()
    for n in ("vlc_score", "vlc_sparsity", "vlc_allocate", "vlc_topk_compact", "vlc_decode_attn",
              "vlc_cache_create", "vlc_cache_destroy", "vlc_workspace_bytes", "vlc_cache_bytes"):
        assert n in names


def test_library_exports_every_declared_symbol(V):
    for n in declared_functions():
        assert hasattr(V.lib, n), f"{n} is declared in include/vlcache.h but not exported"
    assert "gfx950" in V.vlc_version()


def test_shape_validation(V):
    ok = V.make_shape(1, 2, 4, 2, 64, 512, 32, "f32")
    assert V.vlc_workspace_bytes(ok) > 0
    bad = [
        (dict(Hq=4, Hkv=3), V.VLC_ERR_SHAPE), (dict(d=96), V.VLC_ERR_SHAPE), (dict(Hq=18, Hkv=2), V.VLC_ERR_SHAPE),
        (dict(tau=600, m=512), V.VLC_ERR_SHAPE), (dict(tau=0), V.VLC_ERR_SHAPE), (dict(L=0), V.VLC_ERR_SHAPE),
        (dict(tau=4097, m=5000), V.VLC_ERR_SHAPE), (dict(dtype=7), V.VLC_ERR_DTYPE),
    ]
    base = dict(B=1, L=2, Hq=4, Hkv=2, d=64, m=512, tau=32, dtype=V.VLC_F32)
    for kw, code in bad:
        s = V.make_shape(**{**base, **kw})
        assert V.lib.vlc_workspace_bytes(C.byref(s)) == 0
        st = V.lib.vlc_score(C.byref(s), 1, 1, None, 0.01, 1, 1, 1, None, 1, 1 << 30, None)
        assert st == code, (kw, st, V.vlc_last_error_string())
        assert V.vlc_last_error_string()


def test_argument_validation_happens_before_any_launch(V):
    s = V.make_shape(1, 2, 4, 2, 64, 512, 32, "f32")
    sp = C.byref(s)
    assert V.lib.vlc_score(sp, None, 1, None, 0.01, 1, 1, 1, None, 1, 1 << 30, None) == V.VLC_ERR_INVALID_ARG
    assert V.lib.vlc_score(sp, 1, 1, None, 0.01, 1, 1, 1, None, 1, 16, None) == V.VLC_ERR_CAPACITY
    assert V.lib.vlc_score(sp, 1, 1, None, 1.5, 1, 1, 1, 1, 1, 1 << 30, None) == V.VLC_ERR_INVALID_ARG
    assert V.lib.vlc_sparsity(sp, None, None, None, None, 0.01, None, None, None, 0, None) == V.VLC_ERR_INVALID_ARG
    assert V.lib.vlc_allocate(sp, 1, 0, 10, 1, None, None) == V.VLC_ERR_INVALID_ARG
    assert V.lib.vlc_allocate(sp, 1, 11, 10, 1, None, None) == V.VLC_ERR_INVALID_ARG
    assert V.lib.vlc_allocate(sp, None, 1, 10, 1, None, None) == V.VLC_ERR_INVALID_ARG


def test_window_attn_and_score_from_stats_validate_before_any_launch(V):
    f32 = V.make_shape(1, 2, 4, 2, 64, 512, 32, "f32")
    nbytes = C.c_size_t(7)
    assert V.lib.vlc_window_attn_workspace_bytes(C.byref(f32), C.byref(nbytes)) == V.VLC_OK
    assert nbytes.value == 0                                     # the generic kernel (fp32 storage, d = 64) needs no workspace
    assert V.lib.vlc_window_attn_workspace_bytes(C.byref(f32), None) == V.VLC_ERR_INVALID_ARG
    assert V.lib.vlc_window_attn(C.byref(f32), 1, 1, None, None, 1, 1, 1, None, 0, None) == V.VLC_ERR_INVALID_ARG   # v missing
    plain = V.make_shape(1, 2, 8, 2, 128, 3000, 32, "bf16", flags=V.VLC_SHAPE_SCORE_PLAIN_ALU)
    assert V.vlc_window_attn_workspace_bytes(plain) == 0         # the flag sends the matrix-core shape to the generic kernel too
    s = V.make_shape(1, 2, 8, 2, 128, 3000, 32, "bf16")
    sp = C.byref(s)
    need = V.vlc_window_attn_workspace_bytes(s)
    assert need >= 2 * 2 * 4 * 32 * 128 * 4                      # at least one split of fp32 partial outputs
    assert V.lib.vlc_window_attn(sp, 1, 1, None, None, 1, 1, 1, 1, need, None) == V.VLC_ERR_INVALID_ARG     # v missing
    assert V.lib.vlc_window_attn(sp, 1, 1, 1, None, 1, 1, 1, 1, need - 1, None) == V.VLC_ERR_CAPACITY
    assert V.lib.vlc_window_attn(sp, 1, 1, 1, None, 1, 1, 1, None, need, None) == V.VLC_ERR_INVALID_ARG      # workspace missing
    big = V.make_shape(2, 32, 8, 8, 128, 3000, 32, "bf16")         # every KV group has a block of its own: no partials
    assert V.vlc_window_attn_workspace_bytes(big) == 256
    assert V.lib.vlc_score_from_stats(sp, 1, 1, None, 0.01, None, 1, 1, None, None) == V.VLC_ERR_INVALID_ARG
    assert V.lib.vlc_score_from_stats(sp, 1, 1, None, 2.0, 1, 1, 1, 1, None) == V.VLC_ERR_INVALID_ARG
    bad = V.make_shape(1, 2, 8, 3, 128, 3000, 32, "bf16")
    assert V.lib.vlc_score_from_stats(C.byref(bad), 1, 1, None, 0.01, 1, 1, 1, None, None) == V.VLC_ERR_SHAPE


def test_cache_bookkeeping_errors(V):
    s = V.make_shape(1, 2, 4, 2, 64, 512, 32, "f32")
    n = V.vlc_cache_bytes(s, 8, 120)
    assert n > 2 * 4 * 2 * 64 * (120 + 16)           # at least the K and V slabs
    assert V.vlc_cache_bytes(s, 16, 120) > n
    h = C.c_void_p()
    assert V.lib.vlc_cache_create(C.byref(s), 8, 120, 4096, n - 1, C.byref(h)) == V.VLC_ERR_CAPACITY
    assert V.lib.vlc_cache_create(C.byref(s), 8, 120, 4096 + 8, n, C.byref(h)) == V.VLC_ERR_INVALID_ARG   # misaligned
    assert V.lib.vlc_cache_create(C.byref(s), 8, 1, 4096, n, C.byref(h)) == V.VLC_ERR_INVALID_ARG         # sum_k_max < L
    assert V.lib.vlc_cache_create(C.byref(s), 8, 120, 4096, n, C.byref(h)) == V.VLC_OK                    # no device access yet
    lay = V.vlc_cache_layout()
    assert V.lib.vlc_cache_get_layout(h, C.byref(lay)) == V.VLC_OK
    assert lay.total_bytes == n and lay.slots_per_request == 120 + 2 * 8 and lay.kv_off % 256 == 0
    # decode before compaction, bad layer ranges
    assert V.lib.vlc_decode_attn(h, 0, 2, 1, None, None, None, 1, None) == V.VLC_ERR_INVALID_ARG
    assert "vlc_topk_compact" in V.vlc_last_error_string()
    assert V.lib.vlc_decode_attn(None, 0, 1, 1, None, None, None, 1, None) == V.VLC_ERR_INVALID_ARG
    assert V.lib.vlc_topk_compact(h, None, 1, 0, 1, 1, None, None) == V.VLC_ERR_INVALID_ARG
    assert V.lib.vlc_topk_compact(h, 1, 1, -1, 1, 1, None, None) == V.VLC_ERR_INVALID_ARG
    for num, den in ((1, 0), (-1, 10), (11, 10)):                       # recent fraction outside [0, 1]
        assert V.lib.vlc_topk_compact_recent_frac(h, 1, 1, num, den, 1, 1, None, None) == V.VLC_ERR_INVALID_ARG
    assert V.lib.vlc_topk_compact_recent_frac(h, None, 1, 1, 10, 1, 1, None, None) == V.VLC_ERR_INVALID_ARG
    assert V.lib.vlc_cache_hit_rate(h, 1, 1, None, None) == V.VLC_ERR_INVALID_ARG        # cache not filled yet
    assert V.lib.vlc_cache_hit_rate(None, 1, 1, None, None) == V.VLC_ERR_INVALID_ARG
    V.lib.vlc_cache_destroy(h)


def test_cache_options_are_validated_and_reported(V):
    s = V.make_shape(4, 32, 32, 8, 128, 10368, 64, "bf16")
    sum_k = 33177 + 32 * 104
    lay = V.vlc_cache_layout()
    h = C.c_void_p()

    def create(**kw):
        o = V.make_options(**kw)
        n = V.lib.vlc_cache_bytes_opt(C.byref(s), 100, sum_k, C.byref(o))
        if n == 0:
            return None
        assert V.lib.vlc_cache_create_opt(C.byref(s), 100, sum_k, C.byref(o), 4096, n, C.byref(h)) == V.VLC_OK
        assert V.lib.vlc_cache_get_layout(h, C.byref(lay)) == V.VLC_OK and lay.total_bytes == n
        V.lib.vlc_cache_destroy(h)
        return (lay.unit_slots, lay.tail_unit_slots, lay.layer_unit_slots)

    default = create()
    assert default[0] in (256, 512, 1024, 2048) and default[1] <= default[0] and default[2] in (128, 256, 512)
    assert V.vlc_cache_bytes(s, 100, sum_k) == V.vlc_cache_bytes_opt(s, 100, sum_k, None)     # NULL options = the defaults
    assert create(unit_slots=1024, tail_unit_slots=128, layer_unit_slots=256) == (1024, 128, 256)
    assert create(unit_slots=128) == (128, 128, default[2])
    for bad in (dict(unit_slots=100), dict(unit_slots=128, tail_unit_slots=256), dict(layer_unit_slots=4096), dict(gather_rows=256), dict(decode_merge=3),
                dict(decode_order=-1), dict(decode_zigzag=4), dict(gather_rows=48), dict(select_fold=3), dict(kv_fp8=2)):
        assert create(**bad) is None, bad
        assert "options" in V.vlc_last_error_string()
    # an FP8 cache needs bf16 storage
    f32 = V.make_shape(1, 2, 4, 2, 64, 512, 32, "f32")
    o = V.make_options(kv_fp8=1)
    assert V.lib.vlc_cache_bytes_opt(C.byref(f32), 8, 120, C.byref(o)) == 0
    assert V.lib.vlc_cache_create_opt(C.byref(f32), 8, 120, C.byref(o), 4096, 1 << 30, C.byref(h)) == V.VLC_ERR_DTYPE


def test_default_unit_sizes_of_the_benchmark_shapes(V):
    """The library's own choice of block-unit sizes (all-layer list, its tail units, per-layer list) for the four
    benchmark shapes at a 10 % budget and 100 decode steps: few rows keep small units so that the chip fills, many
    rows get units that hold a whole average row."""
    import workloads as W
    lay = V.vlc_cache_layout()
    h = C.c_void_p()
    want = {1: (256, 256, 128), 2: (2048, 2048, 256), 3: (2048, 2048, 256), 4: (1024, 512, 256)}
    for cid, units in want.items():
        cfg = W.CONFIGS[cid]
        s = V.make_shape(cfg.B, cfg.L, cfg.Hq, cfg.Hkv, cfg.d, cfg.m, cfg.tau, cfg.dtype)
        sum_k = cfg.L * cfg.m // 10 + cfg.L * (cfg.m // 100 + 1)
        n = V.vlc_cache_bytes(s, 100, sum_k)
        assert V.lib.vlc_cache_create(C.byref(s), 100, sum_k, 4096, n, C.byref(h)) == V.VLC_OK
        assert V.lib.vlc_cache_get_layout(h, C.byref(lay)) == V.VLC_OK
        V.lib.vlc_cache_destroy(h)
        assert (lay.unit_slots, lay.tail_unit_slots, lay.layer_unit_slots) == units, cid


def test_shape_flags(V):
    s = V.make_shape(1, 2, 8, 2, 128, 3000, 32, "bf16")
    plain = V.make_shape(1, 2, 8, 2, 128, 3000, 32, "bf16", flags=V.VLC_SHAPE_SCORE_PLAIN_ALU)
    assert V.vlc_workspace_bytes(s) > 0 and V.vlc_workspace_bytes(plain) > 0
    bad = V.make_shape(1, 2, 8, 2, 128, 3000, 32, "bf16", flags=6)
    assert V.lib.vlc_workspace_bytes(C.byref(bad)) == 0
    assert V.lib.vlc_score(C.byref(bad), 1, 1, None, 0.01, 1, 1, 1, None, 1, 1 << 30, None) == V.VLC_ERR_INVALID_ARG


def test_library_does_not_read_the_environment():
    """Behaviour depends on the arguments only: no source of the library calls getenv."""
    csrc = os.path.join(ROOT, "paper_2410_23317_amd", "csrc")
    for f in os.listdir(csrc):
        text = open(os.path.join(csrc, f)).read()
        assert "getenv" not in text and "environ" not in text, f


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2410_23317_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower().replace("miracle", ""), f"{f} mentions the oracle"
