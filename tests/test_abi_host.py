"""Host side of the C ABI, no GPU needed: the library loads, exports every
symbol the header declares, sizes its workspace and rejects bad arguments
before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_2506_03762_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2506_03762_amd import build
        build.build()
    return B.load()


def good(**kw):
    base = dict(batch=1, n_q_heads=8, n_kv_heads=2, head_dim=128, seq_len=4096, window=64,
                budget=512, recent=64, dtype=B.AHA_BF16, q_stride=(8 * 4096 * 128, 4096 * 128, 128),
                k_stride=(2 * 4096 * 128, 4096 * 128, 128), v_stride=(2 * 4096 * 128, 4096 * 128, 128))
    base.update(kw)
    return B.Params(**base)


def test_header_symbols_are_exported(lib):
    hdr = open(os.path.join(ROOT, "include", "aha.h")).read()
    declared = set(re.findall(r"\b(aha_[a-z_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert B.version().startswith("aha-gfx950")


def test_struct_layout_matches_header():
    # 14 four-byte fields, nine int64 strides, four four-byte fields
    assert ctypes.sizeof(B.aha_params) == 14 * 4 + 9 * 8 + 4 * 4
    assert B.aha_params.q_stride.offset == 56
    assert B.aha_params.score_pool.offset == 56 + 72
    assert B.aha_params.sink.offset == 56 + 72 + 4
    assert B.aha_params.decode_value_prior.offset == 56 + 72 + 8


def test_workspace_bytes(lib):
    n1 = B.workspace_bytes(good())
    assert n1 > 0 and n1 % 256 == 0
    assert B.workspace_bytes(good(seq_len=32768, budget=2048)) > n1
    assert B.workspace_bytes(good(dtype=B.AHA_F32, head_dim=64)) > 0
    # full accumulation needs row statistics for every row
    assert B.workspace_bytes(good(window=4096)) > n1


DUMMY = ctypes.c_void_p(0x1000)


def call_prefill(lib, p, q=DUMMY, k=DUMMY, v=DUMMY, s=DUMMY, ws=DUMMY, nbytes=1 << 40):
    cp = p.c()
    return lib.aha_prefill_scores(ctypes.byref(cp), q, k, v, s, ws, nbytes, None)


@pytest.mark.parametrize("kw,code", [
    (dict(n_q_heads=7), B.AHA_ERR_INVALID_ARG),
    (dict(head_dim=96), B.AHA_ERR_UNSUPPORTED),
    (dict(budget=0), B.AHA_ERR_INVALID_ARG),
    (dict(budget=5000), B.AHA_ERR_INVALID_ARG),
    (dict(recent=513), B.AHA_ERR_INVALID_ARG),
    (dict(recent=-1), B.AHA_ERR_INVALID_ARG),
    (dict(window=0), B.AHA_ERR_INVALID_ARG),
    (dict(window=4097), B.AHA_ERR_INVALID_ARG),
    (dict(pool_kernel=4), B.AHA_ERR_INVALID_ARG),
    (dict(pool_kernel=257), B.AHA_ERR_INVALID_ARG),
    (dict(dtype=3), B.AHA_ERR_INVALID_ARG),
    (dict(scale_mode=2), B.AHA_ERR_INVALID_ARG),
    (dict(scale_mode=B.AHA_SCALE_FIXED, fixed_scale=-0.1), B.AHA_ERR_INVALID_ARG),
    (dict(k_stride=(0, 0, 100)), B.AHA_ERR_INVALID_ARG),   # not a multiple of 8 elements
    (dict(q_stride=(0, 0, 64)), B.AHA_ERR_INVALID_ARG),    # rows overlap
    (dict(batch=0), B.AHA_ERR_INVALID_ARG),
    (dict(seq_len=(1 << 30) + 8, budget=512), B.AHA_ERR_UNSUPPORTED),
    (dict(batch=70000), B.AHA_ERR_UNSUPPORTED),            # batch * KV heads beyond a grid dimension
    (dict(batch=1 << 30, n_q_heads=64, n_kv_heads=64), B.AHA_ERR_UNSUPPORTED),   # product overflows 32 bits
    (dict(score_pool=4), B.AHA_ERR_INVALID_ARG),
    (dict(score_pool=-1), B.AHA_ERR_INVALID_ARG),
    (dict(score_pool=257), B.AHA_ERR_INVALID_ARG),
    (dict(sink=-1), B.AHA_ERR_INVALID_ARG),
    (dict(sink=449), B.AHA_ERR_INVALID_ARG),               # sink + recent beyond the budget
    (dict(decode_value_prior=2), B.AHA_ERR_INVALID_ARG),
])
def test_bad_params_are_rejected(lib, kw, code):
    assert call_prefill(lib, good(**kw)) == code
    assert len(B.load().aha_last_error()) > 0


def test_bad_pointers_and_workspace(lib):
    p = good()
    assert call_prefill(lib, p, q=None) == B.AHA_ERR_INVALID_ARG
    assert call_prefill(lib, p, k=ctypes.c_void_p(0x1004)) == B.AHA_ERR_INVALID_ARG
    assert call_prefill(lib, p, s=None) == B.AHA_ERR_INVALID_ARG
    assert call_prefill(lib, p, v=None) == B.AHA_ERR_INVALID_ARG
    assert call_prefill(lib, p, ws=None) == B.AHA_ERR_WORKSPACE
    assert call_prefill(lib, p, ws=ctypes.c_void_p(0x1010)) == B.AHA_ERR_WORKSPACE
    assert call_prefill(lib, p, nbytes=B.workspace_bytes(p) - 1) == B.AHA_ERR_WORKSPACE
    assert b"workspace" in lib.aha_last_error()
    cp = p.c()
    assert lib.aha_workspace_bytes(ctypes.byref(cp), None) == B.AHA_ERR_INVALID_ARG
    assert lib.aha_workspace_bytes(None, ctypes.byref(ctypes.c_size_t())) == B.AHA_ERR_INVALID_ARG


def test_prefill_with_given_normalisers_validates(lib):
    """aha_prefill_scores_lse: same checks as aha_prefill_scores, plus the lse pointer."""
    p = good()
    cp = p.c()
    big = 1 << 40
    call = lambda **kw: lib.aha_prefill_scores_lse(
        ctypes.byref(cp), kw.get("q", DUMMY), DUMMY, DUMMY, kw.get("lse", DUMMY), DUMMY,
        kw.get("ws", DUMMY), kw.get("nbytes", big), None)
    assert call(lse=None) == B.AHA_ERR_INVALID_ARG
    assert b"lse" in lib.aha_last_error()
    assert call(lse=ctypes.c_void_p(0x1002)) == B.AHA_ERR_INVALID_ARG   # not 4-byte aligned
    assert call(q=None) == B.AHA_ERR_INVALID_ARG
    assert call(ws=None) == B.AHA_ERR_WORKSPACE
    assert call(nbytes=B.workspace_bytes(p) - 1) == B.AHA_ERR_WORKSPACE
    bad = good(window=0).c()
    assert lib.aha_prefill_scores_lse(ctypes.byref(bad), DUMMY, DUMMY, DUMMY, DUMMY, DUMMY, DUMMY,
                                      big, None) == B.AHA_ERR_INVALID_ARG


def test_scores_over_chosen_rows_validate(lib):
    p = good()
    cp = p.c()
    call = lambda rows=DUMMY, pp=cp: lib.aha_prefill_scores_rows(
        ctypes.byref(pp), DUMMY, DUMMY, DUMMY, rows, DUMMY, DUMMY, 1 << 40, None)
    assert call(rows=None) == B.AHA_ERR_INVALID_ARG
    assert b"rows" in lib.aha_last_error()
    wide = good(window=128).c()                     # 4 query heads x 128 rows: two query tiles
    assert call(pp=wide) == B.AHA_ERR_UNSUPPORTED
    assert b"256" in lib.aha_last_error()


def test_window_attention_validates(lib):
    p = good()
    cp = p.c()
    need = ctypes.c_size_t(0)
    assert lib.aha_window_attention_workspace_bytes(ctypes.byref(cp), ctypes.byref(need)) == B.AHA_OK
    assert need.value > 0 and need.value % 256 == 0
    f32 = good(dtype=B.AHA_F32, q_stride=(0, 0, 128)).c()
    assert lib.aha_window_attention_workspace_bytes(ctypes.byref(f32), ctypes.byref(need)) == B.AHA_OK
    assert need.value == 0
    call = lambda q=DUMMY, out=DUMMY, lse=DUMMY, ws=DUMMY, nbytes=1 << 40: \
        lib.aha_prefill_window_attention(ctypes.byref(cp), q, DUMMY, DUMMY, out, lse, ws, nbytes, None)
    assert call(q=None) == B.AHA_ERR_INVALID_ARG
    assert call(out=None) == B.AHA_ERR_INVALID_ARG
    assert call(lse=ctypes.c_void_p(0x1002)) == B.AHA_ERR_INVALID_ARG
    assert call(ws=None) == B.AHA_ERR_WORKSPACE
    assert call(nbytes=B.window_attention_workspace_bytes(p) - 1) == B.AHA_ERR_WORKSPACE


def test_row_stats_validate(lib):
    """aha_prefill_row_stats: needs q, k and at least one output; the value strides are not looked at."""
    p = good(v_stride=(0, 0, 0))
    cp = p.c()
    big = 1 << 40
    call = lambda q=DUMMY, lse=DUMMY, ent=DUMMY, ws=DUMMY, nbytes=big: lib.aha_prefill_row_stats(
        ctypes.byref(cp), q, DUMMY, lse, ent, ws, nbytes, None)
    assert call(lse=None, ent=None) == B.AHA_ERR_INVALID_ARG
    assert call(q=None) == B.AHA_ERR_INVALID_ARG
    assert call(ent=ctypes.c_void_p(0x1002)) == B.AHA_ERR_INVALID_ARG
    assert call(ws=None) == B.AHA_ERR_WORKSPACE
    assert call(nbytes=B.workspace_bytes(good()) - 1) == B.AHA_ERR_WORKSPACE
    bad = good(q_stride=(0, 0, 64)).c()
    assert lib.aha_prefill_row_stats(ctypes.byref(bad), DUMMY, DUMMY, DUMMY, DUMMY, DUMMY, big,
                                     None) == B.AHA_ERR_INVALID_ARG


def test_other_entry_points_validate(lib):
    p = good()
    cp = p.c()
    # selection on pooled scores keeps them in the workspace
    pooled = good(score_pool=7)
    cpp = pooled.c()
    assert B.workspace_bytes(pooled) >= 4 * pooled.batch * pooled.n_kv_heads * pooled.seq_len
    assert lib.aha_select_topk(ctypes.byref(cpp), DUMMY, DUMMY, None, 0, None) == B.AHA_ERR_WORKSPACE
    assert lib.aha_select_topk(ctypes.byref(cpp), DUMMY, DUMMY, DUMMY, 1024, None) == B.AHA_ERR_WORKSPACE
    cpp.reserved = 1
    assert lib.aha_select_topk(ctypes.byref(cpp), DUMMY, DUMMY, DUMMY, 1 << 40, None) == B.AHA_ERR_INVALID_ARG
    assert lib.aha_select_topk(ctypes.byref(cp), None, DUMMY, None, 0, None) == B.AHA_ERR_INVALID_ARG
    assert lib.aha_compact_kv(ctypes.byref(cp), DUMMY, DUMMY, DUMMY, DUMMY, DUMMY, DUMMY, DUMMY,
                              DUMMY, DUMMY, 512, None) == B.AHA_ERR_INVALID_ARG  # slots < B+1
    assert lib.aha_compact_kv(ctypes.byref(cp), DUMMY, DUMMY, DUMMY, DUMMY, None, DUMMY, DUMMY,
                              DUMMY, DUMMY, 513, None) == B.AHA_ERR_INVALID_ARG
    args = [DUMMY] * 8
    assert lib.aha_decode_step(ctypes.byref(cp), *args, 513, 512, DUMMY, None, 0, None) \
        == B.AHA_ERR_INVALID_ARG                                              # logical_pos too small
    assert lib.aha_decode_step(ctypes.byref(cp), *args, 100, 4097, DUMMY, None, 0, None) \
        == B.AHA_ERR_INVALID_ARG                                              # too few slots
    cp3 = good(n_q_heads=18).c()
    assert lib.aha_decode_step(ctypes.byref(cp3), *args, 513, 4097, DUMMY, None, 0, None) \
        == B.AHA_ERR_UNSUPPORTED                                              # group of 9
    cpb = good(budget=4096, n_q_heads=16, batch=64).c()
    assert lib.aha_decode_step(ctypes.byref(cpb), *args, 4097, 5000, DUMMY, None, 0, None) \
        == B.AHA_ERR_UNSUPPORTED                                              # dots exceed LDS
    # few heads, large budget: the splits' dots must fit 64 KiB of LDS each, or the call is
    # refused before anything is launched (64 splits x 3584 slots at group 4, head_dim 128)
    fits = good(batch=8, n_q_heads=32, n_kv_heads=8, seq_len=1 << 20, budget=229000).c()
    assert lib.aha_decode_step(ctypes.byref(fits), *args, 229001, 229001, DUMMY, None, 0, None) \
        == B.AHA_ERR_WORKSPACE                                                # accepted up to here
    big = good(batch=8, n_q_heads=32, n_kv_heads=8, seq_len=1 << 20, budget=230000).c()
    assert lib.aha_decode_step(ctypes.byref(big), *args, 230001, 230001, DUMMY, DUMMY, 1 << 40, None) \
        == B.AHA_ERR_UNSUPPORTED
    assert b"does not fit" in lib.aha_last_error()
    # compaction looks at the K / V strides only
    kv_only = good(q_stride=(0, 0, 0), window=0, pool_kernel=0).c()
    assert lib.aha_compact_kv(ctypes.byref(kv_only), DUMMY, DUMMY, DUMMY, DUMMY, DUMMY, DUMMY,
                              DUMMY, DUMMY, DUMMY, 512, None) == B.AHA_ERR_INVALID_ARG
    assert b"cache_slots" in lib.aha_last_error()          # the only complaint left
    # a decode-only caller sizes its workspace without a sequence length
    dec_only = good(seq_len=0, window=0).c()
    out = ctypes.c_size_t(0)
    assert lib.aha_workspace_bytes(ctypes.byref(dec_only), ctypes.byref(out)) == B.AHA_OK
    assert out.value > 0 and out.value % 256 == 0
    # few heads: the slots are split over workgroups and the partials need the workspace
    assert lib.aha_decode_step(ctypes.byref(cp), *args, 513, 4097, DUMMY, None, 0, None) \
        == B.AHA_ERR_WORKSPACE


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/libaha.so")
    with pytest.raises(RuntimeError, match="not built"):
        B.load()


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits before touching a device."""
    import os, subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
