"""aha_decode_step_static (the generation step on the library's built-in scratch buffer, for
callers that cannot allocate) against aha_decode_step with a caller workspace: same cache
state, attention output and victims, on two calls in a row, the second on a smaller problem."""
import ctypes

import numpy as np
import pytest

from paper_2506_03762_amd import binding as B
from paper_2506_03762_amd import synth
from tests import harness as H
from tests.harness import Opts


def test_oversized_shapes_are_refused_before_any_launch():
    """No GPU needed: the size check precedes every HIP call."""
    lib = B.load()
    dummy = ctypes.c_void_p(0x1000)
    # 8 KV heads x 4 query heads x budget 16384: 2.2 MiB of dots + partial outputs -> fits
    # 64 heads x 8 query heads x budget 6500: 13 MiB of dots -> refused
    big = B.Params(batch=8, n_q_heads=64, n_kv_heads=8, head_dim=128, seq_len=0, window=0,
                   budget=6500, recent=64).c()
    rc = lib.aha_decode_step_static(ctypes.byref(big), *([dummy] * 8), 6501, 6501, dummy, None)
    assert rc == B.AHA_ERR_UNSUPPORTED
    assert b"built-in buffer" in lib.aha_last_error()
    bad = B.Params(batch=1, n_q_heads=8, n_kv_heads=2, head_dim=128, seq_len=0, window=0,
                   budget=300, recent=400).c()
    assert lib.aha_decode_step_static(ctypes.byref(bad), *([dummy] * 8), 301, 301, dummy, None) \
        == B.AHA_ERR_INVALID_ARG


def _run_both(w, seed, steps):
    """`steps` generation steps through both entry points from the same random cache."""
    import torch
    opts = Opts()
    p = H.gpu_params(w, opts)
    oc = H.random_cache(w, seed)
    ga, gb = H.upload_cache(oc, w, p), H.upload_cache(oc, w, p)
    ws = B.alloc_workspace(p)
    ws.fill_(0xA5)
    shape = (w.batch, w.n_q_heads, w.head_dim)
    oa = torch.full(shape, float("nan"), dtype=B.torch_dtype(p.dtype), device="cuda")
    ob = torch.full(shape, float("nan"), dtype=B.torch_dtype(p.dtype), device="cuda")
    for t in range(steps):
        q, k, v = (H.to_device(a, w.dtype) for a in synth.make_decode_inputs(w, t))
        c_t = w.seq_len + t + 1
        B.aha_decode_step(p, q, k, v, ga.k, ga.v, ga.scores, ga.pos, ga.free_slot, c_t, oa, ws)
        B.aha_decode_step_static(p, q, k, v, gb.k, gb.v, gb.scores, gb.pos, gb.free_slot, c_t, ob)
        torch.cuda.synchronize()
        # integer state bit-exact; the floats come from the same kernels in the same order
        assert torch.equal(ga.pos, gb.pos) and torch.equal(ga.free_slot, gb.free_slot), \
            "victims differ at step %d" % t
        assert torch.equal(ga.scores, gb.scores), "running scores differ at step %d" % t
        assert torch.equal(oa.view(torch.int16) if oa.dtype == torch.bfloat16 else oa,
                           ob.view(torch.int16) if ob.dtype == torch.bfloat16 else ob), \
            "attention outputs differ at step %d" % t
        assert torch.equal(ga.k, gb.k) and torch.equal(ga.v, gb.v)
        assert not torch.isnan(ob.float()).any()


@pytest.mark.gpu
def test_static_scratch_decode_matches_workspace_decode():
    big = synth.scaled(synth.C3, name="static_big", batch=1, n_q_heads=32, n_kv_heads=8,
                       budget=2048, recent=64, seq_len=8192, window=8)      # 0.8 MiB of scratch
    small = synth.scaled(synth.C3, name="static_small", batch=2, n_q_heads=6, n_kv_heads=2,
                         budget=333, recent=5, seq_len=2000, window=8)      # ragged, group of 3
    print("case", big.name, flush=True)
    _run_both(big, 11, steps=3)
    print("case", small.name, "(after the larger one: the buffer holds its leftovers)", flush=True)
    _run_both(small, 12, steps=3)
    # many heads: one workgroup per head, no scratch at all
    wide = synth.scaled(synth.C3, name="static_wide", batch=16, n_q_heads=16, n_kv_heads=8,
                        budget=70, recent=8, seq_len=500, window=8)
    print("case", wide.name, flush=True)
    _run_both(wide, 13, steps=2)
    # fp32 state
    f32 = synth.scaled(synth.C1, name="static_f32", batch=1, n_q_heads=4, n_kv_heads=2,
                       budget=129, recent=3, seq_len=600, window=8)
    print("case", f32.name, flush=True)
    _run_both(f32, 14, steps=2)
