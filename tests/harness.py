"""Shared helpers of the parity tests: run the HIP path through the C ABI, run
the float64 oracle on the same seeded inputs, and compare by the stated rule.

Tolerances (the target's): scores within 1e-5 relative for fp32 inputs and
2e-2 relative for bf16 inputs with fp32 accumulation, plus an absolute floor
of rtol * (mean score) * 1e-3 for entries where fp32 exp underflows; retained
index sets identical except for indices whose oracle score lies within rtol of
the oracle's selection threshold.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

import oracle
from paper_2506_03762_amd import synth


@dataclass
class Opts:
    """Score switches (the paper's three ablation switches and their knobs)."""
    window: Optional[int] = None       # None: the workload's observation window
    scale_mode: int = oracle.SCALE_ADAPTIVE
    fixed_scale: float = 0.0
    lambda_floor: float = -1.0
    value_prior: bool = True
    pool: int = 7
    score_pool: int = 0                # > 1: the selection ranks pooled scores
    sink: int = 0                      # first tokens always retained (selection and decode)
    decode_value_prior: bool = False   # generation: value prior inside the loop


def rtol_of(w: synth.Workload, opts: "Opts | None" = None) -> float:
    """Relative bar on the scores: 1e-5 for fp32 inputs, 2e-2 for bf16 inputs.  The fp32 bar
    is stated for logits of the workloads' size (the standard scale, a window of tens of rows).
    The relative error of exp(x) is the absolute error of x, and a sum of N fp32 terms carries
    about sqrt(N) roundings: with `opts` given, a scale s times the standard 1/sqrt(d) widens
    the fp32 bar s-fold and more than 4096 accumulated rows per key widen it by
    sqrt(rows / 4096) (the random-shape tests draw scales of up to 0.3 and windows of the whole
    sequence)."""
    if w.dtype != "f32":
        return 2e-2
    rtol = 1e-5
    if opts is not None:
        d = w.head_dim
        if opts.scale_mode == oracle.SCALE_FIXED:
            s_eff = abs(opts.fixed_scale)
        else:  # the largest adaptive scale of the observed rows (the last row's)
            floor = d ** -0.5 if opts.lambda_floor < 0 else opts.lambda_floor
            s_eff = max(floor, math.sqrt(2.0 * max(math.log(w.seq_len / w.budget), 0.0) / d))
        rows = w.group * (opts.window or w.window)
        rtol *= max(1.0, s_eff * math.sqrt(d)) * max(1.0, math.sqrt(rows / 4096.0))
    return rtol


def atol_of(w: synth.Workload, opts: Opts) -> float:
    r = opts.window or w.window
    return rtol_of(w) * (w.group * r / w.seq_len) * 1e-3


def oracle_cfg(w: synth.Workload, opts: Opts) -> oracle.Config:
    return oracle.Config(window=opts.window or w.window, budget=w.budget, recent=w.recent,
                         scale_mode=opts.scale_mode, fixed_scale=opts.fixed_scale,
                         lambda_floor=opts.lambda_floor, value_prior=opts.value_prior,
                         pool=opts.pool, sink=opts.sink,
                         decode_value_prior=opts.decode_value_prior)


@dataclass
class Result:
    scores: np.ndarray                 # [b, Hkv, n] float64
    idx: np.ndarray                    # [b, Hkv, B] int32
    cache: Optional[object] = None     # oracle.Cache or device CompactCache
    extra: dict = field(default_factory=dict)


# ------------------------------------------------------------------ oracle --
def run_prefill_oracle(w: synth.Workload, opts: Opts = Opts(), inputs=None, layer=0) -> Result:
    Q, K, V = inputs if inputs is not None else synth.make_prefill(w, layer)
    cfg = oracle_cfg(w, opts)
    S = oracle.prefill_scores(Q, K, V, cfg)
    idx = oracle.select_topk_pooled(S, w.budget, w.recent, opts.score_pool, opts.sink)
    cache = oracle.compact_kv(K.astype(np.float64), V.astype(np.float64), S, idx,
                              slots=w.budget + 1)
    # the scores that ranked the candidates (near-ties are judged on these)
    rank = oracle.pool_scores(S, opts.score_pool) if opts.score_pool > 1 else S
    return Result(S, idx, cache, extra=dict(rank_scores=rank))


# --------------------------------------------------------------------- GPU --
def to_device(a: np.ndarray, dtype: str):
    from paper_2506_03762_amd import workload
    return workload.to_device(a, dtype)


def gpu_params(w: synth.Workload, opts: Opts = Opts()):
    from paper_2506_03762_amd import workload
    return workload.params_for(w, window=opts.window, scale_mode=opts.scale_mode,
                               fixed_scale=opts.fixed_scale, lambda_floor=opts.lambda_floor,
                               value_prior=opts.value_prior, pool=opts.pool,
                               score_pool=opts.score_pool, sink=opts.sink,
                               decode_value_prior=1 if opts.decode_value_prior else 0)


def run_prefill_gpu(w: synth.Workload, opts: Opts = Opts(), inputs=None, layer=0,
                    poison: bool = True) -> Result:
    """scores -> top-k -> compaction through the C ABI; everything copied back."""
    import torch
    from paper_2506_03762_amd import binding as B
    Q, K, V = inputs if inputs is not None else synth.make_prefill(w, layer)
    q, k, v = (to_device(a, w.dtype) for a in (Q, K, V))
    p = gpu_params(w, opts).with_strides(q, k, v)
    ws = B.alloc_workspace(p)
    b, hk, n = w.batch, w.n_kv_heads, w.seq_len
    scores = torch.empty((b, hk, n), dtype=torch.float32, device="cuda")
    idx = torch.empty((b, hk, w.budget), dtype=torch.int32, device="cuda")
    cache = B.CompactCache.empty(p)
    if poison:  # outputs and scratch start from garbage, never from zeros
        ws.fill_(0xA5)
        scores.fill_(float("nan"))
        idx.fill_(-7)
        cache.scores.fill_(float("nan")); cache.pos.fill_(-9); cache.free_slot.fill_(-9)
    B.aha_prefill_scores(p, q, k, v, scores, ws)
    B.aha_select_topk(p, scores, idx, ws)
    B.aha_compact_kv(p, k, v, scores, idx, cache.k, cache.v, cache.scores, cache.pos,
                     cache.free_slot)
    torch.cuda.synchronize()
    return Result(scores.cpu().numpy().astype(np.float64), idx.cpu().numpy(), cache,
                  extra=dict(p=p, q=q, k=k, v=v, scores=scores, idx=idx, ws=ws))


def run_scores_from_lse_gpu(w: synth.Workload, opts: Opts, inputs, lse) -> np.ndarray:
    """aha_prefill_scores_lse through the C ABI: scores [b, Hkv, n] as float64.  `lse` is the
    [b, Hq, window] float32 array handed to the library."""
    import torch
    from paper_2506_03762_amd import binding as B
    Q, K, V = inputs
    q, k, v = (to_device(a, w.dtype) for a in (Q, K, V))
    p = gpu_params(w, opts).with_strides(q, k, v)
    ws = B.alloc_workspace(p)
    ws.fill_(0xA5)
    scores = torch.full((w.batch, w.n_kv_heads, w.seq_len), float("nan"), dtype=torch.float32,
                        device="cuda")
    lse_d = torch.from_numpy(np.ascontiguousarray(lse, dtype=np.float32)).cuda()
    B.aha_prefill_scores_lse(p, q, k, v, lse_d, scores, ws)
    torch.cuda.synchronize()
    return scores.cpu().numpy().astype(np.float64)


# ----------------------------------------------------------------- compare --
def max_rel_err(got, want, w, opts: Opts = Opts()) -> float:
    atol = atol_of(w, opts)
    return float(np.max(np.abs(got - want) / (np.abs(want) + atol / rtol_of(w))))


def assert_scores_close(got, want, w, opts: Opts = Opts()):
    assert got.shape == want.shape
    assert np.all(np.isfinite(got)), "non-finite scores from the GPU path"
    rtol, atol = rtol_of(w, opts), atol_of(w, opts)
    err = np.abs(got - want)
    bad = err > rtol * np.abs(want) + atol
    if bad.any():
        t = np.unravel_index(np.argmax(err / (rtol * np.abs(want) + atol)), err.shape)
        raise AssertionError("scores differ at %d of %d entries; worst at %s: gpu %.9g oracle %.9g"
                             % (bad.sum(), bad.size, t, got[t], want[t]))


def assert_sets_match(idx_gpu, idx_ref, scores_ref, w, max_excused_frac=0.01, sink=0, opts=None):
    """Retained sets equal, except indices whose oracle score is within rtol of
    the oracle's threshold (the B_s-th largest candidate score).  `scores_ref` are the
    oracle's float64 scores that ranked the candidates (the pooled ones when the selection
    ranks pooled scores).  Returns the number of excused indices."""
    # Pooled scores around one dominant token form a plateau: its pool-width neighbours hold
    # the same large term and differ by terms below fp32 resolution, so the kernel (fp32) sees
    # exact ties, broken by position, where float64 sees an order.  Every swapped index must
    # still be a near-tie; with pooling one swap per problem is allowed on top of the 1 %.
    pooled = opts is not None and opts.score_pool > 1
    return sets_match(idx_gpu, idx_ref, scores_ref, w.seq_len, w.budget, w.recent,
                      rtol_of(w, opts), max_excused_frac, sink, swaps_per_problem=1 if pooled else 0)


def sets_match(idx_gpu, idx_ref, scores_ref, n, B, Br, rtol, max_excused_frac=0.01, sink=0,
               swaps_per_problem=0):
    assert idx_gpu.shape == idx_ref.shape
    excused = 0
    problems = int(np.prod(idx_ref.shape[:-1]))
    for p in np.ndindex(idx_ref.shape[:-1]):
        g, r = idx_gpu[p], idx_ref[p]
        assert np.all(np.diff(g) > 0), "GPU indices not strictly ascending at %s" % (p,)
        assert g.min() >= 0 and g.max() < n
        assert np.array_equal(g[B - Br:], np.arange(n - Br, n)), "recent tokens not kept"
        assert np.array_equal(g[:sink], np.arange(sink)), "sink tokens not kept"
        if np.array_equal(g, r):
            continue
        sel = r[(r < n - Br) & (r >= sink)]
        thr = scores_ref[p][sel].min() if sel.size else 0.0
        diff = np.setxor1d(g, r)
        for j in diff:
            s = scores_ref[p][j]
            assert abs(s - thr) <= rtol * abs(thr), \
                "index %d at %s differs and is not a near-tie: score %.9g threshold %.9g" % (j, p, s, thr)
        excused += diff.size
    assert excused <= max_excused_frac * idx_ref.size + 2 + 2 * swaps_per_problem * problems, \
        "too many near-tie flips: %d" % excused
    return excused


def assert_compact_matches(res_gpu: Result, w, K, V):
    """The GPU's compact cache is an exact gather by the GPU's own index list."""
    c = res_gpu.cache
    import torch
    kc = c.k.float().cpu().numpy(); vc = c.v.float().cpu().numpy()
    fc = c.scores.cpu().numpy(); pos = c.pos.cpu().numpy(); fs = c.free_slot.cpu().numpy()
    B = w.budget
    sc32 = res_gpu.extra["scores"].cpu().numpy()
    for p in np.ndindex(res_gpu.idx.shape[:-1]):
        ix = res_gpu.idx[p]
        assert np.array_equal(kc[p][:B], K[p][ix]) and np.array_equal(vc[p][:B], V[p][ix])
        assert np.array_equal(pos[p][:B], ix) and np.all(pos[p][B:] == -1)
        assert np.array_equal(fc[p][:B], sc32[p][ix]) and np.all(fc[p][B:] == 0)
        assert np.all(kc[p][B:] == 0) and np.all(vc[p][B:] == 0)
        assert fs[p] == B


# ------------------------------------------------------------------ decode --
def upload_cache(ref: oracle.Cache, w: synth.Workload, p):
    """Device cache holding the oracle's state (oracle -> GPU direction only)."""
    import torch
    from paper_2506_03762_amd import binding as B
    c = B.CompactCache.empty(p, slots=ref.K.shape[2])
    c.k.copy_(to_device(ref.K.astype(np.float32), w.dtype))
    c.v.copy_(to_device(ref.V.astype(np.float32), w.dtype))
    c.scores.copy_(torch.from_numpy(ref.F.astype(np.float32)).cuda())
    c.pos.copy_(torch.from_numpy(ref.pos).cuda())
    c.free_slot.copy_(torch.from_numpy(ref.free_slot).cuda())
    return c


def random_cache(w: synth.Workload, seed: int, F_fill=None) -> oracle.Cache:
    """A compact cache that no prefill produced: random K/V rows (rounded to the storage
    dtype), `budget` distinct positions below seq_len - the `recent` last ones, as every
    state reached from a prefill holds them, and a random choice of the earlier ones -
    scattered over budget + 1 slots, one free slot; running scores uniform in (0, 1)
    (float32-representable) or `F_fill`."""
    rng = np.random.default_rng(seed)
    b, hk, d, slots = w.batch, w.n_kv_heads, w.head_dim, w.budget + 1
    K = synth.store_round(rng.standard_normal((b, hk, slots, d), dtype=np.float32), w.dtype).astype(np.float64)
    V = synth.store_round(rng.standard_normal((b, hk, slots, d), dtype=np.float32), w.dtype).astype(np.float64)
    pos = np.empty((b, hk, slots), np.int32)
    fs = np.empty((b, hk), np.int32)
    if F_fill is None:
        F = rng.random((b, hk, slots), dtype=np.float32).astype(np.float64)
    else:
        F = np.full((b, hk, slots), float(F_fill))
    for pr in np.ndindex(b, hk):
        perm = rng.permutation(slots)
        held = np.concatenate([np.arange(w.seq_len - w.recent, w.seq_len),
                               rng.choice(w.seq_len - w.recent, w.budget - w.recent, replace=False)])
        held = held[rng.permutation(w.budget)]
        fs[pr] = perm[-1]
        pos[pr][perm[:-1]] = held
        pos[pr][perm[-1]] = -1
        F[pr][perm[-1]] = 0.0
    return oracle.Cache(K, V, F, pos, fs)


def live_state(pos, F):
    """{position: score} of the occupied slots of one (batch, head)."""
    m = pos >= 0
    return dict(zip(pos[m].tolist(), F[m].tolist()))


def run_and_check_decode(w: synth.Workload, res_gpu: Result, ref: Result, steps: int,
                         opts: Opts = Opts(), check_every: int = 1):
    """Lock-step decode on the GPU and in the oracle, both starting from the
    ORACLE's compacted state (scores rounded to fp32 on both sides)."""
    import torch
    from paper_2506_03762_amd import binding as B
    p = gpu_params(w, opts)
    cfg = oracle_cfg(w, opts)
    oc = oracle.Cache(ref.cache.K.copy(), ref.cache.V.copy(),
                      ref.cache.F.astype(np.float32).astype(np.float64), ref.cache.pos.copy(),
                      ref.cache.free_slot.copy())
    gc = upload_cache(oc, w, p)
    ws = B.alloc_workspace(p)
    ws.fill_(0xA5)
    rtol = rtol_of(w, opts)
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=B.torch_dtype(p.dtype),
                      device="cuda")
    flips = 0
    for t in range(steps):
        c_t = w.seq_len + t + 1
        q, k, v = synth.make_decode_inputs(w, t)
        out.fill_(float("nan"))
        B.aha_decode_step(p, to_device(q, w.dtype), to_device(k, w.dtype), to_device(v, w.dtype),
                          gc.k, gc.v, gc.scores, gc.pos, gc.free_slot, c_t, out, ws)
        o_ref = oracle.decode_step(oc, q, k, v, c_t, cfg)
        if (t + 1) % check_every and t != steps - 1:
            continue
        torch.cuda.synchronize()
        o = out.float().cpu().numpy().astype(np.float64)
        tol = rtol * np.abs(o_ref) + rtol * np.sqrt(np.mean(o_ref ** 2))
        assert np.all(np.abs(o - o_ref) <= tol), "decode output differs at step %d: %g" % (
            t, np.max(np.abs(o - o_ref) / tol))
        gpos, gF, gfs = gc.pos.cpu().numpy(), gc.scores.cpu().numpy(), gc.free_slot.cpu().numpy()
        resync = False
        for pr in np.ndindex(gpos.shape[:2]):
            got, want = live_state(gpos[pr], gF[pr]), live_state(oc.pos[pr], oc.F[pr])
            assert len(got) == w.budget and gpos[pr][gfs[pr]] == -1
            if got.keys() != want.keys():
                # a different victim is acceptable only between near-tied scores
                (a,) = got.keys() - want.keys()
                (bb,) = want.keys() - got.keys()
                assert abs(got[a] - want[bb]) <= 2 * rtol * abs(want[bb]) + 1e-30, \
                    "step %d %s: victims differ without a near-tie" % (t, pr)
                flips += 1
                resync = True
                continue
            for pp in want:
                assert abs(got[pp] - want[pp]) <= rtol * abs(want[pp]) + 1e-12, \
                    "step %d %s pos %d: score %.9g vs %.9g" % (t, pr, pp, got[pp], want[pp])
        if resync:
            gc = upload_cache(oc, w, p)
    return flips
