"""Parity of the HIP path (through the C ABI) with the float64 oracle, element
by element on the same seeded inputs: sizes the oracle finishes in seconds,
spanning several tiles and ragged tails, plus the edge cases."""
import math

import numpy as np
import pytest

import oracle
from oracle import SCALE_ADAPTIVE, SCALE_FIXED
from paper_2506_03762_amd import synth
from tests import harness as H
from tests.harness import Opts

pytestmark = pytest.mark.gpu


def check_prefill(w, opts=Opts(), decode_steps=0, layer=0):
    print("case", w.name, w.dtype, "n", w.seq_len, "Hq/Hkv", w.n_q_heads, w.n_kv_heads,
          "d", w.head_dim, "B", w.budget, "Br", w.recent, opts, flush=True)
    inputs = synth.make_prefill(w, layer)
    gpu = H.run_prefill_gpu(w, opts, inputs)
    ref = H.run_prefill_oracle(w, opts, inputs)
    H.assert_scores_close(gpu.scores, ref.scores, w, opts)
    excused = H.assert_sets_match(gpu.idx, ref.idx, ref.extra["rank_scores"], w, sink=opts.sink,
                                  opts=opts)
    H.assert_compact_matches(gpu, w, inputs[1], inputs[2])
    if decode_steps:
        flips = H.run_and_check_decode(w, gpu, ref, decode_steps, opts)
        assert flips <= 1
    return gpu, ref, excused


# ------------------------------------------------------------------- fp32 --
def test_c1_tiny_fp32_exact_config():
    gpu, ref, excused = check_prefill(synth.C1, decode_steps=8)
    assert excused == 0
    assert H.max_rel_err(gpu.scores, ref.scores, synth.C1) < 1e-5


@pytest.mark.parametrize("opts", [
    Opts(value_prior=False),
    Opts(scale_mode=SCALE_FIXED, fixed_scale=0.125),
    Opts(window=512, scale_mode=SCALE_FIXED, fixed_scale=0.125, value_prior=False),  # H2O
    Opts(window=512),                                   # full accumulation, adaptive + floor
    Opts(lambda_floor=0.0, pool=1),
    Opts(window=1, pool=15),
    Opts(scale_mode=SCALE_FIXED, fixed_scale=0.0, value_prior=False),  # uniform rows
])
def test_fp32_switches(opts):
    check_prefill(synth.C1, opts)


@pytest.mark.parametrize("kw", [
    dict(seq_len=515, budget=131, recent=17, window=29),             # ragged everything
    dict(seq_len=300, head_dim=128, n_q_heads=4, n_kv_heads=2, budget=64, recent=8, window=24),
    dict(seq_len=257, batch=3, n_q_heads=6, n_kv_heads=2, budget=40, recent=0, window=16),
    dict(seq_len=96, budget=96, recent=32, window=32),               # keep everything
    dict(seq_len=64, budget=16, recent=16, window=8),                # recents only
    dict(seq_len=33, budget=9, recent=3, window=33),
])
def test_fp32_shapes(kw):
    w = synth.scaled(synth.C1, name="c1_variant", **kw)
    check_prefill(w, decode_steps=3)


# ------------------------------------------------------------------- bf16 --
BF = synth.scaled(synth.C3, name="bf16_small", seq_len=1536, n_q_heads=8, n_kv_heads=2,
                  budget=192, recent=32, window=32)


def test_bf16_small_gqa_with_rope():
    gpu, ref, excused = check_prefill(BF, decode_steps=6)
    assert H.max_rel_err(gpu.scores, ref.scores, BF) < 2e-3   # fp32 accumulation: far inside 2e-2


@pytest.mark.parametrize("opts", [
    Opts(value_prior=False),
    Opts(scale_mode=SCALE_FIXED, fixed_scale=1 / math.sqrt(128), value_prior=False),
    Opts(window=1536, scale_mode=SCALE_FIXED, fixed_scale=1 / math.sqrt(128), value_prior=False),
    Opts(window=1536),
    Opts(window=1, lambda_floor=0.0, pool=3),
    Opts(window=100, pool=31),
])
def test_bf16_switches(opts):
    check_prefill(BF, opts)


@pytest.mark.parametrize("kw", [
    dict(seq_len=1573, window=37, budget=211, recent=19),                      # ragged tail
    dict(seq_len=700, n_q_heads=4, n_kv_heads=4, window=64, budget=128, recent=64),   # MHA
    dict(seq_len=640, n_q_heads=16, n_kv_heads=2, window=48, budget=100, recent=10),  # G=8
    dict(seq_len=520, head_dim=64, n_q_heads=4, n_kv_heads=2, window=20, budget=64, recent=8),
    dict(seq_len=300, batch=3, n_q_heads=2, n_kv_heads=1, window=300, budget=50, recent=5),
    dict(seq_len=200, n_q_heads=6, n_kv_heads=2, window=40, budget=200, recent=40),   # G=3, keep all
    dict(seq_len=31, n_q_heads=2, n_kv_heads=2, window=31, budget=8, recent=8),       # below one tile
])
def test_bf16_shapes(kw):
    w = synth.scaled(BF, name="bf16_variant", **kw)
    check_prefill(w, decode_steps=3)


@pytest.mark.parametrize("kw,pool", [
    (dict(seq_len=1573, n_q_heads=8, n_kv_heads=2, window=64, budget=211, recent=19), 7),   # ragged
    (dict(seq_len=2304, n_q_heads=4, n_kv_heads=1, window=64, budget=300, recent=64), 17),  # widest halo
    (dict(seq_len=2304, n_q_heads=4, n_kv_heads=1, window=64, budget=300, recent=64), 19),  # own launch
    (dict(seq_len=257, n_q_heads=8, n_kv_heads=2, window=57, budget=64, recent=8), 3),      # 1 key in step 2
    (dict(seq_len=100, n_q_heads=4, n_kv_heads=1, window=64, budget=32, recent=4), 1),      # no pooling
    (dict(seq_len=900, batch=2, head_dim=64, n_q_heads=16, n_kv_heads=2, window=32, budget=128,
          recent=32), 5),                                                                   # d = 64
    (dict(seq_len=5000, n_q_heads=12, n_kv_heads=3, window=60, budget=500, recent=60), 9),  # 240 rows
    # 32 problems: key ranges of 1024 keys, pooled in two pieces with the halo between them
    (dict(seq_len=13001, batch=4, n_q_heads=32, n_kv_heads=8, window=64, budget=1000, recent=64), 7),
])
def test_bf16_full_query_tile_forms_the_value_prior_inside_pass_1(kw, pool):
    """Tiles of 225 - 256 flattened rows (eight 32-row blocks): pass 1 loads the value rows
    under its tile arithmetic and pools their norms itself; ragged ends, chunk borders, the
    widest pooling halo it takes (17) and the width beyond it (a launch of its own)."""
    w = synth.scaled(BF, name="bf16_full_tile", **kw)
    assert 224 < (w.n_q_heads // w.n_kv_heads) * w.window <= 256
    check_prefill(w, Opts(pool=pool), decode_steps=2)


def test_c2_llama2_7b_layer():
    gpu, ref, excused = check_prefill(synth.C2, decode_steps=4)
    print("C2 excused near-ties:", excused)


def random_case(seed):
    """One shape and switch set drawn from the whole argument space (seeded)."""
    rng = np.random.default_rng([77, seed])
    bf = bool(rng.integers(2))
    n = int(rng.choice([rng.integers(2, 80), rng.integers(80, 600), rng.integers(600, 2200)]))
    G = int(rng.choice([1, 2, 3, 4, 8]))
    Hkv = int(rng.integers(1, 4))
    budget = int(rng.integers(1, n + 1))
    recent = int(rng.integers(0, budget + 1))
    window = int(rng.choice([1, rng.integers(1, min(n, 96) + 1), n])) if rng.integers(4) == 0 \
        else int(rng.integers(1, min(n, 96) + 1))
    w = synth.scaled(BF if bf else synth.C1, name="random_%d" % seed, seq_len=n,
                     batch=int(rng.integers(1, 3)), n_q_heads=G * Hkv, n_kv_heads=Hkv,
                     head_dim=int(rng.choice([64, 128])), window=window, budget=budget,
                     recent=recent)
    fixed = rng.integers(3) == 0
    opts = Opts(scale_mode=SCALE_FIXED if fixed else SCALE_ADAPTIVE,
                fixed_scale=float(rng.uniform(0.0, 0.3)) if fixed else 0.0,
                lambda_floor=float(rng.choice([-1.0, 0.0, 0.05])),
                value_prior=bool(rng.integers(2)), pool=int(2 * rng.integers(0, 8) + 1),
                score_pool=int(rng.choice([0, 0, 3, 7])))
    return w, opts


@pytest.mark.parametrize("seed", range(64))
def test_random_shapes_and_switches(seed):
    w, opts = random_case(seed)
    check_prefill(w, opts, decode_steps=24 if seed % 4 == 0 else 2)


def test_large_logits_do_not_overflow():
    """Queries and keys 20x larger than usual (raw dots in the thousands, scaled logits in the
    hundreds): both passes work relative to the row maximum, so nothing overflows and the
    near-one-hot rows still match the oracle.  Most keys then score below the float32 range
    (the oracle's float64 still tells them apart), so they count as ties in the selection."""
    for w, opts in ((BF, Opts()), (BF, Opts(window=1536, scale_mode=SCALE_FIXED, fixed_scale=0.3,
                                            value_prior=False)),
                    (synth.C1, Opts(scale_mode=SCALE_FIXED, fixed_scale=1.0))):
        Q, K, V = synth.make_prefill(w, 0)
        big = (synth.round_bf16(Q * 20.0), synth.round_bf16(K * 20.0), V) if w.dtype == "bf16" \
            else ((Q * 20.0).astype(np.float32).astype(np.float64),
                  (K * 20.0).astype(np.float32).astype(np.float64), V)
        gpu = H.run_prefill_gpu(w, opts, big)
        ref = H.run_prefill_oracle(w, opts, big)
        assert np.all(np.isfinite(gpu.scores))
        if w.dtype == "bf16":
            H.assert_scores_close(gpu.scores, ref.scores, w, opts)
        else:
            # the relative error of exp(x) is the absolute error of x, and a float32 dot
            # product 400x larger carries a 400x larger absolute error: 1e-5 becomes 4e-3
            np.testing.assert_allclose(gpu.scores, ref.scores, rtol=4e-3, atol=1e-6)
            continue
        # scores below the float32 range are zero on the kernel's side: equal keys there
        flushed = np.where(ref.scores < 1.2e-38, 0.0, ref.scores)
        H.assert_sets_match(gpu.idx, ref.idx, flushed, w, max_excused_frac=1.0)


# ------------------------------------------- scores from given normalisers --
def check_scores_from_lse(w, opts, layer=0):
    """The row normalisers come from the oracle, rounded to float32 as a forward pass would
    hand them over; the expected scores are the oracle's for exactly those normalisers."""
    print("lse case", w.name, w.dtype, "n", w.seq_len, "Hq/Hkv", w.n_q_heads, w.n_kv_heads,
          opts, flush=True)
    inputs = synth.make_prefill(w, layer)
    cfg = H.oracle_cfg(w, opts)
    lse32 = oracle.row_lse(inputs[0], inputs[1], cfg).astype(np.float32)
    got = H.run_scores_from_lse_gpu(w, opts, inputs, lse32)
    want = oracle.prefill_scores_lse(*inputs, lse32.astype(np.float64), cfg)
    H.assert_scores_close(got, want, w, opts)
    # and they are the scores of the two-pass entry point (float32 rounding of lse aside)
    full = oracle.prefill_scores(*inputs, cfg)
    np.testing.assert_allclose(got, full, rtol=max(H.rtol_of(w), 1e-4), atol=H.atol_of(w, opts))
    return inputs, cfg, lse32, got


@pytest.mark.parametrize("opts", [
    Opts(scale_mode=SCALE_FIXED, fixed_scale=0.125),                       # the forward's scale
    Opts(scale_mode=SCALE_FIXED, fixed_scale=0.125, value_prior=False),
    Opts(window=512, scale_mode=SCALE_FIXED, fixed_scale=0.125, value_prior=False),  # H2O
    Opts(),                                                                # adaptive-scale lse
])
def test_scores_from_lse_fp32(opts):
    check_scores_from_lse(synth.C1, opts)


@pytest.mark.parametrize("opts", [
    Opts(scale_mode=SCALE_FIXED, fixed_scale=1 / math.sqrt(128)),
    Opts(scale_mode=SCALE_FIXED, fixed_scale=1 / math.sqrt(128), value_prior=False),
    Opts(window=1536, scale_mode=SCALE_FIXED, fixed_scale=1 / math.sqrt(128), value_prior=False),
    Opts(window=1536, scale_mode=SCALE_FIXED, fixed_scale=1 / math.sqrt(128)),
    Opts(window=100, pool=31),
])
def test_scores_from_lse_bf16(opts):
    check_scores_from_lse(BF, opts)


@pytest.mark.parametrize("kw", [
    dict(seq_len=1573, window=37, budget=211, recent=19),                      # ragged tail
    dict(seq_len=640, n_q_heads=16, n_kv_heads=2, window=48, budget=100, recent=10),  # G=8
    dict(seq_len=520, head_dim=64, n_q_heads=4, n_kv_heads=2, window=20, budget=64, recent=8),
    dict(seq_len=300, batch=3, n_q_heads=2, n_kv_heads=1, window=300, budget=50, recent=5),
    dict(seq_len=31, n_q_heads=2, n_kv_heads=2, window=31, budget=8, recent=8),       # below one tile
])
def test_scores_from_lse_bf16_shapes(kw):
    w = synth.scaled(BF, name="bf16_lse_variant", **kw)
    check_scores_from_lse(w, Opts(scale_mode=SCALE_FIXED, fixed_scale=w.head_dim ** -0.5))


def test_scores_from_lse_follow_the_given_normaliser():
    """A normaliser shifted by log 2 for one query head halves that head's share: the library
    uses the caller's values, it does not renormalise."""
    opts = Opts(scale_mode=SCALE_FIXED, fixed_scale=1 / math.sqrt(128), value_prior=False)
    inputs, cfg, lse32, _ = check_scores_from_lse(BF, opts)
    shifted = lse32.copy()
    shifted[:, 1] += np.float32(math.log(2.0))
    got = H.run_scores_from_lse_gpu(BF, opts, inputs, shifted)
    want = oracle.prefill_scores_lse(*inputs, shifted.astype(np.float64), cfg)
    H.assert_scores_close(got, want, BF, opts)
    assert np.max(np.abs(got[:, 0] - oracle.prefill_scores(*inputs, cfg)[:, 0])) > 1e-3


@pytest.mark.parametrize("w", [
    BF,
    # a full 256-row tile: pass 1 loads the value rows with the key fragments' addressing
    synth.scaled(BF, name="bf16_full_tile_strided", seq_len=1100, n_q_heads=8, n_kv_heads=2,
                 window=64, budget=150, recent=64),
], ids=lambda w: w.name)
def test_strided_inputs_token_major_layout(w):
    """Q/K/V stored [b, n, h, d] and passed by strides give the same result."""
    import torch
    from paper_2506_03762_amd import binding as B
    Q, K, V = synth.make_prefill(w)
    opts = Opts()
    dense = H.run_prefill_gpu(w, opts, (Q, K, V))
    q, k, v = (H.to_device(np.ascontiguousarray(a.transpose(0, 2, 1, 3)), w.dtype).permute(0, 2, 1, 3)
               for a in (Q, K, V))
    p = H.gpu_params(w, opts).with_strides(q, k, v)
    assert p.q_stride[2] == w.n_q_heads * w.head_dim
    ws = B.alloc_workspace(p)
    scores = torch.empty((w.batch, w.n_kv_heads, w.seq_len), dtype=torch.float32, device="cuda")
    B.aha_prefill_scores(p, q, k, v, scores, ws)
    assert np.array_equal(scores.cpu().numpy().astype(np.float64), dense.scores)


def test_two_host_threads_on_their_own_streams():
    """The boundary is called from two host threads at once, each on a stream of its own with
    its own buffers (the library keeps its last error per thread and its one-time device
    set-up behind a once-flag): every call gives the single-threaded result."""
    import threading
    import torch
    shapes = [BF, synth.scaled(BF, name="bf16_thread_b", seq_len=1100, n_q_heads=8, n_kv_heads=2,
                               window=64, budget=150, recent=64)]
    want = [H.run_prefill_gpu(w) for w in shapes]
    errors = []

    def worker(i):
        try:
            w = shapes[i]
            with torch.cuda.stream(torch.cuda.Stream()):
                for _ in range(6):
                    got = H.run_prefill_gpu(w)
                    assert np.array_equal(got.scores, want[i].scores)
                    assert np.array_equal(got.idx, want[i].idx)
        except BaseException as e:  # noqa: BLE001 - reported by the main thread
            errors.append((i, repr(e)))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors


def test_repeat_calls_are_bit_identical():
    a = H.run_prefill_gpu(BF)
    b = H.run_prefill_gpu(BF)
    assert np.array_equal(a.scores, b.scores) and np.array_equal(a.idx, b.idx)


# ------------------------------------------------------------------ top-k --
def topk_both(scores32, budget, recent, score_pool=0, sink=0):
    import torch
    from paper_2506_03762_amd import binding as B
    b, h, n = scores32.shape
    p = B.Params(batch=b, n_q_heads=h, n_kv_heads=h, head_dim=128, seq_len=n, window=1,
                 budget=budget, recent=recent, score_pool=score_pool, sink=sink)
    idx = torch.full((b, h, budget), -5, dtype=torch.int32, device="cuda")
    ws = B.alloc_workspace(p)
    ws.fill_(0xA5)
    B.aha_select_topk(p, torch.from_numpy(scores32).cuda(), idx, ws)
    return idx.cpu().numpy(), oracle.select_topk_pooled(scores32.astype(np.float64), budget, recent,
                                                        score_pool, sink)


@pytest.mark.parametrize("n,budget,recent", [
    (32768, 2048, 64), (32768, 1024, 64), (16384, 3276, 64), (4096, 512, 64), (1000, 1000, 10),
    (777, 1, 0), (777, 1, 1), (5, 3, 1), (1, 1, 0), (40000, 5000, 100),
    (65600, 4096, 64),      # the last length whose keys still fit the register file
    (100000, 9000, 100),    # beyond it: keys are re-read in every pass
    (131072, 8192, 128),
])
def test_topk_bit_exact_on_random_and_tied_scores(n, budget, recent):
    rng = np.random.default_rng(n + budget)
    heavy = np.exp(rng.standard_normal((2, 3, n)) * 3).astype(np.float32)      # wide range
    tied = (rng.integers(0, 7, (2, 3, n)) / 8.0).astype(np.float32)            # many exact ties
    const = np.full((1, 2, n), 0.25, np.float32)
    zeros = np.zeros((1, 1, n), np.float32)
    narrow = (1.0 + rng.random((1, 2, n)) * 1e-6).astype(np.float32)           # keys differ in low bits
    for s in (heavy, tied, const, zeros, narrow):
        got, want = topk_both(s, budget, recent)
        assert np.array_equal(got, want)


@pytest.mark.parametrize("n,budget,recent,pool", [
    (32768, 2048, 64, 7), (4096, 512, 64, 3), (1000, 300, 10, 15), (100000, 9000, 100, 5),
    (37, 9, 3, 7), (5, 3, 1, 255),
])
def test_topk_on_pooled_scores(n, budget, recent, pool):
    """Selection on smoothed scores.  The kernel pools in float32 (at most `pool` additions of
    non-negative terms and one division: relative error <= (pool + 1) * 2^-24), the oracle in
    float64, so the sets are equal except for candidates whose float64 pooled score lies
    within that bound of the selection threshold; exactly representable inputs agree bit
    for bit."""
    rng = np.random.default_rng(n + pool)
    heavy = np.exp(rng.standard_normal((2, 3, n)) * 3).astype(np.float32)
    tied = (rng.integers(0, 7, (2, 3, n)) / 8.0).astype(np.float32)
    spikes = np.zeros((1, 2, n), np.float32)
    spikes[..., rng.integers(0, n, max(1, n // 50))] = 1.0
    rtol = (pool + 1) * 2.0 ** -24
    for name, s in (("heavy", heavy), ("tied", tied), ("spikes", spikes)):
        got, want = topk_both(s, budget, recent, pool)
        rank = oracle.pool_scores(s.astype(np.float64), pool)
        excused = H.sets_match(got, want, rank, n, budget, recent, rtol)
        print("pooled top-k", name, "excused near-ties:", excused, flush=True)
        if name == "spikes":   # sums of ones are exact in both precisions
            assert excused == 0


def test_prefill_with_pooled_selection_end_to_end():
    """Scores -> pooled selection -> compaction -> decode: the retained set follows the pooled
    ranking, the cache is seeded with the unpooled scores."""
    gpu, ref, excused = check_prefill(BF, Opts(score_pool=7), decode_steps=4)
    plain = H.run_prefill_oracle(BF, Opts(), synth.make_prefill(BF, 0))
    assert not np.array_equal(ref.idx, plain.idx)     # the smoothing changes what is kept
    check_prefill(synth.C1, Opts(score_pool=5), decode_steps=3)


# ----------------------------------------------------------------- decode --
def test_decode_many_steps_gqa4_bf16():
    w = synth.scaled(BF, name="bf16_decode", seq_len=900, n_q_heads=16, n_kv_heads=4,
                     budget=130, recent=20, window=32, batch=2)
    check_prefill(w, decode_steps=40)


def test_decode_many_heads_single_launch_path():
    """128 or more (batch, KV head) problems: one workgroup per head, no split."""
    w = synth.scaled(BF, name="bf16_decode_wide", seq_len=300, n_q_heads=16, n_kv_heads=8,
                     budget=70, recent=8, window=16, batch=16)
    check_prefill(w, decode_steps=5)
    w = synth.scaled(synth.C1, name="f32_decode_wide", seq_len=200, n_q_heads=8, n_kv_heads=8,
                     budget=33, recent=4, window=8, batch=16)
    check_prefill(w, decode_steps=5)


@pytest.mark.parametrize("G,d,budget,recent", [
    (3, 128, 70, 8),      # two whole 32-slot blocks and seven leftover slots
    (4, 128, 31, 4),      # live slots = one block exactly: the free slot sits inside it
    (8, 128, 20, 3),      # fewer live slots than a block: no matrix block at all
    (8, 128, 160, 16),    # five blocks over sixteen waves, one leftover slot
    (8, 64, 95, 9),       # d = 64
    (5, 128, 64, 64),     # every slot protected but the new one's predecessors
])
def test_decode_wide_groups_single_launch_path(G, d, budget, recent):
    """Grouped-query attention with three or more query heads per KV head on the
    one-workgroup-per-head path (bf16): the dots of whole 32-slot blocks come from the matrix
    core, the leftover slots and the free slot from the vector ALU.  Many steps, so that the free
    slot wanders through blocks and leftovers."""
    w = synth.scaled(BF, name="bf16_decode_wide_gqa", seq_len=200, head_dim=d, n_q_heads=8 * G,
                     n_kv_heads=8, budget=budget, recent=recent, window=16, batch=16)
    check_prefill(w, decode_steps=12)


def test_decode_fixed_scale_and_no_recent_fp32():
    w = synth.scaled(synth.C1, name="f32_decode", budget=60, recent=0, window=16)
    check_prefill(w, Opts(scale_mode=SCALE_FIXED, fixed_scale=0.125), decode_steps=20)


def test_decode_extra_slots_are_ignored():
    """cache_slots larger than budget + 1: the surplus slots stay untouched."""
    import torch
    from paper_2506_03762_amd import binding as B
    w = BF
    ref = H.run_prefill_oracle(w)
    p = H.gpu_params(w)
    oc = oracle.compact_kv(ref.cache.K[:, :, :w.budget], ref.cache.V[:, :, :w.budget],
                           ref.cache.F[:, :, :w.budget],
                           np.broadcast_to(np.arange(w.budget, dtype=np.int32),
                                           ref.idx.shape), slots=w.budget + 5)
    oc.pos[:, :, :w.budget] = ref.cache.pos[:, :, :w.budget]
    oc.F = oc.F.astype(np.float32).astype(np.float64)
    gc = H.upload_cache(oc, w, p)
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device="cuda")
    q, k, v = synth.make_decode_inputs(w, 0)
    B.aha_decode_step(p, H.to_device(q, "bf16"), H.to_device(k, "bf16"), H.to_device(v, "bf16"),
                      gc.k, gc.v, gc.scores, gc.pos, gc.free_slot, w.seq_len + 1, out,
                      B.alloc_workspace(p))
    oracle.decode_step(oc, q, k, v, w.seq_len + 1, H.oracle_cfg(w, Opts()))
    assert np.array_equal(gc.pos.cpu().numpy(), oc.pos)
    assert np.array_equal(gc.free_slot.cpu().numpy(), oc.free_slot)
    assert np.all(gc.pos.cpu().numpy()[:, :, w.budget + 1:] == -1)


@pytest.mark.parametrize("base,batch,hq,hkv,budget,recent", [
    (BF, 1, 8, 2, 300, 2),            # few heads: slots split over workgroups, merge launch
    (BF, 16, 8, 8, 70, 3),            # 128 heads: one workgroup per head
    (synth.C1, 1, 2, 2, 129, 1),      # fp32, split path
    (synth.C1, 16, 8, 8, 40, 2),      # fp32, single launch
])
def test_decode_equal_minima_evict_the_highest_position(base, batch, hq, hkv, budget, recent):
    """Tie rule of the generation step on both decode paths.  Scale 0 gives every slot the
    same increment, so equal running scores stay equal and only the rule picks the victim:
    positions and free slots must equal the oracle's exactly (no near-tie allowance), over
    steps in which all, two, or none of the minima tie."""
    import torch
    from paper_2506_03762_amd import binding as B
    w = synth.scaled(base, name="tie_break", batch=batch, n_q_heads=hq, n_kv_heads=hkv,
                     budget=budget, recent=recent, seq_len=4 * budget, window=8)
    opts = Opts(scale_mode=SCALE_FIXED, fixed_scale=0.0)
    p, cfg = H.gpu_params(w, opts), H.oracle_cfg(w, opts)
    d = w.head_dim
    oc = H.random_cache(w, budget, F_fill=0.5)
    for pr in np.ndindex(batch, hkv):
        if pr[1] % 2:   # odd heads: a few equal minima below the rest
            occupied = np.flatnonzero(oc.pos[pr] >= 0)
            oc.F[pr][occupied[:5]] = 0.25
    gc = H.upload_cache(oc, w, p)
    ws = B.alloc_workspace(p)
    out = torch.empty((batch, hq, d), dtype=B.torch_dtype(p.dtype), device="cuda")
    for t in range(4):
        q, k, v = synth.make_decode_inputs(w, t)
        c_t = w.seq_len + t + 1
        B.aha_decode_step(p, H.to_device(q, w.dtype), H.to_device(k, w.dtype),
                          H.to_device(v, w.dtype), gc.k, gc.v, gc.scores, gc.pos, gc.free_slot,
                          c_t, out, ws)
        oracle.decode_step(oc, q, k, v, c_t, cfg)
        torch.cuda.synchronize()
        assert np.array_equal(gc.free_slot.cpu().numpy(), oc.free_slot), "victims differ at step %d" % t
        assert np.array_equal(gc.pos.cpu().numpy(), oc.pos)
        np.testing.assert_allclose(gc.scores.cpu().numpy()[oc.pos >= 0], oc.F[oc.pos >= 0], rtol=1e-6)


def test_decode_split_path_raises_the_split_count_for_large_budgets():
    """Few heads with a budget whose dots do not fit a split workgroup's LDS at the default
    split count (64 heads -> 4 splits of 1626 slots x 8 query heads = 68 KB): the plan must
    use more splits, and the steps must match the oracle."""
    w = synth.scaled(BF, name="decode_large_budget", batch=8, n_q_heads=64, n_kv_heads=8,
                     budget=6500, recent=64, seq_len=20000, window=8)
    oc = H.random_cache(w, 5)
    ref = H.Result(None, None, oc)
    flips = H.run_and_check_decode(w, None, ref, steps=3)
    assert flips == 0


@pytest.mark.parametrize("base", [BF, synth.C1], ids=["bf16", "f32"])
def test_all_zero_value_head_keeps_unrefined_scores(base):
    """A head whose value rows are all zero has max(gamma) = 0: gamma_bar is 1 there on both
    sides, and the other heads are refined as usual."""
    w = synth.scaled(base, name="zero_v", seq_len=700, n_q_heads=4, n_kv_heads=2, budget=90,
                     recent=16, window=24)
    Q, K, V = synth.make_prefill(w)
    V = V.copy()
    V[0, 1] = 0.0
    gpu = H.run_prefill_gpu(w, Opts(), (Q, K, V))
    ref = H.run_prefill_oracle(w, Opts(), (Q, K, V))
    H.assert_scores_close(gpu.scores, ref.scores, w)
    H.assert_sets_match(gpu.idx, ref.idx, ref.scores, w)
    off = H.run_prefill_gpu(w, Opts(value_prior=False), (Q, K, V))
    assert np.array_equal(gpu.scores[0, 1], off.scores[0, 1])


# ------------------------------------------ sink tokens, value prior in the loop --
@pytest.mark.parametrize("n,budget,recent,sink", [
    (32768, 2048, 64, 4), (4096, 512, 64, 4), (1000, 300, 10, 290), (777, 9, 5, 4),   # last: static policy
    (100000, 9000, 100, 7), (131072, 8192, 128, 4), (37, 9, 3, 1), (5, 5, 1, 4),
])
def test_topk_with_sink_tokens_bit_exact(n, budget, recent, sink):
    rng = np.random.default_rng(n + sink)
    heavy = np.exp(rng.standard_normal((2, 3, n)) * 3).astype(np.float32)
    heavy[..., :sink] = 0.0                                          # sinks kept whatever they score
    tied = (rng.integers(0, 7, (2, 3, n)) / 8.0).astype(np.float32)
    const = np.full((1, 2, n), 0.25, np.float32)
    for s in (heavy, tied, const):
        got, want = topk_both(s, budget, recent, sink=sink)
        assert np.array_equal(got, want)
        assert np.array_equal(got[..., :sink], np.broadcast_to(np.arange(sink), got[..., :sink].shape))


def test_sink_policy_end_to_end_with_decode():
    """Scores -> selection with 4 sink tokens -> compaction -> generation steps in which the
    sinks are never evicted, on both decode paths and both dtypes."""
    check_prefill(BF, Opts(sink=4), decode_steps=12)
    check_prefill(synth.C1, Opts(sink=4), decode_steps=12)
    wide = synth.scaled(BF, name="bf16_sink_wide", seq_len=300, n_q_heads=16, n_kv_heads=8,
                        budget=70, recent=8, window=16, batch=16)
    check_prefill(wide, Opts(sink=3), decode_steps=8)
    # sinks with scores far below everything else must still survive generation
    w = synth.scaled(BF, name="sink_low", batch=1, n_q_heads=8, n_kv_heads=2, budget=64,
                     recent=4, seq_len=400, window=8)
    oc = H.random_cache(w, 21)
    for pr in np.ndindex(1, 2):
        pos = oc.pos[pr]
        for sp in range(3):                                         # make sure 0, 1, 2 are cached
            hit = np.flatnonzero(pos == sp)
            slot = hit[0] if hit.size else np.flatnonzero((pos >= 3) & (pos < w.seq_len - w.recent))[0]
            pos[slot] = sp
            oc.F[pr][slot] = 0.0                                    # ... with the lowest scores
    flips = H.run_and_check_decode(w, None, H.Result(None, None, oc), steps=6, opts=Opts(sink=3))
    assert flips == 0


@pytest.mark.parametrize("base,batch,hq,hkv,budget", [
    (BF, 1, 8, 2, 300),            # few heads: split + merge launches
    (BF, 16, 8, 8, 70),            # one workgroup per head
    (synth.C1, 2, 4, 2, 129),      # fp32
])
def test_decode_with_value_prior_in_the_loop(base, batch, hq, hkv, budget):
    """Generation with the value prior applied to what is added to the running scores
    (gamma_bar = ||v||^2 / max over the live slots): lock-step with the oracle; value rows of
    very different norms, so that the option changes the victims."""
    w = synth.scaled(base, name="decode_vp", batch=batch, n_q_heads=hq, n_kv_heads=hkv,
                     budget=budget, recent=8, seq_len=4 * budget, window=8)
    oc = H.random_cache(w, 31 + budget)
    scale = np.random.default_rng(5).uniform(0.1, 3.0, oc.V.shape[:3])[..., None]
    oc.V = synth.store_round((oc.V * scale).astype(np.float32), w.dtype).astype(np.float64)
    ref = H.Result(None, None, oc)
    plain = oracle.Cache(oc.K.copy(), oc.V.copy(), oc.F.copy(), oc.pos.copy(), oc.free_slot.copy())
    flips = H.run_and_check_decode(w, None, ref, steps=10, opts=Opts(decode_value_prior=True))
    assert flips <= 1
    # the option is not a no-op on this state: the plain loop ends elsewhere
    cfg = H.oracle_cfg(w, Opts())
    for t in range(10):
        q, k, v = synth.make_decode_inputs(w, t)
        oracle.decode_step(plain, q, k, v, w.seq_len + t + 1, cfg)
    assert not np.allclose(np.sort(plain.F, axis=-1), np.sort(oc.F, axis=-1))
