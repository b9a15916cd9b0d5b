"""Row statistics of the observed rows from the HIP path (aha_prefill_row_stats): the
log-sum-exp and the information entropy of Sec. 4.2 against the float64 oracle element by
element, the entropy-against-position curves under the standard and the adaptive scale, and
the hand-over of the log-sum-exp to aha_prefill_scores_lse."""
import math

import numpy as np
import pytest

import oracle
from oracle import SCALE_ADAPTIVE, SCALE_FIXED
from paper_2506_03762_amd import synth
from tests import harness as H
from tests.harness import Opts

pytestmark = pytest.mark.gpu

BF = synth.scaled(synth.C3, name="bf16_small", seq_len=1536, n_q_heads=8, n_kv_heads=2,
                  budget=192, recent=32, window=32)


def run_row_stats(w, opts, Q, K):
    import torch
    from paper_2506_03762_amd import binding as B
    q, k = H.to_device(Q, w.dtype), H.to_device(K, w.dtype)
    p = H.gpu_params(w, opts).with_strides(q, k, k)
    ws = B.alloc_workspace(p)
    ws.fill_(0xA5)
    r = opts.window or w.window
    lse = torch.full((w.batch, w.n_q_heads, r), float("nan"), dtype=torch.float32, device="cuda")
    ent = torch.full((w.batch, w.n_q_heads, r), float("nan"), dtype=torch.float32, device="cuda")
    B.aha_prefill_row_stats(p, q, k, lse, ent, ws)
    only = torch.full_like(ent, float("nan"))
    B.aha_prefill_row_stats(p, q, k, None, only, ws)      # either output alone
    torch.cuda.synchronize()
    assert torch.equal(only, ent)
    return lse.cpu().numpy().astype(np.float64), ent.cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("w,opts", [
    (synth.C1, Opts()),
    (synth.C1, Opts(scale_mode=SCALE_FIXED, fixed_scale=0.125)),
    (synth.C1, Opts(window=512, lambda_floor=0.0)),                       # every row, literal formula
    (synth.C1, Opts(scale_mode=SCALE_FIXED, fixed_scale=0.0)),            # uniform rows: ln c
    (BF, Opts()),
    (BF, Opts(window=1536, scale_mode=SCALE_FIXED, fixed_scale=128 ** -0.5)),   # every row, several tiles
    (BF, Opts(window=1536)),
    (synth.scaled(BF, name="ragged", seq_len=1573, window=37, n_q_heads=6, n_kv_heads=2, head_dim=64),
     Opts()),
    (synth.scaled(BF, name="short", seq_len=31, window=31, n_q_heads=2, n_kv_heads=2, budget=8,
                  recent=8), Opts()),
], ids=lambda x: getattr(x, "name", None))
def test_row_stats_match_the_oracle(w, opts):
    """fp32 inputs: 1e-5 relative (+ 5e-5 nats for the entropy, a difference of two numbers of
    size ~ log2 of the row's sum); bf16 inputs with fp32 accumulation: the dots carry ~1e-6
    relative error on logits of size tens, i.e. ~1e-4 in the exponent."""
    print("case", w.name, opts, flush=True)
    Q, K, _ = synth.make_prefill(w)
    cfg = H.oracle_cfg(w, opts)
    lse, ent = run_row_stats(w, opts, Q, K)
    want_lse = oracle.row_lse(Q, K, cfg)
    want_ent = oracle.row_entropy(Q, K, cfg)
    rtol, atol = (1e-5, 5e-5) if w.dtype == "f32" else (1e-4, 1e-3)
    np.testing.assert_allclose(lse, want_lse, rtol=rtol, atol=atol)
    np.testing.assert_allclose(ent, want_ent, rtol=rtol, atol=atol)
    r = opts.window or w.window
    c = np.arange(w.seq_len - r, w.seq_len) + 1
    assert np.all(ent >= 0) and np.all(ent <= np.log(c) + 1e-4)


def test_entropy_against_position_follows_the_two_expectations():
    """The curves behind the adaptive scale (Sec. 4.2) from the HIP path, on iid N(0,1)
    queries and keys, every position observed (window = n): with the standard scale the mean
    entropy of row i follows ln(i + 1) - 1/2, i.e. grows with the context; with
    lambda_i = sqrt(2 ln(c_i / k) / d) it stays at ln k once c_i exceeds k.  (Loose
    bands: the derivation swaps E log for log E.)  The oracle agrees element by element."""
    n, d, heads, k = 4096, 128, 16, 256      # k^2 >> n, where the derivation's swap holds
    w = synth.scaled(synth.C3, name="gaussian_4k", seq_len=n, n_q_heads=heads, n_kv_heads=heads,
                     budget=k, recent=16, window=n)
    rng = np.random.default_rng(404)
    Q = synth.round_bf16(rng.standard_normal((1, heads, n, d), dtype=np.float32))
    K = synth.round_bf16(rng.standard_normal((1, heads, n, d), dtype=np.float32))
    i = np.arange(n)
    std_opts = Opts(window=n, scale_mode=SCALE_FIXED, fixed_scale=d ** -0.5)
    ada_opts = Opts(window=n, lambda_floor=0.0)
    _, std = run_row_stats(w, std_opts, Q, K)
    _, ada = run_row_stats(w, ada_opts, Q, K)
    for opts, got in ((std_opts, std), (ada_opts, ada)):
        want = oracle.row_entropy(Q, K, H.oracle_cfg(w, opts))
        np.testing.assert_allclose(got, want, rtol=1e-4, atol=1e-3)
    std_curve, ada_curve = std.mean(axis=(0, 1)), ada.mean(axis=(0, 1))
    late = i >= 512
    assert np.max(np.abs(std_curve[late] - (np.log(i[late] + 1) - 0.5))) < 0.2
    # (a sharpened row's entropy scatters much more from row to row than a flat row's: the
    # adaptive curve is judged on means over blocks of 256 positions)
    blocks = ada_curve.reshape(-1, 256).mean(axis=1)
    settled = (np.arange(blocks.size) * 256 + 1) > k       # rows with more keys than the budget
    assert np.max(np.abs(blocks[settled] - math.log(k))) < 0.15
    # the standard row keeps flattening with the context, the adaptive one does not
    assert std_curve[-256:].mean() - std_curve[k:2 * k].mean() > 1.5
    assert abs(blocks[-1] - blocks[settled][0]) < 0.15
    print("entropy at i = 511, 2047, 4095: standard %.2f %.2f %.2f, adaptive %.2f %.2f %.2f (ln k = %.2f)"
          % (std_curve[511], std_curve[2047], std_curve[4095], ada_curve[511], ada_curve[2047],
             ada_curve[4095], math.log(k)), flush=True)


def test_log_sum_exp_hands_over_to_the_single_pass_scores():
    """aha_prefill_row_stats produces what aha_prefill_scores_lse consumes: together they give
    the scores of the two-pass entry point."""
    import torch
    from paper_2506_03762_amd import binding as B
    w = BF
    opts = Opts(scale_mode=SCALE_FIXED, fixed_scale=w.head_dim ** -0.5)
    Q, K, V = synth.make_prefill(w)
    lse, _ = run_row_stats(w, opts, Q, K)
    got = H.run_scores_from_lse_gpu(w, opts, (Q, K, V), lse.astype(np.float32))
    two = H.run_prefill_gpu(w, opts, (Q, K, V))
    H.assert_scores_close(got, two.scores, w, opts)
    ref = H.run_prefill_oracle(w, opts, (Q, K, V))
    H.assert_scores_close(got, ref.scores, w, opts)


# ----------------------------------------- accumulators chosen by a Top-k strategy --
def run_scores_rows(w, opts, inputs, rows):
    import torch
    from paper_2506_03762_amd import binding as B
    Q, K, V = inputs
    q, k, v = (H.to_device(a, w.dtype) for a in (Q, K, V))
    p = H.gpu_params(w, opts).with_strides(q, k, v)
    ws = B.alloc_workspace(p)
    ws.fill_(0xA5)
    scores = torch.full((w.batch, w.n_kv_heads, w.seq_len), float("nan"), dtype=torch.float32,
                        device="cuda")
    B.aha_prefill_scores_rows(p, q, k, v, torch.from_numpy(np.ascontiguousarray(rows, np.int32)).cuda(),
                              scores, ws)
    torch.cuda.synchronize()
    return scores.cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("w,opts", [
    (synth.C1, Opts()),
    (synth.C1, Opts(scale_mode=SCALE_FIXED, fixed_scale=0.0, value_prior=False)),   # closed form
    (BF, Opts()),
    (BF, Opts(value_prior=False, lambda_floor=0.0)),
    (synth.scaled(BF, name="ragged", seq_len=1573, window=37, n_q_heads=6, n_kv_heads=2, head_dim=64),
     Opts()),
    (synth.scaled(BF, name="g8", seq_len=640, window=32, n_q_heads=16, n_kv_heads=2), Opts(pool=3)),
    (synth.scaled(BF, name="one_row", seq_len=300, window=1, n_q_heads=2, n_kv_heads=2, budget=50,
                  recent=5), Opts()),
], ids=lambda x: getattr(x, "name", None))
def test_scores_over_chosen_rows_match_the_oracle(w, opts):
    """aha_prefill_scores_rows: random row positions per (batch, query head), anywhere in the
    sequence (early rows see few keys: masks and skipped blocks everywhere), and the most
    recent rows, which must reproduce aha_prefill_scores."""
    print("case", w.name, opts, flush=True)
    inputs = synth.make_prefill(w)
    r = opts.window or w.window
    cfg = H.oracle_cfg(w, opts)
    rng = np.random.default_rng(w.seq_len + r)
    rows = np.stack([[np.sort(rng.choice(w.seq_len, r, replace=False)) for _ in range(w.n_q_heads)]
                     for _ in range(w.batch)]).astype(np.int32)
    got = run_scores_rows(w, opts, inputs, rows)
    want = oracle.prefill_scores_rows(*inputs, rows, cfg)
    H.assert_scores_close(got, want, w, opts)
    last = np.broadcast_to(np.arange(w.seq_len - r, w.seq_len, dtype=np.int32),
                           (w.batch, w.n_q_heads, r))
    plain = H.run_prefill_gpu(w, opts, inputs)
    H.assert_scores_close(run_scores_rows(w, opts, inputs, last), plain.scores, w, opts)
    # the order of the list does not matter
    wild = rows[:, :, ::-1].copy()
    H.assert_scores_close(run_scores_rows(w, opts, inputs, wild), want, w, opts)


def test_lowest_entropy_rows_as_accumulators():
    """One Top-k strategy for the accumulators, composed from the library's own entry points:
    the entropy of every row (aha_prefill_row_stats, window = n), the `window` rows of lowest
    entropy among the later half of each head (picked on the host), and the scores
    accumulated over those rows - against the oracle fed with the same rows."""
    w = synth.scaled(BF, name="topk_rows", seq_len=1024, n_q_heads=8, n_kv_heads=2, window=16)
    inputs = synth.make_prefill(w)
    n, r = w.seq_len, w.window
    _, ent = run_row_stats(w, Opts(window=n), inputs[0], inputs[1])
    cand = ent[:, :, n // 2:]                                   # rows that see at least n/2 keys
    rows = (np.sort(np.argsort(cand, axis=-1)[:, :, :r], axis=-1) + n // 2).astype(np.int32)
    got = run_scores_rows(w, Opts(), inputs, rows)
    want = oracle.prefill_scores_rows(*inputs, rows, H.oracle_cfg(w, Opts()))
    H.assert_scores_close(got, want, w, Opts())
    idx_ref = oracle.select_topk(want, w.budget, w.recent)
    import torch
    from paper_2506_03762_amd import binding as B
    p = H.gpu_params(w, Opts())
    idx = torch.empty((w.batch, w.n_kv_heads, w.budget), dtype=torch.int32, device="cuda")
    B.aha_select_topk(p, torch.from_numpy(got.astype(np.float32)).cuda(), idx)
    H.assert_sets_match(idx.cpu().numpy(), idx_ref, want, w)
