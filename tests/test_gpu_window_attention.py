"""Attention output of the observed rows from the HIP path (aha_prefill_window_attention)
against the float64 oracle, and its log-sum-exp handed on to the single-pass scores."""
import numpy as np
import pytest

import oracle
from oracle import SCALE_FIXED
from paper_2506_03762_amd import synth
from tests import harness as H
from tests.harness import Opts

pytestmark = pytest.mark.gpu

BF = synth.scaled(synth.C3, name="bf16_small", seq_len=1536, n_q_heads=8, n_kv_heads=2,
                  budget=192, recent=32, window=32)


def run_window_attention(w, window, Q, K, V, token_major=False):
    import torch
    from paper_2506_03762_amd import binding as B
    if token_major:  # stored [b, n, h, d], passed by strides
        q, k, v = (H.to_device(np.ascontiguousarray(a.transpose(0, 2, 1, 3)), w.dtype).permute(0, 2, 1, 3)
                   for a in (Q, K, V))
    else:
        q, k, v = (H.to_device(a, w.dtype) for a in (Q, K, V))
    p = H.gpu_params(w, Opts(window=window)).with_strides(q, k, v)
    ws = torch.empty(max(B.window_attention_workspace_bytes(p), 256), dtype=torch.uint8, device="cuda")
    ws.fill_(0xA5)
    out = torch.full((w.batch, w.n_q_heads, window, w.head_dim), float("nan"),
                     dtype=B.torch_dtype(p.dtype), device="cuda")
    lse = torch.full((w.batch, w.n_q_heads, window), float("nan"), dtype=torch.float32, device="cuda")
    B.aha_prefill_window_attention(p, q, k, v, out, lse, ws)
    torch.cuda.synchronize()
    return out.float().cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)


def check(w, window, inputs=None):
    print("case", w.name, w.dtype, "n", w.seq_len, "heads", w.n_q_heads, w.n_kv_heads, "d", w.head_dim,
          "window", window, flush=True)
    Q, K, V = inputs if inputs is not None else synth.make_prefill(w)
    out, lse = run_window_attention(w, window, Q, K, V)
    want = oracle.window_attention(Q, K, V, window)
    cfg = oracle.Config(window=window, budget=w.budget, recent=w.recent, scale_mode=SCALE_FIXED,
                        fixed_scale=w.head_dim ** -0.5)
    want_lse = oracle.row_lse(Q, K, cfg)
    assert np.all(np.isfinite(out)) and np.all(np.isfinite(lse))
    # fp32: 1e-5; bf16: probabilities and the stored output are rounded to bf16 (2^-9 each)
    rtol = 1e-5 if w.dtype == "f32" else 2e-2
    rms = np.sqrt(np.mean(want ** 2, axis=-1, keepdims=True))
    err = np.abs(out - want) / (np.abs(want) + rms)
    assert err.max() <= rtol, "attention output differs: %.3g" % err.max()
    np.testing.assert_allclose(lse, want_lse, rtol=1e-5 if w.dtype == "f32" else 1e-4, atol=1e-3)
    return err.max()


@pytest.mark.parametrize("w,window", [
    (synth.C1, 32),
    (synth.C1, 512),                                                      # every row
    (synth.scaled(synth.C1, name="c1_d128", head_dim=128, seq_len=300, n_q_heads=4, n_kv_heads=2,
                  budget=64, recent=8), 24),
    (BF, 32),
    (BF, 1),
    (BF, 1536),                                                           # every row, 384 row blocks
    (synth.scaled(BF, name="ragged", seq_len=1573, n_q_heads=6, n_kv_heads=2, head_dim=64), 37),
    (synth.scaled(BF, name="g8", seq_len=640, n_q_heads=16, n_kv_heads=2), 48),
    (synth.scaled(BF, name="short", seq_len=31, n_q_heads=2, n_kv_heads=2, budget=8, recent=8), 31),
    (synth.scaled(BF, name="batch3", seq_len=300, batch=3, n_q_heads=2, n_kv_heads=1, budget=50,
                  recent=5), 300),
    # a single block of rows (its own kernel shape) with 64 channels, ragged key ranges
    (synth.scaled(BF, name="one_block_d64", seq_len=2077, n_q_heads=4, n_kv_heads=2, head_dim=64), 9),
    (synth.scaled(BF, name="one_block_d128", seq_len=777, n_q_heads=2, n_kv_heads=2), 32),
], ids=lambda x: getattr(x, "name", x))
def test_window_attention_matches_the_oracle(w, window):
    check(w, window)


@pytest.mark.parametrize("head_dim", [64, 128])
def test_window_attention_with_logits_that_keep_rising(head_dim):
    """Keys whose size grows with the position, aligned with the queries' mean direction: the
    rows' maxima rise all along the sequence, by more than the kernel's slack between its
    softmax reference and the running maximum many times over, and by less than it in
    between (both branches of the lazy reference)."""
    # (128 problems x row-block pairs: four key ranges of eight 128-key steps each)
    w = synth.scaled(BF, name="rising", batch=4, n_q_heads=32, n_kv_heads=16, seq_len=4096,
                     head_dim=head_dim, window=64)
    Q, K, V = synth.make_prefill(w)
    n = w.seq_len
    u = np.random.default_rng(7).standard_normal(head_dim)
    u /= np.linalg.norm(u)
    # logit ~ 3 * ramp / sqrt(d): about 3 (log2 units) more per 128-key step
    ramp = np.linspace(0.0, 20.0 * np.sqrt(head_dim), n)[None, None, :, None]
    Q = synth.store_round((Q * 0.3 + 3.0 * u).astype(np.float32), w.dtype)   # all queries lean on u
    K = synth.store_round((K * 0.5 + ramp * u).astype(np.float32), w.dtype)
    check(w, w.window, (Q, K, V))


def random_attention_case(seed):
    rng = np.random.default_rng(seed)
    d = int(rng.choice([64, 128])); G = int(rng.choice([1, 1, 2, 3, 4, 8]))
    hk = int(rng.integers(1, 4)); b = int(rng.integers(1, 3))
    n = int(rng.choice([rng.integers(1, 200), rng.integers(200, 1500), rng.integers(1500, 5000)]))
    window = int(min(n, rng.choice([1, rng.integers(1, 40), rng.integers(40, 300)])))
    dtype = "bf16" if rng.random() < 0.85 else "f32"
    if dtype == "f32":
        n = min(n, 600); window = min(window, n, 64)
    w = synth.scaled(synth.C3, name="attn_%d" % seed, batch=b, n_q_heads=hk * G, n_kv_heads=hk,
                     head_dim=d, seq_len=n, window=window, budget=max(1, n // 4),
                     recent=min(window, max(1, n // 8)), dtype=dtype)
    return w, window


def test_window_attention_random_shapes():
    """Seeded random shapes: sequence lengths 1 .. 5000, 1 .. 8 query heads per KV head, windows
    of 1 .. 300 rows, both head sizes, both dtypes (single and paired row blocks, ragged key
    ranges, more key ranges than steps)."""
    for seed in range(40):
        check(*random_attention_case(seed))


def test_window_attention_token_major_layout():
    """Q/K/V stored [b, n, h, d] and passed by strides give the same output, bit for bit."""
    w = synth.scaled(BF, name="token_major", seq_len=1100, n_q_heads=8, n_kv_heads=2, window=64)
    Q, K, V = synth.make_prefill(w)
    dense = run_window_attention(w, w.window, Q, K, V)
    strided = run_window_attention(w, w.window, Q, K, V, token_major=True)
    assert np.array_equal(dense[0], strided[0]) and np.array_equal(dense[1], strided[1])


def test_c3_window_attention_and_scores_from_its_log_sum_exp():
    """The 32K-context layer: attention output of the 64 observed rows of all 32 heads against
    the oracle, then the scores from that launch's log-sum-exp (standard scale) against the
    two-pass scores - output and scores with one pass over the keys each."""
    import torch
    w = synth.C3
    inputs = synth.make_prefill(w, threads=16)
    err = check(w, w.window, inputs)
    print("max error relative to |o| + rms: %.3g" % err, flush=True)
    _, lse = run_window_attention(w, w.window, *inputs)
    opts = Opts(scale_mode=SCALE_FIXED, fixed_scale=w.head_dim ** -0.5)
    got = H.run_scores_from_lse_gpu(w, opts, inputs, lse.astype(np.float32))
    two = H.run_prefill_gpu(w, opts, inputs)
    H.assert_scores_close(got, two.scores, w, opts)
