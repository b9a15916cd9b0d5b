"""Pins for the float64 CPU oracle: closed forms, invariants, library routines
and brute force -- nothing here compares the oracle with itself or with the
GPU path."""
import itertools
import math
import os

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

import oracle
from oracle import Config, SCALE_ADAPTIVE, SCALE_FIXED

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rnd(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def harmonic(m):
    return np.concatenate([[0.0], np.cumsum(1.0 / np.arange(1, m + 1))])


# --------------------------------------------------------------- lambda ----
def test_lambda_hand_values():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "lambda_values.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 4
    for i, k, d, val in rows:
        got = oracle.lam(int(i), int(k), int(d), floor=0.0)
        assert abs(got - float(val)) < 5e-7, (i, k, d, got)


def test_lambda_identities():
    d, k = 128, 1000
    assert oracle.lam(k, k, d, floor=0.0) == 0.0
    assert oracle.lam(k // 2, k, d, floor=0.0) == 0.0            # clamped log
    assert oracle.lam(k // 2, k, d, floor=-1.0) == pytest.approx(1 / math.sqrt(d), rel=1e-15)
    # lambda = 1/sqrt(d) exactly where ln(c/k) = 1/2; c is an integer, so check
    # the two integers that bracket k*sqrt(e)
    c = k * math.sqrt(math.e)
    lo, hi = oracle.lam(int(c), k, d, 0.0), oracle.lam(int(c) + 1, k, d, 0.0)
    assert lo < 1 / math.sqrt(d) < hi
    # entropy target: log c - lambda^2 d / 2 == log k  (the equation lambda solves)
    for c_ in (1500, 4096, 32768):
        lam = oracle.lam(c_, k, d, 0.0)
        assert math.log(c_) - lam * lam * d / 2 == pytest.approx(math.log(k), rel=1e-13)
    # floor
    assert oracle.lam(1001, 1000, 64, floor=0.05) == 0.05


# ------------------------------------------------- softmax rows / sums ----
@pytest.mark.parametrize("mode", [SCALE_FIXED, SCALE_ADAPTIVE])
def test_rows_sum_to_one_and_causal(mode):
    b, hq, hk, n, d, r = 2, 4, 2, 96, 16, 20
    Q, K = rnd(1, b, hq, n, d), rnd(2, b, hk, n, d)
    cfg = Config(window=r, budget=24, recent=8, scale_mode=mode, fixed_scale=0.3,
                 value_prior=False)
    P = oracle.attention_rows(Q, K, cfg)
    assert P.shape == (b, hq, r, n)
    np.testing.assert_allclose(P.sum(-1), 1.0, atol=1e-12)
    for ii in range(r):
        i = n - r + ii
        assert np.all(P[:, :, ii, i + 1:] == 0.0)
        assert np.all(P[:, :, ii, :i + 1] > 0.0)


def test_column_sums_total_rows():
    b, hq, hk, n, d, r = 2, 6, 2, 80, 8, 17
    Q, K, V = rnd(3, b, hq, n, d), rnd(4, b, hk, n, d), rnd(5, b, hk, n, d)
    cfg = Config(window=r, budget=20, recent=4, value_prior=False)
    S = oracle.prefill_scores(Q, K, V, cfg)
    np.testing.assert_allclose(S.sum(-1), (hq // hk) * r, rtol=1e-12)
    # scores equal the column sums of the written-out rows, summed per KV group
    P = oracle.attention_rows(Q, K, cfg)
    np.testing.assert_allclose(S, P.sum(2).reshape(b, hk, hq // hk, n).sum(2), rtol=1e-12)


@pytest.mark.parametrize("r", [1, 5, 33, 64])
def test_closed_form_at_scale_zero(r):
    """scale 0 => a_ij = 1/(i+1) => S_j = G (H_n - H_max(j, n-r))."""
    b, hq, hk, n, d = 1, 4, 2, 64, 8
    Q, K, V = rnd(6, b, hq, n, d), rnd(7, b, hk, n, d), rnd(8, b, hk, n, d)
    cfg = Config(window=r, budget=16, recent=4, scale_mode=SCALE_FIXED, fixed_scale=0.0,
                 value_prior=False)
    S = oracle.prefill_scores(Q, K, V, cfg)
    H = harmonic(n)
    j = np.arange(n)
    want = (hq // hk) * (H[n] - H[np.maximum(j, n - r)])
    np.testing.assert_allclose(S[0, 0], want, rtol=1e-13)
    np.testing.assert_allclose(S[0, 1], want, rtol=1e-13)
    if r == n:
        # the paper's bias identity, exact here: S_{j+1} - S_j = -a_jj = -1/(j+1)
        np.testing.assert_allclose(np.diff(S[0, 0]), -(hq // hk) / (j[:-1] + 1.0), rtol=1e-10)


def _library_scores(Q, K, scales_by_row, rows):
    """Independent route: masked logits -> scipy softmax -> column sum."""
    b, hq, n, d = Q.shape
    hk = K.shape[1]
    G = hq // hk
    out = np.zeros((b, hk, n))
    for bi in range(b):
        for h in range(hq):
            W = Q[bi, h] @ K[bi, h // G].T                 # [n, n] raw dots
            for i in rows:
                x = scales_by_row[i] * W[i, :i + 1]
                out[bi, h // G, :i + 1] += sp_softmax(x)
    return out


def test_reduces_to_accumulated_attention_score():
    """window = n, scale 1/sqrt(d), no value prior: the plain accumulated score."""
    b, hq, hk, n, d = 2, 4, 2, 70, 16
    Q, K, V = rnd(9, b, hq, n, d), rnd(10, b, hk, n, d), rnd(11, b, hk, n, d)
    cfg = Config(window=n, budget=16, recent=4, scale_mode=SCALE_FIXED,
                 fixed_scale=1 / math.sqrt(d), value_prior=False)
    S = oracle.prefill_scores(Q, K, V, cfg)
    want = _library_scores(Q, K, {i: 1 / math.sqrt(d) for i in range(n)}, range(n))
    np.testing.assert_allclose(S, want, rtol=1e-11)
    # and via a dense masked softmax, a third route
    for bi in range(b):
        for h in range(hk):
            acc = np.zeros(n)
            for g in range(hq // hk):
                W = (Q[bi, h * (hq // hk) + g] @ K[bi, h].T) / math.sqrt(d)
                W = np.where(np.tril(np.ones((n, n), bool)), W, -np.inf)
                acc += sp_softmax(W, axis=1).sum(0)
            np.testing.assert_allclose(S[bi, h], acc, rtol=1e-11)


def test_adaptive_windowed_matches_library_route():
    b, hq, hk, n, d, r, B = 1, 4, 1, 300, 32, 24, 40
    Q, K, V = rnd(12, b, hq, n, d), rnd(13, b, hk, n, d), rnd(14, b, hk, n, d)
    cfg = Config(window=r, budget=B, recent=8, value_prior=False, lambda_floor=0.0)
    S = oracle.prefill_scores(Q, K, V, cfg)
    sc = {i: math.sqrt(2 * max(math.log((i + 1) / B), 0.0) / d) for i in range(n)}
    want = _library_scores(Q, K, sc, range(n - r, n))
    np.testing.assert_allclose(S, want, rtol=1e-11)


def test_row_lse_matches_library_logsumexp():
    """The row normalisers against scipy's logsumexp of the scaled causal logits (fixed and
    adaptive scale, grouped heads)."""
    from scipy.special import logsumexp
    b, hq, hk, n, d, r, B = 2, 4, 2, 90, 16, 12, 20
    Q, K = rnd(40, b, hq, n, d), rnd(41, b, hk, n, d)
    for cfg, scale_of in (
            (Config(window=r, budget=B, recent=4, scale_mode=SCALE_FIXED, fixed_scale=0.3),
             lambda i: 0.3),
            (Config(window=r, budget=B, recent=4, lambda_floor=0.0),
             lambda i: math.sqrt(2 * max(math.log((i + 1) / B), 0.0) / d))):
        L = oracle.row_lse(Q, K, cfg)
        assert L.shape == (b, hq, r)
        for bi in range(b):
            for h in range(hq):
                for ii in range(r):
                    i = n - r + ii
                    w = K[bi, h // (hq // hk), :i + 1] @ Q[bi, h, i]
                    assert abs(L[bi, h, ii] - logsumexp(scale_of(i) * w)) < 1e-11


def test_scores_from_row_lse():
    """Scores from given normalisers: with the true normalisers they are the scores; the
    normaliser enters as exp(-lse), row by row (a shifted lse rescales that row's share)."""
    b, hq, hk, n, d, r = 1, 4, 2, 80, 16, 8
    Q, K, V = rnd(42, b, hq, n, d), rnd(43, b, hk, n, d), rnd(44, b, hk, n, d)
    for vp in (False, True):
        cfg = Config(window=r, budget=16, recent=4, scale_mode=SCALE_FIXED,
                     fixed_scale=1 / math.sqrt(d), value_prior=vp)
        L = oracle.row_lse(Q, K, cfg)
        S = oracle.prefill_scores(Q, K, V, cfg)
        np.testing.assert_allclose(oracle.prefill_scores_lse(Q, K, V, L, cfg), S, rtol=1e-11)
    # shift the normaliser of one query head's rows by log 2: that head's share halves
    cfg = Config(window=r, budget=16, recent=4, scale_mode=SCALE_FIXED,
                 fixed_scale=1 / math.sqrt(d), value_prior=False)
    L = oracle.row_lse(Q, K, cfg)
    S = oracle.prefill_scores(Q, K, V, cfg)
    share = oracle.prefill_scores(Q[:, 1:2], K[:, 0:1], V[:, 0:1], cfg)  # head 1 alone on KV head 0
    L2 = L.copy()
    L2[:, 1] += math.log(2.0)
    S2 = oracle.prefill_scores_lse(Q, K, V, L2, cfg)
    np.testing.assert_allclose(S2[:, 0], S[:, 0] - 0.5 * share[:, 0], rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(S2[:, 1], S[:, 1], rtol=1e-12)
    # rows still sum to one: the column sums total the number of rows
    np.testing.assert_allclose(S.sum(-1), (hq // hk) * r, rtol=1e-12)


def test_transposed_or_swapped_operands_would_fail():
    """Q and K are not interchangeable: scoring with them swapped differs."""
    b, h, n, d = 1, 1, 40, 8
    Q, K, V = rnd(15, b, h, n, d), rnd(16, b, h, n, d), rnd(17, b, h, n, d)
    cfg = Config(window=8, budget=10, recent=2, value_prior=False)
    a = oracle.prefill_scores(Q, K, V, cfg)
    bb = oracle.prefill_scores(K, Q, V, cfg)
    assert np.abs(a - bb).max() > 1e-3


# ---------------------------------------------- statistical (soft) pins ----
def test_entropy_targets_on_gaussian_inputs():
    """E[H] ~ log c - 1/2 under 1/sqrt(d) and ~ log k under the adaptive scale
    (iid N(0,1) Q, K; loose band, the derivation swaps E log for log E)."""
    b, h, n, d, r, k = 1, 24, 4096, 64, 8, 512
    Q, K = rnd(18, b, h, n, d), rnd(19, b, h, n, d)

    def mean_entropy(cfg):
        P = oracle.attention_rows(Q, K, cfg)
        with np.errstate(divide="ignore", invalid="ignore"):
            H = -(np.where(P > 0, P * np.log(P), 0.0)).sum(-1)
        return H.mean()

    std = mean_entropy(Config(window=r, budget=k, recent=4, scale_mode=SCALE_FIXED,
                              fixed_scale=1 / math.sqrt(d)))
    ada = mean_entropy(Config(window=r, budget=k, recent=4, lambda_floor=0.0))
    assert abs(std - (math.log(n) - 0.5)) < 0.2
    assert abs(ada - math.log(k)) < 0.25
    assert ada < std  # the gain sharpens the rows


def test_row_entropy_closed_forms_and_library_route():
    """Entropy of the observed rows: ln c_i exactly for uniform rows (scale 0), 0 in the
    one-hot limit, scipy.stats.entropy of a library softmax on the masked logits otherwise,
    and 0 <= H <= ln c_i throughout; the two expectations of Sec. 4.2 on Gaussian inputs."""
    from scipy.stats import entropy as sp_entropy
    b, hq, hk, n, d, r = 2, 4, 2, 90, 16, 11
    Q, K = rnd(70, b, hq, n, d), rnd(71, b, hk, n, d)
    c = np.arange(n - r, n) + 1
    uni = oracle.row_entropy(Q, K, Config(r, 20, 3, scale_mode=SCALE_FIXED, fixed_scale=0.0))
    np.testing.assert_allclose(uni, np.broadcast_to(np.log(c), uni.shape), rtol=1e-13)
    hot = oracle.row_entropy(Q, K, Config(r, 20, 3, scale_mode=SCALE_FIXED, fixed_scale=400.0))
    # (a huge gain leaves one key per row, or two if their logits nearly tie)
    assert np.all(hot >= 0) and np.median(hot) < 1e-9 and hot.max() < math.log(2) + 1e-9
    for cfg in (Config(r, 20, 3, scale_mode=SCALE_FIXED, fixed_scale=0.25),
                Config(r, 20, 3), Config(r, 20, 3, lambda_floor=0.0)):
        got = oracle.row_entropy(Q, K, cfg)
        for bb in range(b):
            for h in range(hq):
                for ii in range(r):
                    i = n - r + ii
                    s = cfg.fixed_scale if cfg.scale_mode == SCALE_FIXED else \
                        oracle.lam(i + 1, cfg.budget, d, cfg.lambda_floor)
                    logits = s * (K[bb, h // (hq // hk), :i + 1] @ Q[bb, h, i])
                    want = sp_entropy(sp_softmax(logits))
                    assert got[bb, h, ii] == pytest.approx(want, rel=1e-10, abs=1e-12)
                    assert 0.0 <= got[bb, h, ii] <= math.log(i + 1) + 1e-12
    # expectations on Gaussian inputs (loose band, as in the test above, by the new function)
    b, h, n, d, r, k = 1, 24, 4096, 64, 8, 512
    Q, K = rnd(18, b, h, n, d), rnd(19, b, h, n, d)
    std = oracle.row_entropy(Q, K, Config(r, k, 4, scale_mode=SCALE_FIXED,
                                          fixed_scale=1 / math.sqrt(d))).mean()
    ada = oracle.row_entropy(Q, K, Config(r, k, 4, lambda_floor=0.0)).mean()
    assert abs(std - (math.log(n) - 0.5)) < 0.2 and abs(ada - math.log(k)) < 0.25


def test_accumulated_score_bias_in_expectation():
    """iid Gaussian, full accumulation: E[S_j] = H_n - H_j (each row's entries
    are exchangeable), so the score decays with position."""
    b, h, n, d = 1, 64, 128, 16
    Q, K, V = rnd(20, b, h, n, d), rnd(21, b, h, n, d), rnd(22, b, h, n, d)
    cfg = Config(window=n, budget=16, recent=4, scale_mode=SCALE_FIXED,
                 fixed_scale=1 / math.sqrt(d), value_prior=False)
    S = oracle.prefill_scores(Q, K, V, cfg)[0].mean(0)
    Hn = harmonic(n)
    want = Hn[n] - Hn[np.arange(n)]
    # sampling error of a mean over 64 heads; compare coarse bins
    for lo in range(0, n, 32):
        assert S[lo:lo + 32].mean() == pytest.approx(want[lo:lo + 32].mean(), rel=0.08)
    assert S[:32].mean() > S[32:64].mean() > S[64:96].mean() > S[96:].mean()


# ------------------------------------------------------- value prior ----
def test_value_prior_properties():
    b, hk, n, d = 2, 3, 50, 8
    V = rnd(23, b, hk, n, d)
    for pool in (1, 3, 7):
        g = oracle.value_prior(V, pool)
        assert g.shape == (b, hk, n)
        np.testing.assert_allclose(g.max(-1), 1.0, rtol=1e-15)
        assert np.all(g > 0) and np.all(g <= 1)
        np.testing.assert_allclose(oracle.value_prior(3.7 * V, pool), g, rtol=1e-12)
    nu = (V ** 2).sum(-1)
    np.testing.assert_allclose(oracle.value_prior(V, 1), nu / nu.max(-1, keepdims=True),
                               rtol=1e-13)
    # interior of the pool against numpy's convolution; edges against the
    # truncated mean
    pool, half = 7, 3
    g = oracle.value_prior(V, pool)
    for bi in range(b):
        for h in range(hk):
            gam = np.empty(n)
            gam[half:n - half] = np.convolve(nu[bi, h], np.ones(pool) / pool, mode="valid")
            for j in list(range(half)) + list(range(n - half, n)):
                gam[j] = nu[bi, h, max(0, j - half):min(n, j + half + 1)].mean()
            np.testing.assert_allclose(g[bi, h], gam / gam.max(), rtol=1e-12)


def test_value_prior_equal_norm_rows_is_identity():
    b, hq, hk, n, d = 1, 2, 2, 40, 8
    Q, K, V = rnd(24, b, hq, n, d), rnd(25, b, hk, n, d), rnd(26, b, hk, n, d)
    V /= np.linalg.norm(V, axis=-1, keepdims=True)
    on = oracle.prefill_scores(Q, K, V, Config(8, 10, 2, value_prior=True, pool=5))
    off = oracle.prefill_scores(Q, K, V, Config(8, 10, 2, value_prior=False))
    np.testing.assert_allclose(on, off, rtol=1e-12)


def test_value_prior_of_an_all_zero_head_is_one():
    """max(gamma) = 0 leaves the quotient undefined; the reading taken is gamma_bar = 1, so the
    refined scores of that head equal the unrefined ones while other heads are not touched."""
    Q, K, V = rnd(60, 1, 2, 40, 8), rnd(61, 1, 2, 40, 8), rnd(62, 1, 2, 40, 8)
    V[0, 1] = 0.0
    g = oracle.value_prior(V, 5)
    assert np.all(g[0, 1] == 1.0) and g[0, 0].max() == 1.0 and g[0, 0].min() < 1.0
    on = oracle.prefill_scores(Q, K, V, Config(6, 10, 2, value_prior=True, pool=5))
    off = oracle.prefill_scores(Q, K, V, Config(6, 10, 2, value_prior=False))
    assert np.array_equal(on[0, 1], off[0, 1]) and not np.array_equal(on[0, 0], off[0, 0])


def test_value_prior_multiplies_scores():
    b, hq, hk, n, d = 1, 2, 1, 40, 8
    Q, K, V = rnd(27, b, hq, n, d), rnd(28, b, hk, n, d), rnd(29, b, hk, n, d)
    on = oracle.prefill_scores(Q, K, V, Config(8, 10, 2, value_prior=True, pool=3))
    off = oracle.prefill_scores(Q, K, V, Config(8, 10, 2, value_prior=False))
    nu = (V ** 2).sum(-1)[0, 0]
    gam = np.array([nu[max(0, j - 1):j + 2].mean() for j in range(n)])
    np.testing.assert_allclose(on[0, 0], off[0, 0] * gam / gam.max(), rtol=1e-12)


# -------------------------------------------------------------- GQA ----
def test_gqa_equals_replicated_mha_summed_per_group():
    b, hq, hk, n, d = 1, 8, 2, 60, 8
    G = hq // hk
    Q, K, V = rnd(30, b, hq, n, d), rnd(31, b, hk, n, d), rnd(32, b, hk, n, d)
    cfg = Config(window=12, budget=20, recent=4, value_prior=False)
    gqa = oracle.prefill_scores(Q, K, V, cfg)
    mha = oracle.prefill_scores(Q, np.repeat(K, G, axis=1), np.repeat(V, G, axis=1), cfg)
    np.testing.assert_allclose(gqa, mha.reshape(b, hk, G, n).sum(2), rtol=1e-12)


# ------------------------------------------------------------ top-k ----
def test_topk_brute_force_and_properties():
    rng = np.random.default_rng(33)
    for n, B, Br in [(50, 20, 6), (37, 37, 5), (64, 10, 10), (33, 9, 0), (16, 1, 0)]:
        s = rng.random((3, 2, n))
        idx = oracle.select_topk(s, B, Br)
        assert idx.shape == (3, 2, B) and idx.dtype == np.int32
        for p in np.ndindex(3, 2):
            got = idx[p]
            assert np.all(np.diff(got) > 0)                       # ascending, distinct
            assert set(range(n - Br, n)) <= set(got.tolist())     # recents kept
            cand = np.arange(n - Br)
            order = sorted(cand, key=lambda j: (-s[p][j], j))     # full sort
            want = sorted(order[:B - Br]) + list(range(n - Br, n))
            assert got.tolist() == want
            kept = [j for j in got if j < n - Br]
            drop = [j for j in cand if j not in set(kept)]
            if kept and drop:
                assert s[p][kept].min() >= s[p][drop].max()


def test_topk_exhaustive_subsets_maximise_kept_mass():
    rng = np.random.default_rng(34)
    m, Bs, Br = 11, 4, 2
    s = rng.random(m + Br)
    idx = oracle.select_topk(s, Bs + Br, Br)
    chosen = tuple(j for j in idx if j < m)
    best = max(itertools.combinations(range(m), Bs), key=lambda c: s[list(c)].sum())
    assert chosen == best


def test_topk_ties_keep_lower_index():
    s = np.array([0.5, 0.9, 0.5, 0.5, 0.1, 0.5, 0.0, 0.0])
    assert oracle.select_topk(s, 5, 2).tolist() == [0, 1, 2, 6, 7]
    assert oracle.select_topk(np.zeros(9), 4, 1).tolist() == [0, 1, 2, 8]


# -------------------------------------------------------- compaction ----
def test_pooled_score_selection():
    """Score smoothing before the selection (float64): the interior against numpy.convolve with
    a box of 1/pool, the edges against the mean of the in-range slice, width 1 is the identity,
    a constant stays constant, and the selection is the plain selection of the pooled array."""
    rng = np.random.default_rng(50)
    s = rng.random((3, 97))
    n = s.shape[1]
    for pool in (1, 3, 7, 15):
        h = (pool - 1) // 2
        got = oracle.pool_scores(s, pool)
        for pr in range(s.shape[0]):
            interior = np.convolve(s[pr], np.full(pool, 1.0 / pool), mode="valid")
            np.testing.assert_allclose(got[pr, h:n - h], interior, rtol=1e-13)
            for j in list(range(h)) + list(range(n - h, n)):
                np.testing.assert_allclose(got[pr, j], s[pr, max(0, j - h):j + h + 1].mean(),
                                           rtol=1e-13)
        idx = oracle.select_topk_pooled(s, 20, 5, pool)
        assert np.array_equal(idx, oracle.select_topk(got, 20, 5))
    # an asymmetric input tells a shifted or one-sided window from the centred one
    ramp = np.arange(12, dtype=np.float64)[None] ** 2
    assert oracle.pool_scores(ramp, 3)[0, 5] == (16 + 25 + 36) / 3.0
    assert oracle.pool_scores(ramp, 3)[0, 0] == (0 + 1) / 2.0
    assert oracle.pool_scores(ramp, 5)[0, 11] == (81 + 100 + 121) / 3.0
    assert np.array_equal(oracle.pool_scores(s, 1), s)
    c = np.full((1, 40), 0.375)
    assert np.array_equal(oracle.pool_scores(c, 9), c)
    # a lone spike spreads over its neighbours: with width 3 they outrank a slightly lower lone value
    z = np.zeros((1, 30)); z[0, 10] = 3.0; z[0, 20] = 0.9
    assert set(oracle.select_topk_pooled(z, 3, 0, 3)[0]) == {9, 10, 11}
    assert set(oracle.select_topk(z, 3, 0)[0]) == {0, 10, 20}


def test_compaction_is_a_gather():
    b, hk, n, d, B = 2, 3, 30, 4, 7
    K, V = rnd(35, b, hk, n, d), rnd(36, b, hk, n, d)
    S = np.random.default_rng(37).random((b, hk, n))
    idx = oracle.select_topk(S, B, 2)
    c = oracle.compact_kv(K, V, S, idx, slots=B + 3)
    for p in np.ndindex(b, hk):
        assert np.array_equal(c.K[p][:B], K[p][idx[p]])
        assert np.array_equal(c.V[p][:B], V[p][idx[p]])
        assert np.array_equal(c.F[p][:B], S[p][idx[p]])
        assert np.array_equal(c.pos[p][:B], idx[p])
        assert np.all(c.pos[p][B:] == -1) and np.all(c.F[p][B:] == 0)
        assert c.free_slot[p] == B
    # idempotent on the identity index list
    ident = np.broadcast_to(np.arange(B, dtype=np.int32), (b, hk, B))
    c2 = oracle.compact_kv(c.K[:, :, :B], c.V[:, :, :B], c.F[:, :, :B], ident, slots=B + 1)
    assert np.array_equal(c2.K[:, :, :B], c.K[:, :, :B])


# ------------------------------------------------------------ decode ----
def _python_decode_sim(entries, q, k, v, c_t, B, Br, d, scale, sink=0, value_prior=False):
    """Independent re-simulation on a dict keyed by token position."""
    entries = dict(entries)
    entries[c_t - 1] = [k.copy(), v.copy(), 0.0]
    keys = sorted(entries)
    outs = []
    nu = np.array([float(entries[p][1] @ entries[p][1]) for p in keys])
    gbar = nu / nu.max() if value_prior else np.ones(len(keys))
    for g in range(q.shape[0]):
        w = np.array([float(q[g] @ entries[p][0]) for p in keys])
        po = sp_softmax(w / math.sqrt(d))
        outs.append(sum(po[t] * entries[p][1] for t, p in enumerate(keys)))
        ps = sp_softmax(scale * w)
        for t, p in enumerate(keys):
            entries[p][2] += gbar[t] * ps[t]
    protected = set(keys[len(keys) - Br:]) if Br else set()
    protected |= {p for p in keys if p < sink}
    cands = [p for p in keys if p not in protected]
    victim = min(cands, key=lambda p: (entries[p][2], -p))
    del entries[victim]
    return entries, np.array(outs), victim


@pytest.mark.parametrize("mode", [SCALE_FIXED, SCALE_ADAPTIVE])
def test_decode_against_python_resimulation(mode):
    b, hq, hk, d, n, B, Br = 2, 4, 2, 8, 40, 11, 3
    G = hq // hk
    Q, K, V = rnd(38, b, hq, n, d), rnd(39, b, hk, n, d), rnd(40, b, hk, n, d)
    cfg = Config(window=6, budget=B, recent=Br, scale_mode=mode, fixed_scale=0.4,
                 value_prior=True, pool=3)
    S = oracle.prefill_scores(Q, K, V, cfg)
    idx = oracle.select_topk(S, B, Br)
    cache = oracle.compact_kv(K, V, S, idx, slots=B + 1)
    sims = {p: {int(j): [K[p][j].copy(), V[p][j].copy(), float(S[p][j])] for j in idx[p]}
            for p in np.ndindex(b, hk)}
    rng = np.random.default_rng(41)
    for step in range(8):
        c_t = n + step + 1
        q, k, v = rng.standard_normal((b, hq, d)), rng.standard_normal((b, hk, d)), \
            rng.standard_normal((b, hk, d))
        F_before = cache.F.copy()
        pos_before = cache.pos.copy()
        out = oracle.decode_step(cache, q, k, v, c_t, cfg)
        scale = 0.4 if mode == SCALE_FIXED else oracle.lam(c_t, B, d, cfg.lambda_floor)
        for p in np.ndindex(b, hk):
            sims[p], o, victim = _python_decode_sim(
                sims[p], q[p[0], p[1] * G:(p[1] + 1) * G], k[p], v[p], c_t, B, Br, d, scale)
            np.testing.assert_allclose(out[p[0], p[1] * G:(p[1] + 1) * G], o, rtol=1e-11)
            live = cache.pos[p] >= 0
            assert live.sum() == B                              # constant cache size
            got = {int(pp): float(f) for pp, f in zip(cache.pos[p][live], cache.F[p][live])}
            want = {pp: e[2] for pp, e in sims[p].items()}
            assert got.keys() == want.keys()
            for pp in got:
                assert got[pp] == pytest.approx(want[pp], rel=1e-11)
            assert cache.pos[p][cache.free_slot[p]] == -1       # one eviction
            assert victim not in got
            # recents survive
            assert set(range(c_t - Br, c_t)) <= set(got)
            # the step distributes exactly G units of probability
            Fb = F_before[p].copy()
            Fb[pos_before[p] < 0] = 0.0                         # slot reused by the new token
            total = (cache.F[p] - Fb).sum()
            assert total == pytest.approx(G, rel=1e-11)


def test_decode_output_is_textbook_attention():
    b, hq, hk, d, B = 1, 2, 1, 16, 9
    rng = np.random.default_rng(42)
    Kc, Vc = rng.standard_normal((b, hk, B + 1, d)), rng.standard_normal((b, hk, B + 1, d))
    cache = oracle.Cache(Kc.copy(), Vc.copy(), np.zeros((b, hk, B + 1)),
                         np.concatenate([np.arange(B), [-1]]).astype(np.int32)[None, None].copy(),
                         np.full((b, hk), B, np.int32))
    q, k, v = rng.standard_normal((b, hq, d)), rng.standard_normal((b, hk, d)), \
        rng.standard_normal((b, hk, d))
    out = oracle.decode_step(cache, q, k, v, B + 1, Config(4, B, 2))
    Kf, Vf = Kc[0, 0].copy(), Vc[0, 0].copy()
    Kf[B], Vf[B] = k[0, 0], v[0, 0]
    want = sp_softmax((q[0] @ Kf.T) / math.sqrt(d), axis=-1) @ Vf
    np.testing.assert_allclose(out[0], want, rtol=1e-12)


def _tied_cache(positions, F, d, seed):
    """Compact cache of one head whose slots hold `positions` (in that slot order, -1 = the
    free slot) with running scores F; K and V random."""
    rng = np.random.default_rng(seed)
    slots = len(positions)
    pos = np.array(positions, np.int32)[None, None].copy()
    return oracle.Cache(rng.standard_normal((1, 1, slots, d)), rng.standard_normal((1, 1, slots, d)),
                        np.array(F, np.float64)[None, None].copy(), pos,
                        np.array([[positions.index(-1)]], np.int32))


def test_decode_equal_minima_evict_the_highest_position():
    """Tie rule of the generation step (a reading: the paper is silent).  With scale 0 every
    slot receives the same increment G / (budget + 1), so equal running scores stay equal and
    the rule alone picks the victim; the expected victims below are worked out by hand."""
    d, G = 8, 2
    rng = np.random.default_rng(43)
    q, k, v = rng.standard_normal((1, G, d)), rng.standard_normal((1, 1, d)), rng.standard_normal((1, 1, d))
    cfg = Config(window=4, budget=8, recent=2, scale_mode=SCALE_FIXED, fixed_scale=0.0)
    # slots in scrambled position order; the new token gets position 20 (logical_pos 21).
    # protected: positions 20 and 17; all others hold 0.5 -> victim = position 15 (slot 3)
    positions = [4, 9, 17, 15, -1, 0, 11, 2, 7]
    c = _tied_cache(positions, [0.5] * 9, d, 44)
    oracle.decode_step(c, q, k, v, 21, cfg)
    assert c.free_slot[0, 0] == 3 and c.pos[0, 0, 3] == -1
    assert np.allclose(c.F[0, 0, [0, 1, 2, 5, 6, 7, 8]], 0.5 + G / 9.0)
    # two equal minima (positions 2 and 11) below the rest -> victim = position 11 (slot 6)
    F = [0.5, 0.5, 0.5, 0.5, 0.0, 0.5, 0.25, 0.25, 0.5]
    c = _tied_cache(positions, F, d, 45)
    oracle.decode_step(c, q, k, v, 21, cfg)
    assert c.free_slot[0, 0] == 6
    # a strictly smaller score beats a higher position
    F = [0.5, 0.5, 0.5, 0.5, 0.0, 0.125, 0.25, 0.25, 0.5]
    c = _tied_cache(positions, F, d, 46)
    oracle.decode_step(c, q, k, v, 21, cfg)
    assert c.free_slot[0, 0] == 5
    # a protected slot is never the victim, whatever its score: recent = 3 protects 20, 17, 15
    cfg3 = Config(window=4, budget=8, recent=3, scale_mode=SCALE_FIXED, fixed_scale=0.0)
    F = [0.5, 0.5, 0.5, 0.0, 0.0, 0.5, 0.5, 0.5, 0.5]
    c = _tied_cache(positions, F, d, 47)
    oracle.decode_step(c, q, k, v, 21, cfg3)
    assert c.free_slot[0, 0] == 6          # position 11, the highest unprotected one
    # recent = 0: the new token itself (score 0 + increment) is the unique minimum
    cfg0 = Config(window=4, budget=8, recent=0, scale_mode=SCALE_FIXED, fixed_scale=0.0)
    c = _tied_cache(positions, [0.5] * 9, d, 48)
    oracle.decode_step(c, q, k, v, 21, cfg0)
    assert c.free_slot[0, 0] == 4


# ------------------------------------------- sink tokens, value prior in decode ----
def test_sink_selection_by_definition():
    """First `sink` tokens + `recent` last ones + the best of the rest; sink = 0 is the plain
    selection; budget = sink + recent looks at no score; brute force on random scores."""
    rng = np.random.default_rng(80)
    s = rng.random((4, 60))
    assert np.array_equal(oracle.select_topk_sink(s, 17, 5, 0), oracle.select_topk(s, 17, 5))
    assert oracle.select_topk_sink(s, 9, 5, 4)[2].tolist() == [0, 1, 2, 3, 55, 56, 57, 58, 59]
    for budget, recent, sink in ((17, 5, 4), (20, 0, 3), (12, 3, 9), (60, 10, 4)):
        idx = oracle.select_topk_sink(s, budget, recent, sink)
        for pr in range(s.shape[0]):
            mid = np.arange(sink, 60 - recent)
            order = sorted(mid, key=lambda j: (-s[pr, j], j))[:budget - recent - sink]
            want = sorted(list(range(sink)) + order + list(range(60 - recent, 60)))
            assert idx[pr].tolist() == want
    # a sink token with the lowest score of all is kept, a high score elsewhere is not displaced
    z = np.linspace(1.0, 2.0, 30)[None].copy(); z[0, 0] = 0.0; z[0, 1] = 0.0
    assert oracle.select_topk_sink(z, 6, 2, 2)[0].tolist() == [0, 1, 26, 27, 28, 29]


@pytest.mark.parametrize("sink,vp", [(3, False), (0, True), (2, True)])
def test_decode_with_sink_and_value_prior_against_python_resimulation(sink, vp):
    b, hq, hk, d, n, B, Br = 1, 4, 2, 8, 40, 11, 3
    G = hq // hk
    Q, K, V = rnd(90, b, hq, n, d), rnd(91, b, hk, n, d), rnd(92, b, hk, n, d)
    V *= np.linspace(0.3, 2.0, n)[None, None, :, None]          # value norms that differ a lot
    cfg = Config(window=6, budget=B, recent=Br, value_prior=True, pool=3, sink=sink,
                 decode_value_prior=vp)
    S = oracle.prefill_scores(Q, K, V, cfg)
    idx = oracle.select_topk_sink(S, B, Br, sink)
    cache = oracle.compact_kv(K, V, S, idx, slots=B + 1)
    sims = {p: {int(j): [K[p][j].copy(), V[p][j].copy(), float(S[p][j])] for j in idx[p]}
            for p in np.ndindex(b, hk)}
    rng = np.random.default_rng(93)
    for step in range(10):
        c_t = n + step + 1
        q, k, v = rng.standard_normal((b, hq, d)), rng.standard_normal((b, hk, d)), \
            rng.standard_normal((b, hk, d))
        out = oracle.decode_step(cache, q, k, v, c_t, cfg)
        scale = oracle.lam(c_t, B, d, cfg.lambda_floor)
        for p in np.ndindex(b, hk):
            sims[p], o, victim = _python_decode_sim(
                sims[p], q[p[0], p[1] * G:(p[1] + 1) * G], k[p], v[p], c_t, B, Br, d, scale,
                sink=sink, value_prior=vp)
            np.testing.assert_allclose(out[p[0], p[1] * G:(p[1] + 1) * G], o, rtol=1e-11)
            live = cache.pos[p] >= 0
            got = {int(pp): float(f) for pp, f in zip(cache.pos[p][live], cache.F[p][live])}
            want = {pp: e[2] for pp, e in sims[p].items()}
            assert got.keys() == want.keys()
            for pp in got:
                assert got[pp] == pytest.approx(want[pp], rel=1e-11)
            assert set(range(sink)) <= set(got)                  # sink tokens survive


def test_decode_value_prior_special_cases():
    """Equal value norms leave the step as printed; scaling all values changes nothing; a
    slot with a tiny value row gains next to nothing; the total added is sum gamma_bar p."""
    d, G, B = 8, 2, 8
    rng = np.random.default_rng(94)
    q, k, v = rng.standard_normal((1, G, d)), rng.standard_normal((1, 1, d)), rng.standard_normal((1, 1, d))
    positions = [4, 9, 17, 15, -1, 0, 11, 2, 7]
    def fresh(vscale=1.0, unit=False):
        c = _tied_cache(positions, [0.5] * 9, d, 95)
        if unit:
            c.V /= np.linalg.norm(c.V, axis=-1, keepdims=True)
        c.V *= vscale
        return c
    off = Config(4, B, 2)
    on = Config(4, B, 2, decode_value_prior=True)
    vu = v / np.linalg.norm(v)
    a, bb = fresh(unit=True), fresh(unit=True)
    oracle.decode_step(a, q, k, vu, 21, off); oracle.decode_step(bb, q, k, vu, 21, on)
    np.testing.assert_allclose(a.F, bb.F, rtol=1e-13)            # equal norms: identity
    a, bb = fresh(), fresh(3.0)
    oracle.decode_step(a, q, k, v, 21, on); oracle.decode_step(bb, q, k, 3.0 * v, 21, on)
    np.testing.assert_allclose(a.F, bb.F, rtol=1e-12)            # V -> cV: invariant
    c = fresh(); c.V[0, 0, 2] *= 1e-6
    before = c.F.copy()
    oracle.decode_step(c, q, k, v, 21, on)
    assert c.F[0, 0, 2] - before[0, 0, 2] < 1e-10                # tiny value row: no gain
    ref = fresh(); oracle.decode_step(ref, q, k, v, 21, off)
    gain_on = (c.F - before)[0, 0]; gain_on[4] = c.F[0, 0, 4]
    assert 0 < gain_on.sum() < G                                 # less than the G units of the plain step


# ------------------------------------------------ attention output of the window ----
def test_window_attention_is_textbook_attention():
    """softmax(Q K^T / sqrt(d)) V over the causal prefix, against scipy's softmax and a
    matrix product; the first row of a full window is V_0; constant values come back
    unchanged; every output is a convex combination of the value rows it may see."""
    b, hq, hk, n, d, r = 2, 4, 2, 50, 8, 9
    Q, K, V = rnd(100, b, hq, n, d), rnd(101, b, hk, n, d), rnd(102, b, hk, n, d)
    O = oracle.window_attention(Q, K, V, r)
    for bb in range(b):
        for h in range(hq):
            for ii in range(r):
                i = n - r + ii
                p = sp_softmax((K[bb, h // 2, :i + 1] @ Q[bb, h, i]) / math.sqrt(d))
                np.testing.assert_allclose(O[bb, h, ii], p @ V[bb, h // 2, :i + 1], rtol=1e-12, atol=1e-14)
                assert np.all(O[bb, h, ii] <= V[bb, h // 2, :i + 1].max(0) + 1e-12)
                assert np.all(O[bb, h, ii] >= V[bb, h // 2, :i + 1].min(0) - 1e-12)
    full = oracle.window_attention(Q, K, V, n)
    np.testing.assert_allclose(full[:, :, 0], np.repeat(V[:, :, 0], 2, axis=1), rtol=1e-13)
    np.testing.assert_allclose(full[:, :, n - r:], O, rtol=1e-13)
    const = np.broadcast_to(rnd(103, 1, 1, 1, d), V.shape).copy()
    np.testing.assert_allclose(oracle.window_attention(Q, K, const, r),
                               np.broadcast_to(const[:, :1, :1], (b, hq, r, d)), rtol=1e-12)
    # swapping K and V, or Q and K, is noticed
    assert np.abs(oracle.window_attention(Q, V, K, r) - O).max() > 1e-2


# ------------------------------------------------ accumulation over chosen rows ----
def test_scores_over_given_rows():
    """Accumulators chosen by the caller: the most recent rows give the method's scores; at
    scale 0 the closed form S_j = sum over the chosen rows i >= j of 1 / (i + 1); a library
    route (scipy softmax per row) for random rows; the order of the rows does not matter."""
    b, hq, hk, n, d, r = 2, 4, 2, 70, 8, 6
    Q, K, V = rnd(110, b, hq, n, d), rnd(111, b, hk, n, d), rnd(112, b, hk, n, d)
    last = np.broadcast_to(np.arange(n - r, n, dtype=np.int32), (b, hq, r))
    for cfg in (Config(r, 12, 3), Config(r, 12, 3, value_prior=False, lambda_floor=0.0)):
        np.testing.assert_allclose(oracle.prefill_scores_rows(Q, K, V, last, cfg),
                                   oracle.prefill_scores(Q, K, V, cfg), rtol=1e-13)
    rng = np.random.default_rng(113)
    rows = np.stack([[np.sort(rng.choice(n, r, replace=False)) for _ in range(hq)]
                     for _ in range(b)]).astype(np.int32)
    uni = oracle.prefill_scores_rows(Q, K, V, rows, Config(r, 12, 3, scale_mode=SCALE_FIXED,
                                                           fixed_scale=0.0, value_prior=False))
    for bb in range(b):
        for h in range(hk):
            want = np.zeros(n)
            for g in range(hq // hk):
                for i in rows[bb, h * 2 + g]:
                    want[:i + 1] += 1.0 / (i + 1)
            np.testing.assert_allclose(uni[bb, h], want, rtol=1e-13)
    cfg = Config(r, 12, 3, value_prior=False)
    got = oracle.prefill_scores_rows(Q, K, V, rows, cfg)
    for bb in range(b):
        for h in range(hk):
            want = np.zeros(n)
            for g in range(hq // hk):
                for i in rows[bb, h * 2 + g]:
                    lam = oracle.lam(i + 1, cfg.budget, d, cfg.lambda_floor)
                    want[:i + 1] += sp_softmax(lam * (K[bb, h, :i + 1] @ Q[bb, h * 2 + g, i]))
            np.testing.assert_allclose(got[bb, h], want, rtol=1e-11)
    np.testing.assert_allclose(oracle.prefill_scores_rows(Q, K, V, rows[:, :, ::-1], cfg), got, rtol=1e-12)
    assert np.isclose(got.sum(), b * hq * r)          # every chosen row adds one unit
