"""Where the retained tokens sit, under plain accumulation over every row with the standard
scale (the H2O-style policy the method starts from) and under the method itself, on Gaussian
inputs with planted heavy hitters: the synthetic counterpart of the paper's retained-index
comparison (Sec. 3, the bias of accumulated scores towards early tokens; Sec. 4).  Both
policies run through the HIP path and the oracle; the sets must agree, and with them the
position statistics the comparison is about."""
import math

import numpy as np
import pytest

from oracle import SCALE_FIXED
from paper_2506_03762_amd import synth
from tests import harness as H
from tests.harness import Opts

pytestmark = pytest.mark.gpu

W = synth.scaled(synth.C2, name="retained_positions", seq_len=2048, n_q_heads=4, n_kv_heads=4,
                 budget=512, recent=64, window=64, hh_frac=0.03)
ACCUMULATE_ALL = Opts(window=W.seq_len, scale_mode=SCALE_FIXED,
                      fixed_scale=1 / math.sqrt(W.head_dim), value_prior=False)
METHOD = Opts()


def position_stats(idx, w):
    """Per head: median position of the retained non-recent tokens, planted heavy hitters
    kept, and the late ones (last fifth of the prompt before the recent tokens) kept."""
    out = []
    for b in range(w.batch):
        for h in range(w.n_kv_heads):
            kept = idx[b, h]
            kept = kept[kept < w.seq_len - w.recent]
            hh = synth.heavy_hitter_positions(w, 0, b, h)
            hh = hh[hh < w.seq_len - w.recent]
            late = hh[hh >= int(0.8 * w.seq_len)]
            out.append((float(np.median(kept)), int(np.isin(hh, kept).sum()), hh.size,
                        int(np.isin(late, kept).sum()), late.size))
    return out


def test_accumulated_scores_favour_early_tokens_and_the_method_does_not():
    inputs = synth.make_prefill(W, 0)
    res = {}
    for name, opts in (("all_rows", ACCUMULATE_ALL), ("method", METHOD)):
        print("policy", name, opts, flush=True)
        gpu = H.run_prefill_gpu(W, opts, inputs)
        ref = H.run_prefill_oracle(W, opts, inputs)
        H.assert_scores_close(gpu.scores, ref.scores, W, opts)
        excused = H.assert_sets_match(gpu.idx, ref.idx, ref.extra["rank_scores"], W)
        g, r = position_stats(gpu.idx, W), position_stats(ref.idx, W)
        # histograms of the retained positions: equal up to the excused near-ties
        hg = np.histogram(gpu.idx, bins=16, range=(0, W.seq_len))[0]
        hr = np.histogram(ref.idx, bins=16, range=(0, W.seq_len))[0]
        assert np.abs(hg - hr).sum() <= excused
        if excused == 0:
            assert g == r
        res[name] = g
        print(name, "median position / heavy hitters kept / late kept:", g, flush=True)
    n = W.seq_len
    for (med_a, kept_a, tot, late_a, nlate), (med_m, kept_m, _, late_m, _) in zip(res["all_rows"],
                                                                                 res["method"]):
        # accumulation over every row keeps the head of the prompt; the method spreads out
        assert med_a < 0.25 * n < med_m
        # the method keeps every planted heavy hitter, wherever it sits
        assert kept_m == tot
        # the late ones lose against early ordinary tokens under plain accumulation
        assert nlate > 0 and late_a < late_m == nlate
        assert kept_a < kept_m
