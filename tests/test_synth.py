"""The seeded input generators: reproducible, sliceable, exactly representable."""
import numpy as np
import torch

import oracle
from oracle import Config, SCALE_FIXED
from paper_2506_03762_amd import synth


def test_bf16_rounding_matches_torch():
    x = np.random.default_rng(0).standard_normal(100000).astype(np.float32) * 37.0
    x[:4] = [0.0, -0.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8]   # exact ties
    want = torch.from_numpy(x).to(torch.bfloat16)
    got = synth.round_bf16(x)
    assert np.array_equal(got, want.to(torch.float32).numpy())
    bits = synth.bf16_bits(got)
    assert np.array_equal(bits.view(np.int16), want.view(torch.int16).numpy())


def test_subset_generation_equals_slice_of_full():
    w = synth.scaled(synth.C3, seq_len=256, n_q_heads=8, n_kv_heads=2, batch=2,
                     budget=64)
    Q, K, V = synth.make_prefill(w)
    Q2, K2, V2 = synth.make_prefill(w, batches=[1], kv_heads=[1])
    assert np.array_equal(Q2[0], Q[1, 4:8]) and np.array_equal(K2[0, 0], K[1, 1])
    assert np.array_equal(V2[0, 0], V[1, 1])
    Q3, _, _ = synth.make_prefill(w)
    assert np.array_equal(Q, Q3)                                   # reproducible
    assert np.array_equal(synth.round_bf16(K), K)                  # bf16-representable


def test_structure_sink_and_heavy_hitters_and_layer_knobs():
    w = synth.C1
    Q, K, V = synth.make_prefill(w)
    hh = synth.heavy_hitter_positions(w, 0, 0, 0)
    assert len(hh) == int(np.ceil(0.02 * w.seq_len)) and hh.min() >= 1
    assert hh.max() < w.seq_len - w.window
    norms = np.linalg.norm(K[0, 0], axis=-1)
    assert norms[0] > 2.5 * np.median(norms)                       # sink key scaled x4
    s0, f0 = synth.layer_knobs(synth.C5, 0)
    s31, f31 = synth.layer_knobs(synth.C5, 31)
    assert (s0, s31) == (2.0, 6.0) and abs(f0 - 0.005) < 1e-12 and abs(f31 - 0.03) < 1e-12
    ev = synth.heavy_hitter_positions(synth.C3, 0, 0, 0)
    assert len(ev) == 328 and np.all(np.diff(ev) > 90)             # evenly spread


def test_paper_claim_on_synthetic_inputs():
    """On the tiny workload the accumulated score keeps the left of the
    sequence, the adaptive windowed score does not, and both keep the sink;
    the adaptive score keeps the planted heavy hitters (Sec. 3.1 / Fig. 2c,
    qualitatively)."""
    w = synth.C1
    Q, K, V = synth.make_prefill(w)
    aha = Config(w.window, w.budget, w.recent)
    h2o = Config(w.seq_len, w.budget, w.recent, scale_mode=SCALE_FIXED,
                 fixed_scale=w.head_dim ** -0.5, value_prior=False)
    ia = oracle.select_topk(oracle.prefill_scores(Q, K, V, aha), w.budget, w.recent)
    ih = oracle.select_topk(oracle.prefill_scores(Q, K, V, h2o), w.budget, w.recent)
    assert np.all(ih.mean(-1) + 60 < ia.mean(-1))
    for h in range(w.n_kv_heads):
        hh = set(synth.heavy_hitter_positions(w, 0, 0, h).tolist())
        assert len(hh & set(ia[0, h].tolist())) >= len(hh) - 1
        assert 0 in ia[0, h] and 0 in ih[0, h]
