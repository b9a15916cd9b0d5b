"""Float64 CPU oracle for the AhaKV eviction path -- TEST INFRASTRUCTURE ONLY.

The arithmetic lives in ``aha_oracle.c`` (plain C, double precision, written
from the paper's definitions).  This module only compiles that file with gcc,
loads it with ctypes and marshals numpy arrays.  Nothing here imports or is
imported by the GPU package; only tests, the smoke check and the benchmark's
CPU-baseline leg may use it.

Array layouts (all float64, C-contiguous):
  Q [batch, n_q_heads, n, d]; K, V [batch, n_kv_heads, n, d];
  scores [batch, n_kv_heads, n]; idx [batch, n_kv_heads, budget] int32.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "aha_oracle.c")
_LIB = os.path.join(_HERE, "libaha_oracle.so")

SCALE_FIXED = 0
SCALE_ADAPTIVE = 1


def build(force: bool = False) -> str:
    """Compile the C oracle (gcc -O2 -fopenmp).  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
             "-ffp-contract=off", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.aha_oracle_lambda.restype = ctypes.c_double
        _lib.aha_oracle_lambda.argtypes = [ctypes.c_int64, ctypes.c_int64,
                                           ctypes.c_int64, ctypes.c_double]
    return _lib


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a


def _p(a, ct=ctypes.c_double):
    return a.ctypes.data_as(ctypes.POINTER(ct))


_I64 = ctypes.c_int64


@dataclass
class Config:
    """Knobs of the score (names follow the paper: window r, budget B = k)."""
    window: int                 # r, number of last query rows accumulated
    budget: int                 # B, total cache budget (k in the lambda formula)
    recent: int                 # B_r, most recent tokens always kept
    scale_mode: int = SCALE_ADAPTIVE
    fixed_scale: float = 0.0    # used when scale_mode == SCALE_FIXED
    lambda_floor: float = -1.0  # <0: 1/sqrt(d); 0: literal closed form
    value_prior: bool = True
    pool: int = 7               # odd average-pool width over tokens
    sink: int = 0               # first tokens that are always retained (selection and decode)
    decode_value_prior: bool = False   # generation: refine the added probabilities by the value prior


def lam(c: int, k: int, d: int, floor: float = -1.0) -> float:
    """Adaptive softmax scale for a row over c keys with budget k."""
    return float(_load().aha_oracle_lambda(int(c), int(k), int(d), float(floor)))


def attention_rows(Q, K, cfg: Config):
    """P [batch, n_q_heads, window, n]: the observed (SG-)softmax rows."""
    Q, K = _f64(Q), _f64(K)
    b, hq, n, d = Q.shape
    hk = K.shape[1]
    P = np.empty((b, hq, cfg.window, n), dtype=np.float64)
    _load().aha_oracle_attention_rows(
        _p(Q), _p(K), _I64(b), _I64(hq), _I64(hk), _I64(n), _I64(d),
        _I64(cfg.window), _I64(cfg.budget), ctypes.c_int(cfg.scale_mode),
        ctypes.c_double(cfg.fixed_scale), ctypes.c_double(cfg.lambda_floor), _p(P))
    return P


def value_prior(V, pool: int):
    """gamma_bar [batch, n_kv_heads, n]."""
    V = _f64(V)
    b, hk, n, d = V.shape
    g = np.empty((b, hk, n), dtype=np.float64)
    _load().aha_oracle_value_prior(_p(V), _I64(b), _I64(hk), _I64(n), _I64(d),
                                   _I64(pool), _p(g))
    return g


def prefill_scores(Q, K, V, cfg: Config):
    """Refined eviction scores [batch, n_kv_heads, n]."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    b, hq, n, d = Q.shape
    hk = K.shape[1]
    assert hq % hk == 0 and K.shape == V.shape == (b, hk, n, d)
    assert 1 <= cfg.window <= n
    S = np.empty((b, hk, n), dtype=np.float64)
    _load().aha_oracle_prefill_scores(
        _p(Q), _p(K), _p(V), _I64(b), _I64(hq), _I64(hk), _I64(n), _I64(d),
        _I64(cfg.window), _I64(cfg.budget), ctypes.c_int(cfg.scale_mode),
        ctypes.c_double(cfg.fixed_scale), ctypes.c_double(cfg.lambda_floor),
        ctypes.c_int(1 if cfg.value_prior else 0), _I64(cfg.pool), _p(S))
    return S


def prefill_scores_rows(Q, K, V, rows, cfg: Config):
    """Refined eviction scores [batch, n_kv_heads, n] accumulated over the query rows at the
    positions rows[batch, n_q_heads, window] instead of the most recent ones."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    b, hq, n, d = Q.shape
    hk = K.shape[1]
    assert hq % hk == 0 and K.shape == V.shape == (b, hk, n, d)
    assert rows.shape == (b, hq, cfg.window) and rows.min() >= 0 and rows.max() < n
    S = np.empty((b, hk, n), dtype=np.float64)
    _load().aha_oracle_prefill_scores_rows(
        _p(Q), _p(K), _p(V), _p(rows, ctypes.c_int32), _I64(b), _I64(hq), _I64(hk), _I64(n),
        _I64(d), _I64(cfg.window), _I64(cfg.budget), ctypes.c_int(cfg.scale_mode),
        ctypes.c_double(cfg.fixed_scale), ctypes.c_double(cfg.lambda_floor),
        ctypes.c_int(1 if cfg.value_prior else 0), _I64(cfg.pool), _p(S))
    return S


def row_lse(Q, K, cfg: Config):
    """Natural-log softmax denominators of the observed rows [batch, n_q_heads, window]."""
    Q, K = _f64(Q), _f64(K)
    b, hq, n, d = Q.shape
    hk = K.shape[1]
    assert hq % hk == 0 and K.shape == (b, hk, n, d) and 1 <= cfg.window <= n
    L = np.empty((b, hq, cfg.window), dtype=np.float64)
    _load().aha_oracle_row_lse(
        _p(Q), _p(K), _I64(b), _I64(hq), _I64(hk), _I64(n), _I64(d), _I64(cfg.window),
        _I64(cfg.budget), ctypes.c_int(cfg.scale_mode), ctypes.c_double(cfg.fixed_scale),
        ctypes.c_double(cfg.lambda_floor), _p(L))
    return L


def window_attention(Q, K, V, window: int):
    """Causal attention output (standard scale) of the last `window` rows [b, n_q_heads, window, d]."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    b, hq, n, d = Q.shape
    hk = K.shape[1]
    assert hq % hk == 0 and K.shape == V.shape == (b, hk, n, d) and 1 <= window <= n
    O = np.empty((b, hq, window, d), dtype=np.float64)
    _load().aha_oracle_window_attention(_p(Q), _p(K), _p(V), _I64(b), _I64(hq), _I64(hk), _I64(n),
                                        _I64(d), _I64(window), _p(O))
    return O


def row_entropy(Q, K, cfg: Config):
    """Entropy (nats) of the observed softmax rows [batch, n_q_heads, window]."""
    Q, K = _f64(Q), _f64(K)
    b, hq, n, d = Q.shape
    hk = K.shape[1]
    assert hq % hk == 0 and K.shape == (b, hk, n, d) and 1 <= cfg.window <= n
    H = np.empty((b, hq, cfg.window), dtype=np.float64)
    _load().aha_oracle_row_entropy(
        _p(Q), _p(K), _I64(b), _I64(hq), _I64(hk), _I64(n), _I64(d), _I64(cfg.window),
        _I64(cfg.budget), ctypes.c_int(cfg.scale_mode), ctypes.c_double(cfg.fixed_scale),
        ctypes.c_double(cfg.lambda_floor), _p(H))
    return H


def prefill_scores_lse(Q, K, V, lse, cfg: Config):
    """Refined eviction scores [batch, n_kv_heads, n] from given row normalisers."""
    Q, K, V, lse = _f64(Q), _f64(K), _f64(V), _f64(lse)
    b, hq, n, d = Q.shape
    hk = K.shape[1]
    assert hq % hk == 0 and K.shape == V.shape == (b, hk, n, d)
    assert 1 <= cfg.window <= n and lse.shape == (b, hq, cfg.window)
    S = np.empty((b, hk, n), dtype=np.float64)
    _load().aha_oracle_prefill_scores_lse(
        _p(Q), _p(K), _p(V), _p(lse), _I64(b), _I64(hq), _I64(hk), _I64(n), _I64(d),
        _I64(cfg.window), _I64(cfg.budget), ctypes.c_int(cfg.scale_mode),
        ctypes.c_double(cfg.fixed_scale), ctypes.c_double(cfg.lambda_floor),
        ctypes.c_int(1 if cfg.value_prior else 0), _I64(cfg.pool), _p(S))
    return S


def select_topk(scores, budget: int, recent: int):
    """Ascending retained token indices [..., budget] (int32)."""
    scores = _f64(scores)
    n = scores.shape[-1]
    assert 0 <= recent <= budget <= n
    lead = scores.shape[:-1]
    problems = int(np.prod(lead)) if lead else 1
    idx = np.empty((problems, budget), dtype=np.int32)
    _load().aha_oracle_select_topk(_p(scores), _I64(problems), _I64(n),
                                   _I64(budget), _I64(recent), _p(idx, ctypes.c_int32))
    return idx.reshape(lead + (budget,))


def select_topk_sink(scores, budget: int, recent: int, sink: int):
    """Ascending retained indices [..., budget]: the first `sink` tokens, the `recent` last ones
    and the budget - sink - recent highest scores in between."""
    scores = _f64(scores)
    n = scores.shape[-1]
    assert sink >= 0 and recent >= 0 and sink + recent <= budget <= n
    lead = scores.shape[:-1]
    problems = int(np.prod(lead)) if lead else 1
    idx = np.empty((problems, budget), dtype=np.int32)
    _load().aha_oracle_select_topk_sink(_p(scores), _I64(problems), _I64(n), _I64(budget),
                                        _I64(recent), _I64(sink), _p(idx, ctypes.c_int32))
    return idx.reshape(lead + (budget,))


def pool_scores(scores, pool: int):
    """Average-pooled scores [..., n] (edge-truncated mean over `pool` tokens)."""
    scores = _f64(scores)
    n = scores.shape[-1]
    assert pool >= 1 and pool % 2 == 1
    lead = scores.shape[:-1]
    problems = int(np.prod(lead)) if lead else 1
    out = np.empty((problems, n), dtype=np.float64)
    _load().aha_oracle_pool_scores(_p(scores), _I64(problems), _I64(n), _I64(pool), _p(out))
    return out.reshape(scores.shape)


def select_topk_pooled(scores, budget: int, recent: int, score_pool: int, sink: int = 0):
    """Selection that ranks the candidates by their pooled scores (score_pool <= 1: the scores
    themselves), with `sink` first tokens always retained."""
    ranked = pool_scores(scores, score_pool) if score_pool > 1 else scores
    if sink:
        return select_topk_sink(ranked, budget, recent, sink)
    return select_topk(ranked, budget, recent)


@dataclass
class Cache:
    """Compact cache state; leading dims [batch, n_kv_heads]."""
    K: np.ndarray          # [b, hk, slots, d]
    V: np.ndarray          # [b, hk, slots, d]
    F: np.ndarray          # [b, hk, slots] running score
    pos: np.ndarray        # [b, hk, slots] int32 token position, -1 = free
    free_slot: np.ndarray  # [b, hk] int32


def compact_kv(K, V, scores, idx, slots: int) -> Cache:
    K, V, scores = _f64(K), _f64(V), _f64(scores)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    b, hk, n, d = K.shape
    budget = idx.shape[-1]
    assert slots >= budget + 1
    Kc = np.empty((b, hk, slots, d)); Vc = np.empty((b, hk, slots, d))
    Fc = np.empty((b, hk, slots)); pos = np.empty((b, hk, slots), dtype=np.int32)
    fs = np.empty((b, hk), dtype=np.int32)
    _load().aha_oracle_compact_kv(
        _p(K), _p(V), _p(scores), _p(idx, ctypes.c_int32), _I64(b * hk), _I64(n),
        _I64(d), _I64(budget), _I64(slots), _p(Kc), _p(Vc), _p(Fc),
        _p(pos, ctypes.c_int32), _p(fs, ctypes.c_int32))
    return Cache(Kc, Vc, Fc, pos, fs)


def decode_step(cache: Cache, q, k_new, v_new, logical_pos: int, cfg: Config):
    """One generation step in place on `cache`; returns out [b, n_q_heads, d].

    q [b, n_q_heads, d]; k_new, v_new [b, n_kv_heads, d];
    logical_pos = tokens seen so far including the new one.
    """
    q, k_new, v_new = _f64(q), _f64(k_new), _f64(v_new)
    b, hq, d = q.shape
    hk = k_new.shape[1]
    G = hq // hk
    slots = cache.K.shape[2]
    for a in (cache.K, cache.V, cache.F):
        assert a.dtype == np.float64 and a.flags.c_contiguous
    out = np.empty((b, hq, d), dtype=np.float64)
    _load().aha_oracle_decode_step_ext(
        _p(q), _p(k_new), _p(v_new), _I64(b * hk), _I64(G), _I64(d),
        _I64(cfg.budget), _I64(cfg.recent), _I64(slots), _I64(logical_pos),
        ctypes.c_int(cfg.scale_mode), ctypes.c_double(cfg.fixed_scale),
        ctypes.c_double(cfg.lambda_floor), _I64(cfg.sink),
        ctypes.c_int(1 if cfg.decode_value_prior else 0), _p(cache.K), _p(cache.V), _p(cache.F),
        _p(cache.pos, ctypes.c_int32), _p(cache.free_slot, ctypes.c_int32), _p(out))
    return out


def num_threads() -> int:
    """Threads the OpenMP loops will use (for the CPU-baseline report)."""
    v = os.environ.get("OMP_NUM_THREADS")
    if v:
        try:
            return int(v.split(",")[0])
        except ValueError:
            pass
    return os.cpu_count() or 1
