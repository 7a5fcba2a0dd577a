"""Pins of the oracle's dense preference score (Sec. 4.1, Eq. 6-9)."""
import numpy as np
import pytest

from oracle import preference
from synth import make_layer


def _rand(n_q, hq, hkv, n, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((n_q, hq, 16)).astype(np.float16),
            rng.standard_normal((hkv, n, 16)).astype(np.float16))


def test_uniform_attention_closed_form():
    """All keys equal -> every row of Eq. 6 is 1/n -> P = n_q (1 - k/n)."""
    n_q, n, k = 8, 200, 50
    q = np.random.default_rng(0).standard_normal((n_q, 4, 16))
    keys = np.tile(np.random.default_rng(1).standard_normal((1, 1, 16)), (2, n, 1))
    p = preference.dense_preference(q, keys, k, 0.25)
    assert np.allclose(p, n_q * (1 - k / n), rtol=0, atol=1e-12)
    # k >= n: all the mass is inside the top-k
    assert np.allclose(preference.dense_preference(q, keys, n, 0.25), 0.0, atol=1e-12)
    assert np.allclose(preference.dense_preference(q, keys, n + 7, 0.25), 0.0, atol=1e-12)


def test_one_dominant_key_gives_zero_and_is_sparsity_friendly():
    n_q, n = 4, 100
    q = np.zeros((n_q, 2, 8)); q[..., 0] = 1.0
    keys = np.zeros((1, n, 8)); keys[0, 37, 0] = 200.0       # logit 200 against 0 everywhere else
    p = preference.dense_preference(q, keys, 1, 1.0)
    assert (p < 1e-60).all() and (p >= 0).all()
    assert preference.classify(p, n_q, 0.2) == "sparsity-friendly"
    # flat attention over 1000 keys with k = 10: 99 % of the mass is outside
    keys = np.zeros((1, 1000, 8))
    p = preference.dense_preference(q, keys, 10, 1.0)
    assert np.isclose(preference.layer_score(p, n_q), 0.99)
    assert preference.classify(p, n_q, 0.2) == "quantization-friendly"


def test_brute_force_rows_and_head_mapping():
    """Eq. 6-8 written out with python loops on a tiny case, grouped heads."""
    n_q, hq, hkv, n, k = 3, 4, 2, 11, 4
    q, keys = _rand(n_q, hq, hkv, n, 5)
    got = preference.dense_preference(q, keys, k, 0.3)
    for j in range(hq):
        h = j // (hq // hkv)
        total = 0.0
        for i in range(n_q):
            logits = [0.3 * float(np.dot(q[i, j].astype(np.float64), keys[h, t].astype(np.float64))) for t in range(n)]
            m = max(logits)
            e = [np.exp(x - m) for x in logits]
            a = sorted((x / sum(e) for x in e), reverse=True)
            total += sum(a[:k])
        assert np.isclose(got[j], n_q - total, rtol=1e-12, atol=1e-12)


def test_monotone_in_k_and_bounded():
    q, keys = _rand(6, 4, 2, 300, 9)
    prev = None
    for k in (1, 2, 10, 100, 299, 300):
        p = preference.dense_preference(q, keys, k, 0.25)
        assert (p >= -1e-12).all() and (p <= 6).all()
        if prev is not None:
            assert (p <= prev + 1e-12).all()       # more keys kept, less mass outside
        prev = p
    assert np.allclose(prev, 0.0, atol=1e-12)


def test_synthetic_layers_separate():
    """The workload generator's planted dominant tokens make a layer sparsity-friendly once
    their gain is large; plain Gaussian keys at a long context are quantization-friendly."""
    n, n_q, k = 4096, 8, 64
    sparse_like = make_layer(n, seq=1, dominance_gain=6.0)
    q = np.repeat(sparse_like.q[None], n_q, axis=0)                   # rows near the planted direction
    p_sparse = preference.dense_preference(q, sparse_like.k, k, 128 ** -0.5)
    rng = np.random.default_rng(3)
    qd = rng.standard_normal((n_q, 32, 128)).astype(np.float16) * np.float16(0.3)
    kd = rng.standard_normal((8, n, 128)).astype(np.float16)
    p_dense = preference.dense_preference(qd, kd, k, 128 ** -0.5)
    assert preference.layer_score(p_sparse, n_q) < 0.2 < preference.layer_score(p_dense, n_q)
    assert preference.classify(p_sparse, n_q, 0.2) == "sparsity-friendly"
    assert preference.classify(p_dense, n_q, 0.2) == "quantization-friendly"
