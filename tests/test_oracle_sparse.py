"""Pins of the oracle's sparse path (Sec. 4.2 Stage 2; Sec. 5.1 n_local + n_topk)."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import attention, sparse
from synth import HeadShape, make_layer, static_channels

SMALL = HeadShape(8, 2, 128)


def _brute_topk(scores, k, lo, hi):
    """Selection by repeated scan: the k best by (score desc, index asc)."""
    cand = list(range(lo, hi))
    chosen = []
    for _ in range(min(k, len(cand))):
        best = None
        for t in cand:
            if best is None or scores[t] > scores[best]:
                best = t           # strict '>' keeps the lowest index among ties
        chosen.append(best)
        cand.remove(best)
    return sorted(chosen)


@settings(max_examples=200, deadline=None)
@given(st.lists(st.integers(-3, 3), min_size=1, max_size=40), st.integers(1, 12),
       st.integers(0, 5), st.integers(0, 5))
def test_topk_equals_brute_force_with_heavy_ties(vals, k, n_sink, n_win):
    s = np.array(vals, dtype=np.float32)
    n = len(vals)
    lo, hi = min(n_sink, n), max(n - n_win, min(n_sink, n))
    idx, cnt = sparse.topk_indices(s, k, lo, hi)
    ref = _brute_topk(s, k, lo, hi)
    assert cnt == len(ref)
    assert idx[:cnt].tolist() == ref
    assert (idx[cnt:] == -1).all()


def test_topk_all_equal_scores_takes_lowest_indices():
    s = np.zeros(100, dtype=np.float32)
    idx, cnt = sparse.topk_indices(s, 10, 4, 90)
    assert cnt == 10 and idx.tolist() == list(range(4, 14))
    # +0 and -0 are equal
    s[20] = -0.0
    idx, _ = sparse.topk_indices(s, 10, 4, 90)
    assert idx.tolist() == list(range(4, 14))


def test_scores_exact_on_small_integers():
    """With integer-valued inputs every product and partial sum is exact, so the
    pinned float32 order must equal the float64 sum over channels and heads."""
    rng = np.random.default_rng(3)
    q = rng.integers(-8, 9, size=(8, 128)).astype(np.float16)
    k = rng.integers(-8, 9, size=(2, 300, 128)).astype(np.float16)
    ch = np.stack([np.sort(rng.choice(128, 16, replace=False)) for _ in range(2)]).astype(np.int32)
    summ = sparse.key_summary(k, ch)
    s = sparse.approx_scores(q, summ, ch)
    for h in range(2):
        ref = sum(k[h][:, ch[h]].astype(np.float64) @ q[j][ch[h]].astype(np.float64)
                  for j in range(4 * h, 4 * h + 4))
        assert np.array_equal(s[h].astype(np.float64), ref)


def test_scores_close_to_float64_and_order_sensitive():
    inp = make_layer(2000, shape=SMALL, seq=9)
    ch = static_channels(inp.k, 16)
    summ = sparse.key_summary(inp.k, ch)
    s = sparse.approx_scores(inp.q, summ, ch)
    for h in range(2):
        kk = inp.k[h][:, ch[h]].astype(np.float64)
        qq = inp.q[4 * h:4 * h + 4][:, ch[h]].astype(np.float64)
        ref = (kk @ qq.T).sum(axis=1)
        bound = 64 * 2.0 ** -24 * (np.abs(kk) @ np.abs(qq).T).sum(axis=1)
        assert (np.abs(s[h] - ref) <= bound).all()
    # the channel list contains the planted outlier channels
    for h in range(2):
        assert set(inp.outlier_channels[h]) <= set(ch[h])
    # no -0 in the output
    assert not np.signbit(s[s == 0]).any()


def test_key_summary_uses_listed_channels_per_head():
    rng = np.random.default_rng(4)
    k = rng.standard_normal((2, 10, 128)).astype(np.float16)
    ch = np.array([[1, 5, 9], [0, 2, 127]], dtype=np.int32)
    s = sparse.key_summary(k, ch)
    assert s.shape == (2, 10, 3)
    assert np.array_equal(s[1, 7], k[1, 7, [0, 2, 127]])


def test_attended_set():
    a = sparse.attended_set(1000, np.array([10, 500, 7, -1, -1]), 4, 64)
    assert a.tolist() == [0, 1, 2, 3, 7, 10, 500] + list(range(936, 1000))
    # short sequences: sinks and window overlap, nothing duplicated
    assert sparse.attended_set(3, np.array([-1]), 4, 64).tolist() == [0, 1, 2]
    assert sparse.attended_set(50, np.array([-1]), 4, 64).tolist() == list(range(50))
    assert sparse.attended_set(0, np.array([-1]), 4, 64).tolist() == []


@pytest.mark.parametrize("n", [1, 3, 60, 68, 69, 300])
def test_k_covering_all_candidates_equals_dense(n):
    inp = make_layer(n, shape=SMALL, seq=10)
    ch = static_channels(inp.k, 16)
    summ = sparse.key_summary(inp.k, ch)
    idx, cnt = sparse.estimate_topk(inp.q, summ, ch, n, top_k=256, n_sink=4, n_window=64)
    assert (cnt == max(0, n - 68)).all()
    sm = 1 / np.sqrt(128)
    got = sparse.sparse_attention(inp.q, inp.k, inp.v, idx, cnt, n, sm, n_sink=4, n_window=64)
    ref = attention.decode_attention(inp.q, inp.k, inp.v, sm)
    assert np.abs(got - ref).max() < 1e-12


def test_sparse_attention_reads_only_the_attended_rows():
    inp = make_layer(400, shape=SMALL, seq=11)
    ch = static_channels(inp.k, 16)
    idx, cnt = sparse.estimate_topk(inp.q, sparse.key_summary(inp.k, ch), ch, 400,
                                    top_k=32, n_sink=4, n_window=64)
    sm = 1 / np.sqrt(128)
    base = sparse.sparse_attention(inp.q, inp.k, inp.v, idx, cnt, 400, sm, n_sink=4, n_window=64)
    k2, v2 = inp.k.copy(), inp.v.copy()
    for h in range(2):
        rows = sparse.attended_set(400, idx[h][:cnt[h]], 4, 64)
        mask = np.ones(400, bool)
        mask[rows] = False
        k2[h, mask] = 99
        v2[h, mask] = -99
        assert len(rows) == 4 + 32 + 64
    again = sparse.sparse_attention(inp.q, k2, v2, idx, cnt, 400, sm, n_sink=4, n_window=64)
    assert np.array_equal(base, again)
    # and equals dense attention restricted to those rows, per head
    for h in range(2):
        rows = sparse.attended_set(400, idx[h][:cnt[h]], 4, 64)
        ref = attention.decode_attention(inp.q[4 * h:4 * h + 4], inp.k[h:h + 1, rows], inp.v[h:h + 1, rows], sm)
        assert np.abs(base[4 * h:4 * h + 4] - ref).max() < 1e-13


def test_planted_dominant_tokens_are_recalled_at_small_n():
    """With a strong planted direction the estimate must rank the planted tokens
    on top (sanity of the scoring sign / head grouping, not a paper claim)."""
    inp = make_layer(2048, shape=SMALL, seq=12, dominance_gain=4.0)
    ch = static_channels(inp.k, 16)
    idx, cnt = sparse.estimate_topk(inp.q, sparse.key_summary(inp.k, ch), ch, 2048,
                                    top_k=128, n_sink=4, n_window=64)
    full = static_channels(inp.k, 128)
    idx_full, _ = sparse.estimate_topk(inp.q, sparse.key_summary(inp.k, full), full, 2048,
                                       top_k=128, n_sink=4, n_window=64)
    for h in range(2):
        assert set(inp.dominant_tokens[h]) <= set(idx_full[h])   # all 128 channels: exact logits
        assert len(set(inp.dominant_tokens[h]) & set(idx[h])) >= 4


def test_critical_channels_eq10():
    q_hat = np.array([0.1, -3.0, 0.5, 2.0])
    k = np.array([[1.0, 0.1, -4.0, 0.5], [-2.0, 0.2, 1.0, -0.5]])
    # s = |q| * max|K| = [0.2, 0.6, 2.0, 1.0]
    assert sparse.critical_channels(q_hat, k, 2).tolist() == [2, 3]
    assert sparse.critical_channels(q_hat, k, 3).tolist() == [1, 2, 3]


def test_select_channels_hand_worked_group():
    """Two query heads share one KV head: s_i = (|q_0,i| + |q_1,i|) * max|K_i|."""
    q_hat = np.array([[1.0, -2.0, 0.5, 0.0, 3.0, 1.0],
                      [0.5, 1.0, -0.5, 0.0, -1.0, 1.0]], np.float16)
    k = np.array([[[4.0, 1.0, -10.0, 100.0, 0.5, 2.0],
                   [-2.0, 0.5, 1.0, -7.0, 0.25, -2.0]]], np.float16)
    amax = sparse.channel_absmax(k)
    assert amax.tolist() == [[4.0, 1.0, 10.0, 100.0, 0.5, 2.0]]
    # sums of magnitudes [1.5, 3, 1, 0, 4, 2] -> s = [6, 3, 10, 0, 2, 4]
    assert sparse.select_channels(q_hat, amax, 1).tolist() == [[2]]
    assert sparse.select_channels(q_hat, amax, 3).tolist() == [[0, 2, 5]]
    assert sparse.select_channels(q_hat, amax, 4).tolist() == [[0, 1, 2, 5]]
    # a channel the query does not use is never preferred, however large its keys are
    assert 3 not in sparse.select_channels(q_hat, amax, 5)[0]


def test_select_channels_reduces_to_eq10_for_one_head_and_maximises_the_sum():
    from itertools import combinations
    rng = np.random.default_rng(17)
    for trial in range(20):
        d, ds = 7, 3
        q_hat = rng.standard_normal((1, d)).astype(np.float16)
        k = rng.standard_normal((1, 30, d)).astype(np.float16)
        got = sparse.select_channels(q_hat, sparse.channel_absmax(k), ds)[0]
        assert got.tolist() == sparse.critical_channels(q_hat[0], k[0], ds).tolist()
        s = np.abs(q_hat[0].astype(np.float64)) * np.abs(k[0].astype(np.float64)).max(axis=0)
        best = max(combinations(range(d), ds), key=lambda c: s[list(c)].sum())
        assert np.isclose(s[got].sum(), s[list(best)].sum())


def test_select_channels_ties_invariances_and_outliers():
    # all-equal contributions: the lowest channels win
    q_hat = np.ones((4, 128), np.float16)
    amax = np.ones((1, 128), np.float32)
    assert sparse.select_channels(q_hat, amax, 16)[0].tolist() == list(range(16))
    # positive rescaling of the query does not change the list; permuting channels permutes it
    rng = np.random.default_rng(23)
    inp = make_layer(512, seq=3)
    amax = sparse.channel_absmax(inp.k)
    base = sparse.select_channels(inp.q, amax, 16)
    assert np.array_equal(sparse.select_channels(inp.q * np.float16(2), amax, 16), base)
    perm = rng.permutation(128)
    permuted = sparse.select_channels(inp.q[:, perm], amax[:, perm], 16)
    for h in range(8):
        assert sorted(perm[permuted[h]].tolist()) == base[h].tolist()
    # a flat query picks the planted outlier channels of the keys (x10 by construction)
    flat = np.ones_like(inp.q)
    picked = sparse.select_channels(flat, amax, 16)
    for h in range(8):
        assert set(inp.outlier_channels[h]) <= set(picked[h].tolist())
    # the running maximum over appended pieces equals the maximum over the whole cache
    a = np.maximum(sparse.channel_absmax(inp.k[:, :100]), sparse.channel_absmax(inp.k[:, 100:]))
    assert np.array_equal(a, amax)
