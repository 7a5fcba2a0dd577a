"""GPU parity of the dense preference score (Sec. 4.1, Eq. 6-9) against the oracle, through
the C ABI.  The score is a float32 sum of softmax masses: compared within 1e-4 * n_q per
head (logits are fp16 products accumulated in float32; an entry that swaps places with its
neighbour at the k-th position changes the sum by the difference of two nearly equal
masses)."""
import numpy as np
import pytest
import torch

import paper_2505_19586_amd as tkv
from oracle import preference
from synth import HeadShape, make_layer

pytestmark = pytest.mark.gpu
SM = 1.0 / np.sqrt(128.0)


def _run(q_last, k, top_k, *, shape=(32, 8), capacity=None):
    """q_last [n_q, Hq, D], k [Hkv, n, D] numpy fp16 -> (device scores [Hq], oracle scores [Hq])."""
    n_q, n = q_last.shape[0], k.shape[1]
    dp = tkv.DensePreference(n_q_heads=shape[0], n_kv_heads=shape[1], n_q=n_q, top_k=top_k,
                             capacity=capacity or n)
    qd = torch.from_numpy(q_last)[None].contiguous().cuda()
    kd = torch.from_numpy(np.ascontiguousarray(k.transpose(1, 0, 2)))[None].contiguous().cuda()
    out = dp.score(qd, kd, SM)
    out2 = dp.score(qd, kd, SM)                         # the workspace cleans up after itself
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    return dp, out[0].cpu().numpy().astype(np.float64), preference.dense_preference(q_last, k, top_k, SM)


@pytest.mark.parametrize("n,n_q,top_k", [(4096, 16, 128), (777, 16, 64), (5000, 32, 1024), (100, 16, 128),
                                         (16, 16, 1), (9000, 64, 896)])
def test_matches_oracle(n, n_q, top_k):
    print(f"case preference n={n} n_q={n_q} k={top_k}", flush=True)
    rng = np.random.default_rng(n)
    inp = make_layer(n, config=0, layer=1, seq=n % 31)
    q_last = (inp.q[None].astype(np.float32) + 0.5 * rng.standard_normal((n_q, 32, 128))).astype(np.float16)
    dp, got, want = _run(q_last, inp.k, top_k, capacity=n + 13)
    err = np.abs(got - want).max()
    print(f"   max |P - P_oracle| = {err:.2e} (P up to {want.max():.3f})", flush=True)
    assert err <= 1e-4 * n_q
    for tau in (0.05, 0.2, 0.6):
        friendly, score = dp.classify(torch.from_numpy(got), tau)
        assert abs(score - preference.layer_score(want, n_q)) <= 1e-3
        if abs(preference.layer_score(want, n_q) - tau) > 2e-3:
            assert friendly == (preference.classify(want, n_q, tau) == "quantization-friendly")


def test_closed_forms_on_the_gpu():
    n, n_q, k = 2048, 16, 256
    rng = np.random.default_rng(1)
    q_last = rng.standard_normal((n_q, 32, 128)).astype(np.float16)
    keys = np.tile(rng.standard_normal((8, 1, 128)).astype(np.float16), (1, n, 1))   # all keys of a head equal
    _, got, want = _run(q_last, keys, k)
    assert np.allclose(want, n_q * (1 - k / n), atol=1e-9)
    assert np.abs(got - want).max() <= 1e-4 * n_q
    # top_k >= n: nothing is outside
    _, got, _ = _run(q_last, keys[:, :200], 256)
    assert np.abs(got).max() <= 1e-4


def test_logits_sorted_along_the_sequence():
    """Every query's logit grows with the token index, so a row's top-k keys are its last k
    tokens: they sit in a few adjacent chunks, far more of them in one workgroup's share than its
    per-row list holds (the path that appends straight to memory), and the lower bound from
    the block maxima is at its loosest."""
    n, n_q, k = 20000, 16, 512
    rng = np.random.default_rng(7)
    u = rng.standard_normal((8, 1, 128))
    u /= np.linalg.norm(u, axis=-1, keepdims=True)
    ramp = (np.arange(n, dtype=np.float64) / n)[None, :, None]
    keys = (6.0 * ramp * u).astype(np.float16)
    q_last = (4.0 * np.repeat(u[:, 0], 4, axis=0)[None] + 0.05 * rng.standard_normal((n_q, 32, 128))).astype(np.float16)
    _, got, want = _run(q_last, keys, k)
    print(f"   max |P - P_oracle| = {np.abs(got - want).max():.2e} (P {want.min():.3f} .. {want.max():.3f})", flush=True)
    assert np.abs(got - want).max() <= 1e-4 * n_q
    _, got, want = _run(q_last, keys[:, ::-1].copy(), k)        # and falling
    assert np.abs(got - want).max() <= 1e-4 * n_q


def test_few_distinct_logit_values():
    """Keys drawn from three vectors per head: every row has three distinct logits with
    thousands of ties each; the top-k boundary falls inside a tie class (its mass is shared out
    by count), above it, or exactly on its edge."""
    n, n_q = 6000, 16
    rng = np.random.default_rng(8)
    base = rng.standard_normal((8, 3, 128)).astype(np.float16)
    which = rng.choice(3, size=n, p=[0.7, 0.2, 0.1])
    keys = base[:, which]
    q_last = rng.standard_normal((n_q, 32, 128)).astype(np.float16)
    counts = np.bincount(which, minlength=3)
    for k in (50, int(counts[2]), int(counts[2]) + 1, int(counts[1] + counts[2]), 3000):
        _, got, want = _run(q_last, keys, k)
        assert np.abs(got - want).max() <= 1e-4 * n_q, k


def test_groups_of_eight_and_many_rows():
    """Eight query heads per KV head, and n_q = 256 (1024 or 2048 rows per KV head: several slabs
    of 256 rows)."""
    rng = np.random.default_rng(9)
    for hq, hkv, n_q, n, k in ((16, 2, 256, 3000, 200), (8, 1, 48, 5000, 1000), (4, 4, 256, 2500, 64)):
        qs = rng.standard_normal((n_q, hq, 128)).astype(np.float16)
        ks = (rng.standard_normal((hkv, n, 128)) * 1.5).astype(np.float16)
        _, got, want = _run(qs, ks, k, shape=(hq, hkv))
        print(f"   Hq={hq} Hkv={hkv} n_q={n_q}: max |P - P_oracle| = {np.abs(got - want).max():.2e}", flush=True)
        assert np.abs(got - want).max() <= 1e-4 * n_q


def test_other_head_groupings_and_batch():
    shape = HeadShape(16, 8, 128)
    n, n_q, top_k = 1500, 32, 100
    rng = np.random.default_rng(4)
    qs = rng.standard_normal((2, n_q, 16, 128)).astype(np.float16)
    ks = rng.standard_normal((2, 8, n, 128)).astype(np.float16)
    dp = tkv.DensePreference(n_q_heads=16, n_kv_heads=8, n_q=n_q, top_k=top_k, capacity=n, batch=2)
    kd = torch.from_numpy(np.ascontiguousarray(ks.transpose(0, 2, 1, 3))).cuda()
    out = dp.score(torch.from_numpy(qs).cuda(), kd, SM)
    torch.cuda.synchronize()
    for b in range(2):
        want = preference.dense_preference(qs[b], ks[b], top_k, SM)
        assert np.abs(out[b].cpu().numpy() - want).max() <= 1e-4 * n_q


def test_argument_errors():
    with pytest.raises(tkv.TkvError):
        tkv.DensePreference(n_q=20, capacity=1000)            # n_q not a multiple of 16
    dp = tkv.DensePreference(n_q=16, top_k=8, capacity=64)
    q = torch.zeros(1, 16, 32, 128, dtype=torch.float16, device="cuda")
    k = torch.zeros(1, 65, 8, 128, dtype=torch.float16, device="cuda")
    with pytest.raises(tkv.TkvError):
        dp.score(q, k, SM)                                     # longer than the capacity
