"""Pins for the oracle's elementary operations: invariants, closed forms,
brute force and library routines -- nothing here re-types the oracle's own
formula."""
import itertools

import numpy as np
import pytest
import torch

from oracle import lsq_oracle as O


def test_softmax_rows_sum_to_one_and_shift_invariant():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal((7, 1000)) * 3).astype(np.float32)
    p = O.softmax(x)
    assert np.all(np.abs(p.sum(-1) - 1) < 1e-6)
    assert np.all(p >= 0)
    np.testing.assert_allclose(O.softmax(x + np.float32(11.5)), p, rtol=2e-5, atol=1e-9)
    lp = O.log_softmax(x)
    assert np.all(np.abs(np.exp(lp.astype(np.float64)).sum(-1) - 1) < 1e-5)
    # large offsets must not overflow
    assert np.isfinite(O.log_softmax(x + np.float32(1e4))).all()


def test_log_softmax_matches_torch():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal((5, 333)) * 2).astype(np.float64)
    ref = torch.log_softmax(torch.from_numpy(x), -1).numpy()
    np.testing.assert_allclose(O.log_softmax(x), ref, rtol=0, atol=1e-12)
    ref32 = torch.log_softmax(torch.from_numpy(x.astype(np.float32)), -1).numpy()
    np.testing.assert_allclose(O.log_softmax(x.astype(np.float32)), ref32, rtol=0, atol=2e-6)


def test_softmax_ignores_masked_keys():
    x = np.array([[0.3, -np.inf, 1.2, -np.inf]], np.float32)
    p = O.softmax(x)
    assert p[0, 1] == 0 and p[0, 3] == 0
    np.testing.assert_allclose(p[0, [0, 2]], O.softmax(x[:, [0, 2]])[0], rtol=1e-7)


def test_layer_norm_moments_and_torch():
    rng = np.random.default_rng(2)
    v = (rng.standard_normal((9, 64)) * 4 + 3).astype(np.float64)
    one, zero = np.ones(64), np.zeros(64)
    y = O.layer_norm(v, one, zero, 0.0)
    assert np.abs(y.mean(-1)).max() < 1e-12
    assert np.abs(y.var(-1) - 1).max() < 1e-12          # biased variance
    g, b = rng.standard_normal(64), rng.standard_normal(64)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(v), (64,), torch.from_numpy(g),
                                         torch.from_numpy(b), 1e-5).numpy()
    np.testing.assert_allclose(O.layer_norm(v, g, b, 1e-5), ref, rtol=0, atol=1e-12)
    ref32 = torch.nn.functional.layer_norm(torch.from_numpy(v.astype(np.float32)), (64,),
                                           torch.from_numpy(g.astype(np.float32)),
                                           torch.from_numpy(b.astype(np.float32)), 1e-5).numpy()
    got32 = O.layer_norm(v.astype(np.float32), g.astype(np.float32), b.astype(np.float32), 1e-5)
    np.testing.assert_allclose(got32, ref32, rtol=0, atol=5e-6)


def test_positional_encoding_closed_forms():
    d = 64
    pe0 = O.positional_encoding(0, d, np.float64)[0]
    assert np.array_equal(pe0[0::2], np.zeros(d // 2)) and np.array_equal(pe0[1::2], np.ones(d // 2))
    for p in (1, 7, 100):
        pe = O.positional_encoding(p, d, np.float64)[0]
        assert abs(pe[0] - np.sin(p)) < 1e-15 and abs(pe[1] - np.cos(p)) < 1e-15
        # last pair uses wavelength 10000^((d-2)/d)
        w = 10000.0 ** ((d - 2) / d)
        assert abs(pe[d - 2] - np.sin(p / w)) < 1e-15 and abs(pe[d - 1] - np.cos(p / w)) < 1e-15
        # every (sin, cos) pair lies on the unit circle
        assert np.abs(pe[0::2] ** 2 + pe[1::2] ** 2 - 1).max() < 1e-14
    # angle-addition: PE(p+q) pairs are rotations of PE(p) by q * frequency
    a, b = O.positional_encoding([3, 5, 8], d, np.float64)[:, 0:2], None
    s3, c3, s5, c5, s8, c8 = a[0, 0], a[0, 1], a[1, 0], a[1, 1], a[2, 0], a[2, 1]
    assert abs(s8 - (s3 * c5 + c3 * s5)) < 1e-14 and abs(c8 - (c3 * c5 - s3 * s5)) < 1e-14


def test_attention_single_key_returns_value():
    rng = np.random.default_rng(3)
    q = rng.standard_normal((5, 32)).astype(np.float32)
    K = rng.standard_normal((1, 32)).astype(np.float32)
    V = rng.standard_normal((1, 32)).astype(np.float32)
    out = O.attention(q, K, V, 4)
    assert np.array_equal(out, np.repeat(V, 5, 0))


def test_attention_matches_torch_sdpa():
    rng = np.random.default_rng(4)
    H, dh, nq, nk = 4, 16, 6, 11
    q = rng.standard_normal((nq, H * dh))
    K = rng.standard_normal((nk, H * dh))
    V = rng.standard_normal((nk, H * dh))
    allowed = rng.random((nq, nk)) < 0.7
    allowed[:, 0] = True
    tq = torch.from_numpy(q).view(nq, H, dh).transpose(0, 1)
    tk = torch.from_numpy(K).view(nk, H, dh).transpose(0, 1)
    tv = torch.from_numpy(V).view(nk, H, dh).transpose(0, 1)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=torch.from_numpy(allowed))
    ref = ref.transpose(0, 1).reshape(nq, H * dh).numpy()
    np.testing.assert_allclose(O.attention(q, K, V, H, allowed), ref, rtol=0, atol=1e-12)
    # heads are independent: permuting whole heads of q,K,V permutes the output
    perm = [2, 0, 3, 1]
    cols = np.concatenate([np.arange(h * dh, (h + 1) * dh) for h in perm])
    np.testing.assert_allclose(O.attention(q[:, cols], K[:, cols], V[:, cols], H, allowed), ref[:, cols],
                               rtol=0, atol=1e-12)


def _brute_topk(scores, flat, k):
    """k rounds of linear scan for the best remaining candidate."""
    left = list(range(len(scores)))
    out = []
    for _ in range(min(k, len(left))):
        best = left[0]
        for i in left[1:]:
            if scores[i] > scores[best] or (scores[i] == scores[best] and flat[i] < flat[best]):
                best = i
        out.append(best)
        left.remove(best)
    return out


@pytest.mark.parametrize("case", ["random", "duplicates", "all_equal", "neg_inf", "shuffled_flat"])
def test_topk_full_sort_equals_brute_force(case):
    rng = np.random.default_rng(5)
    n, k = 60, 7
    s = rng.standard_normal(n).astype(np.float32)
    flat = np.arange(n, dtype=np.int64)
    if case == "duplicates":
        s = np.round(s * 2) / 2
    elif case == "all_equal":
        s[:] = 0.25
    elif case == "neg_inf":
        s[rng.random(n) < 0.93] = -np.inf
    elif case == "shuffled_flat":
        s = np.round(s)
        flat = rng.permutation(n).astype(np.int64)
    got = list(O.topk_by_full_sort(s, flat, k))
    assert got == _brute_topk(s, flat, k)


def test_retrieve_threshold_keeps_topk_for_any_partition():
    rng = np.random.default_rng(6)
    V = 500
    for trial in range(200):
        k = int(rng.integers(1, 9))
        x = rng.standard_normal(V).astype(np.float32)
        if trial % 3 == 0:
            x = np.round(x * 4) / 4      # many ties, including at the threshold
        groups = rng.permutation(np.arange(V) % k)
        cand, R = O.hars_retrieve(x, k, groups)
        top = O.topk_by_full_sort(x, np.arange(V), k)
        assert set(top) <= set(cand)
        assert (x[cand] >= R).all() and len(cand) >= k
    # strict ">" would lose an element: two groups, each holding one copy of the maximum
    x = np.array([1.0, 0.0, 1.0, 0.0], np.float32)
    cand, R = O.hars_retrieve(x, 2, np.array([0, 0, 1, 1]))
    assert R == 1.0 and list(cand) == [0, 2] and not (x > R).any()
