"""Pins for the CPU oracle: everything here is fixed by the paper's definitions
or by mathematics, never by the oracle's own output."""
import itertools
import json
import os

import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

from oracle import kvc_oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")
MAX, MEAN = orc.AGG_MAX, orc.AGG_MEAN


def rng(*key):
    return np.random.default_rng(list(key))


# ---------------------------------------------------------------- attention
def test_attention_reduces_to_library_softmax():
    # M = 1, G = 1, Hkv = 1, no head-mean: S is textbook softmax(q K^T / sqrt d).
    r = rng(1)
    d, n = 16, 50
    q = r.standard_normal((1, 1, d))
    k = r.standard_normal((1, n, d))
    s = orc.score_layer(q, k, add_head_mean=False)
    ref = scipy_softmax((k[0] @ q[0, 0]) / np.sqrt(d))
    np.testing.assert_allclose(s[0], ref, rtol=1e-13, atol=0)


def test_handworked_attention_fixture():
    g = json.load(open(os.path.join(GOLD, "handworked_section3_2_2.json")))
    ln2 = np.log(2.0)
    k = np.zeros((1, 3, 4))
    k[0, :, 0] = np.array(g["keys_first_coordinate_over_ln2"]) * ln2
    q = np.zeros((1, 2, 4))
    q[0, :, 0] = g["queries_first_coordinate"]
    a0 = orc.attention(q[0], k[0], 0.5)
    np.testing.assert_allclose(a0 * 7, g["attention_rows_times_7"], rtol=1e-14)
    s_max = orc.score_layer(q, k, agg_task=MAX)
    np.testing.assert_allclose(s_max[0] * 7, g["S_max_task_times_7"], rtol=1e-14)
    s_mean = orc.score_layer(q, k, agg_task=MEAN)
    np.testing.assert_allclose(s_mean[0] * 14, g["S_mean_task_times_14"], rtol=1e-14)


def test_scale_default_is_inverse_sqrt_d_and_override():
    r = rng(2)
    q = r.standard_normal((2, 3, 9))
    k = r.standard_normal((2, 7, 9))
    a = orc.score_layer(q, k)
    b = orc.score_layer(q, k, scale=1.0 / 3.0)
    np.testing.assert_allclose(a, b, rtol=1e-14)
    c = orc.score_layer(q, k, scale=0.7)
    assert np.abs(a - c).max() > 1e-3


def test_identical_keys_closed_form():
    # every key equal -> uniform attention 1/N -> S_group = 1/N, S = 2/N
    r = rng(3)
    hq, hkv, m, d, n = 6, 3, 5, 8, 37
    q = r.standard_normal((hq, m, d))
    k = np.broadcast_to(r.standard_normal((hkv, 1, d)), (hkv, n, d)).copy()
    for at in (MAX, MEAN):
        for ag in (MAX, MEAN):
            s = orc.score_layer(q, k, agg_task=at, agg_group=ag)
            np.testing.assert_allclose(s, 2.0 / n, rtol=1e-13)
            s0 = orc.score_layer(q, k, agg_task=at, agg_group=ag, add_head_mean=False)
            np.testing.assert_allclose(s0, 1.0 / n, rtol=1e-13)


def test_key_shift_invariance():
    r = rng(4)
    q = r.standard_normal((4, 6, 8))
    k = r.standard_normal((2, 33, 8))
    delta = r.standard_normal((2, 1, 8)) * 3.0
    np.testing.assert_allclose(orc.score_layer(q, k), orc.score_layer(q, k + delta),
                               rtol=1e-11)


def test_row_sum_identities():
    r = rng(5)
    q = r.standard_normal((6, 5, 8))
    k = r.standard_normal((3, 41, 8))
    s = orc.score_layer(q, k, agg_task=MEAN, agg_group=MEAN)
    np.testing.assert_allclose(s.sum(axis=1), 2.0, rtol=1e-12)        # rows of A sum to 1
    s0 = orc.score_layer(q, k, agg_task=MEAN, agg_group=MEAN, add_head_mean=False)
    np.testing.assert_allclose(s0.sum(axis=1), 1.0, rtol=1e-12)
    sm = orc.score_layer(q, k, agg_task=MAX, agg_group=MEAN, add_head_mean=False)
    tot = sm.sum(axis=1)
    assert np.all(tot >= 1.0 - 1e-12) and np.all(tot <= min(5, 41) + 1e-12)
    # sum over heads doubles under the augmentation
    np.testing.assert_allclose(orc.score_layer(q, k).sum(axis=0),
                               2.0 * sm.sum(axis=0), rtol=1e-12)


def test_one_hot_limit():
    # orthogonal keys scaled up, each query equal to one key -> indicator attention
    d = n = 8
    k = (np.eye(n) * 1e3)[None]
    targets = [5, 2, 5]
    q = k[0, targets][None]
    s = orc.score_layer(q, k, add_head_mean=False, scale=1.0)
    expect = np.zeros(n)
    expect[[5, 2]] = 1.0
    np.testing.assert_allclose(s[0], expect, atol=1e-300)


def test_gqa_grouping_is_row_major():
    # query head q must read KV head q // G: make only KV head 1 informative
    r = rng(6)
    hq, hkv, m, d, n = 4, 2, 3, 8, 9
    q = r.standard_normal((hq, m, d))
    k = r.standard_normal((hkv, n, d))
    s = orc.score_layer(q, k, add_head_mean=False)
    for h in range(hkv):
        rows = []
        for g in range(2):
            a = scipy_softmax((q[h * 2 + g] @ k[h].T) / np.sqrt(d), axis=1)
            rows.append(a.max(axis=0))
        np.testing.assert_allclose(s[h], np.mean(rows, axis=0), rtol=1e-13)


def test_permutation_invariance_and_equivariance():
    r = rng(7)
    hq, hkv, m, d, n = 6, 2, 4, 8, 21
    q = r.standard_normal((hq, m, d))
    k = r.standard_normal((hkv, n, d))
    base = orc.score_layer(q, k)
    np.testing.assert_allclose(orc.score_layer(q[:, r.permutation(m)], k), base, rtol=1e-12)
    qg = q.reshape(hkv, 3, m, d)[:, r.permutation(3)].reshape(hq, m, d)
    np.testing.assert_allclose(orc.score_layer(qg, k), base, rtol=1e-12)
    p = r.permutation(n)
    np.testing.assert_allclose(orc.score_layer(q, k[:, p]), base[:, p], rtol=1e-12)


def test_single_kv_head_doubles():
    r = rng(8)
    q = r.standard_normal((3, 4, 8))
    k = r.standard_normal((1, 17, 8))
    np.testing.assert_allclose(orc.score_layer(q, k),
                               2 * orc.score_layer(q, k, add_head_mean=False), rtol=1e-14)


def test_widen_bf16_bits():
    bits = np.array([0x3F80, 0xBF80, 0x4049, 0x0000, 0x3DCD], dtype=np.uint16)
    np.testing.assert_array_equal(orc.widen(bits),
                                  [1.0, -1.0, 3.140625, 0.0, 0.10009765625])


# ---------------------------------------------------------------- rank
def test_rank_matches_library_stable_argsort_with_many_ties():
    r = rng(9)
    s = np.round(r.random((5, 200)) * 8) / 8        # 9 distinct values -> many ties
    idx, ss = orc.head_rank(s)
    for h in range(5):
        np.testing.assert_array_equal(idx[h], np.argsort(-s[h], kind="stable"))
        assert sorted(idx[h]) == list(range(200))
        assert np.all(np.diff(ss[h]) <= 0)
        np.testing.assert_array_equal(ss[h], s[h, idx[h]])
        same = ss[h][1:] == ss[h][:-1]
        assert np.all(np.diff(idx[h])[same] > 0)   # ties in ascending index


def test_handworked_composite_fixture():
    g = json.load(open(os.path.join(GOLD, "handworked_section3_3.json")))
    s = np.array(g["S"])
    idx, ss = orc.head_rank(s)
    np.testing.assert_array_equal(idx, g["idx"])
    np.testing.assert_array_equal(ss, g["S_sorted"])
    i_all = np.stack([orc.composite(ss[l]) for l in range(2)])
    np.testing.assert_array_equal(i_all, g["I"])
    i_max = np.stack([orc.composite(ss[l], MAX) for l in range(2)])
    np.testing.assert_array_equal(i_max, g["I_max"])          # head aggregator = max-pooling
    for case in g["select"]:
        lengths, tau = orc.global_select(i_all, case["budget"])
        assert lengths.tolist() == case["lengths"], case
        assert tau == case["tau"], case
    # final selection: which original rows land in K'
    x = np.arange(2 * 2 * 4).reshape(2, 2, 4, 1).astype(np.float32) * 1.0
    lengths, _ = orc.global_select(i_all, 3)
    for l in range(2):
        out = orc.gather(x[l], idx[l], int(lengths[l]))
        rows = g["gather_budget_3_rows"][l]
        for h in range(2):
            np.testing.assert_array_equal(out[h, :, 0], x[l, h, rows[h], 0])


# ---------------------------------------------------------------- composite
def test_composite_properties():
    r = rng(10)
    s = r.random((4, 60))
    _, ss = orc.head_rank(s)
    for ah in (MAX, MEAN):
        i = orc.composite(ss, ah)
        assert np.all(np.diff(i) <= 0)
    assert orc.composite(ss, MEAN)[0] == pytest.approx(s.max(axis=1).mean(), rel=1e-15)
    same = np.broadcast_to(ss[:1], ss.shape)
    np.testing.assert_allclose(orc.composite(same), ss[0], rtol=1e-15)


# ---------------------------------------------------------------- global select
def _brute_lengths(i_all, budget):
    """Enumerate every (N_0..N_{L-1}) with sum = budget; best total prefix mass,
    ties -> lexicographically largest vector (lower layers filled first)."""
    lyr, n = i_all.shape
    pref = np.concatenate([np.zeros((lyr, 1)), np.cumsum(i_all, axis=1)], axis=1)
    best, best_vec = None, None
    for vec in itertools.product(range(n + 1), repeat=lyr):
        if sum(vec) != budget:
            continue
        tot = sum(pref[l, vec[l]] for l in range(lyr))
        if best is None or tot > best + 1e-12 or (abs(tot - best) <= 1e-12 and vec > best_vec):
            best, best_vec = tot, vec
    return list(best_vec)


def _brute_subset(pool, budget):
    """Literal top-B: the size-B subset with the largest sum; among equals the
    lexicographically smallest index tuple."""
    best, best_c = None, None
    for c in itertools.combinations(range(pool.size), budget):
        tot = pool[list(c)].sum()
        if best is None or tot > best + 1e-12:
            best, best_c = tot, c      # combinations() yields lexicographic order
    return best_c


@pytest.mark.parametrize("seed", range(6))
def test_global_select_brute_force(seed):
    r = rng(11, seed)
    lyr, n = 3, 4
    # quantised dyadic scores: exact sums and plenty of ties
    raw = np.round(r.random((lyr, n)) * 6) / 8
    i_all = -np.sort(-raw, axis=1)                      # each layer non-increasing
    for budget in range(lyr * n + 1):
        lengths, tau = orc.global_select(i_all, budget)
        assert lengths.sum() == budget
        assert lengths.tolist() == _brute_lengths(i_all, budget)
        if budget:
            taken = _brute_subset(i_all.reshape(-1), budget)
            assert np.bincount(np.array(taken) // n, minlength=lyr).tolist() == lengths.tolist()
            assert tau == np.partition(i_all.reshape(-1), -budget)[-budget]
            # the taken entries of a layer are a prefix of it
            for l in range(lyr):
                ks = sorted(t % n for t in taken if t // n == l)
                assert ks == list(range(len(ks)))


def test_global_select_special_cases():
    r = rng(12)
    i_all = -np.sort(-r.random((4, 9)), axis=1)
    assert orc.global_select(i_all, 0)[0].tolist() == [0] * 4
    assert orc.global_select(i_all, 36)[0].tolist() == [9] * 4
    assert orc.global_select(i_all[:1], 5)[0].tolist() == [5]
    same = np.broadcast_to(i_all[:1], (4, 9)).copy()
    for b in range(37):
        got = orc.global_select(same, b)[0]
        assert got.sum() == b and got.max() - got.min() <= 1
        assert np.all(np.diff(got) <= 0)               # larger shares on lower layers
    with pytest.raises(ValueError):
        orc.global_select(i_all, 37)


def test_sharper_layer_gets_more_budget():
    r = rng(13)
    hq, hkv, m, d, n, lyr = 4, 2, 8, 16, 128, 3
    qs = [r.standard_normal((hq, m, d)) for _ in range(lyr)]
    ks = [r.standard_normal((hkv, n, d)) for _ in range(lyr)]
    budget = lyr * n // 5
    base = orc.compress(qs, ks, None, budget)["lengths"]
    qs2 = [qs[0], qs[1] * 4.0, qs[2]]
    sharp = orc.compress(qs2, ks, None, budget)["lengths"]
    assert sharp[1] > base[1]


# ---------------------------------------------------------------- per-head sets / gather
def test_per_head_subset_is_optimal_brute_force():
    r = rng(14)
    s = np.round(r.random((3, 7)) * 8) / 8
    idx, _ = orc.head_rank(s)
    for n_keep in range(8):
        for h in range(3):
            chosen = s[h, idx[h, :n_keep]].sum()
            best = max((s[h, list(c)].sum() for c in itertools.combinations(range(7), n_keep)),
                       default=0.0)
            assert chosen == best


def test_gather_definition_and_topk_special_case():
    r = rng(15)
    k = r.standard_normal((1, 30, 4)).astype(np.float32)
    q = r.standard_normal((1, 2, 4))
    res = orc.compress([q], [k], [k], 7)
    assert res["lengths"].tolist() == [7]
    top = np.argsort(-res["S"][0, 0], kind="stable")[:7]
    np.testing.assert_array_equal(res["K_out"][0][0], k[0, top])
    assert res["K_out"][0].dtype == np.float32
    bits = (r.integers(0, 2 ** 16, size=(2, 10, 3))).astype(np.uint16)
    idx = np.stack([r.permutation(10), r.permutation(10)])
    out = orc.gather(bits, idx, 4)
    for h in range(2):
        for kk in range(4):
            np.testing.assert_array_equal(out[h, kk], bits[h, idx[h, kk]])


# ---------------------------------------------------------------- whole pass
def test_whole_pass_invariants():
    r = rng(16)
    hq, hkv, m, d, n, lyr = 4, 2, 4, 8, 40, 3
    qs = [r.standard_normal((hq, m, d)) for _ in range(lyr)]
    ks = [r.standard_normal((hkv, n, d)).astype(np.float32) for _ in range(lyr)]
    vs = [r.standard_normal((hkv, n, d)).astype(np.float32) for _ in range(lyr)]
    for budget in (0, 1, 17, lyr * n // 4, lyr * n):
        res = orc.compress(qs, ks, vs, budget)
        assert res["lengths"].sum() == budget
        for l in range(lyr):
            nl = int(res["lengths"][l])
            assert res["K_out"][l].shape == (hkv, nl, d)       # equal size across heads
            assert res["V_out"][l].shape == (hkv, nl, d)
            assert np.all(np.diff(res["I"][l]) <= 0)
            for h in range(hkv):
                sel = res["idx"][l, h, :nl]
                assert len(set(sel.tolist())) == nl
                np.testing.assert_array_equal(res["K_out"][l][h], ks[l][h, sel])
                np.testing.assert_array_equal(res["V_out"][l][h], vs[l][h, sel])
    full = orc.compress(qs, ks, vs, lyr * n)
    assert full["lengths"].tolist() == [n] * lyr
    for l in range(lyr):
        for h in range(hkv):
            assert sorted(full["idx"][l, h].tolist()) == list(range(n))   # identity as a set


def test_paper_cache_size_example():
    # Section 2.2 example: 32 layers x 8 KV heads x 32000 tokens x 128 dims x 2 (K and V)
    entries = 32 * 8 * 32000 * 128 * 2
    assert entries == 2_097_152_000                   # "about 2 G" entries
    r = 0.9
    assert int((1 - r) * 32 * 32000 + 1e-9) == 102_400   # budget formula at r = 0.9
