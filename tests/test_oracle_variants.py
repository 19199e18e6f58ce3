"""Pins for the oracle's variants: value-norm weighting, position order,
per-layer floor, unstructured selection.  Each is checked against hand-worked
numbers (tests/golden/handworked_variants.json), an invariant the mathematics
fixes, or a brute-force enumeration written independently of the oracle."""
import itertools
import json
import math
import os

import numpy as np
import pytest

from oracle import kvc_oracle as orc

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "handworked_variants.json")))


# ---------------------------------------------------------------- value norm
def test_vnorm_handworked_attention_and_scores():
    g = GOLD["vnorm"]
    q, k, v = np.array(g["q"]), np.array(g["k"]), np.array(g["v"])
    for qh in range(2):
        a = orc.attention(q[qh], k[0], g["scale"])
        np.testing.assert_allclose(a, np.array(g["attention"][qh]), rtol=0, atol=1e-15)
    s_w = orc.score_layer(q, k, scale=g["scale"], v=v)
    s_p = orc.score_layer(q, k, scale=g["scale"])
    np.testing.assert_allclose(s_w, np.array(g["S_weighted"]), rtol=1e-14)
    np.testing.assert_allclose(s_p, np.array(g["S_plain"]), rtol=1e-14)


def test_vnorm_uses_euclidean_norm_of_the_value_row():
    g = GOLD["vnorm_norm"]   # uniform attention 1/2; norms 5 and 2; one KV head doubles under the head mean
    s = orc.score_layer(np.array(g["q"]), np.array(g["k"]), v=np.array(g["v"]))
    np.testing.assert_allclose(s, np.array(g["S_weighted"]), rtol=1e-15)


def _brute_weighted_scores(q, k, v, agg_task, agg_group, add_head_mean):
    """Element-by-element loops over the weighted attention matrix."""
    hq, m, d = q.shape
    hkv, n, _ = k.shape
    g = hq // hkv
    scale = 1.0 / math.sqrt(d)
    s_task = [[0.0] * n for _ in range(hq)]
    for qh in range(hq):
        h = qh // g
        rows = []
        for mm in range(m):
            logits = [scale * sum(q[qh, mm, j] * k[h, c, j] for j in range(d)) for c in range(n)]
            top = max(logits)
            ex = [math.exp(x - top) for x in logits]
            z = sum(ex)
            rows.append([ex[c] / z * math.sqrt(sum(v[h, c, j] ** 2 for j in range(d))) for c in range(n)])
        for c in range(n):
            col = [rows[mm][c] for mm in range(m)]
            s_task[qh][c] = max(col) if agg_task == orc.AGG_MAX else sum(col) / m
    s_group = [[0.0] * n for _ in range(hkv)]
    for h in range(hkv):
        for c in range(n):
            col = [s_task[h * g + gg][c] for gg in range(g)]
            s_group[h][c] = max(col) if agg_group == orc.AGG_MAX else sum(col) / g
    out = np.array(s_group)
    if add_head_mean:
        out = out + np.array([sum(s_group[h][c] for h in range(hkv)) / hkv for c in range(n)])[None, :]
    return out


@pytest.mark.parametrize("agg_task,agg_group,add", [(0, 1, True), (1, 0, False), (1, 1, True), (0, 0, True)])
def test_vnorm_matches_bruteforce(agg_task, agg_group, add):
    rng = np.random.default_rng(5)
    q = rng.standard_normal((4, 3, 5))
    k = rng.standard_normal((2, 7, 5))
    v = rng.standard_normal((2, 7, 5)) * rng.uniform(0.1, 10.0, size=(2, 7, 1))
    got = orc.score_layer(q, k, agg_task=agg_task, agg_group=agg_group, add_head_mean=add, v=v)
    want = _brute_weighted_scores(q, k, v, agg_task, agg_group, add)
    np.testing.assert_allclose(got, want, rtol=1e-12)


def test_vnorm_unit_rows_change_nothing_and_scaling_is_homogeneous():
    rng = np.random.default_rng(6)
    q = rng.standard_normal((4, 3, 8))
    k = rng.standard_normal((2, 9, 8))
    v = rng.standard_normal((2, 9, 8))
    unit = v / np.linalg.norm(v, axis=2, keepdims=True)
    plain = orc.score_layer(q, k)
    np.testing.assert_allclose(orc.score_layer(q, k, v=unit), plain, rtol=1e-13)
    np.testing.assert_allclose(orc.score_layer(q, k, v=3.5 * v), 3.5 * orc.score_layer(q, k, v=v), rtol=1e-13)
    # the weight depends on the KV head and the token only: per head it is a column scaling
    w = np.linalg.norm(v, axis=2)
    np.testing.assert_allclose(orc.score_layer(q, k, v=v, add_head_mean=False),
                               w * orc.score_layer(q, k, add_head_mean=False), rtol=1e-13)


# ------------------------------------------------------------- per-layer floor
def test_floor_handworked():
    g = GOLD["floor"]
    i_all = np.array(g["I"])
    lengths, tau = orc.global_select(i_all, g["budget"])
    assert lengths.tolist() == g["plain_lengths"] and tau == g["plain_tau"]
    lengths, tau = orc.global_select(i_all, g["budget"], g["min_per_layer"])
    assert lengths.tolist() == g["floor_lengths"] and tau == g["floor_tau"]


def _brute_select(pool_rows, budget, floor):
    """Tuple sort, written without numpy indexing tricks."""
    rows, n = len(pool_rows), len(pool_rows[0])
    f = min(floor, n)
    forced = [(r, kk) for r in range(rows) for kk in range(f)]
    free = [(-pool_rows[r][kk], r * n + kk) for r in range(rows) for kk in range(f, n)]
    free.sort()
    chosen = forced + [(flat // n, flat % n) for _, flat in free[:budget - len(forced)]]
    lengths = [0] * rows
    for r, _ in chosen:
        lengths[r] += 1
    return lengths, chosen


@pytest.mark.parametrize("seed", range(6))
def test_floor_and_ties_match_bruteforce(seed):
    rng = np.random.default_rng(seed)
    rows, n = 3, 5
    # few distinct values -> many ties, non-increasing rows like real composite scores
    raw = np.sort(rng.integers(0, 4, size=(rows, n)).astype(np.float64), axis=1)[:, ::-1]
    for floor in (0, 1, 2, 7):
        f = min(floor, n)
        for budget in range(rows * f, rows * n + 1):
            lengths, tau = orc.global_select(raw, budget, floor)
            want, chosen = _brute_select(raw.tolist(), budget, floor)
            assert lengths.tolist() == want
            assert int(lengths.sum()) == budget and int(lengths.min()) >= f
            # non-increasing rows: the chosen entries of a row are a prefix
            for r in range(rows):
                assert sorted(kk for rr, kk in chosen if rr == r) == list(range(want[r]))


def test_floor_budget_below_the_floor_is_an_error():
    with pytest.raises(ValueError):
        orc.global_select(np.zeros((4, 6)), 7, 2)
    lengths, tau = orc.global_select(np.zeros((4, 6)), 8, 2)
    assert lengths.tolist() == [2, 2, 2, 2] and tau is None


# --------------------------------------------------------------- unstructured
def test_unstructured_handworked():
    g = GOLD["unstructured"]
    s3 = np.array(g["S_sorted"])
    lyr, hkv, n = s3.shape
    lengths, tau = orc.global_select(s3.reshape(lyr * hkv, n), g["budget"])
    assert lengths.reshape(lyr, hkv).tolist() == g["lengths"] and tau == g["tau"]


def test_unstructured_compress_is_per_head_topk_of_the_global_pool():
    rng = np.random.default_rng(11)
    lyr, hq, hkv, n, m, d = 2, 4, 2, 12, 3, 8
    q = [rng.standard_normal((hq, m, d)).astype(np.float32) for _ in range(lyr)]
    k = [rng.standard_normal((hkv, n, d)).astype(np.float32) for _ in range(lyr)]
    v = [rng.standard_normal((hkv, n, d)).astype(np.float32) for _ in range(lyr)]
    budget = 17
    out = orc.compress(q, k, v, budget, unstructured=True)
    assert out["I"] is None and out["lengths"].shape == (lyr, hkv) and int(out["lengths"].sum()) == budget
    # brute force: the 17 largest of all Lyr*Hkv*N scores S (the same multiset as S')
    entries = sorted(((-out["S"][l, h, c], l, h, c) for l in range(lyr) for h in range(hkv) for c in range(n)))
    keep = {(l, h): set() for l in range(lyr) for h in range(hkv)}
    for _, l, h, c in entries[:budget]:
        keep[(l, h)].add(c)
    for l in range(lyr):
        for h in range(hkv):
            nl = int(out["lengths"][l, h])
            assert set(out["idx"][l, h, :nl].tolist()) == keep[(l, h)]
            np.testing.assert_array_equal(out["K_out"][l][h], k[l][h, out["idx"][l, h, :nl]])
            np.testing.assert_array_equal(out["V_out"][l][h], v[l][h, out["idx"][l, h, :nl]])


# ------------------------------------------------------------- position order
def test_position_order_handworked():
    g = GOLD["position"]
    idx = np.array(g["idx"])
    x = np.arange(2 * 4 * 1).reshape(2, 4, 1) % 4          # row content = its own position
    rank = orc.gather(x, idx, g["n_keep"])
    pos = orc.gather(x, idx, g["n_keep"], position_order=True)
    assert rank[..., 0].tolist() == g["rows_rank"] and pos[..., 0].tolist() == g["rows_position"]


def test_position_order_full_budget_is_the_identity_and_sets_agree():
    rng = np.random.default_rng(3)
    lyr, hq, hkv, n, m, d = 2, 4, 2, 10, 2, 4
    q = [rng.standard_normal((hq, m, d)).astype(np.float32) for _ in range(lyr)]
    k = [rng.standard_normal((hkv, n, d)).astype(np.float32) for _ in range(lyr)]
    v = [rng.standard_normal((hkv, n, d)).astype(np.float32) for _ in range(lyr)]
    full = orc.compress(q, k, v, lyr * n, position_order=True)
    for l in range(lyr):
        np.testing.assert_array_equal(full["K_out"][l], k[l])
        np.testing.assert_array_equal(full["V_out"][l], v[l])
    a = orc.compress(q, k, v, 9)
    b = orc.compress(q, k, v, 9, position_order=True)
    assert a["lengths"].tolist() == b["lengths"].tolist()
    for l in range(lyr):
        nl = int(a["lengths"][l])
        for h in range(hkv):
            rows = a["idx"][l, h, :nl]
            np.testing.assert_array_equal(b["K_out"][l][h], k[l][h, np.sort(rows)])
            assert sorted(map(bytes, a["K_out"][l][h])) == sorted(map(bytes, b["K_out"][l][h]))


# ---------------------------------------------------------------- causal tail
def test_causal_tail_handworked():
    g = GOLD["causal_tail"]
    q, k = np.array(g["q"]), np.array(g["k"])
    a = orc.attention(q[0], k[0], g["scale"], causal_tail=True)
    np.testing.assert_allclose(a, np.array(g["attention"]), rtol=0, atol=1e-15)
    np.testing.assert_allclose(orc.score_layer(q, k, scale=g["scale"], causal_tail=True), np.array(g["S"]), rtol=1e-14)
    np.testing.assert_allclose(orc.score_layer(q, k, scale=g["scale"]), np.array(g["S_unmasked"]), rtol=1e-14)


def test_causal_tail_rows_are_softmaxes_over_their_visible_prefix():
    rng = np.random.default_rng(8)
    m, n, d = 5, 11, 6
    q, k = rng.standard_normal((m, d)), rng.standard_normal((n, d))
    a = orc.attention(q, k, 0.3, causal_tail=True)
    for mm in range(m):
        vis = n - m + mm + 1                                   # keys 0 .. N-M+m
        assert np.all(a[mm, vis:] == 0.0)
        # brute force over the visible keys only
        logits = [0.3 * sum(q[mm, j] * k[c, j] for j in range(d)) for c in range(vis)]
        z = sum(math.exp(x) for x in logits)
        np.testing.assert_allclose(a[mm, :vis], [math.exp(x) / z for x in logits], rtol=1e-13)
    np.testing.assert_allclose(a.sum(axis=1), 1.0, rtol=1e-14)
    # the last task token sees everything: its row equals the unmasked one; one task token = no mask
    np.testing.assert_allclose(a[-1], orc.attention(q, k, 0.3)[-1], rtol=1e-14)
    np.testing.assert_allclose(orc.attention(q[:1], k, 0.3, causal_tail=True), orc.attention(q[:1], k, 0.3), rtol=1e-14)
    with pytest.raises(ValueError):
        orc.attention(q, k[:4], 0.3, causal_tail=True)


# ------------------------------------------------------------ forced retention
def test_force_keep_marks_exactly_the_named_tokens():
    s = np.arange(12.0).reshape(2, 6)
    out = orc.force_keep(s, 2, 1)
    assert np.isinf(out[:, [0, 1, 5]]).all() and np.array_equal(out[:, 2:5], s[:, 2:5])
    assert orc.force_keep(s, 0, 0) is s
    assert np.isinf(orc.force_keep(s, 4, 4)).all()            # overlapping ranges cover everything
    with pytest.raises(ValueError):
        orc.force_keep(s, -1, 0)


def test_forced_tokens_are_retained_in_every_head_and_come_first():
    rng = np.random.default_rng(13)
    lyr, hq, hkv, n, m, d = 3, 4, 2, 20, 3, 8
    q = [rng.standard_normal((hq, m, d)).astype(np.float32) for _ in range(lyr)]
    k = [rng.standard_normal((hkv, n, d)).astype(np.float32) for _ in range(lyr)]
    v = [rng.standard_normal((hkv, n, d)).astype(np.float32) for _ in range(lyr)]
    forced = [0, 1, 17, 18, 19]
    budget = lyr * len(forced) + 4
    out = orc.compress(q, k, v, budget, keep_first=2, keep_last=3)
    plain = orc.compress(q, k, v, budget)
    assert int(out["lengths"].sum()) == budget and int(out["lengths"].min()) >= len(forced)
    for l in range(lyr):
        for h in range(hkv):
            assert out["idx"][l, h, :len(forced)].tolist() == forced      # +inf ties: ascending position
            # the others keep the order they have without forcing
            rest = [c for c in plain["idx"][l, h].tolist() if c not in forced]
            assert out["idx"][l, h, len(forced):].tolist() == rest
    # with exactly Lyr * forced slots every layer keeps the forced tokens and nothing else
    tight = orc.compress(q, k, v, lyr * len(forced), keep_first=2, keep_last=3)
    assert tight["lengths"].tolist() == [len(forced)] * lyr
