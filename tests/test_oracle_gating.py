"""Pins of the group-limited gate of the oracle (oracle/gating_oracle.c).  CPU only."""
import os

import numpy as np
import pytest

import oracle
from paper_2602_00509_amd import workload as wl

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "gating_example.txt")


def read_example():
    rows = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *vals = line.split()
        rows[key] = np.array([float(v) for v in vals])
    return rows


def one_token_gate(scores):
    """H = 1, x = 1: the gate weight of expert e IS its logit; logit = log(p / (1 - p))."""
    x = wl.f32_to_bf16_bits(np.ones((1, 1), np.float32))
    w = np.log(scores / (1.0 - scores)).astype(np.float32).reshape(-1, 1)
    return x, w


def rand_case(seed, T, H, E):
    rng = np.random.default_rng(seed)
    x = wl.f32_to_bf16_bits(rng.standard_normal((T, H)).astype(np.float32))
    w = (rng.standard_normal((E, H)) * 0.3).astype(np.float32)
    sb = (rng.standard_normal(E) * 0.1).astype(np.float32)
    return x, w, sb


def test_hand_worked_example():
    ex = read_example()
    x, w = one_token_gate(ex["scores"])
    kw = dict(select_bias=ex["select_bias"].astype(np.float32), scoring="sigmoid", n_group=4, topk_group=2,
              group_top=2, k=3, renormalize=True, routed_scale=2.5)
    o = oracle.route_grouped(x, w, **kw)
    np.testing.assert_allclose(o["scores"][0], ex["scores"], atol=1e-6)
    np.testing.assert_allclose(o["group_scores"][0], ex["group_scores"], atol=1e-6)
    assert o["groups"][0].tolist() == ex["groups"].astype(int).tolist()
    assert o["idx"][0].tolist() == ex["idx"].astype(int).tolist()
    np.testing.assert_allclose(o["w"][0], ex["w"], atol=1e-6)
    assert o["counts"].sum() == 3 and o["counts"][[12, 4, 5]].tolist() == [1, 1, 1]
    # the mistakes the fixture lists really would show on this example
    top1 = oracle.route_grouped(x, w, **dict(kw, group_top=1))
    assert top1["groups"][0].tolist() == [0, 3]
    nobias = oracle.route_grouped(x, w, **dict(kw, select_bias=None))
    assert nobias["groups"][0].tolist() == [1, 2]
    unlimited = oracle.route_grouped(x, w, **dict(kw, topk_group=4))
    assert unlimited["idx"][0].tolist() == [0, 12, 8]
    assert abs(o["w"][0, 0] - 0.75 / 1.90 * 2.5) > 0.1


def brute_force(x_bits, w, sb, scoring, n_group, topk_group, group_top, k, renorm, scale):
    """The same gate with sorts instead of repeated arg-max scans."""
    xf = oracle.bf16_bits_to_f64(x_bits)
    l = xf @ w.astype(np.float64).T
    if scoring == "sigmoid":
        s = 1.0 / (1.0 + np.exp(-l))
    else:
        z = np.exp(l - l.max(1, keepdims=True))
        s = z / z.sum(1, keepdims=True)
    c = s + (0.0 if sb is None else sb.astype(np.float64))
    T, E = c.shape
    gs = E // n_group
    grp = np.sort(c.reshape(T, n_group, gs), axis=2)[:, :, gs - group_top:].sum(2)
    idx = np.empty((T, k), np.int64)
    wout = np.empty((T, k))
    for t in range(T):
        order = sorted(range(n_group), key=lambda j: (-grp[t, j], j))[:topk_group]
        cand = [e for e in range(E) if e // gs in order]
        cand.sort(key=lambda e: (-c[t, e], e))
        idx[t] = cand[:k]
        wv = s[t, idx[t]]
        wout[t] = (wv / wv.sum() if renorm else wv) * scale
    return idx, wout, grp


@pytest.mark.parametrize("scoring", ["sigmoid", "softmax"])
@pytest.mark.parametrize("E,n_group,topk_group,group_top,k", [(16, 4, 2, 2, 3), (32, 8, 4, 2, 8), (24, 3, 1, 3, 4),
                                                              (64, 8, 3, 1, 6), (8, 1, 1, 2, 2), (12, 12, 5, 1, 5)])
def test_against_sort_based_brute_force(scoring, E, n_group, topk_group, group_top, k):
    x, w, sb = rand_case(E * 7 + k, 40, 24, E)
    for renorm, scale, bias in ((True, 2.5, sb), (False, 1.0, None)):
        o = oracle.route_grouped(x, w, select_bias=bias, scoring=scoring, n_group=n_group, topk_group=topk_group,
                                 group_top=group_top, k=k, renormalize=renorm, routed_scale=scale)
        idx, wout, grp = brute_force(x, w, bias, scoring, n_group, topk_group, group_top, k, renorm, scale)
        np.testing.assert_array_equal(o["idx"], idx)
        np.testing.assert_allclose(o["w"], wout, rtol=1e-12)
        np.testing.assert_allclose(o["group_scores"], grp, rtol=1e-12, atol=1e-15)   # order of the additions differs
        assert np.bincount(idx.ravel(), minlength=E).tolist() == o["counts"].tolist()


def test_one_group_softmax_is_the_plain_router():
    x, w, _ = rand_case(5, 64, 32, 16)
    bias = (np.random.default_rng(1).standard_normal((2, 16))).astype(np.float32)
    for renorm in (True, False):
        a = oracle.route_topk(x, w, bias, tokens_per_group=32, k=4, renormalize=renorm)
        b = oracle.route_grouped(x, w, bias, tokens_per_group=32, scoring="softmax", n_group=1, topk_group=1,
                                 group_top=1, k=4, renormalize=renorm)
        np.testing.assert_array_equal(a["idx"], b["idx"])
        np.testing.assert_allclose(a["w"], b["w"], rtol=1e-14)
        np.testing.assert_allclose(a["probs"], b["scores"], rtol=1e-14)
        np.testing.assert_array_equal(a["counts"], b["counts"])


def test_sigmoid_without_bias_orders_like_the_logits():
    x, w, _ = rand_case(6, 64, 32, 16)
    a = oracle.route_topk(x, w, k=4)
    b = oracle.route_grouped(x, w, scoring="sigmoid", n_group=1, topk_group=1, group_top=1, k=4, renormalize=False)
    np.testing.assert_array_equal(a["idx"], b["idx"])
    np.testing.assert_allclose(b["w"], 1.0 / (1.0 + np.exp(-np.take_along_axis(a["logits"], a["idx"].astype(np.int64), 1))),
                               rtol=1e-12)


def test_softmax_over_the_chosen_equals_renormalised_softmax():
    """A gate that takes the k largest logits and then a softmax over those k (the GPT-OSS form) is
    the renormalised softmax-top-k gate: p_e / sum_chosen p = exp(l_e) / sum_chosen exp(l)."""
    x, w, _ = rand_case(7, 50, 16, 32)
    o = oracle.route_topk(x, w, k=4, renormalize=True)
    lsel = np.take_along_axis(o["logits"], o["idx"].astype(np.int64), 1)
    z = np.exp(lsel - lsel.max(1, keepdims=True))
    np.testing.assert_allclose(o["w"], z / z.sum(1, keepdims=True), rtol=1e-12)


def test_invariants():
    E, n_group, topk_group, k = 64, 8, 4, 8
    x, w, sb = rand_case(9, 200, 48, E)
    o = oracle.route_grouped(x, w, select_bias=sb, scoring="sigmoid", n_group=n_group, topk_group=topk_group,
                             group_top=2, k=k, renormalize=True, routed_scale=2.5)
    gs = E // n_group
    for t in range(200):
        assert set((o["idx"][t] // gs).tolist()) <= set(o["groups"][t].tolist())
        assert len(set(o["idx"][t].tolist())) == k
        assert len(set(o["groups"][t].tolist())) == topk_group
        assert (np.diff(o["choice"][t, o["idx"][t]]) <= 0).all()
    np.testing.assert_allclose(o["w"].sum(1), 2.5, rtol=1e-12)
    assert o["counts"].sum() == 200 * k
    np.testing.assert_allclose(o["choice"] - o["scores"], np.broadcast_to(sb.astype(np.float64), (200, E)), atol=1e-15)
    # a large selection bias forces an expert into every token's choice without changing its gating value
    sb2 = sb.copy()
    sb2[37] += 10.0
    o2 = oracle.route_grouped(x, w, select_bias=sb2, scoring="sigmoid", n_group=n_group, topk_group=topk_group,
                              group_top=2, k=k, renormalize=False, routed_scale=1.0)
    assert (o2["idx"][:, 0] == 37).all()
    np.testing.assert_allclose(o2["w"][:, 0], o2["scores"][:, 37], rtol=0, atol=0)
    assert o2["counts"][37] == 200


def test_ties_go_to_the_lower_index():
    x = wl.f32_to_bf16_bits(np.ones((1, 1), np.float32))
    w = np.zeros((12, 1), np.float32)          # all scores equal: 0.5
    o = oracle.route_grouped(x, w, scoring="sigmoid", n_group=4, topk_group=2, group_top=2, k=5, renormalize=True)
    assert o["groups"][0].tolist() == [0, 1]
    assert o["idx"][0].tolist() == [0, 1, 2, 3, 4]
    np.testing.assert_allclose(o["w"][0], 0.2)


def test_bad_arguments():
    x, w, _ = rand_case(1, 4, 8, 16)
    for kw in (dict(n_group=3), dict(n_group=4, topk_group=5), dict(n_group=4, topk_group=1, k=5),
               dict(n_group=4, topk_group=2, group_top=5)):
        with pytest.raises(ValueError):
            oracle.route_grouped(x, w, **dict(dict(scoring="sigmoid", n_group=1, topk_group=1, group_top=1, k=2), **kw))
