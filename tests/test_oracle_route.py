"""Pins of the oracle's router / predictor against what the mathematics fixes.

Nothing here re-types the oracle's own loop: the checks are a brute-force stable sort,
closed forms (Zipf prior, uniform prior, a hand-computed 4-expert example), library routines
(numpy matmul, torch.softmax in fp64) and invariants (Table 1: sum_e n_e = B*k).
"""
import numpy as np
import pytest
import torch

from paper_2602_00509_amd import workload as wl


def _rand_case(seed, T, H, E):
    rng = np.random.default_rng(seed)
    x = wl.f32_to_bf16_bits(rng.standard_normal((T, H), dtype=np.float32))
    w = (rng.standard_normal((E, H), dtype=np.float32) * np.float32(0.3))
    b = rng.standard_normal((E,), dtype=np.float32)
    return x, w, b


@pytest.mark.parametrize("E", [2, 5, 16])
def test_topk_equals_full_stable_sort(oracle, E):
    """Brute force: a full stable sort of every row by descending logit, for every k."""
    T, H = 48, 24
    x, w, b = _rand_case(10 + E, T, H, E)
    logits = wl.bf16_bits_to_f32(x).astype(np.float64) @ w.astype(np.float64).T + b.astype(np.float64)
    order = np.argsort(-logits, axis=1, kind="stable")
    for k in range(1, E + 1):
        r = oracle.route_topk(x, w, b, k=k, renormalize=False)
        np.testing.assert_allclose(r["logits"], logits, rtol=0, atol=1e-12)
        np.testing.assert_array_equal(r["idx"], order[:, :k])
        # property: every unselected logit <= every selected one
        sel_min = np.take_along_axis(r["logits"], r["idx"], 1).min(1)
        mask = np.ones_like(logits, bool)
        np.put_along_axis(mask, r["idx"], False, 1)
        if k < E:
            assert (np.where(mask, logits, -np.inf).max(1) <= sel_min).all()


def test_exact_ties_go_to_lower_index(oracle):
    """W = 0, b = 0: uniform probabilities 1/E and idx = (0..k-1)."""
    T, H, E, k = 5, 8, 7, 3
    x = wl.f32_to_bf16_bits(np.random.default_rng(0).standard_normal((T, H), dtype=np.float32))
    r = oracle.route_topk(x, np.zeros((E, H), np.float32), np.zeros(E, np.float32), k=k, renormalize=False)
    np.testing.assert_allclose(r["probs"], 1.0 / E, rtol=0, atol=1e-15)
    np.testing.assert_array_equal(r["idx"], np.tile(np.arange(k), (T, 1)))
    np.testing.assert_allclose(r["w"], 1.0 / E, atol=1e-15)
    # duplicated logits in the middle: experts 1 and 4 tie for first place
    b = np.array([0.0, 2.0, 1.0, -1.0, 2.0, 0.5, 0.0], np.float32)
    r = oracle.route_topk(x, np.zeros((E, H), np.float32), b, k=4, renormalize=True)
    np.testing.assert_array_equal(r["idx"], np.tile(np.array([1, 4, 2, 5]), (T, 1)))


def test_bias_only_softmax_is_zipf(oracle):
    """W = 0, b_e = -s ln(rank_e)  =>  p_e = rank_e^-s / sum_j j^-s (closed form)."""
    E, s = 16, 1.2
    order = np.random.default_rng(3).permutation(E)
    rank = np.empty(E, np.int64)
    rank[order] = np.arange(1, E + 1)
    b = (-s * np.log(rank.astype(np.float64))).astype(np.float32)
    x = wl.f32_to_bf16_bits(np.ones((3, 8), np.float32))
    r = oracle.route_topk(x, np.zeros((E, 8), np.float32), b, k=4, renormalize=False)
    expect = rank.astype(np.float64) ** (-s)
    expect /= expect.sum()
    np.testing.assert_allclose(r["probs"][0], expect, rtol=2e-7)   # bias is fp32
    np.testing.assert_array_equal(r["idx"][0], order[:4])           # hottest first


def test_hand_computed_four_experts(oracle):
    """x = (1, 2); W rows give logits ln1, ln2, ln4, ln1 -> p = (1,2,4,1)/8.

    W is [E,H] = [4,2] with E != H, so a transposed operand cannot pass."""
    x = wl.f32_to_bf16_bits(np.array([[1.0, 2.0]], np.float32))
    W = np.array([[0.0, 0.0], [np.log(2.0), 0.0], [0.0, np.log(2.0)], [2.0, -1.0]], np.float32)
    r = oracle.route_topk(x, W, None, k=2, renormalize=True)
    np.testing.assert_allclose(r["logits"][0], [0.0, np.log(2.0), np.log(4.0), 0.0], atol=1e-7)
    np.testing.assert_allclose(r["probs"][0], [0.125, 0.25, 0.5, 0.125], atol=1e-7)
    np.testing.assert_array_equal(r["idx"][0], [2, 1])
    np.testing.assert_allclose(r["w"][0], [2.0 / 3.0, 1.0 / 3.0], atol=1e-7)
    r = oracle.route_topk(x, W, None, k=3, renormalize=False)
    np.testing.assert_array_equal(r["idx"][0], [2, 1, 0])           # tie 0 vs 3 -> lower index
    np.testing.assert_allclose(r["w"][0], [0.5, 0.25, 0.125], atol=1e-7)
    np.testing.assert_array_equal(r["counts"], [1, 1, 1, 0])


def test_softmax_matches_torch_fp64(oracle):
    T, H, E, k = 33, 40, 12, 3
    x, w, b = _rand_case(77, T, H, E)
    r = oracle.route_topk(x, w, b, k=k, renormalize=True)
    xt = torch.from_numpy(wl.bf16_bits_to_f32(x)).double()
    logits = xt @ torch.from_numpy(w).double().T + torch.from_numpy(b).double()
    p = torch.softmax(logits, dim=1)
    np.testing.assert_allclose(r["probs"], p.numpy(), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(r["probs"].sum(1), 1.0, atol=1e-14)
    tv, ti = torch.topk(p, k, dim=1)
    np.testing.assert_array_equal(r["idx"], ti.numpy())             # no ties in random data
    np.testing.assert_allclose(r["w"], (tv / tv.sum(1, keepdim=True)).numpy(), rtol=1e-12)
    np.testing.assert_allclose(r["w"].sum(1), 1.0, atol=1e-14)
    r2 = oracle.route_topk(x, w, b, k=k, renormalize=False)
    np.testing.assert_allclose(r2["w"], np.take_along_axis(r2["probs"], r2["idx"], 1), rtol=0, atol=0)


def test_counts_conservation(oracle):
    """Table 1: sum_e n_e = B*k, and n_e is the histogram of the chosen experts."""
    T, H, E, k = 200, 16, 10, 4
    x, w, b = _rand_case(5, T, H, E)
    r = oracle.route_topk(x, w, b, k=k)
    assert int(r["counts"].sum()) == T * k
    np.testing.assert_array_equal(r["counts"], np.bincount(r["idx"].ravel(), minlength=E))
    # every token picks k distinct experts
    assert all(len(set(row.tolist())) == k for row in r["idx"])


def test_bias_groups_equal_per_chunk_calls(oracle):
    """Token t uses bias row min(t // tokens_per_group, G-1): same as routing chunk by chunk."""
    T, H, E, k, tpg = 70, 16, 9, 2, 16
    x, w, _ = _rand_case(6, T, H, E)
    G = 3                                       # fewer rows than chunks: last row is reused
    bias = np.random.default_rng(8).standard_normal((G, E)).astype(np.float32) * 3
    r = oracle.route_topk(x, w, bias, tokens_per_group=tpg, k=k)
    for c0 in range(0, T, tpg):
        g = min(c0 // tpg, G - 1)
        rc = oracle.route_topk(x[c0:c0 + tpg], w, bias[g], k=k)
        np.testing.assert_array_equal(r["idx"][c0:c0 + tpg], rc["idx"])
        np.testing.assert_allclose(r["probs"][c0:c0 + tpg], rc["probs"], rtol=0, atol=0)


def test_predictor_is_cloned_router_at_zero_residual(oracle):
    """Sec. 4.2: the residual is zero-initialised, so the predictor equals the cloned router."""
    T, H, E, k = 64, 32, 16, 4
    x, w, b = _rand_case(9, T, H, E)
    r = oracle.route_topk(x, w, b, k=k)
    p = oracle.predict_topk(x, w, b, k=k)
    np.testing.assert_array_equal(r["idx"], p["idx"])
    np.testing.assert_array_equal(r["counts"], p["counts"])
    np.testing.assert_allclose(r["probs"], p["probs"], rtol=0, atol=0)
    assert oracle.topk_overlap(p["idx"], r["idx"]) == 1.0
    # overlap metric on a hand case: {0,1} vs {1,2} and {3,4} vs {3,4} -> (1+2)/4
    assert oracle.topk_overlap(np.array([[0, 1], [3, 4]]), np.array([[1, 2], [4, 3]])) == 0.75


def test_imbalance_ratio_eq1(oracle):
    assert oracle.imbalance_ratio(np.array([5.0, 5.0, 5.0, 5.0])) == 1.0
    assert oracle.imbalance_ratio(np.array([8.0, 0.0, 0.0, 0.0])) == 4.0
    assert abs(oracle.imbalance_ratio(np.array([3.0, 1.0])) - 1.5) < 1e-15


# ---------------------------------------------------------------- Eq. 7 with its residual

def test_residual_with_zero_output_layer_is_the_router(oracle):
    """Eq. 7 at the initialisation the paper prescribes (W2_hat = 0): logits, order and weights of the router."""
    T, H, E, D = 40, 32, 12, 24
    x, w, b = _rand_case(70, T, H, E)
    rng = np.random.default_rng(71)
    w1 = wl.f32_to_bf16_bits(rng.standard_normal((D, H), dtype=np.float32))
    w2 = np.zeros((E, D), np.float32)
    r = oracle.route_topk(x, w, b, k=3)
    p = oracle.predict_topk_residual(x, w, b, None, w1, w2, k=3)
    np.testing.assert_array_equal(p["logits"], r["logits"])
    np.testing.assert_array_equal(p["idx"], r["idx"])
    np.testing.assert_array_equal(p["w"], r["w"])


def test_residual_one_hot_closed_form(oracle):
    """W1_hat picks one coordinate of h, W2_hat sends it to one expert: exactly one logit moves, by
    c * silu(h_j).  silu(1) = 0.7310585786300049 and silu(-2) = -0.2384058440442351 are typed in.
    H, D and E all differ and the ones sit off the diagonal, so a transposed operand moves another
    logit or another token."""
    T, H, E, D = 2, 5, 7, 3
    xf = np.zeros((T, H), np.float32)
    xf[0, 2], xf[1, 2] = 1.0, -2.0
    xf[0, 4], xf[1, 0] = 0.5, 3.0            # coordinates the residual must ignore
    x = wl.f32_to_bf16_bits(xf)
    w = np.zeros((E, H), np.float32)
    w1f = np.zeros((D, H), np.float32)
    w1f[1, 2] = 1.0
    w2 = np.zeros((E, D), np.float32)
    w2[3, 1] = 2.0
    p = oracle.predict_topk_residual(x, w, None, None, wl.f32_to_bf16_bits(w1f), w2, k=1)
    want = np.zeros((T, E))
    want[0, 3] = 2.0 * 0.7310585786300049
    want[1, 3] = 2.0 * -0.2384058440442351
    np.testing.assert_allclose(p["logits"], want, rtol=0, atol=1e-15)
    assert p["idx"][0, 0] == 3                       # raised logit wins
    assert p["idx"][1, 0] == 0                       # lowered logit loses to the tie at 0, lowest index


def test_residual_is_additive_in_the_output_layer(oracle):
    """The logits are affine in W2_hat: the shift from W2a + W2b is the sum of the two shifts."""
    T, H, E, D = 30, 48, 9, 16
    x, w, b = _rand_case(72, T, H, E)
    rng = np.random.default_rng(73)
    w1 = wl.f32_to_bf16_bits(rng.standard_normal((D, H), dtype=np.float32) * np.float32(0.2))
    # entries with few significant bits, so that W2a + W2b is exact in fp32
    w2a = (rng.integers(-8, 9, (E, D)) / 16.0).astype(np.float32)
    w2b = (rng.integers(-8, 9, (E, D)) / 16.0).astype(np.float32)
    base = oracle.route_topk(x, w, b, k=2)["logits"]
    la = oracle.predict_topk_residual(x, w, b, None, w1, w2a, k=2)["logits"] - base
    lb = oracle.predict_topk_residual(x, w, b, None, w1, w2b, k=2)["logits"] - base
    lab = oracle.predict_topk_residual(x, w, b, None, w1, w2a + w2b, k=2)["logits"] - base
    np.testing.assert_allclose(lab, la + lb, rtol=0, atol=1e-11)
    assert np.abs(la).max() > 0.1                    # the residual is not trivially zero here


def test_residual_matches_torch_fp64(oracle):
    """Library cross-check: torch matmul + torch.nn.functional.silu in fp64."""
    T, H, E, D = 25, 40, 11, 20
    x, w, b = _rand_case(74, T, H, E)
    rng = np.random.default_rng(75)
    w1 = wl.f32_to_bf16_bits(rng.standard_normal((D, H), dtype=np.float32) * np.float32(0.3))
    w2 = rng.standard_normal((E, D)).astype(np.float32)
    p = oracle.predict_topk_residual(x, w, b, None, w1, w2, k=4)
    h = torch.from_numpy(wl.bf16_bits_to_f32(x).astype(np.float64))
    l = h @ torch.from_numpy(w.astype(np.float64)).T + torch.from_numpy(b.astype(np.float64))
    l = l + torch.nn.functional.silu(h @ torch.from_numpy(wl.bf16_bits_to_f32(w1).astype(np.float64)).T) \
        @ torch.from_numpy(w2.astype(np.float64)).T
    np.testing.assert_allclose(p["logits"], l.numpy(), rtol=0, atol=1e-11)
    np.testing.assert_allclose(p["probs"], torch.softmax(l, 1).numpy(), rtol=0, atol=1e-13)
    assert p["counts"].sum() == T * 4


def test_cross_entropy_closed_forms(oracle):
    """CE(p, p) is the entropy; a one-hot target picks -log q_e; uniform against uniform is log E."""
    E = 8
    u = np.full((3, E), 1.0 / E)
    assert abs(oracle.cross_entropy_sum(u, u) - 3 * np.log(E)) < 1e-12
    onehot = np.zeros((1, E)); onehot[0, 5] = 1.0
    q = np.full((1, E), 0.05); q[0, 5] = 0.65
    assert abs(oracle.cross_entropy_sum(onehot, q) + np.log(0.65)) < 1e-15
    p = np.array([[0.5, 0.25, 0.25, 0, 0, 0, 0, 0]])
    assert abs(oracle.cross_entropy_sum(p, np.where(p > 0, p, 1.0)) - 1.5 * np.log(2.0)) < 1e-15      # entropy: 1.5 bits
    # Gibbs: CE(p, q) >= CE(p, p)
    rng = np.random.default_rng(0)
    a, b = rng.random((4, E)), rng.random((4, E))
    a /= a.sum(1, keepdims=True); b /= b.sum(1, keepdims=True)
    assert oracle.cross_entropy_sum(a, b) >= oracle.cross_entropy_sum(a, a)
