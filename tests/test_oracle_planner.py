"""Pins of the planner oracle (Algorithm 1 of the paper) against what the problem statement fixes:
the two constraints of the optimisation problem of Sec. 4.3 (conservation, validity), the budgets,
monotone bottleneck latency, locality, a fixed point, and two hand-worked examples whose numbers are
written out here step by step (computed by hand from the paper's description, not by the oracle)."""
import numpy as np
import pytest


def _random_nhat(seed, R, E, scale=200, zipf=1.2):
    rng = np.random.default_rng(seed)
    pop = (np.arange(1, E + 1) ** -zipf)[rng.permutation(E)]
    lam = scale * pop / pop.mean()
    return rng.poisson(lam, size=(R, E)).astype(np.int32)


def _latencies(n, n0, g_num, g_den):
    """Sec. 3.2 / 3.3 written with array operations (a second, vectorised statement of the model)."""
    R = n.shape[0]
    ner = n.sum(0)                                           # [E, rt]
    comp = np.where(ner > 0, ner + n0, 0).sum(0)             # per rt
    recv = n.sum(1)                                          # [rs, rt]
    vin = recv.sum(0) - np.diag(recv)
    vout = recv.sum(1) - np.diag(recv)
    return g_den * comp + 2 * g_num * np.maximum(vin, vout)


@pytest.mark.parametrize("seed,R,E,E_loc", [(1, 4, 16, 4), (2, 8, 64, 8), (3, 8, 256, 32), (4, 3, 10, 4), (5, 16, 128, 8)])
@pytest.mark.parametrize("cost", [(0, 0, 1), (64, 1, 4), (16, 3, 2)])
def test_constraints_budgets_and_monotone_bottleneck(oracle, seed, R, E, E_loc, cost):
    n0, g_num, g_den = cost
    nh = _random_nhat(seed, R, E)
    r = oracle.plan_greedy(nh, E_loc, max_replicas=3, budget=2, k_max=16, eps=0, n0=n0, g_num=g_num, g_den=g_den)
    n = r["n"]
    # conservation: sum_r n_{e,r} = n_e, per origin
    np.testing.assert_array_equal(n.sum(2), nh)
    assert (n >= 0).all()
    # validity: n_{e,r} > 0 only where rank r holds e
    host = np.zeros((E, R), bool)
    host[np.arange(E), np.arange(E) // E_loc] = True
    for rr in range(R):
        for e in r["delta_in"][rr]:
            if e >= 0:
                assert not host[e, rr]                       # never a second copy on one rank
                host[e, rr] = True
    assert (n.sum(0)[~host] == 0).all()
    # budgets: replicas per rank, transfers in and out per rank, accepted moves
    assert ((r["delta_in"] >= 0).sum(1) <= 2).all() and ((r["delta_out"] >= 0).sum(1) <= 2).all()
    assert r["n_moves"] <= 16 and (r["moves"][: r["n_moves"]] >= 0).all() and (r["moves"][r["n_moves"]:] == -1).all()
    # the reported latencies are those of the model, and the bottleneck never got worse
    base = np.zeros_like(n)
    for rs in range(R):
        base[rs, np.arange(E), np.arange(E) // E_loc] = nh[rs]
    assert r["L_before"] == _latencies(base, n0, g_num, g_den).max()
    assert r["L_after"] == _latencies(n, n0, g_num, g_den).max()
    assert r["L_after"] <= r["L_before"]
    if r["n_moves"]:
        assert r["L_after"] < r["L_before"]
    # locality first: tokens whose origin holds the expert are processed there
    for rs in range(R):
        for e in np.nonzero(host[:, rs])[0]:
            assert n[rs, e].sum() == n[rs, e, rs]
    # each accepted move strictly lowers the bottleneck: replay the moves' prefix plans
    for k in range(r["n_moves"] + 1):
        rk = oracle.plan_greedy(nh, E_loc, max_replicas=3, budget=2, k_max=k, eps=0, n0=n0, g_num=g_num, g_den=g_den)
        if k:
            assert rk["L_after"] < prev
            np.testing.assert_array_equal(rk["moves"][:k], r["moves"][:k])
        prev = rk["L_after"]


def test_balanced_input_is_a_fixed_point(oracle):
    """Every rank already carries the same load: no move can lower the bottleneck, the plan is the baseline."""
    R, E, E_loc = 4, 16, 4
    nh = np.full((R, E), 25, np.int32)
    r = oracle.plan_greedy(nh, E_loc, n0=32, g_num=1, g_den=2)
    assert r["n_moves"] == 0 and (r["delta_in"] == -1).all() and r["L_after"] == r["L_before"]
    for rs in range(R):
        for e in range(E):
            assert r["n"][rs, e, e // E_loc] == 25


def test_hand_worked_three_ranks_compute_only(oracle):
    """R = 3, one expert per rank, cost = tokens processed (n0 = 0, no network term).
    Origins send 20 / 30 / 40 tokens to expert 0 (home: rank 0); origin 1 sends 10 to expert 1, origin 2
    sends 10 to expert 2.  Loads 90 / 10 / 10, total 110, average ceil(110/3) = 37.
    Move 1: bottleneck 0, helper 1 (tie with 2, lower rank).  Expert 0 is copied to rank 1; origin 1's 30
      tokens come home to rank 1; rank 0 is left with 60, wants to shed 60 - 37 = 23; the only origin without
      a copy is 2 (40 tokens on rank 0): 23 of them go to rank 1.  Loads 37 / 63 / 10, bottleneck 90 -> 63.
    Move 2: bottleneck 1, helper 2.  Rank 1 holds expert 1 (10) and a copy of expert 0 (53): expert 0.  Origin
      2's tokens (17 on rank 0, 23 on rank 1) come home to rank 2; no origin without a copy is left.
      Loads 20 / 40 / 50, bottleneck 63 -> 50.
    Then: bottleneck 2 holds expert 2 (all its tokens are local, nothing to move) and a copy of expert 0
      (already everywhere): both helpers are marked invalid, the loop ends."""
    nh = np.array([[20, 0, 0], [30, 10, 0], [40, 0, 10]], np.int32)
    r = oracle.plan_greedy(nh, 1, max_replicas=2, budget=2, k_max=16)
    assert r["n_moves"] == 2 and r["L_before"] == 90 and r["L_after"] == 50 and r["max_load"] == 50
    np.testing.assert_array_equal(r["moves"][:2], [[0, 0, 1], [0, 1, 2]])
    np.testing.assert_array_equal(r["delta_in"], [[-1, -1], [0, -1], [0, -1]])
    np.testing.assert_array_equal(r["delta_out"], [[0, -1], [0, -1], [-1, -1]])
    want = np.zeros((3, 3, 3), np.int32)
    want[0, 0, 0], want[1, 0, 1], want[2, 0, 2] = 20, 30, 40          # expert 0: everybody local
    want[1, 1, 1], want[2, 2, 2] = 10, 10
    np.testing.assert_array_equal(r["n"], want)
    # stopping after one move gives the intermediate state of the derivation
    r1 = oracle.plan_greedy(nh, 1, max_replicas=2, budget=2, k_max=1)
    assert r1["L_after"] == 63
    assert r1["n"][2, 0].tolist() == [17, 23, 0] and r1["n"][1, 0].tolist() == [0, 30, 0]


def test_hand_worked_with_fragmentation_and_network_cost(oracle):
    """Same traffic, cost with n0 = 8 (per-expert fixed cost) and a network term g = 1/2:
    L_r = 2 * sum_{e: n>0} (n_{e,r} + 8) + 2 * 1 * max(V_in, V_out).
    Baseline: rank 0 processes 90 tokens of one expert, 70 of them remote: L0 = 2*(90+8) + 2*70 = 336.
      rank 1: 2*(10+8) + 2*max(0, 30) = 96;  rank 2: 2*(10+8) + 2*max(0, 40) = 116.  Bottleneck 336.
    Move 1 (bottleneck 0, helper 1 = smallest L): as in the compute-only example, rank 0 keeps 20 + 17, rank 1
      gets 30 (local) + 23 (from origin 2).  L0 = 2*(37+8) + 2*max(17, 0) = 124;
      L1 = 2*((53+8) + (10+8)) + 2*max(23, 0) = 204;  L2 = 2*(10+8) + 2*max(0, 40) = 116.  Bottleneck 204, gain 132.
    Move 2 (bottleneck 1, helper 2): expert 0 again; origin 2's 40 tokens come home.
      L0 = 2*(20+8) = 56;  L1 = 2*((30+8) + (10+8)) = 112;  L2 = 2*((40+8) + (10+8)) = 132.  Bottleneck 132, gain 72.
    Then nothing movable on rank 2: the loop ends."""
    nh = np.array([[20, 0, 0], [30, 10, 0], [40, 0, 10]], np.int32)
    r = oracle.plan_greedy(nh, 1, max_replicas=2, budget=2, k_max=16, n0=8, g_num=1, g_den=2)
    assert (r["L_before"], r["L_after"], r["n_moves"]) == (336, 132, 2)
    r1 = oracle.plan_greedy(nh, 1, max_replicas=2, budget=2, k_max=1, n0=8, g_num=1, g_den=2)
    assert r1["L_after"] == 204
    # a gain threshold above the second move's gain (72) stops after the first
    r2 = oracle.plan_greedy(nh, 1, max_replicas=2, budget=2, k_max=16, eps=72, n0=8, g_num=1, g_den=2)
    assert r2["n_moves"] == 1 and r2["L_after"] == 204


def test_budget_zero_and_replica_cap(oracle):
    nh = _random_nhat(9, 4, 16)
    assert oracle.plan_greedy(nh, 4, max_replicas=3, budget=0)["n_moves"] == 0
    assert oracle.plan_greedy(nh, 4, max_replicas=0, budget=3)["n_moves"] == 0
    r = oracle.plan_greedy(nh, 4, max_replicas=1, budget=3, k_max=16)
    assert ((r["delta_in"] >= 0).sum(1) <= 1).all()


def test_plan_for_rank_layout(oracle):
    """The per-rank view lists one replica per holding rank in ascending rank order with the planned token
    counts as weights; local copies carry their slot (native first, replicas after), others -1."""
    nh = np.array([[20, 0, 0], [30, 10, 0], [40, 0, 10]], np.int32)
    r = oracle.plan_greedy(nh, 1, max_replicas=2, budget=2, k_max=16)
    p = oracle.plan_for_rank(r["n"], r["delta_in"], 1, rank=1)
    np.testing.assert_array_equal(p["rep_off"], [0, 3, 4, 5])
    np.testing.assert_array_equal(p["rep_weight"], [20, 30, 40, 10, 10])
    np.testing.assert_array_equal(p["rep_slot"], [-1, 1, -1, 0, -1])      # expert 0's copy sits in slot 1 of rank 1
    np.testing.assert_array_equal(p["slot_expert"], [1, 0, -1])
    p0 = oracle.plan_for_rank(r["n"], r["delta_in"], 1, rank=0)
    np.testing.assert_array_equal(p0["rep_slot"], [0, -1, -1, -1, -1])
    # an expert nobody is predicted to use keeps a unit weight on its home copy
    nh2 = np.array([[5, 0], [7, 0]], np.int32)
    r2 = oracle.plan_greedy(nh2, 1, max_replicas=1, budget=1)
    p2 = oracle.plan_for_rank(r2["n"], r2["delta_in"], 1, rank=1)
    e1 = slice(p2["rep_off"][1], p2["rep_off"][2])
    assert p2["rep_weight"][e1].tolist() == [1] and p2["rep_slot"][e1].tolist() == [0]
    # the per-replica token split that permute derives from these weights conserves every expert's tokens
    for e in range(3):
        assert p["rep_weight"][p["rep_off"][e]:p["rep_off"][e + 1]].sum() == nh[:, e].sum()


def test_plan_dispatch_hand_worked_and_ties_to_the_receiving_plan(oracle):
    """The plan as a source rank applies it to its own tokens: one slot per (destination rank, expert copy).
    Hand-worked on the state after the first move of the three-rank example: expert 0 is held by ranks 0
    (home) and 1 (copy), experts 1 and 2 by their homes.  Slots by destination rank, then expert:
    rank 0: (e0) = slot 0;  rank 1: (e0) = 1, (e1) = 2;  rank 2: (e2) = 3.  Origin 2's 40 tokens of expert 0
    are planned 17 on rank 0 and 23 on rank 1; its own expert 2 keeps its 10 tokens at home; it predicted
    nothing for expert 1, whose home is rank 1."""
    nh = np.array([[20, 0, 0], [30, 10, 0], [40, 0, 10]], np.int32)
    r1 = oracle.plan_greedy(nh, 1, max_replicas=2, budget=2, k_max=1)
    d2 = oracle.plan_dispatch(r1["n"], r1["delta_in"], 1, rank=2)
    np.testing.assert_array_equal(d2["rep_off"], [0, 2, 3, 4])
    np.testing.assert_array_equal(d2["rep_slot"], [0, 1, 2, 3])
    np.testing.assert_array_equal(d2["rep_weight"], [17, 23, 1, 10])
    np.testing.assert_array_equal(d2["rank_off"], [0, 1, 3, 4])
    np.testing.assert_array_equal(d2["slot_expert"], [0, 0, 1, 2])
    # origin 1 holds the copy: locality first, all 30 of its tokens of expert 0 stay on rank 1
    d1 = oracle.plan_dispatch(r1["n"], r1["delta_in"], 1, rank=1)
    np.testing.assert_array_equal(d1["rep_weight"], [0, 30, 10, 1])
    np.testing.assert_array_equal(d1["rep_slot"], [0, 1, 2, 3])
    # random cases: same replica lists as the receiving plan, slots unique and ordered by rank then expert,
    # the weights of all origins add up to the receiving plan's weights, every origin's weights add up to what
    # it predicted, and an origin that holds a copy of an expert keeps its own tokens of it
    for seed, R, E, E_loc in ((1, 4, 16, 4), (2, 8, 64, 8), (3, 5, 20, 4)):
        nh = _random_nhat(seed, R, E)
        r = oracle.plan_greedy(nh, E_loc, max_replicas=3, budget=2, k_max=16, n0=16, g_num=1, g_den=4)
        assert r["n_moves"] >= 2
        recv = oracle.plan_for_rank(r["n"], r["delta_in"], E_loc, rank=0)
        total = np.zeros_like(recv["rep_weight"])
        for rs in range(R):
            d = oracle.plan_dispatch(r["n"], r["delta_in"], E_loc, rank=rs)
            np.testing.assert_array_equal(d["rep_off"], recv["rep_off"])
            used = int(d["rep_off"][E])
            assert sorted(d["rep_slot"].tolist()) == list(range(used)) and d["rank_off"][R] == used
            slot_rank = np.searchsorted(d["rank_off"], np.arange(used), side="right") - 1
            for r_ in range(R):                                   # inside a rank, slots follow the expert order
                assert (np.diff(d["slot_expert"][slot_rank == r_]) > 0).all()
            for e in range(E):
                sl = slice(d["rep_off"][e], d["rep_off"][e + 1])
                w, ranks = d["rep_weight"][sl], slot_rank[d["rep_slot"][sl]]
                assert (d["slot_expert"][d["rep_slot"][sl]] == e).all()
                assert (np.diff(ranks) > 0).all() and (e // E_loc) in ranks
                if nh[rs, e] > 0:
                    assert w.sum() == nh[rs, e]
                    if rs in ranks:
                        assert w[list(ranks).index(rs)] == nh[rs, e]          # locality first
                    total[sl] += w
                else:
                    assert w.sum() == 1 and w[list(ranks).index(rs if rs in ranks else e // E_loc)] == 1
        planned = nh.sum(0)
        for e in range(E):
            sl = slice(recv["rep_off"][e], recv["rep_off"][e + 1])
            if planned[e] > 0:
                np.testing.assert_array_equal(total[sl], recv["rep_weight"][sl])
