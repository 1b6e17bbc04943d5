"""Pins of the oracle's grouped SwiGLU FFN, combine and whole layer: hand-computed values,
torch fp64 library cross-check, exact scaling laws, identity experts, plan invariance."""
import numpy as np
import torch

from paper_2602_00509_amd import workload as wl


def _bits(a):
    return wl.f32_to_bf16_bits(np.asarray(a, np.float32))


def test_ffn_hand_computed(oracle):
    """H=2, F=1: x=(1,2), W1=(1,0) -> a=1; W3=(0,1) -> c=2; h = silu(1)*2 = 2/(1+e^-1);
    W2 = (1,-2)^T -> y = (h, -2h).  Swapping W1 and W3 would give silu(2)*1 instead."""
    xp = _bits([[1.0, 2.0]])
    w13 = _bits([[1.0, 0.0], [0.0, 1.0]])
    w2 = _bits([[1.0], [-2.0]])
    y = oracle.grouped_ffn(xp, np.array([0, 1], np.int32), [w13], [w2])
    h = 2.0 / (1.0 + np.exp(-1.0))
    np.testing.assert_allclose(y, [[h, -2.0 * h]], rtol=1e-15)


def test_ffn_matches_torch_fp64(oracle):
    rng = np.random.default_rng(4)
    H, F, S = 24, 40, 3
    offs = np.array([0, 5, 5, 12], np.int32)              # middle slot empty
    xp = _bits(rng.standard_normal((14, H)))
    w13 = [_bits(rng.standard_normal((2 * F, H)) * 0.2) for _ in range(S)]
    w2 = [_bits(rng.standard_normal((H, F)) * 0.2) for _ in range(S)]
    y = oracle.grouped_ffn(xp, offs, w13, w2)
    assert y.shape == (12, H)
    xt = torch.from_numpy(wl.bf16_bits_to_f32(xp)).double()
    for s in range(S):
        a13 = torch.from_numpy(wl.bf16_bits_to_f32(w13[s])).double()
        a2 = torch.from_numpy(wl.bf16_bits_to_f32(w2[s])).double()
        rows = slice(int(offs[s]), int(offs[s + 1]))
        g = xt[rows] @ a13[:F].T
        u = xt[rows] @ a13[F:].T
        ref = (torch.nn.functional.silu(g) * u) @ a2.T
        np.testing.assert_allclose(y[rows], ref.numpy(), rtol=1e-11, atol=1e-13)
    # sampled rows give the same values as the full pass; rows outside any slot stay zero
    ys = oracle.grouped_ffn(xp, offs, w13, w2, rows=np.array([11, 0, 13, 6], np.int32))
    np.testing.assert_array_equal(ys[[0, 1, 3]], y[[11, 0, 6]])
    assert not ys[2].any()


def test_ffn_exact_properties(oracle):
    rng = np.random.default_rng(5)
    H, F = 16, 24
    xp = _bits(rng.standard_normal((6, H)))
    wa = (_bits(rng.standard_normal((2 * F, H)) * 0.3), _bits(rng.standard_normal((H, F)) * 0.3))
    wb = (_bits(rng.standard_normal((2 * F, H)) * 0.3), _bits(rng.standard_normal((H, F)) * 0.3))
    offs = np.array([0, 4, 6], np.int32)
    y = oracle.grouped_ffn(xp, offs, [wa[0], wb[0]], [wa[1], wb[1]])
    # silu(0) = 0: a zero row gives a zero output
    z = oracle.grouped_ffn(np.zeros((2, H), np.uint16), np.array([0, 2], np.int32), [wa[0]], [wa[1]])
    assert not z.any()
    # doubling W2 (exact in bf16) doubles y exactly
    w2x2 = _bits(wl.bf16_bits_to_f32(wa[1]) * 2)
    y2 = oracle.grouped_ffn(xp, offs, [wa[0], wb[0]], [w2x2, wb[1]])
    np.testing.assert_array_equal(y2[:4], 2 * y[:4])
    np.testing.assert_array_equal(y2[4:], y[4:])
    # a slot's output does not depend on which slot index holds the weights
    xq = np.concatenate([xp[4:], xp[:4]])
    yq = oracle.grouped_ffn(xq, np.array([0, 2, 6], np.int32), [wb[0], wa[0]], [wb[1], wa[1]])
    np.testing.assert_array_equal(yq[:2], y[4:])
    np.testing.assert_array_equal(yq[2:], y[:4])
    # an empty slot list / M = 0 does nothing
    assert oracle.grouped_ffn(xp, np.array([0, 0], np.int32), [wa[0]], [wa[1]]).shape == (0, H)


def test_combine_identity_experts_and_remote(oracle):
    """If every expert is the identity (y[row] = x[token]) the renormalised combine returns x."""
    rng = np.random.default_rng(6)
    T, H, E, k = 50, 16, 6, 3
    x = _bits(rng.standard_normal((T, H)))
    w = (rng.standard_normal((E, H)) * 0.5).astype(np.float32)
    r = oracle.route_topk(x, w, None, k=k, renormalize=True)
    plan = dict(rep_off=np.arange(E + 1, dtype=np.int32), rep_slot=np.arange(E, dtype=np.int32),
                rep_weight=np.ones(E, np.int32))
    p = oracle.permute(r["idx"], plan["rep_off"], plan["rep_slot"], plan["rep_weight"], E, x)
    y = wl.bf16_bits_to_f32(p["xp"]).astype(np.float64)
    out = oracle.combine(y, p["pair_row"], r["w"])
    np.testing.assert_allclose(out, wl.bf16_bits_to_f32(x).astype(np.float64), rtol=1e-14, atol=1e-15)
    # all pairs remote -> zeros
    out0 = oracle.combine(y, np.full((T, k), -1, np.int32), r["w"])
    assert not out0.any()
    # hand case: out = 0.25*y[2] + 0.5*y[0], the pair with row -1 is skipped
    yy = np.array([[1.0, 2.0], [10.0, 20.0], [100.0, 200.0]])
    o = oracle.combine(yy, np.array([[2, -1, 0]], np.int32), np.array([[0.25, 0.125, 0.5]]))
    np.testing.assert_array_equal(o, [[25.5, 51.0]])


def test_combine_with_a_shared_expert(oracle):
    """Identity routed experts and an identity shared expert: out = (sum of weights + scale) * x; a hand case;
    a zero shared output gives the plain combine."""
    rng = np.random.default_rng(8)
    T, H, E, k = 40, 8, 5, 2
    x = _bits(rng.standard_normal((T, H)))
    xf = wl.bf16_bits_to_f32(x).astype(np.float64)
    w = (rng.standard_normal((E, H)) * 0.5).astype(np.float32)
    r = oracle.route_topk(x, w, None, k=k, renormalize=False)
    ident = dict(rep_off=np.arange(E + 1, dtype=np.int32), rep_slot=np.arange(E, dtype=np.int32),
                 rep_weight=np.ones(E, np.int32))
    p = oracle.permute(r["idx"], ident["rep_off"], ident["rep_slot"], ident["rep_weight"], E, x)
    y = wl.bf16_bits_to_f32(p["xp"]).astype(np.float64)
    out = oracle.combine_shared(y, p["pair_row"], r["w"], xf, 0.75)
    np.testing.assert_allclose(out, (r["w"].sum(1, keepdims=True) + 0.75) * xf, rtol=1e-13, atol=1e-15)
    np.testing.assert_array_equal(oracle.combine_shared(y, p["pair_row"], r["w"], np.zeros_like(xf), 3.0),
                                  oracle.combine(y, p["pair_row"], r["w"]))
    yy = np.array([[1.0, 2.0], [10.0, 20.0], [100.0, 200.0]])
    o = oracle.combine_shared(yy, np.array([[2, -1, 0]], np.int32), np.array([[0.25, 0.125, 0.5]]),
                              np.array([[4.0, -8.0]]), 0.5)
    np.testing.assert_array_equal(o, [[27.5, 47.0]])      # 25.5 + 0.5*4, 51 + 0.5*(-8)


def test_layer_plan_invariance(oracle):
    """Sec. 4.1 / 4.2: the main track is semantically equivalent to standard execution, so with
    every replica local the layer output under any plan equals the output with no replication."""
    cfg = wl.small_config(T=80, H=32, E=6, k=2, F=48, E_loc=6, n_rep=2, ep=1, chunk=0)
    x = wl.activations(cfg)
    wg, b = wl.gate_weights(cfg), wl.zipf_bias(cfg)
    ew = {e: wl.expert_weights(cfg, e) for e in range(cfg.E)}
    base = wl.no_replica_plan(cfg)
    ref = oracle.moe_layer(x, wg, b, None, cfg.k, True, base, [ew[e][0] for e in range(cfg.E)],
                           [ew[e][1] for e in range(cfg.E)])
    plan = wl.build_plan(cfg, ref["route"]["counts"])
    se = plan["slot_expert"]
    rep = oracle.moe_layer(x, wg, b, None, cfg.k, True, plan, [ew[int(e)][0] for e in se],
                           [ew[int(e)][1] for e in se])
    assert rep["permute"]["n_local"] == cfg.N == ref["permute"]["n_local"]
    assert (rep["permute"]["slot_counts"][cfg.E_loc:] > 0).all()      # replicas really used
    np.testing.assert_array_equal(rep["out"], ref["out"])
    # and the layer equals a dense per-token evaluation with torch fp64
    xt = torch.from_numpy(wl.bf16_bits_to_f32(x)).double()
    dense = torch.zeros_like(xt)
    for t in range(cfg.T):
        for s in range(cfg.k):
            e = int(ref["route"]["idx"][t, s])
            a13 = torch.from_numpy(wl.bf16_bits_to_f32(ew[e][0])).double()
            a2 = torch.from_numpy(wl.bf16_bits_to_f32(ew[e][1])).double()
            g, u = a13[:cfg.F] @ xt[t], a13[cfg.F:] @ xt[t]
            dense[t] += ref["route"]["w"][t, s] * (a2 @ (torch.nn.functional.silu(g) * u))
    np.testing.assert_allclose(ref["out"], dense.numpy(), rtol=1e-10, atol=1e-14)
