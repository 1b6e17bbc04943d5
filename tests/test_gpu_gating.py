"""GPU parity of probe_route_grouped (group-limited gate) against oracle/gating_oracle.c."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_00509_amd import probe
from paper_2602_00509_amd import workload as wl
from gpu_util import dev_bf16, PROB_ATOL

pytestmark = pytest.mark.gpu

TAU_C = 2e-6   # selection-score gap below which a decision is declared ambiguous (scores are <= 1 + |bias|)


def make_case(seed, T, H, E, scale=0.05):
    rng = np.random.default_rng(seed)
    x = wl.f32_to_bf16_bits(rng.standard_normal((T, H)).astype(np.float32))
    w = (rng.standard_normal((E, H)) * scale).astype(np.float32)
    sb = (rng.standard_normal(E) * 0.05).astype(np.float32)
    bias = (rng.standard_normal((2, E)) * 0.5).astype(np.float32)
    return x, w, sb, bias


def clear_tokens(o, k, topk_group, n_group):
    """Tokens where no decision of the oracle is within TAU_C of flipping."""
    T = o["choice"].shape[0]
    gsc = -np.sort(-o["group_scores"], axis=1)
    ok = np.ones(T, bool)
    if topk_group < n_group:
        ok &= (gsc[:, topk_group - 1] - gsc[:, topk_group]) > 2 * TAU_C
    # (the order among the allowed groups is not an output)
    E = o["choice"].shape[1]
    gs = E // n_group
    allowed = np.zeros((T, E), bool)
    for r in range(topk_group):
        g = o["groups"][:, r]
        for t in range(T):
            allowed[t, g[t] * gs:(g[t] + 1) * gs] = True
    c = np.where(allowed, o["choice"], -np.inf)
    top = -np.sort(-c, axis=1)[:, :min(k + 1, E)]
    gaps = np.abs(np.diff(top, axis=1))
    gaps = np.where(np.isfinite(gaps), gaps, np.inf)
    ok &= (gaps > TAU_C).all(axis=1)
    return ok


def check(g, o, k, topk_group, n_group, scale):
    idx = g["idx"].cpu().numpy()
    w = g["w"].cpu().numpy().astype(np.float64)
    clear = clear_tokens(o, k, topk_group, n_group)
    assert clear.mean() > 0.9, clear.mean()
    np.testing.assert_array_equal(idx[clear], o["idx"][clear])
    np.testing.assert_allclose(w[clear], o["w"][clear], rtol=0, atol=PROB_ATOL * max(scale, 1.0))
    # ambiguous tokens: the choice must still be a valid one within the tolerance
    E = o["choice"].shape[1]
    gs = E // n_group
    for t in np.nonzero(~clear)[0]:
        chosen = idx[t]
        assert len(set(chosen.tolist())) == k
        gsc = o["group_scores"][t]
        kth_group = np.sort(gsc)[-topk_group]
        groups = set((chosen // gs).tolist())
        assert len(groups) <= topk_group
        assert all(gsc[j] >= kth_group - 2 * TAU_C for j in groups)
        cc = o["choice"][t, chosen]
        assert (np.diff(cc) <= TAU_C).all()
    if "scores" in g:
        np.testing.assert_allclose(g["scores"].cpu().numpy().astype(np.float64), o["scores"], rtol=0, atol=PROB_ATOL)
    if "counts" in g:
        cnt = g["counts"].cpu().numpy()
        assert cnt.sum() == idx.size
        np.testing.assert_array_equal(cnt, np.bincount(idx.ravel(), minlength=E))
    return int((~clear).sum())


CASES = [
    # T, H, E, k, n_group, topk_group, group_top, scoring, renorm, scale, logit bias, selection bias
    (300, 256, 256, 8, 8, 4, 2, "sigmoid", True, 2.5, False, True),     # the DeepSeek-V3 gate
    (257, 192, 256, 8, 8, 4, 2, "softmax", False, 1.0, True, True),
    (130, 128, 128, 8, 4, 2, 2, "sigmoid", True, 1.0, True, False),
    (99, 64, 64, 6, 16, 3, 1, "sigmoid", True, 1.0, False, True),
    (65, 72, 96, 4, 3, 1, 3, "softmax", True, 2.0, False, False),      # H % 64 != 0, E % 64 != 0
    (64, 64, 8, 2, 1, 1, 2, "sigmoid", False, 1.0, False, True),
    (33, 64, 10, 3, 5, 2, 2, "sigmoid", True, 1.0, True, True),        # E % 4 != 0: scalar loads
    (1, 64, 256, 8, 8, 4, 2, "sigmoid", True, 2.5, False, True),
    (0, 64, 256, 8, 8, 4, 2, "sigmoid", True, 2.5, False, True),
]


@pytest.mark.parametrize("T,H,E,k,n_group,topk_group,group_top,scoring,renorm,scale,lbias,sbias", CASES)
def test_route_grouped_parity(T, H, E, k, n_group, topk_group, group_top, scoring, renorm, scale, lbias, sbias):
    x, w, sb, bias = make_case(T * 31 + E, T, H, E)
    tpg = max((T + 1) // 2, 1)
    o = oracle.route_grouped(x, w, bias if lbias else None, tpg, sb if sbias else None, scoring=scoring,
                             n_group=n_group, topk_group=topk_group, group_top=group_top, k=k, renormalize=renorm,
                             routed_scale=scale)
    g = probe.route_grouped(dev_bf16(x) if T else torch.empty((0, H), dtype=torch.bfloat16, device="cuda"),
                            torch.from_numpy(w).cuda(), torch.from_numpy(bias).cuda() if lbias else None, tpg,
                            torch.from_numpy(sb).cuda() if sbias else None, scoring=scoring, n_group=n_group,
                            topk_group=topk_group, group_top=group_top, k=k, renormalize=renorm, routed_scale=scale,
                            want_scores=True)
    torch.cuda.synchronize()
    if T == 0:
        assert g["counts"].cpu().numpy().sum() == 0
        return
    check(g, o, k, topk_group, n_group, scale)


def test_one_group_softmax_equals_route_topk_bitwise():
    x, w, sb, bias = make_case(5, 500, 256, 128)
    dx, dw, db = dev_bf16(x), torch.from_numpy(w).cuda(), torch.from_numpy(bias).cuda()
    a = probe.route_topk(dx, dw, db, 250, k=8, renormalize=True, want_probs=True)
    b = probe.route_grouped(dx, dw, db, 250, None, scoring="softmax", n_group=1, topk_group=1, group_top=1, k=8,
                            renormalize=True, want_scores=True)
    torch.cuda.synchronize()
    assert torch.equal(a["idx"], b["idx"]) and torch.equal(a["counts"], b["counts"])
    assert torch.equal(a["probs"], b["scores"])
    np.testing.assert_allclose(a["w"].cpu().numpy(), b["w"].cpu().numpy(), rtol=0, atol=1e-6)


def test_deepseek_shape_sampled():
    """Configuration-3 shape (8192 tokens, 256 experts in 8 groups, 4 allowed, top-8): a token sample against the oracle."""
    cfg = wl.CONFIGS[3]
    x = wl.activations(cfg, 0)
    w = wl.gate_weights(cfg, 0)
    rng = np.random.default_rng(11)
    sb = (rng.standard_normal(cfg.E) * 0.02).astype(np.float32)
    g = probe.route_grouped(dev_bf16(x), torch.from_numpy(w).cuda(), None, None, torch.from_numpy(sb).cuda(),
                            scoring="sigmoid", n_group=8, topk_group=4, group_top=2, k=8, renormalize=True,
                            routed_scale=2.5, want_scores=True)
    torch.cuda.synchronize()
    tokens = np.sort(rng.choice(cfg.T, 256, replace=False))
    o = oracle.route_grouped(x[tokens], w, None, None, sb, scoring="sigmoid", n_group=8, topk_group=4, group_top=2, k=8,
                             renormalize=True, routed_scale=2.5)
    sub = dict(idx=g["idx"][tokens], w=g["w"][tokens], scores=g["scores"][tokens])
    check(sub, o, 8, 4, 8, 2.5)
    cnt = g["counts"].cpu().numpy()
    np.testing.assert_array_equal(cnt, np.bincount(g["idx"].cpu().numpy().ravel(), minlength=cfg.E))
    # every token stays inside four groups of 32 experts
    grp = (g["idx"].cpu().numpy() // 32)
    assert max(len(set(r.tolist())) for r in grp) <= 4


@pytest.mark.parametrize("T,H,F,k,scale", [(300, 128, 192, 4, 1.0), (65, 64, 64, 8, 0.5), (1, 64, 64, 1, 1.0)])
def test_combine_with_shared_expert(T, H, F, k, scale):
    """probe_combine_shared against the oracle; the shared expert's output comes from the grouped FFN run on x
    itself with one slot of T rows (checked against the oracle's FFN too)."""
    from gpu_util import bits_of, f64_of, rel_err, BF16_RTOL
    rng = np.random.default_rng(T + k)
    x = wl.f32_to_bf16_bits(rng.standard_normal((T, H)).astype(np.float32))
    w13 = wl.f32_to_bf16_bits((rng.standard_normal((2 * F, H)) * 0.05).astype(np.float32))
    w2 = wl.f32_to_bf16_bits((rng.standard_normal((H, F)) * 0.05).astype(np.float32))
    n_rows = T * k // 2 + 3
    y = wl.f32_to_bf16_bits(rng.standard_normal((n_rows, H)).astype(np.float32))
    pair_row = rng.integers(-1, n_rows, size=(T, k)).astype(np.int32)
    w = rng.random((T, k)).astype(np.float32)
    so = np.array([0, T], np.int32)
    d_x = dev_bf16(x)
    shared = probe.grouped_ffn(d_x, torch.from_numpy(so).cuda(), probe.WeightTable([dev_bf16(w13)], [dev_bf16(w2)]))
    out = probe.combine_shared(dev_bf16(y), torch.from_numpy(pair_row).cuda(), torch.from_numpy(w).cuda(), shared, scale)
    plain = probe.combine(dev_bf16(y), torch.from_numpy(pair_row).cuda(), torch.from_numpy(w).cuda())
    zero = probe.combine_shared(dev_bf16(y), torch.from_numpy(pair_row).cuda(), torch.from_numpy(w).cuda(),
                                torch.zeros_like(shared), 3.0)
    torch.cuda.synchronize()
    o_shared = oracle.grouped_ffn(x, so, [w13], [w2])
    assert rel_err(f64_of(shared), o_shared) <= BF16_RTOL
    yf = wl.bf16_bits_to_f32(y).astype(np.float64)
    # fed with the GPU's own (bf16) shared output: one fp32 accumulation and one rounding
    o = oracle.combine_shared(yf, pair_row, w.astype(np.float64), f64_of(shared), scale)
    assert rel_err(f64_of(out), o) <= 4e-3
    # and end to end against the oracle's own shared expert
    o2 = oracle.combine_shared(yf, pair_row, w.astype(np.float64), o_shared, scale)
    assert rel_err(f64_of(out), o2) <= BF16_RTOL
    assert torch.equal(zero, plain)
