"""GPU parity of probe_predict_topk_residual (Eq. 7 with its residual MLP) against the oracle."""
import numpy as np
import pytest
import torch

from paper_2602_00509_amd import workload as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def probe():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2602_00509_amd import probe as p
    p.lib()
    return p


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


def _case(seed, T, H, E, D, groups):
    rng = np.random.default_rng(seed)
    x = wl.f32_to_bf16_bits(rng.standard_normal((T, H), dtype=np.float32))
    wg = rng.standard_normal((E, H), dtype=np.float32) * np.float32(0.05)
    b = rng.standard_normal((groups, E)).astype(np.float32)
    w1 = wl.f32_to_bf16_bits(rng.standard_normal((D, H), dtype=np.float32) * np.float32(1.5 / np.sqrt(H)))
    w2 = (rng.standard_normal((E, D)) * (1.0 / np.sqrt(D))).astype(np.float32)
    return x, wg, b, w1, w2


@pytest.mark.parametrize("T,H,E,D,k", [(300, 128, 64, 64, 4), (2100, 256, 256, 256, 8), (8200, 512, 256, 128, 8),
                                       (150, 72, 20, 24, 3), (77, 64, 9, 8, 2), (513, 192, 130, 1024, 6)])
def test_predictor_with_residual_matches_oracle(oracle, probe, G, T, H, E, D, k):
    """Every token: indices bit-exact outside the ambiguity margin, weights and probabilities within 1e-5.
    The shapes cover both GEMM kernels (H % 64 == 0 or not), both token-tile heights, widths D that are
    not multiples of 128 and the largest D, E not a multiple of 4."""
    print("case predictor T=%d H=%d E=%d D=%d" % (T, H, E, D), flush=True)
    x, wg, b, w1, w2 = _case(T + D, T, H, E, D, 3)
    tpg = max(T // 3, 1)
    g = probe.predict_topk_residual(G.dev_bf16(x), torch.from_numpy(wg).cuda(), torch.from_numpy(b).cuda(), tpg,
                                    G.dev_bf16(w1), torch.from_numpy(w2).cuda(), k, True, want_probs=True)
    torch.cuda.synchronize()
    o = oracle.predict_topk_residual(x, wg, b, tpg, w1, w2, k, True)
    # the residual must matter in this test: it changes the top-k of a good share of the tokens
    base = oracle.route_topk(x, wg, b, tpg, k, True)
    assert (base["idx"] != o["idx"]).any(axis=1).mean() > 0.2
    G.check_route(g, o, k, True)
    np.testing.assert_allclose(g["probs"].cpu().numpy(), o["probs"], rtol=0, atol=G.PROB_ATOL)
    np.testing.assert_array_equal(g["counts"].cpu().numpy(), np.bincount(g["idx"].cpu().numpy().ravel(), minlength=E))


def test_zero_output_layer_is_bitwise_the_plain_predictor(probe, G):
    """W2_hat = 0 (the paper's initialisation) adds a plane of zeros: same bits as probe_predict_topk."""
    T, H, E, D, k = 1000, 256, 128, 64, 8
    x, wg, b, w1, _ = _case(5, T, H, E, D, 2)
    dx, dwg, db = G.dev_bf16(x), torch.from_numpy(wg).cuda(), torch.from_numpy(b).cuda()
    p0 = probe.predict_topk(dx, dwg, db, 500, k, True, want_probs=True)
    p1 = probe.predict_topk_residual(dx, dwg, db, 500, G.dev_bf16(w1), torch.zeros((E, D), device="cuda"), k, True,
                                     want_probs=True)
    torch.cuda.synchronize()
    for key in ("idx", "w", "probs", "counts"):
        assert torch.equal(p0[key], p1[key]), key


def test_predictor_with_residual_at_the_benchmark_shape(oracle, probe, G):
    """DeepSeek-V3-shaped shard (T = 8192, H = 7168, E = 256, top-8) with a residual of width 256, in the
    launch configuration the benchmark uses; 192 sampled tokens against the oracle."""
    cfg = wl.CONFIGS[3]
    T, H, E, k, D = cfg.T, cfg.H, cfg.E, cfg.k, 256
    x = wl.activations(cfg, 1)
    wg = wl.gate_weights(cfg, 1)
    b = wl.zipf_bias(cfg, 1, 1)
    rng = np.random.default_rng(33)
    w1 = wl.f32_to_bf16_bits(rng.standard_normal((D, H), dtype=np.float32) * np.float32(1.5 / np.sqrt(H)))
    w2 = (rng.standard_normal((E, D)) * (1.0 / np.sqrt(D))).astype(np.float32)
    tpg = wl.tokens_per_group(cfg)
    g = probe.predict_topk_residual(G.dev_bf16(x), torch.from_numpy(wg).cuda(), torch.from_numpy(b).cuda(), tpg,
                                    G.dev_bf16(w1), torch.from_numpy(w2).cuda(), k, True, want_probs=True)
    torch.cuda.synchronize()
    tok = np.sort(rng.choice(T, size=192, replace=False))
    o = oracle.predict_topk_residual(x[tok], wg, G.gather_bias(b, tpg, tok), 1, w1, w2, k, True)
    G.check_route(g, o, k, True, tokens=tok)
    np.testing.assert_allclose(g["probs"].cpu().numpy()[tok], o["probs"], rtol=0, atol=G.PROB_ATOL)
    idx = g["idx"].cpu().numpy()
    np.testing.assert_array_equal(g["counts"].cpu().numpy(), np.bincount(idx.ravel(), minlength=E))


@pytest.mark.parametrize("T,H,E,k", [(300, 128, 64, 4), (2100, 256, 256, 8), (8200, 512, 128, 8), (150, 72, 9, 3)])
def test_fused_router_and_predictor_match_their_oracles(oracle, probe, G, T, H, E, k):
    """One pass over x for this layer's router and the next layer's (zero-residual) predictor: each output
    set against the oracle of its own gate, and against the two separate calls (same decisions)."""
    print("case fused T=%d H=%d E=%d" % (T, H, E), flush=True)
    rng = np.random.default_rng(T)
    x = wl.f32_to_bf16_bits(rng.standard_normal((T, H), dtype=np.float32))
    w1 = rng.standard_normal((E, H), dtype=np.float32) * np.float32(0.05)
    w2 = rng.standard_normal((E, H), dtype=np.float32) * np.float32(0.05)
    b1 = rng.standard_normal((2, E)).astype(np.float32)
    b2 = rng.standard_normal((2, E)).astype(np.float32)
    tpg = (T + 1) // 2
    dx = G.dev_bf16(x)
    d = lambda a: torch.from_numpy(a).cuda()
    r, p = probe.route_predict_topk(dx, d(w1), d(b1), d(w2), d(b2), tpg, k, True, want_probs=True)
    torch.cuda.synchronize()
    for got, w, b in ((r, w1, b1), (p, w2, b2)):
        o = oracle.route_topk(x, w, b, tpg, k, True)
        G.check_route(got, o, k, True)
        np.testing.assert_allclose(got["probs"].cpu().numpy(), o["probs"], rtol=0, atol=G.PROB_ATOL)
        np.testing.assert_array_equal(got["counts"].cpu().numpy(),
                                      np.bincount(got["idx"].cpu().numpy().ravel(), minlength=E))
    # a missing bias on one side only
    r2, p2 = probe.route_predict_topk(dx, d(w1), None, d(w2), d(b2), tpg, k, False)
    torch.cuda.synchronize()
    G.check_route(r2, oracle.route_topk(x, w1, None, tpg, k, False), k, False)
    G.check_route(p2, oracle.route_topk(x, w2, b2, tpg, k, False), k, False)


def test_predictor_metrics_match_the_oracle(oracle, probe, G):
    """Top-k accuracy, top-half-k hit rate (exact integers) and the cross-entropy sum of the predictor
    against the next layer's router on drifted hidden states; zero drift gives accuracy 1."""
    cfg = wl.small_config(T=1500, H=128, E=64, k=8, F=128, E_loc=8, n_rep=0, zipf_s=1.5, ep=8, cid=95)
    T, E, k = cfg.T, cfg.E, cfg.k
    x = wl.activations(cfg, 0)
    wg = wl.gate_weights(cfg, 1)
    b = wl.zipf_bias(cfg, 0, 1)
    tpg = wl.tokens_per_group(cfg)
    d = lambda a: torch.from_numpy(a).cuda()
    for alpha in (0.0, 0.5):
        x2 = wl.drifted_activations(cfg, x, alpha, 0) if alpha else x
        pred = probe.predict_topk(G.dev_bf16(x), d(wg), d(b), tpg, k, True, want_probs=True)
        true = probe.route_topk(G.dev_bf16(x2), d(wg), d(b), tpg, k, True, want_probs=True)
        hits, ce = probe.predictor_metrics(pred["idx"], true["idx"], pred_probs=pred["probs"], true_probs=true["probs"])
        half, _ = probe.predictor_metrics(pred["idx"], true["idx"], kp=k, kt=k // 2)
        torch.cuda.synchronize()
        pi, ti = pred["idx"].cpu().numpy(), true["idx"].cpu().numpy()
        assert int(hits) == round(oracle.topk_overlap(pi, ti) * T * k)
        assert int(half) == round(oracle.topk_overlap(pi, ti[:, : k // 2]) * T * (k // 2))
        ref = oracle.cross_entropy_sum(true["probs"].cpu().numpy(), pred["probs"].cpu().numpy())
        assert abs(float(ce) - ref) <= 1e-9 * abs(ref)
        if alpha == 0.0:
            assert int(hits) == T * k and int(half) == T * (k // 2)
        else:
            assert 0.3 * T * k < int(hits) < T * k
