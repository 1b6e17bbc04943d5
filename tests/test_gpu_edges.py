"""GPU edge cases through the C ABI: empty and degenerate inputs, determinism, plan
invariance, the predictor identity, HIP-graph replay of the five-call sequence."""
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


def _layer(G, probe, cfg, batch=0):
    L = G.Layer(cfg, batch)
    r = probe.route_topk(L.d_x, L.d_wg, L.d_bias, L.tpg, cfg.k, True, want_probs=True)
    torch.cuda.synchronize()
    return L, r


def test_empty_batch(probe):
    print("case empty batch", flush=True)
    dev = "cuda"
    H, E, k, S, F = 64, 8, 2, 3, 64
    x = torch.empty((0, H), dtype=torch.bfloat16, device=dev)
    wg = torch.zeros((E, H), dtype=torch.float32, device=dev)
    r = probe.route_topk(x, wg, None, None, k, True, out=dict(counts=torch.full((E,), 7, dtype=torch.int32, device=dev)))
    assert r["idx"].shape == (0, k) and int(r["counts"].abs().sum()) == 0
    plan = probe.Plan(np.arange(E + 1), np.array([0, 1, 2, -1, -1, -1, -1, -1]), np.ones(E), S)
    p = probe.permute(r["idx"], plan, x)
    torch.cuda.synchronize()
    assert int(p["n_local"]) == 0 and p["slot_offsets"].tolist() == [0] * (S + 1) and p["slot_counts"].tolist() == [0] * S
    w13 = [torch.zeros((2 * F, H), dtype=torch.bfloat16, device=dev) for _ in range(S)]
    w2 = [torch.zeros((H, F), dtype=torch.bfloat16, device=dev) for _ in range(S)]
    y = probe.grouped_ffn(p["xp"], p["slot_offsets"], probe.WeightTable(w13, w2))
    out = probe.combine(y, p["pair_row"], r["w"])
    torch.cuda.synchronize()
    assert y.shape == (0, H) and out.shape == (0, H)


def test_all_remote_and_zero_weight_replica(oracle, probe, G):
    print("case all remote / zero weight", flush=True)
    cfg = wl.small_config(T=200, H=128, E=12, k=3, F=128, E_loc=4, n_rep=2, ep=3, chunk=0, cid=80)
    L, r = _layer(G, probe, cfg)
    E, S = cfg.E, cfg.S
    # every expert remote: no rows, pair_row all -1, combine gives zeros, FFN launches do nothing
    plan = probe.Plan(np.arange(E + 1), -np.ones(E), np.ones(E), S)
    p = probe.permute(r["idx"], plan, L.d_x)
    L.load_weights(np.arange(S) % E, probe)
    y = torch.full((cfg.N, cfg.H), float("nan"), dtype=torch.bfloat16, device="cuda")
    probe.grouped_ffn(p["xp"], p["slot_offsets"], L.weights, out=y)
    out = probe.combine(torch.zeros_like(y), p["pair_row"], r["w"])
    torch.cuda.synchronize()
    assert int(p["n_local"]) == 0 and bool((p["pair_row"] == -1).all()) and bool((p["row_pair"] == -1).all())
    assert bool(torch.isnan(y.float()).all()) and float(out.float().abs().max()) == 0.0
    # a zero-weight replica receives nothing; its partner takes everything
    g_idx = r["idx"].cpu().numpy()
    rep_off = np.r_[0, 2, np.arange(3, E + 2)]
    rep_slot = np.r_[0, 4, np.where(np.arange(1, E) < 4, np.arange(1, E), -1)]
    rep_weight = np.r_[0, 5, np.ones(E - 1, np.int64)]
    plan = probe.Plan(rep_off, rep_slot, rep_weight, S)
    p = probe.permute(r["idx"], plan, L.d_x)
    torch.cuda.synchronize()
    o = oracle.permute(g_idx, rep_off.astype(np.int32), rep_slot.astype(np.int32), rep_weight.astype(np.int32), S, L.x)
    assert int(p["slot_counts"][0]) == 0 and int(p["slot_counts"][4]) == int((g_idx == 0).sum())
    np.testing.assert_array_equal(p["pair_row"].cpu().numpy(), o["pair_row"])
    np.testing.assert_array_equal(p["row_pair"].cpu().numpy(), o["row_pair"])
    np.testing.assert_array_equal(p["slot_offsets"].cpu().numpy(), o["slot_offsets"])


def test_topk_equals_all_experts_and_predictor_identity(oracle, probe, G):
    print("case k == E, predictor identity", flush=True)
    cfg = wl.small_config(T=77, H=64, E=8, k=8, F=64, E_loc=8, n_rep=0, ep=1, chunk=0, cid=81)
    L, r = _layer(G, probe, cfg)
    o = oracle.route_topk(L.x, L.wg, L.bias, L.tpg, cfg.k, True)
    G.check_route(r, o, cfg.k, True)
    assert bool((torch.sort(r["idx"], dim=1).values == torch.arange(8, device="cuda", dtype=torch.int32)).all())
    np.testing.assert_allclose(r["w"].sum(1).cpu().numpy(), 1.0, atol=1e-6)
    assert r["counts"].tolist() == [cfg.T] * 8
    # Sec. 4.2: at the zero-initialised residual the predictor is the cloned router
    pr = probe.predict_topk(L.d_x, L.d_wg, L.d_bias, L.tpg, cfg.k, True, want_probs=True)
    torch.cuda.synchronize()
    for key in ("idx", "w", "probs", "counts"):
        assert torch.equal(r[key], pr[key]), key


@pytest.mark.parametrize("T,H,E,k", [(150, 72, 20, 3), (300, 200, 130, 8), (64, 8, 5, 2), (129, 1000, 256, 8)])
def test_route_when_hidden_size_is_not_a_multiple_of_64(oracle, probe, G, T, H, E, k):
    """H % 8 == 0 is all the router asks for; these shapes take the kernel that zero-fills the K tail."""
    print("case route H=%d" % H, flush=True)
    rng = np.random.default_rng(H)
    x = wl.f32_to_bf16_bits(rng.standard_normal((T, H), dtype=np.float32))
    wg = (rng.standard_normal((E, H), dtype=np.float32) * np.float32(0.05))
    b = rng.standard_normal((2, E)).astype(np.float32)
    tpg = 100
    g = probe.route_topk(G.dev_bf16(x), torch.from_numpy(wg).cuda(), torch.from_numpy(b).cuda(), tpg, k, True,
                         want_probs=True)
    torch.cuda.synchronize()
    o = oracle.route_topk(x, wg, b, tpg, k, True)
    G.check_route(g, o, k, True)
    np.testing.assert_array_equal(g["counts"].cpu().numpy(), np.bincount(g["idx"].cpu().numpy().ravel(), minlength=E))


@pytest.mark.parametrize("T,H,E,k", [(8200, 256, 256, 8), (4100, 1024, 200, 6), (2049, 128, 130, 4)])
def test_route_on_256_token_tiles_with_a_ragged_last_tile(oracle, probe, G, T, H, E, k):
    """Large batches take the 256-token tile of the gate GEMM; T is not a multiple of the tile, E not
    always one of 128, and the K range of one split is as short as one step."""
    print("case route T=%d H=%d E=%d" % (T, H, E), flush=True)
    rng = np.random.default_rng(T)
    x = wl.f32_to_bf16_bits(rng.standard_normal((T, H), dtype=np.float32))
    wg = (rng.standard_normal((E, H), dtype=np.float32) * np.float32(0.05))
    b = rng.standard_normal((3, E)).astype(np.float32)
    tpg = 1500
    g = probe.route_topk(G.dev_bf16(x), torch.from_numpy(wg).cuda(), torch.from_numpy(b).cuda(), tpg, k, True,
                         want_probs=True)
    torch.cuda.synchronize()
    o = oracle.route_topk(x, wg, b, tpg, k, True)
    G.check_route(g, o, k, True)
    np.testing.assert_allclose(g["probs"].cpu().numpy(), o["probs"], rtol=0, atol=G.PROB_ATOL)
    np.testing.assert_array_equal(g["counts"].cpu().numpy(), np.bincount(g["idx"].cpu().numpy().ravel(), minlength=E))


def test_determinism_and_plan_invariance(oracle, probe, G):
    """Two runs are bit-identical; with every replica local, any plan gives the same layer output."""
    print("case determinism / plan invariance", flush=True)
    cfg = wl.small_config(T=900, H=256, E=6, k=2, F=320, E_loc=6, n_rep=2, ep=1, chunk=256, cid=82)
    L, r = _layer(G, probe, cfg)
    counts = r["counts"].cpu().numpy()

    def run(plan):
        d_plan = probe.Plan(plan["rep_off"], plan["rep_slot"], plan["rep_weight"], plan["num_slots"])
        p = probe.permute(r["idx"], d_plan, L.d_x)
        L.load_weights(plan["slot_expert"], probe)
        y = torch.zeros((cfg.N, cfg.H), dtype=torch.bfloat16, device="cuda")
        probe.grouped_ffn(p["xp"], p["slot_offsets"], L.weights, out=y)
        out = probe.combine(y, p["pair_row"], r["w"])
        torch.cuda.synchronize()
        return p, y, out

    base = wl.no_replica_plan(cfg)
    rep = wl.build_plan(cfg, counts)
    p0, y0, out0 = run(base)
    p0b, y0b, out0b = run(base)
    assert torch.equal(out0, out0b) and torch.equal(y0, y0b) and torch.equal(p0["row_pair"], p0b["row_pair"])
    p1, y1, out1 = run(rep)
    assert int(p1["n_local"]) == cfg.N == int(p0["n_local"])
    assert bool((p1["slot_counts"][cfg.E_loc:] > 0).all())
    # a row's K loop does not depend on where the row sits, so the outputs agree bit for bit
    assert torch.equal(out0, out1)


def test_predictor_overlap_matches_oracle(oracle, probe, G):
    """Top-k overlap of the lookahead predictor against the next layer's router: the GPU's
    integer metric equals the oracle's on unambiguous tokens; drift 0 gives overlap 1."""
    print("case predictor overlap", flush=True)
    cfg = wl.small_config(T=512, H=256, E=64, k=8, F=64, E_loc=16, n_rep=0, ep=4, chunk=128, cid=83)
    h = wl.activations(cfg, 0)
    wn, bn = wl.gate_weights(cfg, 1), wl.zipf_bias(cfg, 0, 1)
    d_w, d_b = torch.from_numpy(wn).cuda(), torch.from_numpy(bn).cuda()
    tpg = wl.tokens_per_group(cfg)
    for alpha, lo, hi in ((0.0, 1.0, 1.0), (0.2, 0.6, 1.0), (0.5, 0.4, 0.95)):
        h2 = wl.drifted_activations(cfg, h, alpha, 0) if alpha > 0 else h
        pred = probe.predict_topk(G.dev_bf16(h), d_w, d_b, tpg, cfg.k, True)
        true = probe.route_topk(G.dev_bf16(h2), d_w, d_b, tpg, cfg.k, True)
        torch.cuda.synchronize()
        g_ov = oracle.topk_overlap(pred["idx"].cpu().numpy(), true["idx"].cpu().numpy())
        o_pred = oracle.predict_topk(h, wn, bn, tpg, cfg.k, True)
        o_true = oracle.route_topk(h2, wn, bn, tpg, cfg.k, True)
        o_ov = oracle.topk_overlap(o_pred["idx"], o_true["idx"])
        amb = G.ambiguous_tokens(o_pred["logits"], cfg.k) | G.ambiguous_tokens(o_true["logits"], cfg.k)
        assert abs(g_ov - o_ov) <= amb.sum() * cfg.k / (cfg.T * cfg.k) + 1e-12
        assert lo <= g_ov <= hi, (alpha, g_ov)


def test_graph_replay(oracle, probe, G):
    """The five calls record into a HIP graph (no allocation, no host sync, no memset nodes);
    every replay, with eager work in between, reproduces the eager results."""
    print("case graph replay", flush=True)
    cfg = wl.small_config(T=300, H=128, E=16, k=4, F=128, E_loc=8, n_rep=2, ep=2, chunk=0, cid=84)
    L, r0 = _layer(G, probe, cfg)
    plan = wl.build_plan(cfg, r0["counts"].cpu().numpy())
    d_plan = probe.Plan(plan["rep_off"], plan["rep_slot"], plan["rep_weight"], plan["num_slots"])
    L.load_weights(plan["slot_expert"], probe)
    T, H, E, k, S, F, N = cfg.T, cfg.H, cfg.E, cfg.k, cfg.S, cfg.F, cfg.N
    dev = "cuda"
    mk = lambda shape, dt: torch.zeros(shape, dtype=dt, device=dev)
    bufs = dict(r=dict(idx=mk((T, k), torch.int32), w=mk((T, k), torch.float32), counts=mk((E,), torch.int32)),
                pr=dict(idx=mk((T, k), torch.int32), w=mk((T, k), torch.float32), counts=mk((E,), torch.int32)),
                p=dict(slot_counts=mk((S,), torch.int32), slot_offsets=mk((S + 1,), torch.int32),
                       row_pair=mk((N,), torch.int32), pair_row=mk((T, k), torch.int32),
                       xp=mk((N, H), torch.bfloat16), n_local=mk((1,), torch.int32)),
                y=mk((N, H), torch.bfloat16), out=mk((T, H), torch.bfloat16))
    ws_r = torch.empty(probe.route_topk_workspace_bytes(T, H, E, k), dtype=torch.uint8, device=dev)
    ws_p = torch.empty(max(256, probe.permute_workspace_bytes(T, E, k, S)), dtype=torch.uint8, device=dev)
    ws_f = torch.empty(probe.grouped_ffn_workspace_bytes(S, H, F, N), dtype=torch.uint8, device=dev)

    def step():
        probe.predict_topk(L.d_x, L.d_wg, L.d_bias, L.tpg, k, True, out=bufs["pr"], workspace=ws_r)
        probe.route_topk(L.d_x, L.d_wg, L.d_bias, L.tpg, k, True, out=bufs["r"], workspace=ws_r)
        probe.permute(bufs["r"]["idx"], d_plan, L.d_x, out=bufs["p"], workspace=ws_p)
        probe.grouped_ffn(bufs["p"]["xp"], bufs["p"]["slot_offsets"], L.weights, out=bufs["y"], workspace=ws_f)
        probe.combine(bufs["y"], bufs["p"]["pair_row"], bufs["r"]["w"], out=bufs["out"])

    step()                                   # eager (also the one-time LDS opt-in of the FFN kernels)
    torch.cuda.synchronize()
    ref = {k_: bufs[k_].clone() for k_ in ("y", "out")}
    ref_idx, ref_rows = bufs["r"]["idx"].clone(), bufs["p"]["row_pair"].clone()
    nl = int(bufs["p"]["n_local"])
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            step()
    torch.cuda.synchronize()
    for i in range(3):
        for t in (bufs["y"], bufs["out"], bufs["r"]["idx"], bufs["p"]["row_pair"]):
            t.fill_(0)                       # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(bufs["r"]["idx"], ref_idx) and torch.equal(bufs["p"]["row_pair"], ref_rows), i
        assert torch.equal(bufs["y"][:nl], ref["y"][:nl]) and torch.equal(bufs["out"], ref["out"]), i


def test_ffn_every_way_a_slot_is_cut_into_tiles(oracle, probe, G):
    """Slot sizes on both sides of every tile-height boundary (the FFN cuts a slot into row tiles of
    several heights and lets taller tiles absorb small remainders), empty slots in between: every
    output element against the oracle."""
    cfg = wl.small_config(T=64, H=128, E=4, k=2, F=192, cid=93)
    sizes = [0, 1, 63, 64, 65, 128, 129, 191, 192, 193, 255, 256, 257, 0, 300, 320, 321, 384, 385, 449,
             512, 513, 576, 577, 640, 641, 700, 768 + 1, 768 + 65, 768 + 129, 768 + 192, 768 + 193, 1024 + 130, 7]
    S = len(sizes)
    so = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    n = int(so[-1])
    ws = wl.expert_weights_many(cfg, [s % 4 for s in range(S)])
    rng = np.random.default_rng(5)
    xp = wl.f32_to_bf16_bits(rng.standard_normal((n + 9, cfg.H)).astype(np.float32))
    d_w = {e: (G.dev_bf16(ws[e][0]), G.dev_bf16(ws[e][1])) for e in range(4)}
    tab = probe.WeightTable([d_w[s % 4][0] for s in range(S)], [d_w[s % 4][1] for s in range(S)])
    d_xp = G.dev_bf16(xp)
    y = torch.full((n + 9, cfg.H), 7.0, dtype=torch.bfloat16, device="cuda")
    probe.grouped_ffn(d_xp, torch.from_numpy(so).cuda(), tab, out=y)
    torch.cuda.synchronize()
    ref = oracle.grouped_ffn(xp, so, [ws[s % 4][0] for s in range(S)], [ws[s % 4][1] for s in range(S)])
    got = G.f64_of(y)
    assert G.rel_err(got[:n], ref) < G.BF16_RTOL
    assert (got[n:] == 7.0).all()          # rows past the last slot are not written


def _ffn_against_oracle(oracle, probe, G, cfg, sizes, n_weights, seed, extra_rows=9):
    """probe_grouped_ffn on slots of the given sizes, every output element against the oracle."""
    S = len(sizes)
    so = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    n = int(so[-1])
    ws = wl.expert_weights_many(cfg, list(range(n_weights)))
    rng = np.random.default_rng(seed)
    xp = wl.f32_to_bf16_bits(rng.standard_normal((n + extra_rows, cfg.H)).astype(np.float32))
    d_w = {e: (G.dev_bf16(ws[e][0]), G.dev_bf16(ws[e][1])) for e in range(n_weights)}
    tab = probe.WeightTable([d_w[s % n_weights][0] for s in range(S)], [d_w[s % n_weights][1] for s in range(S)])
    y = torch.full((n + extra_rows, cfg.H), 7.0, dtype=torch.bfloat16, device="cuda")
    probe.grouped_ffn(G.dev_bf16(xp), torch.from_numpy(so).cuda(), tab, out=y)
    torch.cuda.synchronize()
    ref = oracle.grouped_ffn(xp, so, [ws[s % n_weights][0] for s in range(S)], [ws[s % n_weights][1] for s in range(S)])
    got = G.f64_of(y)
    err = G.rel_err(got[:n], ref)
    assert err < G.BF16_RTOL, err
    assert (got[n:] == 7.0).all()          # rows past the last slot are not written
    return err


def test_ffn_decode_schedule_every_element(oracle, probe, G):
    """A decode-sized row space (at most 64 rows per slot on average): the call takes the schedule of skinny
    tiles (64 rows x 64 h columns / 128 output columns).  Slot sizes around the 64-row tile boundary, empty
    slots, slots of several row tiles; F and H that leave a partial last column block."""
    for (H, F, cid) in ((192, 320, 96), (128, 64, 97), (256, 448, 98)):
        cfg = wl.small_config(T=64, H=H, E=4, k=2, F=F, cid=cid)
        sizes = [0, 1, 40, 63, 64, 65, 0, 130, 17, 33, 5, 0, 90, 2]
        assert sum(sizes) + 9 <= 64 * len(sizes)
        print("case decode schedule H=%d F=%d" % (H, F), flush=True)
        _ffn_against_oracle(oracle, probe, G, cfg, sizes, 4, seed=H + F)


def test_ffn_every_tile_height_at_full_depth(oracle, probe, G):
    """One slot per tile height (320, 256, 192, 128, 64 rows) and a ragged one, at the depth of the benchmark's
    main configuration (K = 7168 in the first GEMM, 2048 in the second: 112 and 32 steps of the main loop):
    every output element against the oracle."""
    cfg = wl.CONFIGS[3]
    print("case full-depth tile heights", flush=True)
    _ffn_against_oracle(oracle, probe, G, cfg, [320, 256, 192, 128, 64, 37, 0, 321], 3, seed=77)


@pytest.mark.parametrize("cid", [1, 4])
def test_ffn_with_rows_gathered_on_load_equals_ffn_on_the_permuted_copy(oracle, probe, G, cid):
    """probe_permute without the row copy + probe_grouped_ffn_gather give bit for bit the y of the standard
    pair (same kernels, only the source of the activation rows differs), and match the oracle."""
    cfg = wl.CONFIGS[cid]
    L, r = _layer(G, probe, cfg)
    counts = r["counts"].cpu().numpy()
    plan = wl.build_plan(cfg, counts)
    d_plan = probe.Plan(plan["rep_off"], plan["rep_slot"], plan["rep_weight"], plan["num_slots"])
    full = probe.permute(r["idx"], d_plan, L.d_x)
    lean = probe.permute(r["idx"], d_plan, L.d_x, copy_rows=False)
    assert "xp" not in lean
    for key in ("slot_counts", "slot_offsets", "pair_row", "n_local"):
        assert torch.equal(full[key], lean[key]), key
    nl = int(full["n_local"].item())
    assert torch.equal(full["row_pair"][:nl], lean["row_pair"][:nl])
    L.load_weights(plan["slot_expert"], probe)
    y0 = torch.full((cfg.N, cfg.H), 3.0, dtype=torch.bfloat16, device="cuda")
    y1 = torch.full((cfg.N, cfg.H), 3.0, dtype=torch.bfloat16, device="cuda")
    probe.grouped_ffn(full["xp"], full["slot_offsets"], L.weights, out=y0)
    probe.grouped_ffn_gather(L.d_x, lean["row_pair"], cfg.k, lean["slot_offsets"], L.weights, out=y1)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)
    ws = [wl.expert_weights(cfg, int(e)) for e in plan["slot_expert"]]
    o_p = oracle.permute(r["idx"].cpu().numpy(), plan["rep_off"], plan["rep_slot"], plan["rep_weight"],
                         plan["num_slots"], L.x)
    ref = oracle.grouped_ffn(o_p["xp"], o_p["slot_offsets"], [w[0] for w in ws], [w[1] for w in ws])
    assert G.rel_err(G.f64_of(y1)[:nl], ref) < G.BF16_RTOL


def test_largest_slot_and_expert_counts(oracle, probe, G):
    """The limits of the build at once: 256 experts, top-8, 1024 weight slots (four local copies of every
    expert with unequal shares).  Permute is checked completely, the FFN on a row sample from every slot."""
    E, k, T, H, F, S = 256, 8, 2048, 64, 64, 1024
    cfg = wl.small_config(T=T, H=H, E=E, k=k, F=F, E_loc=E, n_rep=0, zipf_s=1.0, chunk=0, ep=1, cid=95)
    L, r = _layer(G, probe, cfg)
    rep_off = np.arange(0, 4 * E + 1, 4, dtype=np.int32)
    rng = np.random.default_rng(95)
    rep_slot = rng.permutation(S).astype(np.int32)                  # copies of an expert sit in scattered slots
    rep_weight = rng.integers(0, 4, size=S).astype(np.int32)
    rep_weight[::4] = np.maximum(rep_weight[::4], 1)                # every expert keeps a positive share
    slot_expert = np.empty(S, np.int32)
    slot_expert[rep_slot] = np.repeat(np.arange(E, dtype=np.int32), 4)
    plan = probe.Plan(rep_off, rep_slot, rep_weight, S)
    p = probe.permute(r["idx"], plan, L.d_x)
    torch.cuda.synchronize()
    idx = r["idx"].cpu().numpy()
    o = oracle.permute(idx, rep_off, rep_slot, rep_weight, S, L.x)
    for key in ("slot_counts", "slot_offsets", "pair_row"):
        np.testing.assert_array_equal(p[key].cpu().numpy(), o[key])
    nl = int(o["n_local"])
    assert int(p["n_local"].item()) == nl == T * k
    np.testing.assert_array_equal(p["row_pair"].cpu().numpy()[:nl], o["row_pair"][:nl])
    np.testing.assert_array_equal(G.bits_of(p["xp"][:nl]), o["xp"][:nl])
    ws = wl.expert_weights_many(cfg, list(range(E)))
    d_w = [(G.dev_bf16(a), G.dev_bf16(b)) for a, b in ws]
    tab = probe.WeightTable([d_w[e][0] for e in slot_expert], [d_w[e][1] for e in slot_expert])
    y = probe.grouped_ffn(p["xp"], p["slot_offsets"], tab)
    torch.cuda.synchronize()
    so = o["slot_offsets"]
    rows = np.unique(np.concatenate([so[:-1][np.diff(so) > 0], so[1:][np.diff(so) > 0] - 1,
                                     rng.choice(nl, 512, replace=False)])).astype(np.int32)
    ref = oracle.grouped_ffn(o["xp"], so, [ws[e][0] for e in slot_expert], [ws[e][1] for e in slot_expert], rows=rows)
    got = G.f64_of(y[torch.from_numpy(rows.astype(np.int64)).cuda()])
    assert G.rel_err(got, ref) < G.BF16_RTOL
    assert (np.diff(so) == 0).any() and (np.diff(so) > 64).any()    # empty slots and slots of several tiles' worth


def test_more_tokens_than_one_pass_of_any_grid(oracle, probe, G):
    """140001 tokens: the top-k kernel's grid covers 131072 tokens per pass and wraps, permute walks 274 blocks
    of pairs, the FFN table holds hundreds of tiles.  Routing and permutation are checked completely, the
    floating-point stages on samples."""
    cfg = wl.small_config(T=140001, H=64, E=16, k=2, F=64, E_loc=8, n_rep=2, zipf_s=1.1, chunk=0, ep=2, cid=96)
    print("case many tokens", flush=True)
    res = G.run_layer_parity(oracle, probe, cfg, batch=0, route_sample=None, ffn_sample=64, seed=96)
    assert res["n_local"] > 100000


def test_graph_replay_of_the_variant_entry_points(oracle, probe, G):
    """The planner, the dispatch plan, the group-limited gate, permute without the row copy, the FFN with rows
    gathered on load and the combine with a shared expert record into one HIP graph; every replay, with eager
    work in between, reproduces the eager results bit for bit."""
    print("case graph replay, variants", flush=True)
    cfg = wl.small_config(T=384, H=128, E=32, k=4, F=128, E_loc=8, n_rep=0, ep=4, chunk=0, cid=98)
    T, H, E, k, F, R, E_loc = cfg.T, cfg.H, cfg.E, cfg.k, cfg.F, 4, 8
    L = G.Layer(cfg, 0)
    rng = np.random.default_rng(98)
    nh = torch.from_numpy(rng.poisson(60, size=(R, E)).astype(np.int32)).cuda()
    nh[:, 3] *= 6                                                  # a hot expert, so that the planner moves something
    sb = torch.from_numpy((rng.standard_normal(E) * 0.05).astype(np.float32)).cuda()
    kw = dict(max_replicas=2, budget=2, k_max=8, n0=16, g_num=1, g_den=2)
    S = E_loc + 2
    ws = wl.expert_weights_many(cfg, list(range(E)))
    d_w = [(G.dev_bf16(a), G.dev_bf16(b)) for a, b in ws]
    shared_tab = probe.WeightTable([d_w[0][0]], [d_w[0][1]])
    so_shared = torch.tensor([0, T], dtype=torch.int32, device="cuda")
    res = {}

    def step():
        g = probe.plan_greedy(nh, E_loc, rank=0, want_assignment=True, **kw)
        d = probe.plan_dispatch(g["n"], g["delta_in"], E_loc, 0)
        r = probe.route_grouped(L.d_x, L.d_wg, None, None, sb, scoring="sigmoid", n_group=4, topk_group=2, group_top=2,
                                k=k, renormalize=True, routed_scale=2.5)
        p = probe.permute(r["idx"], g["plan"], L.d_x, copy_rows=False)
        res.update(g=g, d=d, r=r, p=p)
        return g, d, r, p

    # the weight table follows the planner's slot_expert, which is fixed for a fixed n_hat: build it once, eagerly
    g0, _, _, _ = step()
    torch.cuda.synchronize()
    se = g0["slot_expert"].cpu().numpy()
    assert (se[E_loc:] >= 0).any()
    tab = probe.WeightTable([d_w[max(int(e), 0)][0] for e in se], [d_w[max(int(e), 0)][1] for e in se])

    def full():
        g, d, r, p = step()
        y = probe.grouped_ffn_gather(L.d_x, p["row_pair"], k, p["slot_offsets"], tab)
        shared = probe.grouped_ffn(L.d_x, so_shared, shared_tab)
        y0 = torch.where(torch.arange(y.shape[0], device="cuda")[:, None] < p["n_local"], y, torch.zeros_like(y))
        out = probe.combine_shared(y0, p["pair_row"], r["w"], shared, 1.0)
        res.update(out=out, y0=y0)

    full()
    torch.cuda.synchronize()
    ref = dict(out=res["out"].clone(), idx=res["r"]["idx"].clone(), rows=res["p"]["pair_row"].clone(),
               rep_w=res["g"]["rep_weight"].clone(), dslot=res["d"]["rep_slot"].clone(), y0=res["y0"].clone())
    assert (ref["rows"] >= 0).any() and ref["out"].float().abs().sum() > 0
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            full()
    torch.cuda.synchronize()
    cap = dict(out=res["out"], idx=res["r"]["idx"], rows=res["p"]["pair_row"], rep_w=res["g"]["rep_weight"],
               dslot=res["d"]["rep_slot"], y0=res["y0"])
    used = int(res["g"]["rep_off"][-1])
    for i in range(3):
        for t in cap.values():
            t.zero_()                        # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(cap["idx"], ref["idx"]) and torch.equal(cap["rows"], ref["rows"]), i
        assert torch.equal(cap["rep_w"][:used], ref["rep_w"][:used]) and torch.equal(cap["dslot"][:used], ref["dslot"][:used]), i
        assert torch.equal(cap["y0"], ref["y0"]) and torch.equal(cap["out"], ref["out"]), i
