"""Helpers shared by the GPU parity tests: tensor marshalling, error metrics, and one function
that runs a whole layer through libprobe and checks every stage against the CPU oracle."""
from __future__ import annotations

import numpy as np
import torch

from paper_2602_00509_amd import workload as wl

TAU = 1e-5          # logit gap below which a token's top-k order is declared ambiguous (the gate's fp32 logits
                    # are within a few 1e-6 of the fp64 ones: exact bf16 x bf16 products, fp32 accumulation)
PROB_ATOL = 1e-5    # gate probabilities / weights, absolute
BF16_RTOL = 2e-2    # bf16 outputs: max |g-o| / (|o| + rms(o))


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def bits_of(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def f64_of(t: torch.Tensor) -> np.ndarray:
    return wl.bf16_bits_to_f32(bits_of(t)).astype(np.float64)


def rel_err(g: np.ndarray, o: np.ndarray) -> float:
    """max_i |g_i - o_i| / (|o_i| + rms(o)); plain relative error is undefined near zeros."""
    if o.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(o * o)))
    if rms == 0.0:
        return float(np.abs(g - o).max())
    return float((np.abs(g - o) / (np.abs(o) + rms)).max())


def rel_err_rows(g: np.ndarray, o: np.ndarray) -> float:
    """max over rows t and elements i of |g_ti - o_ti| / (|o_ti| + rms(o_t)): the same metric with the scale taken
    per row, for tensors whose rows differ in scale by construction (a layer-output row scales with the gate-weight
    mass of the token's local pairs, which without renormalisation spans more than an order of magnitude)."""
    if o.size == 0:
        return 0.0
    rms = np.sqrt(np.mean(o * o, axis=1, keepdims=True))
    den = np.abs(o) + rms
    err = np.abs(g - o)
    return float(np.where(den > 0, err / np.where(den > 0, den, 1.0), err).max())


def ambiguous_tokens(logits: np.ndarray, k: int) -> np.ndarray:
    """Tokens whose k+1 largest logits contain an adjacent gap below TAU."""
    E = logits.shape[1]
    top = -np.sort(-logits, axis=1)[:, :min(k + 1, E)]
    return (np.abs(np.diff(top, axis=1)) < TAU).any(axis=1)


def check_route(gpu: dict, ora: dict, k: int, renormalize: bool, tokens=None):
    """gpu: tensors from probe.route_topk; ora: oracle dict (possibly for a token subset)."""
    sel = slice(None) if tokens is None else tokens
    g_idx = gpu["idx"].cpu().numpy()[sel]
    g_w = gpu["w"].cpu().numpy()[sel].astype(np.float64)
    amb = ambiguous_tokens(ora["logits"], k)
    clear = ~amb
    # bit-exact indices wherever the oracle's order is unambiguous
    np.testing.assert_array_equal(g_idx[clear], ora["idx"][clear])
    np.testing.assert_allclose(g_w[clear], ora["w"][clear], rtol=0, atol=PROB_ATOL)
    # ambiguous tokens: the chosen set must still be a valid top-k within TAU
    for t in np.nonzero(amb)[0]:
        lg = ora["logits"][t]
        kth = np.sort(lg)[-k]
        chosen = g_idx[t]
        assert len(set(chosen.tolist())) == k
        assert (lg[chosen] >= kth - TAU).all()
        must = np.nonzero(lg > kth + TAU)[0]
        assert set(must.tolist()) <= set(chosen.tolist())
        assert (np.diff(lg[chosen]) <= TAU).all()          # descending up to TAU
    if "probs" in gpu and gpu["probs"] is not None:
        g_p = gpu["probs"].cpu().numpy()[sel].astype(np.float64)
        np.testing.assert_allclose(g_p, ora["probs"], rtol=0, atol=PROB_ATOL)
        if not renormalize:
            np.testing.assert_array_equal(np.take_along_axis(g_p, g_idx.astype(np.int64), 1), g_w)
    return int(amb.sum())


def gather_bias(bias, tpg, tokens):
    """Bias rows for a token subset, for an oracle call with tokens_per_group = 1."""
    if bias is None:
        return None
    g = np.minimum(np.asarray(tokens) // tpg, bias.shape[0] - 1)
    return np.ascontiguousarray(bias[g])


class Layer:
    """Device copies of one configuration's inputs plus the host originals."""

    def __init__(self, cfg, batch=0, plan=None, threads=8):
        self.cfg, self.batch = cfg, batch
        self.x = wl.activations(cfg, batch)
        self.wg = wl.gate_weights(cfg, 0)
        self.bias = wl.zipf_bias(cfg, batch, 0)
        self.tpg = wl.tokens_per_group(cfg)
        self.d_x = dev_bf16(self.x)
        self.d_wg = torch.from_numpy(self.wg).cuda()
        self.d_bias = torch.from_numpy(self.bias).cuda()
        self.plan = plan
        self.threads = threads
        self.weights = None

    def load_weights(self, slot_expert, probe):
        ew = wl.expert_weights_many(self.cfg, slot_expert, threads=self.threads)
        self.w13 = [w[0] for w in ew]
        self.w2 = [w[1] for w in ew]
        self.weights = probe.WeightTable([dev_bf16(w) for w in self.w13], [dev_bf16(w) for w in self.w2])


def run_layer_parity(oracle, probe, cfg, batch=0, plan_fn=None, route_sample=None, ffn_sample=None,
                     renormalize=True, seed=0, report=None):
    """Route -> permute -> FFN -> combine on the GPU, every stage checked against the oracle.

    route_sample / ffn_sample: number of tokens / rows the oracle evaluates (None = all)."""
    rng = np.random.default_rng(seed)
    L = Layer(cfg, batch)
    T, H, E, k = cfg.T, cfg.H, cfg.E, cfg.k
    torch.cuda.synchronize()

    # ---- route
    g_r = probe.route_topk(L.d_x, L.d_wg, L.d_bias, L.tpg, k, renormalize, want_probs=True)
    torch.cuda.synchronize()
    g_idx = g_r["idx"].cpu().numpy()
    if route_sample is None or route_sample >= T:
        o_r = oracle.route_topk(L.x, L.wg, L.bias, L.tpg, k, renormalize)
        n_amb = check_route(g_r, o_r, k, renormalize)
        if n_amb == 0 or (g_idx == o_r["idx"]).all():
            np.testing.assert_array_equal(g_r["counts"].cpu().numpy(), o_r["counts"])
    else:
        tok = np.sort(rng.choice(T, size=route_sample, replace=False))
        o_r = oracle.route_topk(L.x[tok], L.wg, gather_bias(L.bias, L.tpg, tok), 1, k, renormalize)
        n_amb = check_route(g_r, o_r, k, renormalize, tokens=tok)
    # counts are the histogram of the GPU's own indices, always
    np.testing.assert_array_equal(g_r["counts"].cpu().numpy(), np.bincount(g_idx.ravel(), minlength=E))
    srt = np.sort(g_idx, axis=1)
    assert (srt[:, 1:] != srt[:, :-1]).all()          # k distinct experts per token

    # ---- plan (input recipe) from the routed counts, then permute
    counts = np.bincount(g_idx.ravel(), minlength=E)
    plan = plan_fn(cfg, counts) if plan_fn else wl.build_plan(cfg, counts)
    d_plan = probe.Plan(plan["rep_off"], plan["rep_slot"], plan["rep_weight"], plan["num_slots"])
    g_p = probe.permute(g_r["idx"], d_plan, L.d_x)
    torch.cuda.synchronize()
    o_p = oracle.permute(g_idx, plan["rep_off"], plan["rep_slot"], plan["rep_weight"], plan["num_slots"], L.x)
    nl = o_p["n_local"]
    assert int(g_p["n_local"].item()) == nl
    np.testing.assert_array_equal(g_p["slot_counts"].cpu().numpy(), o_p["slot_counts"])
    np.testing.assert_array_equal(g_p["slot_offsets"].cpu().numpy(), o_p["slot_offsets"])
    np.testing.assert_array_equal(g_p["pair_row"].cpu().numpy(), o_p["pair_row"])
    np.testing.assert_array_equal(g_p["row_pair"].cpu().numpy(), o_p["row_pair"])
    np.testing.assert_array_equal(bits_of(g_p["xp"][:nl]), o_p["xp"][:nl])

    # ---- grouped FFN
    L.load_weights(plan["slot_expert"], probe)
    y = torch.full((cfg.N, H), float("nan"), dtype=torch.bfloat16, device="cuda")
    probe.grouped_ffn(g_p["xp"], g_p["slot_offsets"], L.weights, out=y)
    torch.cuda.synchronize()
    e2e_tokens = None
    if ffn_sample is None or ffn_sample >= nl:
        rows = np.arange(nl, dtype=np.int32)
    else:
        # Stratified sample: the FFN cuts a slot into row tiles whose heights are multiples of 64 counted from the
        # slot's first row, and a wave owns 32-row blocks of a tile, so one random row from every 32-row block
        # of every slot touches every (tile, wave row block) of the schedule whatever the cut.  If that is more
        # than ffn_sample rows, a random subset of the blocks is kept.  The first and last row of every
        # non-empty slot (tile edges) and every local row of a few tokens (for the layer output) are added.
        picks, edges = [], []
        for s in range(plan["num_slots"]):
            a, b = int(o_p["slot_offsets"][s]), int(o_p["slot_offsets"][s + 1])
            if b > a:
                edges += [a, b - 1]
                for blk in range(a, b, 32):
                    picks.append(int(rng.integers(blk, min(blk + 32, b))))
        picks = np.asarray(picks, np.int64)
        if picks.size > ffn_sample:
            picks = rng.choice(picks, size=ffn_sample, replace=False)
        e2e_tokens = np.sort(rng.choice(T, size=min(T, 48), replace=False))
        tok_rows = o_p["pair_row"][e2e_tokens].ravel()
        rows = np.unique(np.concatenate([np.asarray(edges, np.int64), picks, tok_rows[tok_rows >= 0]])).astype(np.int32)
    o_y = oracle.grouped_ffn(o_p["xp"], o_p["slot_offsets"], L.w13, L.w2, rows=rows)
    g_y = f64_of(y[torch.from_numpy(rows.astype(np.int64)).cuda()])
    assert np.isfinite(g_y).all()
    e_ffn = rel_err(g_y, o_y)
    assert e_ffn <= BF16_RTOL, "FFN rel err %.3e" % e_ffn
    if nl < cfg.N:                                     # rows past n_local are never written
        assert torch.isnan(y[nl:].float()).all()

    # ---- combine, fed with the GPU's own y and weights
    y_in = torch.where(torch.isnan(y), torch.zeros_like(y), y)
    out = probe.combine(y_in, g_p["pair_row"], g_r["w"])
    torch.cuda.synchronize()
    if ffn_sample is None or ffn_sample >= nl:
        toks = np.arange(T)
    else:
        toks = np.sort(rng.choice(T, size=min(T, 4 * ffn_sample), replace=False))
    o_c = oracle.combine(f64_of(y_in[:max(nl, 1)]) if nl else np.zeros((1, H)), o_p["pair_row"][toks],
                         g_r["w"].cpu().numpy().astype(np.float64)[toks])
    e_comb = rel_err(f64_of(out[torch.from_numpy(toks).cuda()]), o_c)
    assert e_comb <= 4e-3, "combine rel err %.3e" % e_comb

    # ---- end to end against the unrounded oracle chain (same routing decisions): every token when the oracle
    # computed every row, otherwise the tokens whose local rows were all added to the sample
    e_e2e = e_out = None
    o_w = o_r["w"] if (route_sample is None or route_sample >= T) and (g_idx == o_r["idx"]).all() \
        else g_r["w"].cpu().numpy().astype(np.float64)
    if e2e_tokens is None:
        e2e_tokens, y_full = np.arange(T), o_y
    else:
        y_full = np.zeros((max(nl, 1), H))
        y_full[rows] = o_y
    if nl > 0 and len(e2e_tokens):
        pr = o_p["pair_row"][e2e_tokens]
        o_out = oracle.combine(y_full, pr, o_w[e2e_tokens])
        g_out = f64_of(out[torch.from_numpy(e2e_tokens).cuda()])
        # The FFN tolerance carried through the weighted sum, element by element: a row of y may be off by
        # BF16_RTOL * (|y| + rms(y)), so out[t] may be off by sum_s w[t,s] times that, plus its own rounding.
        rms_y = float(np.sqrt(np.mean(o_y * o_y))) if o_y.size else 0.0
        scale = oracle.combine(np.abs(y_full) + rms_y, pr, np.abs(o_w[e2e_tokens]))
        tol = BF16_RTOL * scale + 2.0 ** -8 * np.abs(o_out) + 1e-30
        e_e2e = float((np.abs(g_out - o_out) / tol).max()) * BF16_RTOL
        assert e_e2e <= BF16_RTOL, "layer err %.3e of the propagated FFN tolerance" % e_e2e
        # and the plain metric on the layer output with the scale of each token's own row,
        # max |g - o| / (|o| + rms(o[t])): a row of `out` scales with the gate-weight mass of the token's local pairs
        # (zero for a token without one, and spread over more than an order of magnitude without renormalisation),
        # so one rms over the whole tensor is not the scale of any row
        e_out = rel_err_rows(g_out, o_out)
        assert e_out <= BF16_RTOL, "layer output rel err %.3e" % e_out
    res = dict(cfg=cfg.name, batch=batch, n_local=nl, ambiguous=n_amb, ffn_err=e_ffn, combine_err=e_comb,
               e2e_err=e_e2e, out_err=e_out, sampled_rows=int(len(rows)), slot_rows=o_p["slot_counts"].tolist())
    if report is not None:
        report.append(res)
    return res
