"""probe_pack_gate + the *_packed router / predictor calls against the calls that split the fp32 gate
themselves: same kernels on the same planes, so every output must agree bit for bit."""
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


def _inputs(seed, T, H, E, groups):
    rng = np.random.default_rng(seed)
    x = torch.from_numpy(wl.f32_to_bf16_bits(rng.standard_normal((T, H), dtype=np.float32)).view(np.int16)).cuda()
    x = x.view(torch.bfloat16)
    wg = torch.from_numpy(rng.standard_normal((E, H), dtype=np.float32) * np.float32(0.05)).cuda()
    wn = torch.from_numpy(rng.standard_normal((E, H), dtype=np.float32) * np.float32(0.05)).cuda()
    b = torch.from_numpy(rng.standard_normal((groups, E)).astype(np.float32)).cuda()
    return x, wg, wn, b


def _same(a, b, names=("idx", "w", "probs", "counts")):
    for n in names:
        assert torch.equal(a[n], b[n]), n


SHAPES = [(8192, 512, 256, 8), (300, 128, 64, 4), (128, 4096, 128, 8), (150, 72, 20, 3), (2100, 256, 130, 6)]


@pytest.mark.parametrize("T,H,E,k", SHAPES)
def test_packed_router_and_predictor_are_bitwise_the_unpacked_ones(probe, T, H, E, k):
    print("case packed T=%d H=%d E=%d k=%d" % (T, H, E, k), flush=True)
    x, wg, wn, b = _inputs(T + E, T, H, E, 3)
    tpg = max(T // 3, 1)
    pg = probe.PackedGate(wg)
    # the planes carry the fp32 weight exactly: hi + mid + lo == w
    pl = pg.planes.float()
    assert torch.equal(pl[0] + pl[1] + pl[2], wg)
    for renorm in (True, False):
        _same(probe.route_topk(x, wg, b, tpg, k, renorm, want_probs=True),
              probe.route_topk(x, pg, b, tpg, k, renorm, want_probs=True))
    _same(probe.predict_topk(x, wg, b, tpg, k, True, want_probs=True),
          probe.predict_topk(x, pg, b, tpg, k, True, want_probs=True))
    # counts start from zero on every call, also when the output buffer holds the previous call's counts
    out = probe.route_topk(x, pg, b, tpg, k, True)
    again = probe.route_topk(x, pg, b, tpg, k, True, out=out)
    assert int(again["counts"].sum().item()) == T * k
    # fused router + next layer's predictor on one stack of 2E rows
    r0, p0 = probe.route_predict_topk(x, wg, b, wn, b, tpg, k, True, want_probs=True)
    r1, p1 = probe.route_predict_topk(x, probe.PackedGate(wg, wn), b, None, b, tpg, k, True, want_probs=True)
    _same(r0, r1)
    _same(p0, p1)
    torch.cuda.synchronize()


def test_packed_group_limited_gate(probe):
    T, H, E, k = 1000, 256, 256, 8
    x, wg, _, b = _inputs(3, T, H, E, 1)
    sb = torch.from_numpy(np.random.default_rng(4).standard_normal(E).astype(np.float32) * 0.01).cuda()
    kw = dict(scoring="sigmoid", n_group=8, topk_group=4, group_top=2, k=k, renormalize=True, routed_scale=2.5,
              want_scores=True)
    a = probe.route_grouped(x, wg, b, T, sb, **kw)
    c = probe.route_grouped(x, probe.PackedGate(wg), b, T, sb, **kw)
    _same(a, c, ("idx", "w", "scores", "counts"))


def test_packed_empty_batch_clears_the_counts(probe):
    H, E, k = 64, 8, 2
    x, wg, _, b = _inputs(5, 4, H, E, 1)
    out = dict(counts=torch.full((E,), 9, dtype=torch.int32, device="cuda"))
    r = probe.route_topk(x[:0], probe.PackedGate(wg), b, 1, k, True, out=out)
    assert int(r["counts"].abs().sum().item()) == 0
