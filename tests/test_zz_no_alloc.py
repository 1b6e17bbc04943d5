"""probe_permute_static (the entry point that allocates nothing: block histograms in the library's static
device array) against probe_permute, bit for bit, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

from paper_2602_00509_amd import probe

pytestmark = pytest.mark.gpu


def _case(seed, T, H, E, k, S):
    rng = np.random.default_rng(seed)
    # skewed expert choice, k distinct experts per token
    p = 1.0 / np.arange(1, E + 1) ** 1.1
    p /= p.sum()
    idx = np.stack([rng.choice(E, size=k, replace=False, p=p) for _ in range(T)]).astype(np.int32)
    # plan: experts 0..S-3 native in slots 0..S-3, the two hottest of them get a second local slot with
    # weights 3:2 and 1:1, every other expert lives elsewhere
    rep_off, rep_slot, rep_w = [0], [], []
    for e in range(E):
        if e == 0:
            rep_slot += [0, S - 2]; rep_w += [3, 2]
        elif e == 1:
            rep_slot += [1, S - 1]; rep_w += [1, 1]
        elif e < S - 2:
            rep_slot += [e]; rep_w += [1]
        else:
            rep_slot += [-1]; rep_w += [1]
        rep_off.append(len(rep_slot))
    x = torch.randn((T, H), device="cuda").to(torch.bfloat16)
    return torch.from_numpy(idx).cuda(), probe.Plan(rep_off, rep_slot, rep_w, S), x


def _outs(T, H, k, S):
    N = T * k
    i32 = dict(dtype=torch.int32, device="cuda")
    return dict(slot_counts=torch.full((S,), -7, **i32), slot_offsets=torch.full((S + 1,), -7, **i32),
                row_pair=torch.full((N,), -7, **i32), pair_row=torch.full((T, k), -7, **i32),
                xp=torch.zeros((N, H), dtype=torch.bfloat16, device="cuda"), n_local=torch.full((1,), -7, **i32))


def _compare(idx, plan, x):
    T, k = idx.shape
    H, S = x.shape[1], plan.num_slots
    ref = probe.permute(idx, plan, x, out=_outs(T, H, k, S))
    got = probe.permute_static(idx, plan, x, out=_outs(T, H, k, S))
    torch.cuda.synchronize()
    for name in ("slot_counts", "slot_offsets", "row_pair", "pair_row", "n_local"):
        assert torch.equal(ref[name], got[name]), name
    nl = int(ref["n_local"].item())
    assert nl > 0
    assert torch.equal(ref["xp"][:nl].view(torch.int16), got["xp"][:nl].view(torch.int16))
    return nl


def test_static_scratch_permute_matches_workspace_permute_twice():
    # first call: 32 blocks of 1024 pairs in the scratch array; second call: a smaller batch (8 blocks, fewer
    # experts) that reuses the front of the same array; third: a decode-sized batch (one block, array untouched)
    big = _case(11, 4096, 256, 256, 8, 36)
    small = _case(12, 1000, 128, 64, 8, 18)
    tiny = _case(13, 100, 64, 32, 4, 10)
    n1 = _compare(*big)
    n2 = _compare(*small)
    n3 = _compare(*tiny)
    assert n1 > n2 > n3
    # and the large one again after the small ones
    assert _compare(*big) == n1


def test_static_scratch_limit_is_enforced():
    E = 256
    cap = probe.permute_static_max_pairs(E)
    assert cap == 256 * 1024 // (E * 4) * 1024
    k = 8
    T = cap // k + 1024            # one block more than the array holds
    idx = torch.zeros((T, k), dtype=torch.int32, device="cuda")
    plan = probe.Plan(list(range(E + 1)), [-1] * E, [1] * E, 4)
    x = torch.zeros((T, 8), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(probe.ProbeError) as ei:
        probe.permute_static(idx, plan, x, out=_outs(T, 8, k, 4))
    assert ei.value.code == -2 and "static" in str(ei.value)
