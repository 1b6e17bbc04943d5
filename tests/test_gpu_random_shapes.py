"""Randomised shapes and plans through the whole layer on the GPU, every stage against the oracle.

Shapes are drawn from a seeded generator: token counts around tile and wave boundaries, hidden and FFN
widths that are and are not multiples of 256, expert counts from 2 to 200, any top-k up to 8, and plans
with several replicas per expert, zero weights, remote copies and empty slots."""
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


def random_plan(rng, E, max_slots):
    """A random valid plan: every expert gets 1-3 replicas, each local (a fresh slot) or remote, with
    weights 0-5 (at least one positive); some slots stay empty."""
    rep_off, rep_slot, rep_weight, slot_expert = [0], [], [], []
    p_local = min(0.6, 0.75 * max_slots / E)             # spread the local slots over all experts
    for e in range(E):
        n = int(rng.integers(1, 4))
        w = rng.integers(0, 6, size=n)
        if w.sum() == 0:
            w[int(rng.integers(0, n))] = int(rng.integers(1, 6))
        for i in range(n):
            local = rng.random() < p_local and len(slot_expert) < max_slots
            if local:
                rep_slot.append(len(slot_expert))
                slot_expert.append(e)
            else:
                rep_slot.append(-1)
            rep_weight.append(int(w[i]))
        rep_off.append(len(rep_slot))
    if not slot_expert:                                   # at least one local slot
        rep_slot[0] = 0
        slot_expert.append(0)
    spare = int(rng.integers(0, 3))                       # slots that hold weights but get no token
    for _ in range(spare):
        slot_expert.append(int(rng.integers(0, E)))
    return dict(rep_off=np.asarray(rep_off, np.int32), rep_slot=np.asarray(rep_slot, np.int32),
                rep_weight=np.asarray(rep_weight, np.int32), num_slots=len(slot_expert),
                slot_expert=np.asarray(slot_expert, np.int32))


def _cases():
    rng = np.random.default_rng(20260127)
    out = []
    for i in range(14):
        T = int(rng.choice([1, 2, 31, 63, 64, 65, 127, 129, 255, 257, 300, 511, 640, 1023, 1025, 1500]))
        H = int(rng.choice([64, 128, 192, 256, 320, 512]))
        F = int(rng.choice([64, 128, 192, 256, 448]))
        E = int(rng.choice([2, 3, 5, 8, 17, 40, 64, 130, 200]))
        k = int(rng.integers(1, min(8, E) + 1))
        out.append((i, T, H, E, k, F, 1.0, 0, 24))
    # a second, wider draw: one expert, the largest expert counts, strong and no skew, bias groups inside the
    # call, one to sixty local slots
    for i in range(14, 40):
        T = int(rng.choice([1, 3, 17, 64, 65, 100, 128, 129, 255, 256, 257, 383, 512, 513, 700, 1024, 1300, 2049]))
        H = int(rng.choice([64, 128, 192, 256, 320, 448, 512, 704]))
        F = int(rng.choice([64, 128, 192, 256, 320, 448, 576]))
        E = int(rng.choice([1, 2, 3, 4, 7, 8, 16, 33, 64, 100, 128, 129, 255, 256]))
        k = int(rng.integers(1, min(8, E) + 1))
        out.append((i, T, H, E, k, F, float(rng.choice([0.0, 1.0, 2.0])), int(rng.choice([0, 0, 64])),
                    int(rng.choice([1, 4, 24, 60]))))
    return out


@pytest.mark.parametrize("case,T,H,E,k,F,zipf_s,chunk,max_slots", _cases())
def test_random_shape_and_plan(oracle, probe, G, case, T, H, E, k, F, zipf_s, chunk, max_slots):
    print("case random %d: T=%d H=%d E=%d k=%d F=%d zipf=%.1f chunk=%d slots<=%d" % (case, T, H, E, k, F, zipf_s, chunk,
                                                                                    max_slots), flush=True)
    cfg = wl.small_config(T=T, H=H, E=E, k=k, F=F, E_loc=min(E, 4), n_rep=0, zipf_s=zipf_s, chunk=chunk, ep=1,
                          cid=200 + case)
    rng = np.random.default_rng(case)
    plan = random_plan(rng, E, max_slots=max_slots)
    res = G.run_layer_parity(oracle, probe, cfg, batch=0, plan_fn=lambda c, counts: plan, renormalize=bool(case % 2))
    assert res["n_local"] <= T * k


@pytest.mark.parametrize("case,T,H,E,k,F,max_slots", [(0, 6001, 256, 8, 6, 1024, 24), (1, 8192, 320, 16, 8, 512, 60),
                                                       (2, 4096, 512, 4, 3, 1536, 4)])
def test_every_element_on_the_work_queue_path(oracle, probe, G, case, T, H, E, k, F, max_slots):
    """Mid-size layers with tens of thousands of local rows: the FFN runs as the persistent launch (more work items
    than CUs, tickets drawn from the per-XCD counters, stealing at the end) and EVERY element of h's consumer y and of
    the layer output is compared with the oracle, not a sample."""
    print("case queue %d: T=%d H=%d E=%d k=%d F=%d slots<=%d" % (case, T, H, E, k, F, max_slots), flush=True)
    cfg = wl.small_config(T=T, H=H, E=E, k=k, F=F, E_loc=min(E, 4), n_rep=0, zipf_s=1.0, chunk=0, ep=1,
                          cid=400 + case)
    plan = random_plan(np.random.default_rng(9000 + case), E, max_slots=max_slots)
    res = G.run_layer_parity(oracle, probe, cfg, batch=0, plan_fn=lambda c, counts: plan, renormalize=True)
    assert res["sampled_rows"] == res["n_local"] and res["n_local"] >= 4096
