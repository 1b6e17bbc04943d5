"""Host-side logic that needs neither the GPU nor the oracle: the seeded input generators and the
plan recipe of workload.py, and the command-line contract of bench.py."""
import os
import subprocess
import sys

import numpy as np
import pytest

from paper_2602_00509_amd import workload as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "one-GPU" in r.stderr and r.stdout.strip() == ""


def test_generators_are_seeded_and_shaped():
    cfg = wl.small_config(T=37, H=64, E=12, k=3, F=64, E_loc=4, n_rep=2, ep=3, chunk=16, cid=77)
    for fn, args in ((wl.activations, (cfg, 1)), (wl.gate_weights, (cfg, 0)), (wl.zipf_bias, (cfg, 1, 0))):
        a, b = fn(*args), fn(*args)
        assert a.dtype == b.dtype and np.array_equal(a, b)
    assert wl.activations(cfg, 0).shape == (37, 64) and wl.activations(cfg, 0).dtype == np.uint16
    assert not np.array_equal(wl.activations(cfg, 0), wl.activations(cfg, 1))
    assert wl.gate_weights(cfg).shape == (12, 64) and wl.gate_weights(cfg).dtype == np.float32
    w13, w2 = wl.expert_weights(cfg, 5)
    assert w13.shape == (128, 64) and w2.shape == (64, 64) and w13.dtype == np.uint16
    a, _ = wl.expert_weights(cfg, 5, copy=1)
    assert np.array_equal(a, w13)                        # a replica holds a copy of the same expert


def test_zipf_bias_is_minus_s_log_rank_of_a_permutation():
    for cid in (1, 2, 3, 5, 7):
        cfg = wl.CONFIGS[cid]
        b = wl.zipf_bias(cfg, 1, 0).astype(np.float64)
        assert b.shape == (cfg.G, cfg.E)
        for g in range(min(cfg.G, 3)):
            rank = np.exp(-b[g] / cfg.zipf_s)
            np.testing.assert_allclose(np.sort(rank), np.arange(1, cfg.E + 1), rtol=1e-5)
    # the rotating configurations move one base order by E_loc experts per batch
    cfg = wl.CONFIGS[3]
    order = lambda batch: np.argsort(-wl.zipf_bias(cfg, batch, 0)[0], kind="stable")    # most popular expert first
    np.testing.assert_array_equal(order(2), np.roll(order(0), 2 * cfg.E_loc))


def test_bf16_rounding_helpers():
    # bf16 keeps 8 significand bits: the spacing at 1 is 2^-7
    x = np.array([1.0, 1.0 + 2.0 ** -7, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -2.5, 0.0, 3.0e38], np.float32)
    bits = wl.f32_to_bf16_bits(x)
    back = wl.bf16_bits_to_f32(bits)
    # ties to even: 1 + 2^-8 lies halfway between 1 and 1 + 2^-7 -> 1; 1 + 3*2^-8 -> 1 + 2^-6
    np.testing.assert_array_equal(back[:5], np.array([1.0, 1.0078125, 1.0, 1.015625, -2.5], np.float32))
    assert back[5] == 0.0 and np.isfinite(back[6])
    np.testing.assert_array_equal(wl.f32_to_bf16_bits(back), bits)      # idempotent


@pytest.mark.parametrize("cid", sorted(wl.CONFIGS))
def test_plan_recipe_is_a_valid_plan(cid):
    cfg = wl.CONFIGS[cid]
    rng = np.random.default_rng(cid)
    counts = rng.integers(0, 1000, size=cfg.E)
    p = wl.build_plan(cfg, counts)
    E, S = cfg.E, cfg.S
    assert p["num_slots"] == S and p["slot_expert"].shape == (S,)
    off, slot, wgt = p["rep_off"], p["rep_slot"], p["rep_weight"]
    assert off[0] == 0 and (np.diff(off) >= 1).all() and off[-1] == len(slot) == len(wgt)
    local = slot[slot >= 0]
    assert len(set(local.tolist())) == len(local) and (local < S).all()      # a slot holds one replica
    for e in range(E):
        w = wgt[off[e]:off[e + 1]]
        assert (w >= 0).all() and w.sum() >= 1
        for i in range(off[e], off[e + 1]):
            if slot[i] >= 0:
                assert p["slot_expert"][slot[i]] == e
    # native experts stay in their own slot; replicas go to the most loaded other experts
    for e in range(cfg.E_loc):
        assert e in slot[off[e]:off[e + 1]]
    assert len(local) <= S
    q = wl.no_replica_plan(cfg)
    assert (q["rep_weight"] == 1).all() and (np.diff(q["rep_off"]) == 1).all()
