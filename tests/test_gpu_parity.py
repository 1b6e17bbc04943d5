"""GPU parity: libprobe (HIP, through the C ABI) against the CPU oracle, stage by stage.

Bars: integer outputs bit-exact (top-k indices wherever the oracle's order is unambiguous at
1e-5 in the logits, otherwise a valid top-k within that margin); gate probabilities and
weights within 1e-5 absolute; bf16 outputs within 2e-2 of the fp64 oracle in the metric
max |g-o| / (|o| + rms(o))."""
import json
import os

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
    p.lib()                     # raises if libprobe.so is missing: there is no fallback
    return p


@pytest.fixture(scope="module")
def G():
    import gpu_util
    return gpu_util


REPORT = []


def _flush_report():
    """Error magnitudes of every case, written where PROBE_REPORT_DIR points (if set)."""
    out = os.environ.get("PROBE_REPORT_DIR")
    if not out:
        return
    os.makedirs(out, exist_ok=True)
    with open(os.path.join(out, "parity_report.json"), "w") as f:
        json.dump(REPORT, f, indent=1, default=str)


SMALL = [
    # ragged tails everywhere: T not a multiple of 64/128, odd expert counts, several tiles
    dict(T=96, H=128, E=16, k=4, F=192, E_loc=4, n_rep=2, ep=4, chunk=32),
    dict(T=333, H=256, E=10, k=3, F=320, E_loc=10, n_rep=2, ep=1, chunk=0),
    dict(T=1, H=64, E=8, k=1, F=64, E_loc=8, n_rep=1, ep=1, chunk=0),
    dict(T=700, H=192, E=200, k=8, F=128, E_loc=50, n_rep=3, ep=4, chunk=128),
    dict(T=1100, H=64, E=3, k=2, F=64, E_loc=3, n_rep=1, ep=1, chunk=0),     # slots of > 128 rows
    dict(T=257, H=512, E=256, k=8, F=448, E_loc=32, n_rep=4, ep=8, chunk=0),
]


@pytest.mark.parametrize("i", range(len(SMALL)))
@pytest.mark.parametrize("renorm", [True, False])
def test_small_layers(oracle, probe, G, i, renorm):
    cfg = wl.small_config(cid=90 + i, **SMALL[i])
    print("case small", i, SMALL[i], "renorm", renorm, flush=True)
    G.run_layer_parity(oracle, probe, cfg, batch=0, renormalize=renorm, seed=i, report=REPORT)
    _flush_report()


@pytest.mark.parametrize("cid,batch", [(1, 0), (1, 1), (4, 0), (4, 3)])
def test_full_configs_every_element(oracle, probe, G, cid, batch):
    """Configurations small enough for the oracle to compute every output element."""
    print("case full", cid, batch, flush=True)
    G.run_layer_parity(oracle, probe, wl.CONFIGS[cid], batch=batch, seed=cid, report=REPORT)
    _flush_report()


@pytest.mark.parametrize("cid,batch", [(2, 0), (3, 0), (3, 5), (5, 0)])
def test_full_configs_sampled(oracle, probe, G, cid, batch):
    """Full benchmark sizes: integer stages and the router (every token) checked completely; the FFN on a
    stratified sample of about a thousand rows that reaches every row tile and every 32-row block of it, the
    layer output on the tokens whose rows are all in the sample."""
    print("case sampled", cid, batch, flush=True)
    G.run_layer_parity(oracle, probe, wl.CONFIGS[cid], batch=batch, route_sample=None,
                       ffn_sample=320 if cid == 2 else 1024, seed=cid, report=REPORT)
    _flush_report()


# The two models the paper evaluates (Sec. 5): GPT-OSS-120B-shaped (128 experts, top-4, hidden and FFN width
# 2880, neither a multiple of 256) and Qwen3-MoE-235B-shaped (128 experts, top-8, hidden 4096, FFN width
# 1536), one rank's share at ep = 8 with two replica slots, a 2048-token prefill chunk.  Shapes only: the
# gate is the renormalised softmax top-k (the GPT-OSS form, softmax over the chosen logits, equals it).
PAPER_MODELS = [
    dict(T=2048, H=2880, E=128, k=4, F=2880, E_loc=16, n_rep=2, ep=8, chunk=0),
    dict(T=2048, H=4096, E=128, k=8, F=1536, E_loc=16, n_rep=2, ep=8, chunk=0),
]


@pytest.mark.parametrize("i", range(len(PAPER_MODELS)))
def test_shapes_of_the_models_the_paper_evaluates(oracle, probe, G, i):
    cfg = wl.small_config(cid=300 + i, **PAPER_MODELS[i])
    print("case paper model shape", i, PAPER_MODELS[i], flush=True)
    G.run_layer_parity(oracle, probe, cfg, batch=0, route_sample=256, ffn_sample=32, seed=300 + i, report=REPORT)
    _flush_report()

