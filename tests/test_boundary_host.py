"""Host-side checks of the C-ABI boundary that need no GPU: the library loads, exports every
symbol the header declares, sizes its workspaces, and rejects bad arguments before launching
anything.  No compute call is made here."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "probe.h")


@pytest.fixture(scope="module")
def L():
    from paper_2602_00509_amd import probe, build
    if not os.path.exists(probe.LIB_PATH):
        build.build()
    return probe.lib()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(probe_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_functions()
    for must in ("probe_route_topk", "probe_predict_topk", "probe_permute", "probe_grouped_ffn",
                 "probe_combine", "probe_last_error_string", "probe_version"):
        assert must in names
    for n in names:
        assert hasattr(L, n), "libprobe.so does not export %s" % n
    assert L.probe_version().decode()


def test_workspace_sizes(L):
    from paper_2602_00509_amd import probe
    # route: three bf16 planes of the gate plus split-K partial logits
    assert probe.route_topk_workspace_bytes(8192, 7168, 256, 8) >= 3 * 256 * 7168 * 2 + 8192 * 256 * 4
    assert probe.route_topk_workspace_bytes(0, 64, 8, 2) > 0
    assert probe.permute_workspace_bytes(8192, 256, 8, 36) >= 256 * 4
    # ffn: the intermediate activation h [max_rows, F] in bf16
    assert probe.grouped_ffn_workspace_bytes(36, 7168, 2048, 65536) >= 65536 * 2048 * 2


def test_bad_arguments_are_rejected_without_a_launch(L):
    from paper_2602_00509_amd.probe import _Plan
    err = lambda: L.probe_last_error_string().decode()
    fake = C.c_void_p(0x1000)          # aligned, never dereferenced: validation fails first
    odd = C.c_void_p(0x1008)
    big = C.c_size_t(1 << 40)
    # combine
    assert L.probe_combine(None, None, None, 4, 64, 2, None, None) == -1 and "null" in err()
    assert L.probe_combine(fake, fake, fake, 4, 60, 2, fake, None) == -2
    assert L.probe_combine(fake, fake, fake, 4, 64, 9, fake, None) == -2
    assert L.probe_combine(odd, fake, fake, 4, 64, 2, fake, None) == -3
    assert L.probe_combine(fake, fake, fake, -1, 64, 2, fake, None) == -1
    assert L.probe_combine(None, None, None, 0, 64, 2, None, None) == 0          # empty batch is legal
    assert L.probe_combine_shared(fake, fake, fake, None, 1.0, 4, 64, 2, fake, None) == -1   # shared output missing
    assert L.probe_combine_shared(fake, fake, fake, odd, 1.0, 4, 64, 2, fake, None) == -3
    assert L.probe_combine_shared(fake, fake, fake, fake, 1.0, 4, 60, 2, fake, None) == -2
    # route / predict
    for fn in (L.probe_route_topk, L.probe_predict_topk):
        assert fn(fake, fake, None, 1, 1, 16, 64, 8, 9, 1, fake, fake, None, None, fake, big, None) == -1   # k > E
        assert fn(fake, fake, None, 1, 1, 16, 64, 300, 2, 1, fake, fake, None, None, fake, big, None) == -2  # E > 256
        assert fn(fake, fake, None, 1, 1, 16, 60, 8, 2, 1, fake, fake, None, None, fake, big, None) == -2    # H % 8
        assert fn(odd, fake, None, 1, 1, 16, 64, 8, 2, 1, fake, fake, None, None, fake, big, None) == -3
        assert fn(fake, fake, None, 1, 1, 16, 64, 8, 2, 1, fake, fake, None, None, fake, C.c_size_t(16), None) == -4
        assert fn(fake, fake, fake, 0, 1, 16, 64, 8, 2, 1, fake, fake, None, None, fake, big, None) == -1    # G < 1
        assert "probe_" in err()
    # predictor with its residual MLP
    pr = L.probe_predict_topk_residual
    ok_tail = (16, 64, 8, 2, 1, fake, fake, None, None, fake, big, None)
    assert pr(fake, fake, None, 1, 1, fake, fake, 0, *ok_tail) == -1                  # D <= 0
    assert pr(fake, fake, None, 1, 1, None, fake, 16, *ok_tail) == -1                 # w1_hat NULL
    assert pr(fake, fake, None, 1, 1, fake, fake, 12, *ok_tail) == -2                 # D % 8
    assert pr(fake, fake, None, 1, 1, fake, fake, 2048, *ok_tail) == -2               # D > 1024
    assert pr(fake, fake, None, 1, 1, odd, fake, 16, *ok_tail) == -3
    assert pr(fake, fake, None, 1, 1, fake, fake, 16, 16, 64, 8, 2, 1, fake, fake, None, None, fake,
              C.c_size_t(L.probe_route_topk_workspace_bytes(16, 64, 8, 2)), None) == -4   # needs more than the router
    assert L.probe_predict_topk_residual_workspace_bytes(16, 64, 8, 2, 16) > L.probe_route_topk_workspace_bytes(16, 64, 8, 2)
    # group-limited gate
    from paper_2602_00509_amd.probe import _Gating
    rg = lambda gt, E=64, k=4, sb=fake: L.probe_route_grouped(
        fake, fake, None, 1, 1, sb, C.byref(gt) if gt else None, 16, 64, E, k, fake, fake, None, None, fake, big, None)
    assert rg(None) == -1 and "gating" in err()
    assert rg(_Gating(2, 8, 4, 2, 1, 1.0)) == -1                         # unknown scoring
    assert rg(_Gating(1, 7, 4, 2, 1, 1.0)) == -1                         # n_group does not divide E
    assert rg(_Gating(1, 8, 9, 2, 1, 1.0)) == -1                         # topk_group > n_group
    assert rg(_Gating(1, 8, 4, 9, 1, 1.0)) == -1                         # group_top > group size
    assert rg(_Gating(1, 32, 1, 1, 1, 1.0)) == -1                        # k does not fit the allowed groups
    assert rg(_Gating(1, 32, 4, 1, 1, 1.0)) == -2                        # n_group > 16
    assert rg(_Gating(1, 8, 4, 2, 1, 1.0), sb=odd) == -3
    assert rg(_Gating(1, 8, 4, 2, 1, 1.0), E=300) == -2
    # planner
    from paper_2602_00509_amd.probe import _PlannerParams
    pp = _PlannerParams(3, 3, 16, 0, 0, 0, 1)
    pg = lambda R, E, El, rank, par, ws=big, nh=fake: L.probe_plan_greedy(
        nh, R, E, El, rank, C.byref(par) if par else None, fake, fake, fake, fake, fake, fake, fake, fake, None, fake, ws, None)
    assert pg(8, 64, 8, 0, None) == -1                                   # params NULL
    assert pg(8, 64, 4, 0, pp) == -1                                     # E_loc * R < E
    assert pg(8, 64, 8, 8, pp) == -1                                     # rank out of range
    assert pg(8, 64, 8, 0, _PlannerParams(3, 3, 16, 0, 0, 0, 0)) == -1   # g_den < 1
    assert pg(32, 64, 2, 0, pp) == -2                                    # R > 16
    assert pg(8, 512, 64, 0, pp) == -2                                   # E > 256
    assert pg(8, 64, 8, 0, _PlannerParams(9, 3, 16, 0, 0, 0, 1)) == -2   # max_replicas > 8
    assert pg(8, 64, 8, 0, _PlannerParams(3, 3, 65, 0, 0, 0, 1)) == -2   # k_max > 64
    assert pg(8, 64, 8, 0, pp, nh=None) == -1
    assert pg(8, 64, 8, 0, pp, ws=C.c_size_t(64)) == -4 and "workspace" in err()
    assert L.probe_plan_greedy_workspace_bytes(8, 64) >= 64 * 8 * 8 * 4
    pd = lambda R, E, El, mr, rank, na=fake: L.probe_plan_dispatch(na, fake, R, E, El, mr, rank, fake, fake, fake, fake, fake, None)
    assert pd(8, 64, 8, 3, 8) == -1 and pd(8, 64, 4, 3, 0) == -1 and pd(8, 64, 8, 3, 0, na=None) == -1
    assert pd(32, 64, 2, 3, 0) == -2 and pd(8, 64, 8, 9, 0) == -2
    # permute
    plan = _Plan(0x1000, 0x1000, 0x1000, 4)
    args = lambda **kw: None
    assert L.probe_permute(fake, None, fake, 16, 64, 8, 2, fake, fake, fake, fake, fake, fake, fake, big, None) == -1
    assert L.probe_permute(fake, C.byref(plan), fake, 16, 60, 8, 2, fake, fake, fake, fake, fake, fake, fake, big, None) == -2
    assert L.probe_permute(fake, C.byref(plan), fake, 16, 64, 8, 2, fake, fake, fake, fake, fake, fake, fake, C.c_size_t(0), None) == -4
    bad = _Plan(0x1000, 0x1000, 0x1000, 2000)
    assert L.probe_permute(fake, C.byref(bad), fake, 16, 64, 8, 2, fake, fake, fake, fake, fake, fake, fake, big, None) == -2
    # permute without a workspace: larger batches than the static scratch array holds are refused
    assert L.probe_permute_static(fake, C.byref(plan), fake, 40000, 64, 256, 8, fake, fake, fake, fake, fake, fake, None) == -2
    assert "static" in err() and L.probe_permute_static_max_pairs(256) == 262144
    assert L.probe_permute_static(fake, None, fake, 16, 64, 8, 2, fake, fake, fake, fake, fake, fake, None) == -1
    assert L.probe_permute_static(fake, C.byref(plan), odd, 16, 64, 8, 2, fake, fake, fake, fake, fake, fake, None) == -3
    # packed gate
    assert L.probe_pack_gate_bytes(7168, 256) >= 3 * 256 * 7168 * 2
    assert L.probe_pack_gate(None, 64, 8, 8, 0, fake, None) == -1
    assert L.probe_pack_gate(fake, 64, 8, 8, 1, fake, None) == -1                    # rows past the stack
    assert L.probe_pack_gate(fake, 60, 8, 8, 0, fake, None) == -2
    assert L.probe_pack_gate(fake, 64, 8, 8, 0, odd, None) == -3
    for fn in (L.probe_route_topk_packed, L.probe_predict_topk_packed):
        assert fn(fake, None, None, 1, 1, 16, 64, 8, 2, 1, fake, fake, None, None, fake, big, None) == -1   # planes NULL
        assert fn(fake, odd, None, 1, 1, 16, 64, 8, 2, 1, fake, fake, None, None, fake, big, None) == -3
        assert fn(fake, fake, None, 1, 1, 16, 64, 8, 2, 1, fake, fake, None, None, fake, C.c_size_t(16), None) == -4
    assert L.probe_route_topk_packed_workspace_bytes(16, 64, 8, 2) < L.probe_route_topk_workspace_bytes(16, 64, 8, 2)
    # bias and probability outputs are read / written with 16-byte accesses: misaligned ones are refused
    for fn in (L.probe_route_topk, L.probe_predict_topk):
        assert fn(fake, fake, C.c_void_p(0x1004), 1, 1, 16, 64, 8, 2, 1, fake, fake, None, None, fake, big, None) == -3
        assert fn(fake, fake, None, 1, 1, 16, 64, 8, 2, 1, fake, fake, C.c_void_p(0x1004), None, fake, big, None) == -3
    # grouped ffn
    assert L.probe_grouped_ffn(fake, fake, fake, fake, 4, 100, 128, 64, fake, fake, big, None) == -2      # H % 64
    assert L.probe_grouped_ffn(fake, fake, fake, fake, 4, 128, 96, 64, fake, fake, big, None) == -2       # F % 64
    assert L.probe_grouped_ffn(fake, fake, fake, fake, 4, (1 << 21) + 64, 64, 64, fake, fake, big, None) == -2  # H > 2^21
    assert b"2^21" in L.probe_last_error_string()
    assert L.probe_grouped_ffn(fake, fake, fake, fake, 0, 128, 128, 64, fake, fake, big, None) == -1
    assert L.probe_grouped_ffn(None, fake, fake, fake, 4, 128, 128, 64, fake, fake, big, None) == -1
    assert L.probe_grouped_ffn(fake, fake, fake, fake, 4, 128, 128, 64, fake, fake, C.c_size_t(8), None) == -4
    assert L.probe_grouped_ffn(fake, fake, fake, fake, 4, 128, 128, 0, fake, None, C.c_size_t(0), None) == 0  # no rows


def test_missing_library_fails_loudly(monkeypatch):
    from paper_2602_00509_amd import probe
    monkeypatch.setattr(probe, "_lib", None)
    monkeypatch.setattr(probe, "LIB_PATH", "/nonexistent/libprobe.so")
    with pytest.raises(FileNotFoundError):
        probe.lib()


def test_product_path_does_not_touch_the_oracle():
    """The binding, the kernels' build script and the workload generators never import oracle/."""
    pkg = os.path.join(ROOT, "paper_2602_00509_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "probe_oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2602_00509_amd" not in text and "libprobe.so" not in text, f
