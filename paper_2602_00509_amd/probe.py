"""Thin ctypes binding of libprobe.so (include/probe.h).

Argument marshalling only: every step of the layer runs in the HIP kernels of the library.
PyTorch appears here for device memory (tensors as buffers) and streams, nothing else.  There
is no CPU fallback: if the library is missing or a call fails, an exception is raised.

Function names follow the C entry points (``route_topk`` -> ``probe_route_topk`` ...).
Outputs and workspaces may be passed in (``out=...``, ``workspace=...``) so that a caller can
pre-allocate everything; otherwise they are allocated with torch on the input's device.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libprobe.so")
_lib = None

MAX_EXPERTS, MAX_TOPK, MAX_SLOTS = 256, 8, 1024


class ProbeError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("libprobe error %d: %s" % (code, text))
        self.code = code


class _PlannerParams(C.Structure):
    _fields_ = [("max_replicas", C.c_int32), ("budget", C.c_int32), ("k_max", C.c_int32), ("eps", C.c_int64),
                ("n0", C.c_int64), ("g_num", C.c_int64), ("g_den", C.c_int64)]


class _Plan(C.Structure):
    _fields_ = [("rep_off", C.c_void_p), ("rep_slot", C.c_void_p), ("rep_weight", C.c_void_p),
                ("num_slots", C.c_int32)]


def lib():
    """Load libprobe.so (built in-tree by build.py); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                "%s not found: build it with `python -m paper_2602_00509_amd.build` "
                "(there is no fallback path)" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        L.probe_last_error_string.restype = C.c_char_p
        L.probe_version.restype = C.c_char_p
        for name in ("probe_route_topk_workspace_bytes", "probe_predict_topk_workspace_bytes"):
            getattr(L, name).restype = C.c_size_t
            getattr(L, name).argtypes = [C.c_int] * 4
        L.probe_permute_workspace_bytes.restype = C.c_size_t
        L.probe_permute_workspace_bytes.argtypes = [C.c_int] * 4
        L.probe_grouped_ffn_workspace_bytes.restype = C.c_size_t
        L.probe_grouped_ffn_workspace_bytes.argtypes = [C.c_int] * 4
        route_args = ([C.c_void_p] * 3 + [C.c_int] * 7 + [C.c_void_p] * 5 + [C.c_size_t, C.c_void_p])
        L.probe_route_topk.argtypes = route_args
        L.probe_predict_topk.argtypes = route_args
        L.probe_predict_topk_residual.argtypes = ([C.c_void_p] * 3 + [C.c_int] * 2 + [C.c_void_p] * 2 +
                                                  [C.c_int] * 6 + [C.c_void_p] * 5 + [C.c_size_t, C.c_void_p])
        L.probe_predict_topk_residual.restype = C.c_int
        L.probe_predict_topk_residual_workspace_bytes.restype = C.c_size_t
        L.probe_predict_topk_residual_workspace_bytes.argtypes = [C.c_int] * 5
        L.probe_permute.argtypes = ([C.c_void_p, C.POINTER(_Plan), C.c_void_p] + [C.c_int] * 4 +
                                    [C.c_void_p] * 7 + [C.c_size_t, C.c_void_p])
        L.probe_permute_static.restype = C.c_int
        L.probe_permute_static.argtypes = ([C.c_void_p, C.POINTER(_Plan), C.c_void_p] + [C.c_int] * 4 +
                                           [C.c_void_p] * 7)
        L.probe_permute_static_max_pairs.restype = C.c_size_t
        L.probe_permute_static_max_pairs.argtypes = [C.c_int]
        L.probe_grouped_ffn.argtypes = ([C.c_void_p] * 4 + [C.c_int] * 4 + [C.c_void_p] * 2 +
                                        [C.c_size_t, C.c_void_p])
        L.probe_grouped_ffn_gather.argtypes = ([C.c_void_p] * 2 + [C.c_int] * 2 + [C.c_void_p] * 3 + [C.c_int] * 4 +
                                               [C.c_void_p] * 2 + [C.c_size_t, C.c_void_p])
        L.probe_grouped_ffn_gather.restype = C.c_int
        L.probe_combine.argtypes = [C.c_void_p] * 3 + [C.c_int] * 3 + [C.c_void_p] * 2
        L.probe_combine_shared.restype = C.c_int
        L.probe_combine_shared.argtypes = [C.c_void_p] * 4 + [C.c_float] + [C.c_int] * 3 + [C.c_void_p] * 2
        L.probe_route_grouped_workspace_bytes.restype = C.c_size_t
        L.probe_route_grouped_workspace_bytes.argtypes = [C.c_int] * 4
        L.probe_route_grouped.restype = C.c_int
        L.probe_route_grouped.argtypes = ([C.c_void_p] * 3 + [C.c_int] * 2 + [C.c_void_p, C.POINTER(_Gating)] +
                                          [C.c_int] * 4 + [C.c_void_p] * 5 + [C.c_size_t, C.c_void_p])
        L.probe_pack_gate_bytes.restype = C.c_size_t
        L.probe_pack_gate_bytes.argtypes = [C.c_int, C.c_int]
        L.probe_pack_gate.restype = C.c_int
        L.probe_pack_gate.argtypes = [C.c_void_p] + [C.c_int] * 4 + [C.c_void_p, C.c_void_p]
        for name in ("probe_route_topk_packed_workspace_bytes", "probe_route_predict_topk_packed_workspace_bytes"):
            getattr(L, name).restype = C.c_size_t
            getattr(L, name).argtypes = [C.c_int] * 4
        L.probe_route_topk_packed.argtypes = route_args
        L.probe_predict_topk_packed.argtypes = route_args
        L.probe_route_topk_packed.restype = L.probe_predict_topk_packed.restype = C.c_int
        L.probe_route_grouped_packed.restype = C.c_int
        L.probe_route_grouped_packed.argtypes = ([C.c_void_p] * 3 + [C.c_int] * 2 + [C.c_void_p, C.POINTER(_Gating)] +
                                                 [C.c_int] * 4 + [C.c_void_p] * 5 + [C.c_size_t, C.c_void_p])
        L.probe_route_predict_topk_packed.restype = C.c_int
        L.probe_route_predict_topk_packed.argtypes = ([C.c_void_p] * 4 + [C.c_int] * 7 + [C.c_void_p] * 9 +
                                                      [C.c_size_t, C.c_void_p])
        L.probe_route_predict_topk_workspace_bytes.restype = C.c_size_t
        L.probe_route_predict_topk_workspace_bytes.argtypes = [C.c_int] * 4
        L.probe_route_predict_topk.restype = C.c_int
        L.probe_route_predict_topk.argtypes = ([C.c_void_p] * 5 + [C.c_int] * 7 + [C.c_void_p] * 9 +
                                               [C.c_size_t, C.c_void_p])
        L.probe_plan_greedy_workspace_bytes.restype = C.c_size_t
        L.probe_plan_greedy_workspace_bytes.argtypes = [C.c_int, C.c_int]
        L.probe_plan_greedy.restype = C.c_int
        L.probe_plan_greedy.argtypes = ([C.c_void_p] + [C.c_int] * 4 + [C.POINTER(_PlannerParams)] +
                                        [C.c_void_p] * 10 + [C.c_size_t, C.c_void_p])
        L.probe_plan_dispatch.restype = C.c_int
        L.probe_plan_dispatch.argtypes = [C.c_void_p] * 2 + [C.c_int] * 5 + [C.c_void_p] * 6
        L.probe_predictor_metrics.restype = C.c_int
        L.probe_predictor_metrics.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_int,
                                              C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
        for name in ("probe_route_topk", "probe_predict_topk", "probe_permute", "probe_grouped_ffn",
                     "probe_combine"):
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise ProbeError(rc, lib().probe_last_error_string().decode())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _want(t, dtype, shape, name):
    if t.dtype != dtype or tuple(t.shape) != tuple(shape) or not t.is_contiguous() or not t.is_cuda:
        raise ValueError("%s: expected contiguous cuda %s %s, got %s %s" %
                         (name, dtype, tuple(shape), t.dtype, tuple(t.shape)))
    return t


def _ws(workspace, nbytes, device):
    if workspace is None:
        workspace = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
    return workspace


# --------------------------------------------------------------------- route / predict

def route_topk_workspace_bytes(T, H, E, k):
    return int(lib().probe_route_topk_workspace_bytes(T, H, E, k))


predict_topk_workspace_bytes = route_topk_workspace_bytes


def predict_topk_residual_workspace_bytes(T, H, E, k, D):
    return int(lib().probe_predict_topk_residual_workspace_bytes(T, H, E, k, D))


class PackedGate:
    """probe_pack_gate: the bf16 planes of one gate, or of two gates stacked (for route_predict_topk).

    ``planes`` is bf16 [3, stack_rows, H]; pass the object wherever a w_gate tensor is accepted."""

    def __init__(self, w_gate, w_gate_next=None, *, stream=None):
        E, H = w_gate.shape
        _want(w_gate, torch.float32, (E, H), "w_gate")
        gates = [w_gate]
        if w_gate_next is not None:
            _want(w_gate_next, torch.float32, (E, H), "w_gate_next")
            gates.append(w_gate_next)
        self.E, self.H, self.stack_rows = E, H, E * len(gates)
        nbytes = int(lib().probe_pack_gate_bytes(H, self.stack_rows))
        self.buf = torch.empty(nbytes, dtype=torch.uint8, device=w_gate.device)
        for i, g in enumerate(gates):
            _check(lib().probe_pack_gate(_ptr(g), H, E, self.stack_rows, i * E, _ptr(self.buf), _stream(stream)))
        self.planes = self.buf[:3 * self.stack_rows * H * 2].view(torch.bfloat16).view(3, self.stack_rows, H)
        self.device = w_gate.device

    def data_ptr(self):
        return self.buf.data_ptr()


def route_topk_packed_workspace_bytes(T, H, E, k):
    return int(lib().probe_route_topk_packed_workspace_bytes(T, H, E, k))


def _route(fn, x, w_gate, bias, tokens_per_group, k, renormalize, want_probs, want_counts, out,
           workspace, stream, residual=None):
    T, H = x.shape
    packed = isinstance(w_gate, PackedGate)
    _want(x, torch.bfloat16, (T, H), "x")
    if packed:
        if w_gate.stack_rows != w_gate.E or w_gate.H != H or residual is not None:
            raise ValueError("a single packed gate with H = %d is needed here" % H)
        E = w_gate.E
        fn = {"probe_route_topk": lib().probe_route_topk_packed,
              "probe_predict_topk": lib().probe_predict_topk_packed}[fn.__name__]
    else:
        E = w_gate.shape[0]
        _want(w_gate, torch.float32, (E, H), "w_gate")
    G = 1
    if bias is not None:
        if bias.dim() == 1:
            bias = bias.view(1, E)
        G = bias.shape[0]
        _want(bias, torch.float32, (G, E), "bias")
    tpg = int(tokens_per_group) if tokens_per_group else max(T, 1)
    out = dict(out) if out else {}
    dev = x.device
    if "idx" not in out:
        out["idx"] = torch.empty((T, k), dtype=torch.int32, device=dev)
    if "w" not in out:
        out["w"] = torch.empty((T, k), dtype=torch.float32, device=dev)
    if want_probs and "probs" not in out:
        out["probs"] = torch.empty((T, E), dtype=torch.float32, device=dev)
    if want_counts and "counts" not in out:
        out["counts"] = torch.empty((E,), dtype=torch.int32, device=dev)
    _want(out["idx"], torch.int32, (T, k), "idx")
    _want(out["w"], torch.float32, (T, k), "w")
    probs = out.get("probs") if want_probs else None
    counts = out.get("counts") if want_counts else None
    tail = (T, H, E, k, int(bool(renormalize)), _ptr(out["idx"]), _ptr(out["w"]), _ptr(probs), _ptr(counts))
    if residual is None:
        need = route_topk_packed_workspace_bytes(T, H, E, k) if packed else route_topk_workspace_bytes(T, H, E, k)
        workspace = _ws(workspace, need, dev)
        rc = fn(_ptr(x), _ptr(w_gate), _ptr(bias), G, tpg, *tail, _ptr(workspace), workspace.numel(),
                _stream(stream))
    else:
        w1_hat, w2_hat = residual
        D = w1_hat.shape[0]
        _want(w1_hat, torch.bfloat16, (D, H), "w1_hat")
        _want(w2_hat, torch.float32, (E, D), "w2_hat")
        workspace = _ws(workspace, predict_topk_residual_workspace_bytes(T, H, E, k, D), dev)
        rc = fn(_ptr(x), _ptr(w_gate), _ptr(bias), G, tpg, _ptr(w1_hat), _ptr(w2_hat), D, *tail,
                _ptr(workspace), workspace.numel(), _stream(stream))
    _check(rc)
    return out


def route_topk(x, w_gate, bias=None, tokens_per_group=None, k=2, renormalize=True, *,
               want_probs=False, want_counts=True, out=None, workspace=None, stream=None):
    """probe_route_topk: returns dict(idx int32 [T,k], w fp32 [T,k], probs?, counts?)."""
    return _route(lib().probe_route_topk, x, w_gate, bias, tokens_per_group, k, renormalize,
                  want_probs, want_counts, out, workspace, stream)


class _Gating(C.Structure):
    _fields_ = [("scoring", C.c_int32), ("n_group", C.c_int32), ("topk_group", C.c_int32),
                ("group_top", C.c_int32), ("renormalize", C.c_int32), ("routed_scale", C.c_float)]


SCORE_SOFTMAX, SCORE_SIGMOID = 0, 1


def route_grouped(x, w_gate, bias=None, tokens_per_group=None, select_bias=None, *, scoring="sigmoid",
                  n_group=1, topk_group=1, group_top=2, k=2, renormalize=True, routed_scale=1.0,
                  want_scores=False, want_counts=True, out=None, workspace=None, stream=None):
    """probe_route_grouped: group-limited gate; returns dict(idx, w, scores?, counts?)."""
    T, H = x.shape
    packed = isinstance(w_gate, PackedGate)
    _want(x, torch.bfloat16, (T, H), "x")
    if packed:
        if w_gate.stack_rows != w_gate.E or w_gate.H != H:
            raise ValueError("a single packed gate with H = %d is needed here" % H)
        E = w_gate.E
    else:
        E = w_gate.shape[0]
        _want(w_gate, torch.float32, (E, H), "w_gate")
    G = 1
    if bias is not None:
        if bias.dim() == 1:
            bias = bias.view(1, E)
        G = bias.shape[0]
        _want(bias, torch.float32, (G, E), "bias")
    if select_bias is not None:
        _want(select_bias, torch.float32, (E,), "select_bias")
    tpg = int(tokens_per_group) if tokens_per_group else max(T, 1)
    gating = _Gating({"softmax": SCORE_SOFTMAX, "sigmoid": SCORE_SIGMOID}[scoring], int(n_group), int(topk_group),
                     int(group_top), int(bool(renormalize)), float(routed_scale))
    out = dict(out) if out else {}
    dev = x.device
    out.setdefault("idx", torch.empty((T, k), dtype=torch.int32, device=dev))
    out.setdefault("w", torch.empty((T, k), dtype=torch.float32, device=dev))
    if want_scores:
        out.setdefault("scores", torch.empty((T, E), dtype=torch.float32, device=dev))
    if want_counts:
        out.setdefault("counts", torch.empty((E,), dtype=torch.int32, device=dev))
    _want(out["idx"], torch.int32, (T, k), "idx")
    _want(out["w"], torch.float32, (T, k), "w")
    workspace = _ws(workspace, int(lib().probe_route_grouped_workspace_bytes(T, H, E, k)), dev)
    fn = lib().probe_route_grouped_packed if packed else lib().probe_route_grouped
    rc = fn(_ptr(x), _ptr(w_gate), _ptr(bias), G, tpg, _ptr(select_bias), C.byref(gating),
                                   T, H, E, k, _ptr(out["idx"]), _ptr(out["w"]),
                                   _ptr(out.get("scores") if want_scores else None),
                                   _ptr(out.get("counts") if want_counts else None), _ptr(workspace),
                                   workspace.numel(), _stream(stream))
    _check(rc)
    return out


def predict_topk(h_prev, w_gate_next, bias_next=None, tokens_per_group=None, k=2,
                 renormalize=True, *, want_probs=False, want_counts=True, out=None, workspace=None,
                 stream=None):
    """probe_predict_topk: lookahead predictor; ``counts`` is the predicted workload n-hat."""
    return _route(lib().probe_predict_topk, h_prev, w_gate_next, bias_next, tokens_per_group, k,
                  renormalize, want_probs, want_counts, out, workspace, stream)


def predict_topk_residual(h_prev, w_gate_next, bias_next, tokens_per_group, w1_hat, w2_hat, k=2,
                          renormalize=True, *, want_probs=False, want_counts=True, out=None,
                          workspace=None, stream=None):
    """probe_predict_topk_residual: Eq. 7 in full; w1_hat bf16 [D,H], w2_hat fp32 [E,D]."""
    return _route(lib().probe_predict_topk_residual, h_prev, w_gate_next, bias_next, tokens_per_group, k,
                  renormalize, want_probs, want_counts, out, workspace, stream, residual=(w1_hat, w2_hat))


def route_predict_topk_workspace_bytes(T, H, E, k):
    return int(lib().probe_route_predict_topk_workspace_bytes(T, H, E, k))


def route_predict_topk(x, w_gate, bias, w_gate_next, bias_next, tokens_per_group=None, k=2, renormalize=True, *,
                       want_probs=False, out=None, pred_out=None, workspace=None, stream=None):
    """probe_route_predict_topk: router and zero-residual predictor of the next layer in one pass over x.

    Returns (route dict, predict dict), each with idx, w, counts and optionally probs."""
    T, H = x.shape
    packed = isinstance(w_gate, PackedGate)
    _want(x, torch.bfloat16, (T, H), "x")
    if packed:
        if w_gate.stack_rows != 2 * w_gate.E or w_gate.H != H or w_gate_next is not None:
            raise ValueError("route_predict_topk takes ONE PackedGate(w_gate, w_gate_next) and w_gate_next=None")
        E = w_gate.E
    else:
        E = w_gate.shape[0]
        _want(w_gate, torch.float32, (E, H), "w_gate")
        _want(w_gate_next, torch.float32, (E, H), "w_gate_next")
    G = 1
    biases = []
    for b in (bias, bias_next):
        if b is not None:
            if b.dim() == 1:
                b = b.view(1, E)
            G = b.shape[0]
            _want(b, torch.float32, (G, E), "bias")
        biases.append(b)
    if biases[0] is not None and biases[1] is not None:
        assert biases[0].shape == biases[1].shape
    tpg = int(tokens_per_group) if tokens_per_group else max(T, 1)
    dev = x.device
    outs = []
    for o in (out, pred_out):
        o = dict(o) if o else {}
        o.setdefault("idx", torch.empty((T, k), dtype=torch.int32, device=dev))
        o.setdefault("w", torch.empty((T, k), dtype=torch.float32, device=dev))
        o.setdefault("counts", torch.empty((E,), dtype=torch.int32, device=dev))
        if want_probs:
            o.setdefault("probs", torch.empty((T, E), dtype=torch.float32, device=dev))
        _want(o["idx"], torch.int32, (T, k), "idx")
        _want(o["w"], torch.float32, (T, k), "w")
        outs.append(o)
    r, p = outs
    tail = (G, tpg, T, H, E, k, int(bool(renormalize)), _ptr(r["idx"]), _ptr(r["w"]),
            _ptr(r.get("probs") if want_probs else None), _ptr(r["counts"]), _ptr(p["idx"]), _ptr(p["w"]),
            _ptr(p.get("probs") if want_probs else None), _ptr(p["counts"]))
    if packed:
        workspace = _ws(workspace, int(lib().probe_route_predict_topk_packed_workspace_bytes(T, H, E, k)), dev)
        rc = lib().probe_route_predict_topk_packed(_ptr(x), _ptr(w_gate), _ptr(biases[0]), _ptr(biases[1]), *tail,
                                                   _ptr(workspace), workspace.numel(), _stream(stream))
    else:
        workspace = _ws(workspace, route_predict_topk_workspace_bytes(T, H, E, k), dev)
        rc = lib().probe_route_predict_topk(_ptr(x), _ptr(w_gate), _ptr(biases[0]), _ptr(w_gate_next),
                                            _ptr(biases[1]), *tail, _ptr(workspace), workspace.numel(),
                                            _stream(stream))
    _check(rc)
    return r, p


# ------------------------------------------------------------------------------ planner

def plan_greedy(n_hat, E_loc, rank=0, max_replicas=3, budget=3, k_max=16, eps=0, n0=0, g_num=0, g_den=1, *,
                want_assignment=False, workspace=None, stream=None):
    """probe_plan_greedy: Algorithm 1 on n_hat int32 [R,E]; every output stays on the device.

    Returns dict(plan=Plan usable by permute, rep_off, rep_slot, rep_weight, slot_expert, delta_in,
    delta_out, moves, stats int64 [4], n (optional))."""
    R, E = n_hat.shape
    _want(n_hat, torch.int32, (R, E), "n_hat")
    dev = n_hat.device
    i32 = dict(dtype=torch.int32, device=dev)
    out = dict(rep_off=torch.empty((E + 1,), **i32), rep_slot=torch.empty((E + R * max_replicas,), **i32),
               rep_weight=torch.empty((E + R * max_replicas,), **i32),
               slot_expert=torch.empty((E_loc + max_replicas,), **i32),
               delta_in=torch.empty((R, max_replicas), **i32), delta_out=torch.empty((R, budget), **i32),
               moves=torch.empty((k_max, 3), **i32), stats=torch.empty((4,), dtype=torch.int64, device=dev))
    if want_assignment:
        out["n"] = torch.empty((R, E, R), **i32)
    params = _PlannerParams(max_replicas, budget, k_max, eps, n0, g_num, g_den)
    workspace = _ws(workspace, int(lib().probe_plan_greedy_workspace_bytes(R, E)), dev)
    rc = lib().probe_plan_greedy(_ptr(n_hat), R, E, E_loc, rank, C.byref(params), _ptr(out["rep_off"]),
                                 _ptr(out["rep_slot"]), _ptr(out["rep_weight"]), _ptr(out["slot_expert"]),
                                 _ptr(out["delta_in"]), _ptr(out["delta_out"]), _ptr(out["moves"]),
                                 _ptr(out["stats"]), _ptr(out.get("n")), _ptr(workspace), workspace.numel(),
                                 _stream(stream))
    _check(rc)
    out["plan"] = Plan(out["rep_off"], out["rep_slot"], out["rep_weight"], E_loc + max_replicas, dev)
    return out


def plan_dispatch(n_assign, delta_in, E_loc, rank, *, stream=None):
    """probe_plan_dispatch: the plan as source rank ``rank`` applies it to its own tokens; one slot per
    (destination rank, expert copy), ranks first.

    n_assign int32 [R,E,R] and delta_in int32 [R,max_replicas] as written by plan_greedy(want_assignment=True).
    Returns dict(plan=Plan with num_slots = E + R*max_replicas, rep_off, rep_slot, rep_weight, rank_off, slot_expert)."""
    R, E, _ = n_assign.shape
    max_replicas = delta_in.shape[1]
    _want(n_assign, torch.int32, (R, E, R), "n_assign")
    _want(delta_in, torch.int32, (R, max_replicas), "delta_in")
    dev = n_assign.device
    i32 = dict(dtype=torch.int32, device=dev)
    cap = E + R * max_replicas
    out = dict(rep_off=torch.empty((E + 1,), **i32), rep_slot=torch.empty((cap,), **i32),
               rep_weight=torch.empty((cap,), **i32), rank_off=torch.empty((R + 1,), **i32),
               slot_expert=torch.full((cap,), -1, **i32))
    rc = lib().probe_plan_dispatch(_ptr(n_assign), _ptr(delta_in), R, E, int(E_loc), max_replicas, int(rank),
                                   _ptr(out["rep_off"]), _ptr(out["rep_slot"]), _ptr(out["rep_weight"]),
                                   _ptr(out["rank_off"]), _ptr(out["slot_expert"]), _stream(stream))
    _check(rc)
    out["plan"] = Plan(out["rep_off"], out["rep_slot"], out["rep_weight"], cap, dev)
    return out


# ------------------------------------------------------------------------------ permute

class Plan:
    """Device copy of a balance plan (rep_off [E+1], rep_slot [R], rep_weight [R], S)."""

    def __init__(self, rep_off, rep_slot, rep_weight, num_slots, device="cuda"):
        def dev(a):
            return torch.as_tensor(a, dtype=torch.int32).contiguous().to(device)
        self.rep_off, self.rep_slot, self.rep_weight = dev(rep_off), dev(rep_slot), dev(rep_weight)
        self.num_slots = int(num_slots)
        self.num_experts = self.rep_off.numel() - 1
        self.c = _Plan(self.rep_off.data_ptr(), self.rep_slot.data_ptr(), self.rep_weight.data_ptr(),
                       self.num_slots)


def permute_workspace_bytes(T, E, k, S):
    return int(lib().probe_permute_workspace_bytes(T, E, k, S))


def permute_static_max_pairs(E):
    return int(lib().probe_permute_static_max_pairs(E))


def permute_static(topk_idx, plan: Plan, x, *, out, stream=None, copy_rows=True):
    """probe_permute_static: probe_permute without a workspace (the library's static scratch array).

    Every output tensor must be passed in ``out`` (this wrapper allocates nothing either)."""
    return permute(topk_idx, plan, x, out=out, stream=stream, copy_rows=copy_rows, _static=True)


def permute(topk_idx, plan: Plan, x, *, out=None, workspace=None, stream=None, copy_rows=True, _static=False):
    """probe_permute: returns dict(slot_counts, slot_offsets, row_pair, pair_row, xp, n_local).

    copy_rows=False passes xp = NULL: index outputs only (for grouped_ffn_gather); no "xp" in the result."""
    T, k = topk_idx.shape
    H = x.shape[1]
    E, S = plan.num_experts, plan.num_slots
    _want(topk_idx, torch.int32, (T, k), "topk_idx")
    _want(x, torch.bfloat16, (T, H), "x")
    dev = x.device
    out = dict(out) if out else {}
    N = T * k
    spec = dict(slot_counts=((S,), torch.int32), slot_offsets=((S + 1,), torch.int32),
                row_pair=((N,), torch.int32), pair_row=((T, k), torch.int32),
                xp=((N, H), torch.bfloat16), n_local=((1,), torch.int32))
    if not copy_rows:
        del spec["xp"]
        out.pop("xp", None)
    for name, (shape, dt) in spec.items():
        if name not in out:
            if _static:
                raise ValueError("permute_static: output %r must be pre-allocated" % name)
            out[name] = torch.empty(shape, dtype=dt, device=dev)
        _want(out[name], dt, shape, name)
    if _static:
        rc = lib().probe_permute_static(_ptr(topk_idx), C.byref(plan.c), _ptr(x), T, H, E, k,
                                        _ptr(out["slot_counts"]), _ptr(out["slot_offsets"]),
                                        _ptr(out["row_pair"]), _ptr(out["pair_row"]), _ptr(out.get("xp")),
                                        _ptr(out["n_local"]), _stream(stream))
        _check(rc)
        return out
    workspace = _ws(workspace, permute_workspace_bytes(T, E, k, S), dev)
    rc = lib().probe_permute(_ptr(topk_idx), C.byref(plan.c), _ptr(x), T, H, E, k,
                             _ptr(out["slot_counts"]), _ptr(out["slot_offsets"]),
                             _ptr(out["row_pair"]), _ptr(out["pair_row"]), _ptr(out.get("xp")),
                             _ptr(out["n_local"]), _ptr(workspace), workspace.numel(),
                             _stream(stream))
    _check(rc)
    return out


# -------------------------------------------------------------------------- grouped FFN

class WeightTable:
    """Device arrays of per-slot weight pointers; keeps the weight tensors alive."""

    def __init__(self, w13_list, w2_list):
        assert len(w13_list) == len(w2_list) and len(w13_list) >= 1
        self.S = len(w13_list)
        self.F, self.H = w2_list[0].shape[1], w2_list[0].shape[0]
        for a, b in zip(w13_list, w2_list):
            _want(a, torch.bfloat16, (2 * self.F, self.H), "w13")
            _want(b, torch.bfloat16, (self.H, self.F), "w2")
        self.w13, self.w2 = list(w13_list), list(w2_list)
        dev = w13_list[0].device
        self.w13_ptrs = torch.tensor([t.data_ptr() for t in w13_list], dtype=torch.int64).to(dev)
        self.w2_ptrs = torch.tensor([t.data_ptr() for t in w2_list], dtype=torch.int64).to(dev)


def grouped_ffn_workspace_bytes(S, H, F, max_rows):
    return int(lib().probe_grouped_ffn_workspace_bytes(S, H, F, max_rows))


def grouped_ffn(xp, slot_offsets, weights: WeightTable, *, out=None, workspace=None, stream=None):
    """probe_grouped_ffn: y bf16 [max_rows,H]; rows >= slot_offsets[-1] are left untouched."""
    max_rows, H = xp.shape
    S, F = weights.S, weights.F
    _want(xp, torch.bfloat16, (max_rows, H), "xp")
    _want(slot_offsets, torch.int32, (S + 1,), "slot_offsets")
    assert H == weights.H
    if out is None:
        out = torch.empty((max_rows, H), dtype=torch.bfloat16, device=xp.device)
    _want(out, torch.bfloat16, (max_rows, H), "y")
    workspace = _ws(workspace, grouped_ffn_workspace_bytes(S, H, F, max_rows), xp.device)
    rc = lib().probe_grouped_ffn(_ptr(xp), _ptr(slot_offsets), _ptr(weights.w13_ptrs),
                                 _ptr(weights.w2_ptrs), S, H, F, max_rows, _ptr(out),
                                 _ptr(workspace), workspace.numel(), _stream(stream))
    _check(rc)
    return out


def grouped_ffn_gather(x, row_pair, k, slot_offsets, weights: WeightTable, *, out=None, workspace=None,
                       stream=None):
    """probe_grouped_ffn_gather: the FFN on rows x[row_pair[r] / k] gathered on load (no xp)."""
    T, H = x.shape
    max_rows = row_pair.numel()
    S, F = weights.S, weights.F
    _want(x, torch.bfloat16, (T, H), "x")
    _want(row_pair, torch.int32, (max_rows,), "row_pair")
    _want(slot_offsets, torch.int32, (S + 1,), "slot_offsets")
    assert H == weights.H
    if out is None:
        out = torch.empty((max_rows, H), dtype=torch.bfloat16, device=x.device)
    _want(out, torch.bfloat16, (max_rows, H), "y")
    workspace = _ws(workspace, grouped_ffn_workspace_bytes(S, H, F, max_rows), x.device)
    rc = lib().probe_grouped_ffn_gather(_ptr(x), _ptr(row_pair), T, k, _ptr(slot_offsets), _ptr(weights.w13_ptrs),
                                        _ptr(weights.w2_ptrs), S, H, F, max_rows, _ptr(out), _ptr(workspace),
                                        workspace.numel(), _stream(stream))
    _check(rc)
    return out


# ------------------------------------------------------------------------------ combine

def combine(y, pair_row, topk_w, *, out=None, stream=None):
    """probe_combine: out bf16 [T,H]."""
    T, k = pair_row.shape
    H = y.shape[1]
    _want(y, torch.bfloat16, (y.shape[0], H), "y")
    _want(pair_row, torch.int32, (T, k), "pair_row")
    _want(topk_w, torch.float32, (T, k), "topk_w")
    if out is None:
        out = torch.empty((T, H), dtype=torch.bfloat16, device=y.device)
    _want(out, torch.bfloat16, (T, H), "out")
    rc = lib().probe_combine(_ptr(y), _ptr(pair_row), _ptr(topk_w), T, H, k, _ptr(out),
                             _stream(stream))
    _check(rc)
    return out


def combine_shared(y, pair_row, topk_w, shared_y, shared_scale=1.0, *, out=None, stream=None):
    """probe_combine_shared: combine plus shared_scale * shared_y[t]; out bf16 [T,H]."""
    T, k = pair_row.shape
    H = y.shape[1]
    _want(y, torch.bfloat16, (y.shape[0], H), "y")
    _want(pair_row, torch.int32, (T, k), "pair_row")
    _want(topk_w, torch.float32, (T, k), "topk_w")
    _want(shared_y, torch.bfloat16, (T, H), "shared_y")
    if out is None:
        out = torch.empty((T, H), dtype=torch.bfloat16, device=y.device)
    _want(out, torch.bfloat16, (T, H), "out")
    rc = lib().probe_combine_shared(_ptr(y), _ptr(pair_row), _ptr(topk_w), _ptr(shared_y), C.c_float(shared_scale),
                                    T, H, k, _ptr(out), _stream(stream))
    _check(rc)
    return out


# names of the C entry points, for callers that prefer them
probe_route_topk = route_topk
probe_predict_topk = predict_topk
probe_permute = permute
probe_grouped_ffn = grouped_ffn
probe_combine = combine


def predictor_metrics(pred_idx, true_idx, kp=None, kt=None, pred_probs=None, true_probs=None, *, stream=None):
    """probe_predictor_metrics: (hits int64 [1], cross-entropy sum float64 [1] or None), on the device.

    hits / (T * kt) with kp = kt = k is the top-k accuracy of the predictor."""
    T = pred_idx.shape[0]
    kp = kp or pred_idx.shape[1]
    kt = kt or true_idx.shape[1]
    _want(pred_idx, torch.int32, (T, pred_idx.shape[1]), "pred_idx")
    _want(true_idx, torch.int32, (T, true_idx.shape[1]), "true_idx")
    hits = torch.empty((1,), dtype=torch.int64, device=pred_idx.device)
    ce, E = None, 0
    if pred_probs is not None:
        E = pred_probs.shape[1]
        _want(pred_probs, torch.float32, (T, E), "pred_probs")
        _want(true_probs, torch.float32, (T, E), "true_probs")
        ce = torch.empty((1,), dtype=torch.float64, device=pred_idx.device)
    _check(lib().probe_predictor_metrics(_ptr(pred_idx), pred_idx.shape[1], kp, _ptr(true_idx), true_idx.shape[1], kt,
                                         T, _ptr(pred_probs), _ptr(true_probs), E, _ptr(hits), _ptr(ce),
                                         _stream(stream)))
    return hits, ce


def version() -> str:
    return lib().probe_version().decode()
