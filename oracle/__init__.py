"""ctypes front end of the CPU oracle (``probe_oracle.c``, ``planner_oracle.c``, ``gating_oracle.c``).

TEST INFRASTRUCTURE ONLY: the tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline``
leg of ``bench.py`` may import this package; the product path never does.  It imports
nothing from the HIP package and shares no code with it.

The C files are compiled with gcc on first use (``build()``), into ``oracle/libprobe_oracle.so``.
All arrays are numpy; bf16 tensors travel as ``uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, f) for f in ("probe_oracle.c", "planner_oracle.c", "gating_oracle.c")]
_LIB = os.path.join(_HERE, "libprobe_oracle.so")
_lock = threading.Lock()
_lib = None


# PROBE_ORACLE_SANITIZE=1 (set by oracle/run_sanitized.py for its child process) selects a second build of the
# same sources with AddressSanitizer and UndefinedBehaviorSanitizer, kept in its own file.
_SANITIZE = os.environ.get("PROBE_ORACLE_SANITIZE") == "1"
if _SANITIZE:
    _LIB = os.path.join(_HERE, "libprobe_oracle_san.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C99 + OpenMP).  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < max(os.path.getmtime(f) for f in _SRCS)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        flags = (["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"]
                 if _SANITIZE else ["-O2"])
        cmd = ["gcc"] + flags + ["-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", tmp] + _SRCS + ["-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            build()
            lib = C.CDLL(_LIB)
            lib.oracle_imbalance_ratio.restype = C.c_double
            _lib = lib
    return _lib


def _p(a, ty):
    if a is None:
        return None
    return a.ctypes.data_as(C.POINTER(ty))


def _chk(a, dtype, shape=None):
    a = np.ascontiguousarray(a, dtype=dtype)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError("expected shape %s, got %s" % (shape, a.shape))
    return a


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) exactly to float64."""
    u = bits.astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _route(fn, x_bits, w_gate, bias, tokens_per_group, k, renormalize):
    x_bits = _chk(x_bits, np.uint16)
    T, H = x_bits.shape
    w_gate = _chk(w_gate, np.float32)
    E = w_gate.shape[0]
    assert w_gate.shape == (E, H)
    if bias is not None:
        bias = _chk(bias, np.float32)
        if bias.ndim == 1:
            bias = bias.reshape(1, E)
        G = bias.shape[0]
        assert bias.shape == (G, E)
    else:
        G = 1
    tpg = int(tokens_per_group) if tokens_per_group else max(T, 1)
    logits = np.empty((T, E), np.float64)
    probs = np.empty((T, E), np.float64)
    idx = np.empty((T, k), np.int32)
    w = np.empty((T, k), np.float64)
    counts = np.empty((E,), np.int32)
    rc = fn(_p(x_bits, C.c_uint16), _p(w_gate, C.c_float), _p(bias, C.c_float), G, tpg, T, H,
            E, k, int(bool(renormalize)), _p(logits, C.c_double), _p(probs, C.c_double),
            _p(idx, C.c_int32), _p(w, C.c_double), _p(counts, C.c_int32))
    if rc != 0:
        raise ValueError("oracle route failed: %d" % rc)
    return dict(logits=logits, probs=probs, idx=idx, w=w, counts=counts)


def route_topk(x_bits, w_gate, bias=None, tokens_per_group=None, k=2, renormalize=True):
    """Router: logits, softmax over all experts, k largest, weights, counts n_e (fp64)."""
    return _route(_load().oracle_route_topk, x_bits, w_gate, bias, tokens_per_group, k,
                  renormalize)


def predict_topk(h_prev_bits, w_gate_next, bias_next=None, tokens_per_group=None, k=2,
                 renormalize=True):
    """Lookahead predictor at its zero-initialised residual; ``counts`` is n-hat."""
    return _route(_load().oracle_predict_topk, h_prev_bits, w_gate_next, bias_next,
                  tokens_per_group, k, renormalize)


def predict_topk_residual(h_prev_bits, w_gate_next, bias_next, tokens_per_group, w1_hat_bits, w2_hat,
                          k=2, renormalize=True):
    """Eq. 7 in full: cloned router plus W2_hat silu(W1_hat h); w1_hat bf16 bits [D,H], w2_hat fp32 [E,D]."""
    w1_hat_bits = _chk(w1_hat_bits, np.uint16)
    w2_hat = _chk(w2_hat, np.float32)
    D = w1_hat_bits.shape[0]
    assert w1_hat_bits.shape == (D, h_prev_bits.shape[1]) and w2_hat.shape == (w_gate_next.shape[0], D)
    fn = _load().oracle_predict_topk_residual

    def bound(*a):
        # a = (x, w_gate, bias, G, tpg, T, H, E, k, renorm, outputs...): insert the residual after tpg
        return fn(*a[:5], _p(w1_hat_bits, C.c_uint16), _p(w2_hat, C.c_float), D, *a[5:])
    return _route(bound, h_prev_bits, w_gate_next, bias_next, tokens_per_group, k, renormalize)


def route_grouped(x_bits, w_gate, bias=None, tokens_per_group=None, select_bias=None, scoring="sigmoid",
                  n_group=1, topk_group=1, group_top=2, k=2, renormalize=True, routed_scale=1.0):
    """Group-limited gate (``gating_oracle.c``): scores, selection scores, group scores, allowed
    groups, chosen experts, gating values, counts; all floating point in fp64."""
    x_bits = _chk(x_bits, np.uint16)
    T, H = x_bits.shape
    w_gate = _chk(w_gate, np.float32)
    E = w_gate.shape[0]
    assert w_gate.shape == (E, H)
    if bias is not None:
        bias = _chk(bias, np.float32)
        if bias.ndim == 1:
            bias = bias.reshape(1, E)
        G = bias.shape[0]
        assert bias.shape == (G, E)
    else:
        G = 1
    if select_bias is not None:
        select_bias = _chk(select_bias, np.float32, (E,))
    tpg = int(tokens_per_group) if tokens_per_group else max(T, 1)
    mode = {"softmax": 0, "sigmoid": 1}[scoring]
    out = dict(logits=np.empty((T, E)), scores=np.empty((T, E)), choice=np.empty((T, E)),
               group_scores=np.empty((T, n_group)), groups=np.empty((T, topk_group), np.int32),
               idx=np.empty((T, k), np.int32), w=np.empty((T, k)), counts=np.empty((E,), np.int32))
    fn = _load().oracle_route_grouped
    fn.argtypes = None
    rc = fn(_p(x_bits, C.c_uint16), _p(w_gate, C.c_float), _p(bias, C.c_float), G, tpg,
            _p(select_bias, C.c_float), mode, int(n_group), int(topk_group), int(group_top),
            int(bool(renormalize)), C.c_double(float(routed_scale)), T, H, E, int(k),
            _p(out["logits"], C.c_double), _p(out["scores"], C.c_double), _p(out["choice"], C.c_double),
            _p(out["group_scores"], C.c_double), _p(out["groups"], C.c_int32), _p(out["idx"], C.c_int32),
            _p(out["w"], C.c_double), _p(out["counts"], C.c_int32))
    if rc != 0:
        raise ValueError("oracle route_grouped failed: %d" % rc)
    return out


def plan_dispatch(n, delta_in, E_loc, rank):
    """The plan of plan_greedy as source rank ``rank`` applies it to its own tokens: one slot per
    (destination rank, expert copy), numbered by rank first; rank_off [R+1] delimits the ranks' slots."""
    n = _chk(n, np.int32)
    R, E, _ = n.shape
    delta_in = _chk(delta_in, np.int32)
    max_replicas = delta_in.shape[1]
    rep_off = np.zeros((E + 1,), np.int32)
    cap = E + R * max_replicas
    rep_slot = np.full((cap,), -1, np.int32)
    rep_weight = np.zeros((cap,), np.int32)
    rank_off = np.zeros((R + 1,), np.int32)
    slot_expert = np.full((cap,), -1, np.int32)
    rc = _load().oracle_plan_dispatch(_p(n, C.c_int32), _p(delta_in, C.c_int32), R, E, int(E_loc), max_replicas,
                                      int(rank), _p(rep_off, C.c_int32), _p(rep_slot, C.c_int32),
                                      _p(rep_weight, C.c_int32), _p(rank_off, C.c_int32), _p(slot_expert, C.c_int32))
    if rc != 0:
        raise ValueError("oracle plan_dispatch failed: %d" % rc)
    used = int(rep_off[E])
    return dict(rep_off=rep_off, rep_slot=rep_slot[:used].copy(), rep_weight=rep_weight[:used].copy(), num_slots=cap,
                rank_off=rank_off, slot_expert=slot_expert[:used].copy())


def permute(topk_idx, rep_off, rep_slot, rep_weight, num_slots, x_bits=None):
    """Sequential weighted round-robin assignment and stable grouping by slot."""
    topk_idx = _chk(topk_idx, np.int32)
    T, k = topk_idx.shape
    rep_off = _chk(rep_off, np.int32)
    E = rep_off.shape[0] - 1
    rep_slot = _chk(rep_slot, np.int32)
    rep_weight = _chk(rep_weight, np.int32)
    S = int(num_slots)
    N = T * k
    H = 0
    xp = None
    if x_bits is not None:
        x_bits = _chk(x_bits, np.uint16)
        H = x_bits.shape[1]
        assert x_bits.shape[0] == T
        xp = np.empty((N, H), np.uint16)
    slot_counts = np.empty((S,), np.int32)
    slot_offsets = np.empty((S + 1,), np.int32)
    row_pair = np.empty((N,), np.int32)
    pair_row = np.empty((T, k), np.int32)
    n_local = np.zeros((1,), np.int32)
    rc = _load().oracle_permute(_p(topk_idx, C.c_int32), _p(rep_off, C.c_int32),
                                _p(rep_slot, C.c_int32), _p(rep_weight, C.c_int32), S,
                                _p(x_bits, C.c_uint16), T, H, E, k, _p(slot_counts, C.c_int32),
                                _p(slot_offsets, C.c_int32), _p(row_pair, C.c_int32),
                                _p(pair_row, C.c_int32), _p(xp, C.c_uint16),
                                _p(n_local, C.c_int32))
    if rc != 0:
        raise ValueError("oracle permute failed: %d" % rc)
    return dict(slot_counts=slot_counts, slot_offsets=slot_offsets, row_pair=row_pair,
                pair_row=pair_row, xp=xp, n_local=int(n_local[0]))


def grouped_ffn(xp_bits, slot_offsets, w13_list, w2_list, rows=None):
    """SwiGLU expert FFN for the rows listed (all rows below slot_offsets[-1] if None).

    Returns fp64 [len(rows), H]."""
    xp_bits = _chk(xp_bits, np.uint16)
    H = xp_bits.shape[1]
    slot_offsets = _chk(slot_offsets, np.int32)
    S = slot_offsets.shape[0] - 1
    assert len(w13_list) == S and len(w2_list) == S
    w13_list = [_chk(w, np.uint16) for w in w13_list]
    w2_list = [_chk(w, np.uint16) for w in w2_list]
    F = w2_list[0].shape[1] if S else 1
    for a, b in zip(w13_list, w2_list):
        assert a.shape == (2 * F, H) and b.shape == (H, F)
    if rows is None:
        rows = np.arange(int(slot_offsets[-1]), dtype=np.int32)
    rows = _chk(rows, np.int32)
    if rows.size:
        assert rows.min() >= 0 and rows.max() < xp_bits.shape[0]
    PT = C.POINTER(C.c_uint16)
    a13 = (PT * max(S, 1))(*[_p(w, C.c_uint16) for w in w13_list])
    a2 = (PT * max(S, 1))(*[_p(w, C.c_uint16) for w in w2_list])
    y = np.zeros((rows.shape[0], H), np.float64)
    rc = _load().oracle_grouped_ffn(_p(xp_bits, C.c_uint16), _p(slot_offsets, C.c_int32), a13,
                                    a2, S, H, F, _p(rows, C.c_int32), int(rows.shape[0]),
                                    _p(y, C.c_double))
    if rc != 0:
        raise ValueError("oracle grouped_ffn failed: %d" % rc)
    return y


def combine(y, pair_row, w):
    """Gate-weighted sum over a token's local pairs, ascending top-k position (fp64)."""
    y = _chk(y, np.float64)
    H = y.shape[1]
    pair_row = _chk(pair_row, np.int32)
    T, k = pair_row.shape
    w = _chk(w, np.float64, (T, k))
    if pair_row.size:
        assert pair_row.max() < y.shape[0]
    out = np.empty((T, H), np.float64)
    rc = _load().oracle_combine(_p(y, C.c_double), _p(pair_row, C.c_int32), _p(w, C.c_double),
                                T, H, k, _p(out, C.c_double))
    if rc != 0:
        raise ValueError("oracle combine failed: %d" % rc)
    return out


def combine_shared(y, pair_row, w, shared, shared_scale=1.0):
    """combine() plus shared_scale times the shared expert's output of every token (fp64)."""
    y = _chk(y, np.float64)
    H = y.shape[1]
    pair_row = _chk(pair_row, np.int32)
    T, k = pair_row.shape
    w = _chk(w, np.float64, (T, k))
    shared = _chk(shared, np.float64, (T, H))
    if pair_row.size:
        assert pair_row.max() < y.shape[0]
    out = np.empty((T, H), np.float64)
    rc = _load().oracle_combine_shared(_p(y, C.c_double), _p(pair_row, C.c_int32), _p(w, C.c_double),
                                       _p(shared, C.c_double), C.c_double(float(shared_scale)), T, H, k,
                                       _p(out, C.c_double))
    if rc != 0:
        raise ValueError("oracle combine_shared failed: %d" % rc)
    return out


def imbalance_ratio(rank_load) -> float:
    """Eq. 1: max rank load over mean rank load."""
    rank_load = _chk(rank_load, np.float64)
    return float(_load().oracle_imbalance_ratio(_p(rank_load, C.c_double), int(rank_load.size)))


def topk_overlap(pred_idx, true_idx) -> float:
    """Mean over tokens of |pred_k intersect true_k| / k (the predictor's top-k accuracy)."""
    pred_idx = np.asarray(pred_idx)
    true_idx = np.asarray(true_idx)
    T, k = true_idx.shape
    hit = 0
    for t in range(T):
        hit += len(set(pred_idx[t].tolist()) & set(true_idx[t].tolist()))
    return hit / float(max(T, 1) * k)


def moe_layer(x_bits, w_gate, bias, tokens_per_group, k, renormalize, plan, w13_list, w2_list):
    """Whole layer: route -> permute -> FFN -> combine, nothing rounded in between."""
    r = route_topk(x_bits, w_gate, bias, tokens_per_group, k, renormalize)
    p = permute(r["idx"], plan["rep_off"], plan["rep_slot"], plan["rep_weight"],
                plan["num_slots"], x_bits)
    y = grouped_ffn(p["xp"], p["slot_offsets"], w13_list, w2_list)
    out = combine(y, p["pair_row"], r["w"])
    return dict(route=r, permute=p, y=y, out=out)


def cross_entropy_sum(true_probs, pred_probs) -> float:
    """Sum over tokens of - sum_e p_true log p_pred (the distillation loss of Sec. 4.2), fp64.
    Terms with p_true = 0 contribute nothing."""
    p = np.asarray(true_probs, np.float64)
    q = np.asarray(pred_probs, np.float64)
    total = 0.0
    for t in range(p.shape[0]):
        for e in range(p.shape[1]):
            if p[t, e] > 0.0:
                total -= p[t, e] * np.log(q[t, e])
    return float(total)


# ------------------------------------------------------------------------------ planner

def plan_greedy(n_hat, E_loc, max_replicas=3, budget=3, k_max=16, eps=0, n0=0, g_num=0, g_den=1):
    """Algorithm 1 (greedy balance-optimal planning) on predicted tokens n_hat [R,E] (source rank, expert).

    Returns dict(n [R,E,R] tokens by (origin, expert, processing rank), delta_in [R,max_replicas],
    delta_out [R,budget], moves [k_max,3] rows (expert, r_src, r_dst), L_before, L_after, max_load,
    n_moves)."""
    n_hat = _chk(n_hat, np.int32)
    R, E = n_hat.shape
    n = np.zeros((R, E, R), np.int32)
    delta_in = np.full((R, max(max_replicas, 1)), -1, np.int32)[:, :max_replicas]
    delta_in = np.ascontiguousarray(delta_in)
    delta_out = np.ascontiguousarray(np.full((R, max(budget, 1)), -1, np.int32)[:, :budget])
    moves = np.ascontiguousarray(np.full((max(k_max, 1), 3), -1, np.int32)[:k_max])
    stats = np.zeros((4,), np.int64)
    i64 = C.c_int64
    rc = _load().oracle_plan_greedy(_p(n_hat, C.c_int32), R, E, int(E_loc), int(max_replicas), int(budget),
                                    int(k_max), i64(int(eps)), i64(int(n0)), i64(int(g_num)), i64(int(g_den)),
                                    _p(n, C.c_int32), _p(delta_in, C.c_int32), _p(delta_out, C.c_int32),
                                    _p(moves, C.c_int32), _p(stats, C.c_int64))
    if rc != 0:
        raise ValueError("oracle plan_greedy failed: %d" % rc)
    return dict(n=n, delta_in=delta_in, delta_out=delta_out, moves=moves, L_before=int(stats[0]),
                L_after=int(stats[1]), max_load=int(stats[2]), n_moves=int(stats[3]))


def plan_for_rank(n, delta_in, E_loc, rank):
    """The plan of plan_greedy in the layout probe_permute consumes, as seen from one rank."""
    n = _chk(n, np.int32)
    R, E, _ = n.shape
    delta_in = _chk(delta_in, np.int32)
    max_replicas = delta_in.shape[1]
    rep_off = np.zeros((E + 1,), np.int32)
    cap = E + R * max_replicas
    rep_slot = np.full((cap,), -1, np.int32)
    rep_weight = np.zeros((cap,), np.int32)
    slot_expert = np.full((E_loc + max_replicas,), -1, np.int32)
    rc = _load().oracle_plan_for_rank(_p(n, C.c_int32), _p(delta_in, C.c_int32), R, E, int(E_loc), max_replicas,
                                      int(rank), _p(rep_off, C.c_int32), _p(rep_slot, C.c_int32),
                                      _p(rep_weight, C.c_int32), _p(slot_expert, C.c_int32))
    if rc != 0:
        raise ValueError("oracle plan_for_rank failed: %d" % rc)
    used = int(rep_off[E])
    return dict(rep_off=rep_off, rep_slot=rep_slot[:used].copy(), rep_weight=rep_weight[:used].copy(),
                num_slots=E_loc + max_replicas, slot_expert=slot_expert)
