"""ctypes front end of the CPU oracle (oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this, and this
never imports the product's HIP binding.

All arrays are numpy, host memory.  Storage dtypes: 0 = fp32, 1 = bf16 bit
patterns (uint16), 2 = fp64.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

F32, BF16, F64 = 0, 1, 2
GATE_FULL, GATE_RENORM = 0, 1
MARGIN = 1e-4          # near-tie margin on logits, relative to max(1, max|logit|)

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(path)
        _lib.oracle_route.restype = C.c_int
        _lib.oracle_expert_norm.restype = C.c_int
        _lib.oracle_importance.restype = C.c_int
        _lib.oracle_permute.restype = C.c_int
        _lib.oracle_expert_ffn.restype = C.c_int
        _lib.oracle_combine.restype = C.c_int
        _lib.oracle_select_resident.restype = C.c_int
        _lib.oracle_policy_scores.restype = C.c_int
        _lib.oracle_on_demand.restype = C.c_int
        _lib.oracle_round_bf16.restype = None
        _lib.oracle_num_threads.restype = C.c_int
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _dtype_of(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.float64:
        return F64
    raise TypeError(f"unsupported storage dtype {a.dtype}")


def _c(a, dt=None):
    a = np.ascontiguousarray(a) if dt is None else np.ascontiguousarray(a, dtype=dt)
    return a


def route(x, Wr, expert_to_slot, gate_mode=GATE_FULL, margin=MARGIN):
    """Returns dict(orig_expert, orig_gate, slot, gate, xnorm, logits, ambiguous)."""
    x = _c(x); Wr = _c(Wr, np.float32); e2s = _c(expert_to_slot, np.int32)
    T, d = x.shape
    E = Wr.shape[0]
    assert Wr.shape[1] == d and e2s.shape == (E,)
    out = dict(orig_expert=np.empty(T, np.int32), orig_gate=np.empty(T, np.float32),
               slot=np.empty(T, np.int32), gate=np.empty(T, np.float32),
               xnorm=np.empty(T, np.float32), logits=np.empty((T, E), np.float64),
               ambiguous=np.empty(T, np.uint8))
    rc = lib().oracle_route(_p(x), _dtype_of(x), T, d, _p(Wr), E, _p(e2s), int(gate_mode),
                            _p(out["orig_expert"]), _p(out["orig_gate"]), _p(out["slot"]),
                            _p(out["gate"]), _p(out["xnorm"]), _p(out["logits"]),
                            _p(out["ambiguous"]), C.c_double(margin))
    if rc:
        raise ValueError(f"oracle_route rc={rc}")
    out["ambiguous"] = out["ambiguous"].astype(bool)
    return out


def expert_norm(W1, W2):
    """|E_i| for each expert of a bank: W1 [n,d,f], W2 [n,f,d] -> float64 [n]."""
    W1 = _c(W1); W2 = _c(W2)
    n, d, f = W1.shape
    assert W2.shape == (n, f, d) and W1.dtype == W2.dtype
    out = np.empty(n, np.float64)
    rc = lib().oracle_expert_norm(_p(W1), _p(W2), _dtype_of(W1), n, d, f, _p(out))
    assert rc == 0
    return out


def importance(orig_expert, orig_gate, xnorm, expert_norm_, state=None):
    """Returns (count int32 [E], gsum f64 [E], score f64 [E]); if `state` (a
    previous return value) is given, accumulates into copies of it."""
    oe = _c(orig_expert, np.int32); og = _c(orig_gate, np.float32); xn = _c(xnorm, np.float32)
    en = _c(expert_norm_, np.float64)
    E = en.shape[0]
    if state is None:
        count, gsum, score = np.zeros(E, np.int32), np.zeros(E, np.float64), np.zeros(E, np.float64)
        acc = 0
    else:
        count, gsum, score = (np.array(s, copy=True) for s in state)
        acc = 1
    rc = lib().oracle_importance(_p(oe), _p(og), _p(xn), oe.shape[0], _p(en), E,
                                 _p(count), _p(gsum), _p(score), acc)
    if rc:
        raise ValueError(f"oracle_importance rc={rc}")
    return count, gsum, score


def permute(x, slot, K):
    """Returns (x_perm, perm, inv_perm, offsets).  x may be None."""
    slot = _c(slot, np.int32)
    T = slot.shape[0]
    perm = np.empty(T, np.int32); inv = np.empty(T, np.int32); offsets = np.empty(K + 1, np.int32)
    if x is not None:
        x = _c(x)
        xp = np.empty_like(x)
        row_bytes = x.strides[0] if T else 0
    else:
        xp, row_bytes = None, 0
    rc = lib().oracle_permute(_p(x), C.c_size_t(row_bytes), _p(slot), T, K, _p(xp), _p(perm),
                              _p(inv), _p(offsets))
    if rc:
        raise ValueError(f"oracle_permute rc={rc}")
    return xp, perm, inv, offsets


def expert_ffn(x_perm, W1, W2, offsets, rows=None):
    """y [T,d] float64 (unrounded).  W1 [K,d,f], W2 [K,f,d] are the SLOT arrays.
    With `rows`, only those rows are computed; the others are NaN."""
    xp = _c(x_perm); W1 = _c(W1); W2 = _c(W2); offsets = _c(offsets, np.int32)
    T, d = xp.shape
    K, d1, f = W1.shape
    assert d1 == d and W2.shape == (K, f, d) and offsets.shape == (K + 1,)
    y = np.full((T, d), np.nan, np.float64)
    if rows is not None:
        rows = _c(rows, np.int32)
        assert rows.size == 0 or (rows.min() >= 0 and rows.max() < T)
    rc = lib().oracle_expert_ffn(_p(xp), _dtype_of(xp), _p(W1), _p(W2), _dtype_of(W1), _p(offsets),
                                 K, d, f, T, _p(rows), 0 if rows is None else rows.shape[0], _p(y))
    if rc:
        raise ValueError(f"oracle_expert_ffn rc={rc}")
    return y


def combine(y_perm, inv_perm, gate, out_dtype, residual=None):
    """out [T,d] in out_dtype storage (fp32 / bf16 bits / fp64)."""
    y = _c(y_perm); inv = _c(inv_perm, np.int32); gate = _c(gate, np.float32)
    T, d = y.shape
    np_dt = {F32: np.float32, BF16: np.uint16, F64: np.float64}[out_dtype]
    out = np.empty((T, d), np_dt)
    res = None if residual is None else _c(residual)
    rc = lib().oracle_combine(_p(y), _dtype_of(y), _p(inv), _p(gate), _p(res),
                              0 if res is None else _dtype_of(res), T, d, _p(out), out_dtype)
    assert rc == 0
    return out


def select_resident(score, slot_to_expert, expert_to_slot):
    """Applies the update rule to copies of the maps.
    Returns (slot_to_expert, expert_to_slot, [(slot, expert), ...] to load)."""
    score = _c(score, np.float64)
    s2e = np.array(slot_to_expert, np.int32, copy=True)
    e2s = np.array(expert_to_slot, np.int32, copy=True)
    K, E = s2e.shape[0], e2s.shape[0]
    cs = np.empty(K, np.int32); ce = np.empty(K, np.int32)
    n = lib().oracle_select_resident(_p(score), E, K, _p(s2e), _p(e2s), _p(cs), _p(ce))
    if n < 0:
        raise ValueError(f"oracle_select_resident rc={n}")
    return s2e, e2s, [(int(cs[i]), int(ce[i])) for i in range(n)]


POLICY_IMPORTANCE, POLICY_COUNT, POLICY_MAGNITUDE = 0, 1, 2


def policy_scores(policy, count, score, expert_norm_):
    """What ranks the experts at an update under `policy` (float64 [E])."""
    count = _c(count, np.int32); score = _c(score, np.float64); en = _c(expert_norm_, np.float64)
    rank = np.empty(en.shape[0], np.float64)
    rc = lib().oracle_policy_scores(int(policy), en.shape[0], _p(count), _p(score), _p(en), _p(rank))
    if rc:
        raise ValueError(f"oracle_policy_scores rc={rc}")
    return rank


class OnDemand:
    """State of the load-on-miss baseline: a batch counter and per-slot use stamps."""

    def __init__(self, K):
        self.clock = np.zeros(1, np.int64)
        self.last_use = np.zeros(K, np.int64)

    def plan(self, orig_expert, expert_to_slot):
        """[(slot, expert), ...] to load after a batch with these original choices."""
        oe = _c(orig_expert, np.int32); e2s = _c(expert_to_slot, np.int32)
        K = self.last_use.shape[0]
        cs = np.empty(K, np.int32); ce = np.empty(K, np.int32)
        n = lib().oracle_on_demand(_p(oe), oe.shape[0], e2s.shape[0], K, _p(e2s), _p(self.clock),
                                   _p(self.last_use), _p(cs), _p(ce))
        if n < 0:
            raise ValueError(f"oracle_on_demand rc={n}")
        return [(int(cs[i]), int(ce[i])) for i in range(n)]


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def round_bf16(a):
    a = _c(a, np.float64)
    out = np.empty(a.shape, np.uint16)
    lib().oracle_round_bf16(_p(a), C.c_size_t(a.size), _p(out))
    return out


def layer_forward(x, Wr, W1_slots, W2_slots, expert_to_slot, gate_mode=GATE_FULL, out_dtype=None,
                  residual=None):
    """One whole layer, the steps chained with nothing rounded in between
    except what the interfaces fix (gates and norms are fp32 values).
    Returns a dict with every intermediate."""
    K = W1_slots.shape[0]
    r = route(x, Wr, expert_to_slot, gate_mode)
    xp, perm, inv, offsets = permute(x, r["slot"], K)
    y = expert_ffn(xp, W1_slots, W2_slots, offsets)
    od = _dtype_of(np.ascontiguousarray(x)) if out_dtype is None else out_dtype
    out = combine(y, inv, r["gate"], od, residual)
    r.update(x_perm=xp, perm=perm, inv_perm=inv, offsets=offsets, y_perm=y, out=out)
    return r
