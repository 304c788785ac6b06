"""ctypes binding of libswapmoe: argument marshalling only.

Every function here has the name and argument order of the C entry point it
calls (include/swapmoe.h) and does nothing but turn torch tensors into device
pointers, pass the current HIP stream, and raise on a non-zero status.  PyTorch
supplies device memory and streams; no arithmetic of the layer happens in
Python, and there is no fallback: importing this module fails if the HIP
library has not been built.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# SMOE_LIBRARY points at another build of the same library (e.g. an instrumented one)
LIB_PATH = os.environ.get("SMOE_LIBRARY") or os.path.join(_HERE, "libswapmoe.so")

SMOE_OK, SMOE_EINVAL, SMOE_ESTATE, SMOE_EHIP, SMOE_ENOMEM = 0, -1, -2, -3, -4
SMOE_F32, SMOE_BF16 = 0, 1
SMOE_GATE_FULL, SMOE_GATE_RENORM = 0, 1
SMOE_POLICY_IMPORTANCE, SMOE_POLICY_COUNT, SMOE_POLICY_MAGNITUDE = 0, 1, 2

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first (python -m paper_2308_15030_amd.build, or "
        "__graft_entry__.build()).  There is no CPU or PyTorch fallback for this library.")

_lib = C.CDLL(LIB_PATH)


class smoe_config(C.Structure):
    _fields_ = [("E", C.c_int32), ("K", C.c_int32), ("d_model", C.c_int32), ("d_ff", C.c_int32),
                ("max_tokens", C.c_int32), ("dtype", C.c_int32), ("gate_mode", C.c_int32),
                ("spare_slots", C.c_int32)]


_vp, _i = C.c_void_p, C.c_int
_SIGS = {
    "smoe_create": (C.c_int, [C.POINTER(smoe_config), C.POINTER(_vp)]),
    "smoe_destroy": (C.c_int, [_vp]),
    "smoe_last_error": (C.c_char_p, []),
    "smoe_workspace_bytes": (C.c_size_t, [_vp]),
    "smoe_slot_weight_bytes": (C.c_size_t, [_vp]),
    "smoe_bind": (C.c_int, [_vp, _vp, _vp, _vp, _vp, _vp]),
    "smoe_expert_norm": (C.c_int, [_vp, _vp, _vp, _i, _vp, _vp]),
    "smoe_set_resident": (C.c_int, [_vp, _i, _i, _vp, _vp, _vp]),
    "smoe_get_maps": (C.c_int, [_vp, _vp, _vp]),
    "smoe_select_resident": (C.c_int, [_vp, _vp, _vp, _vp]),
    "smoe_update_begin": (C.c_int, [_vp, _vp]),
    "smoe_update_tick": (C.c_int, [_vp, _vp, _vp, _vp, _vp]),
    "smoe_update_pending": (C.c_int, [_vp]),
    "smoe_route": (C.c_int, [_vp, _vp, _i, _vp, _vp, _vp, _vp, _vp, _vp]),
    "smoe_importance": (C.c_int, [_vp, _vp, _vp, _vp, _i, _vp, _vp, _vp, _i, _vp]),
    "smoe_permute": (C.c_int, [_vp, _vp, _vp, _i, _vp, _vp, _vp, _vp, _vp]),
    "smoe_permute_static": (C.c_int, [_vp, _vp, _vp, _i, _vp, _vp, _vp, _vp, _vp]),
    "smoe_expert_ffn": (C.c_int, [_vp, _vp, _vp, _i, _vp, _vp]),
    "smoe_combine": (C.c_int, [_vp, _vp, _vp, _vp, _vp, _i, _vp, _vp]),
    "smoe_set_profile_events": (C.c_int, [_vp, _vp, _vp, _vp, _vp]),
    "smoe_policy_scores": (C.c_int, [_i, _i, _vp, _vp, _vp, _vp]),
    "smoe_on_demand_plan": (C.c_int, [_vp, _vp, _i, _vp, _vp]),
    "smoe_profile_memory": (C.c_int, [C.POINTER(smoe_config), _vp]),
    "smoe_profile_begin": (C.c_int, [_vp, _vp]),
    "smoe_profile_end": (C.c_int, [_vp, _vp, C.POINTER(C.c_float)]),
    "smoe_period_inflection": (C.c_int, [_vp, _i, C.c_float]),
    "smoe_describe_ffn": (C.c_int, [_vp, _i, _i, C.c_char_p, C.c_size_t]),
    "smoe_update_on_device": (C.c_int, [_vp, _vp, _vp, _vp, _vp]),
    "smoe_profile_stream_read": (C.c_int, [_vp, _i, _vp]),
    "smoe_forward": (C.c_int, [_vp, _vp, _i, _vp, _vp, _i] + [_vp] * 12),
}
EXPORTS = tuple(_SIGS)
for _name, (_res, _args) in _SIGS.items():
    _fn = getattr(_lib, _name)
    _fn.restype, _fn.argtypes = _res, _args


class SmoeError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"libswapmoe status {status}: {message}")
        self.status = status


def smoe_last_error() -> str:
    return _lib.smoe_last_error().decode()


def _check(rc: int) -> int:
    if rc < 0:
        raise SmoeError(rc, smoe_last_error())
    return rc


def _ptr(t):
    """Device (or host) address of a tensor / numpy array; None -> NULL."""
    if t is None:
        return None
    if isinstance(t, torch.Tensor):
        return t.data_ptr()
    return t.ctypes.data


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def smoe_create(E, K, d_model, d_ff, max_tokens, dtype, gate_mode=SMOE_GATE_FULL, spare_slots=0):
    cfg = smoe_config(E, K, d_model, d_ff, max_tokens, dtype, gate_mode, spare_slots)
    h = _vp()
    _check(_lib.smoe_create(C.byref(cfg), C.byref(h)))
    return h


def smoe_destroy(layer):
    _check(_lib.smoe_destroy(layer))


def smoe_workspace_bytes(layer) -> int:
    return _lib.smoe_workspace_bytes(layer)


def smoe_slot_weight_bytes(layer) -> int:
    return _lib.smoe_slot_weight_bytes(layer)


def smoe_bind(layer, router_w, slot_w1, slot_w2, expert_norm, workspace):
    _check(_lib.smoe_bind(layer, _ptr(router_w), _ptr(slot_w1), _ptr(slot_w2), _ptr(expert_norm),
                          _ptr(workspace)))


def smoe_expert_norm(layer, w1, w2, n, out, stream=None):
    _check(_lib.smoe_expert_norm(layer, _ptr(w1), _ptr(w2), n, _ptr(out), _stream(stream)))


def smoe_set_resident(layer, slot, expert, w1_src, w2_src, stream=None):
    _check(_lib.smoe_set_resident(layer, slot, expert, _ptr(w1_src), _ptr(w2_src), _stream(stream)))


def smoe_get_maps(layer, slot_to_expert, expert_to_slot):
    _check(_lib.smoe_get_maps(layer, _ptr(slot_to_expert), _ptr(expert_to_slot)))


def smoe_select_resident(layer, score, changed_slots, changed_experts) -> int:
    return _check(_lib.smoe_select_resident(layer, _ptr(score), _ptr(changed_slots), _ptr(changed_experts)))


def smoe_route(layer, x, T, orig_expert, orig_gate, slot, gate, xnorm, stream=None):
    _check(_lib.smoe_route(layer, _ptr(x), T, _ptr(orig_expert), _ptr(orig_gate), _ptr(slot), _ptr(gate),
                           _ptr(xnorm), _stream(stream)))


def smoe_importance(layer, orig_expert, orig_gate, xnorm, T, count, gsum, score, accumulate, stream=None):
    _check(_lib.smoe_importance(layer, _ptr(orig_expert), _ptr(orig_gate), _ptr(xnorm), T, _ptr(count),
                                _ptr(gsum), _ptr(score), int(accumulate), _stream(stream)))


def smoe_permute(layer, x, slot, T, x_perm, perm, inv_perm, offsets, stream=None):
    _check(_lib.smoe_permute(layer, _ptr(x), _ptr(slot), T, _ptr(x_perm), _ptr(perm), _ptr(inv_perm),
                             _ptr(offsets), _stream(stream)))


def smoe_permute_static(layer, x, slot, T, x_perm, perm, inv_perm, offsets, stream=None):
    _check(_lib.smoe_permute_static(layer, _ptr(x), _ptr(slot), T, _ptr(x_perm), _ptr(perm), _ptr(inv_perm),
                                    _ptr(offsets), _stream(stream)))


def smoe_expert_ffn(layer, x_perm, offsets, T, y_perm, stream=None):
    _check(_lib.smoe_expert_ffn(layer, _ptr(x_perm), _ptr(offsets), T, _ptr(y_perm), _stream(stream)))


def smoe_combine(layer, y_perm, inv_perm, gate, residual, T, out, stream=None):
    _check(_lib.smoe_combine(layer, _ptr(y_perm), _ptr(inv_perm), _ptr(gate), _ptr(residual), T,
                             _ptr(out), _stream(stream)))


def smoe_forward(layer, x, T, residual, out, accumulate, orig_expert, orig_gate, slot, gate, xnorm, count,
                 gsum, score, perm, inv_perm, offsets, stream=None):
    _check(_lib.smoe_forward(layer, _ptr(x), T, _ptr(residual), _ptr(out), int(accumulate), _ptr(orig_expert),
                             _ptr(orig_gate), _ptr(slot), _ptr(gate), _ptr(xnorm), _ptr(count), _ptr(gsum),
                             _ptr(score), _ptr(perm), _ptr(inv_perm), _ptr(offsets), _stream(stream)))


def smoe_set_profile_events(layer, g1_begin, g1_end, g2_begin, g2_end):
    """Events are torch.cuda.Event(enable_timing=True) objects (or None)."""
    def h(e):
        if e is None:
            return None
        if e.cuda_event == 0:      # torch creates the HIP event lazily, on first record
            e.record()
        return e.cuda_event
    _check(_lib.smoe_set_profile_events(layer, h(g1_begin), h(g1_end), h(g2_begin), h(g2_end)))


# ---------------------------------------------------------------------------
# Buffer plumbing: one object that owns the torch allocations a layer needs.
# ---------------------------------------------------------------------------

def _act_dtype(dtype):
    # bf16 activations travel as raw bit patterns so host-side test data can be
    # handed over unchanged
    return torch.float32 if dtype == SMOE_F32 else torch.int16


class smoe_memory_profile(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("expert_bytes", "resident_bytes", "workspace_bytes", "bank_bytes",
                                          "router_bytes")]


def smoe_policy_scores(policy, E, count, score, expert_norm, rank):
    _check(_lib.smoe_policy_scores(policy, E, _ptr(count), _ptr(score), _ptr(expert_norm), _ptr(rank)))


def smoe_on_demand_plan(layer, orig_expert_host, T, changed_slots, changed_experts) -> int:
    return _check(_lib.smoe_on_demand_plan(layer, _ptr(orig_expert_host), T, _ptr(changed_slots),
                                           _ptr(changed_experts)))


def smoe_profile_memory(E, K, d_model, d_ff, max_tokens, dtype, gate_mode=SMOE_GATE_FULL, spare_slots=0) -> dict:
    cfg = smoe_config(E, K, d_model, d_ff, max_tokens, dtype, gate_mode, spare_slots)
    out = smoe_memory_profile()
    _check(_lib.smoe_profile_memory(C.byref(cfg), C.byref(out)))
    return {n: int(getattr(out, n)) for n, _ in smoe_memory_profile._fields_}


def smoe_profile_begin(layer, stream=None):
    _check(_lib.smoe_profile_begin(layer, _stream(stream)))


def smoe_profile_end(layer, stream=None) -> float:
    us = C.c_float(0.0)
    _check(_lib.smoe_profile_end(layer, _stream(stream), C.byref(us)))
    return float(us.value)


def smoe_profile_stream_read(layer, which, stream=None):
    _check(_lib.smoe_profile_stream_read(layer, int(which), _stream(stream)))


def smoe_period_inflection(latency_us, tolerance) -> int:
    import numpy as np
    lat = np.ascontiguousarray(latency_us, np.float32)
    return _check(_lib.smoe_period_inflection(_ptr(lat), int(lat.shape[0]), C.c_float(tolerance)))


def smoe_describe_ffn(layer, T, fused=True) -> str:
    buf = C.create_string_buffer(256)
    _check(_lib.smoe_describe_ffn(layer, T, int(fused), buf, 256))
    return buf.value.decode()


def smoe_update_on_device(layer, score_dev, bank_w1, bank_w2, stream=None):
    _check(_lib.smoe_update_on_device(layer, _ptr(score_dev), _ptr(bank_w1), _ptr(bank_w2), _stream(stream)))


def smoe_update_begin(layer, score_host) -> int:
    return _check(_lib.smoe_update_begin(layer, _ptr(score_host)))


def smoe_update_tick(layer, bank_w1, bank_w2, load_stream, compute_stream=None) -> int:
    return _check(_lib.smoe_update_tick(layer, _ptr(bank_w1), _ptr(bank_w2), _stream(load_stream),
                                              _stream(compute_stream)))


def smoe_update_pending(layer) -> int:
    return _check(_lib.smoe_update_pending(layer))


class Layer:
    """Handle + the device buffers it is bound to + reusable output buffers.

    Methods only allocate (once) and marshal; each maps to one C entry point.
    """

    def __init__(self, E, K, d_model, d_ff, max_tokens, dtype, gate_mode=SMOE_GATE_FULL,
                 router_w=None, expert_norm=None, device="cuda:0", spare_slots=0):
        self.E, self.K, self.d_model, self.d_ff = E, K, d_model, d_ff
        self.max_tokens, self.dtype, self.gate_mode = max_tokens, dtype, gate_mode
        self.device = torch.device(device)
        self.spare_slots = spare_slots
        self.handle = smoe_create(E, K, d_model, d_ff, max_tokens, dtype, gate_mode, spare_slots)
        dev = self.device
        nb = smoe_slot_weight_bytes(self.handle)
        self.slot_w1 = torch.empty(nb, dtype=torch.uint8, device=dev)
        self.slot_w2 = torch.empty(nb, dtype=torch.uint8, device=dev)
        self.workspace = torch.empty(smoe_workspace_bytes(self.handle), dtype=torch.uint8, device=dev)
        self.router_w = (torch.zeros(E, d_model, dtype=torch.float32, device=dev) if router_w is None
                         else router_w.to(dev, torch.float32).contiguous())
        self.expert_norm = (torch.ones(E, dtype=torch.float32, device=dev) if expert_norm is None
                            else expert_norm.to(dev, torch.float32).contiguous())
        smoe_bind(self.handle, self.router_w, self.slot_w1, self.slot_w2, self.expert_norm, self.workspace)
        T, act = max_tokens, _act_dtype(dtype)
        i32, f32 = torch.int32, torch.float32
        self.orig_expert = torch.empty(T, dtype=i32, device=dev)
        self.orig_gate = torch.empty(T, dtype=f32, device=dev)
        self.slot = torch.empty(T, dtype=i32, device=dev)
        self.gate = torch.empty(T, dtype=f32, device=dev)
        self.xnorm = torch.empty(T, dtype=f32, device=dev)
        self.count = torch.zeros(E, dtype=i32, device=dev)
        self.gsum = torch.zeros(E, dtype=f32, device=dev)
        self.score = torch.zeros(E, dtype=f32, device=dev)
        self.x_perm = torch.empty(T, d_model, dtype=act, device=dev)
        self.perm = torch.empty(T, dtype=i32, device=dev)
        self.inv_perm = torch.empty(T, dtype=i32, device=dev)
        self.offsets = torch.empty(K + 1, dtype=i32, device=dev)
        self.y_perm = torch.empty(T, d_model, dtype=act, device=dev)
        self.out = torch.empty(T, d_model, dtype=act, device=dev)

    def rebind(self):
        """Binds the same buffers again: every slot becomes empty."""
        smoe_bind(self.handle, self.router_w, self.slot_w1, self.slot_w2, self.expert_norm, self.workspace)

    def close(self):
        if self.handle is not None:
            smoe_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # one method per entry point ------------------------------------------------
    def expert_norm_of(self, w1_bank, w2_bank):
        n = w1_bank.shape[0]
        out = torch.empty(n, dtype=torch.float32, device=self.device)
        smoe_expert_norm(self.handle, w1_bank, w2_bank, n, out)
        return out

    def set_resident(self, slot, expert, w1_src, w2_src):
        smoe_set_resident(self.handle, slot, expert, w1_src, w2_src)

    def update_on_device(self, bank_w1, bank_w2, score=None):
        """Update rule and slot loads on the device, from self.score unless another ranking is given."""
        smoe_update_on_device(self.handle, self.score if score is None else score, bank_w1, bank_w2)

    def maps(self):
        import numpy as np
        s2e = np.empty(self.K, np.int32)
        e2s = np.empty(self.E, np.int32)
        smoe_get_maps(self.handle, s2e, e2s)
        return s2e, e2s

    def select_resident(self, score_host):
        import numpy as np
        score_host = np.ascontiguousarray(score_host, np.float32)
        cs = np.empty(self.K, np.int32)
        ce = np.empty(self.K, np.int32)
        n = smoe_select_resident(self.handle, score_host, cs, ce)
        return [(int(cs[i]), int(ce[i])) for i in range(n)]

    def policy_rank(self, policy):
        """Host copy of what `policy` ranks the experts by (one read-back of E numbers)."""
        import numpy as np
        rank = np.empty(self.E, np.float32)
        src = {SMOE_POLICY_IMPORTANCE: self.score, SMOE_POLICY_COUNT: self.count,
               SMOE_POLICY_MAGNITUDE: self.expert_norm}[policy].cpu().numpy()
        smoe_policy_scores(policy, self.E, src if policy == SMOE_POLICY_COUNT else None,
                           src if policy == SMOE_POLICY_IMPORTANCE else None,
                           src if policy == SMOE_POLICY_MAGNITUDE else None, rank)
        return rank

    def on_demand_plan(self, T):
        """Load-on-miss plan for the batch just served (reads back its orig_expert)."""
        import numpy as np
        oe = self.orig_expert[:T].cpu().numpy()
        cs = np.empty(self.K, np.int32)
        ce = np.empty(self.K, np.int32)
        n = smoe_on_demand_plan(self.handle, oe, T, cs, ce)
        return [(int(cs[i]), int(ce[i])) for i in range(n)]

    def update_begin(self, score_host):
        import numpy as np
        return smoe_update_begin(self.handle, np.ascontiguousarray(score_host, np.float32))

    def update_tick(self, bank_w1, bank_w2, load_stream):
        return smoe_update_tick(self.handle, bank_w1, bank_w2, load_stream)

    def update_pending(self):
        return smoe_update_pending(self.handle)

    def route(self, x, T):
        smoe_route(self.handle, x, T, self.orig_expert, self.orig_gate, self.slot, self.gate, self.xnorm)

    def importance(self, T, accumulate):
        smoe_importance(self.handle, self.orig_expert, self.orig_gate, self.xnorm, T, self.count,
                        self.gsum, self.score, accumulate)

    def permute(self, x, T):
        smoe_permute(self.handle, x, self.slot, T, self.x_perm, self.perm, self.inv_perm, self.offsets)

    def expert_ffn(self, T):
        smoe_expert_ffn(self.handle, self.x_perm, self.offsets, T, self.y_perm)

    def combine(self, T, residual=None, out=None):
        smoe_combine(self.handle, self.y_perm, self.inv_perm, self.gate, residual, T,
                     self.out if out is None else out)

    def forward_fused(self, x, T, accumulate=1, residual=None, out=None):
        """The whole hot path through the single-call entry point (bf16 layers)."""
        out = self.out if out is None else out
        smoe_forward(self.handle, x, T, residual, out, accumulate, self.orig_expert, self.orig_gate, self.slot,
                     self.gate, self.xnorm, self.count, self.gsum, self.score, self.perm, self.inv_perm,
                     self.offsets)
        return out

    def forward(self, x, T, accumulate=1, residual=None, out=None):
        """The whole hot path as the five per-step calls on the current stream."""
        self.route(x, T)
        self.importance(T, accumulate)
        self.permute(x, T)
        self.expert_ffn(T)
        self.combine(T, residual, out)
        return self.out if out is None else out
