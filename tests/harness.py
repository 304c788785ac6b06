"""Shared plumbing of the GPU parity tests: builds a HIP layer and the oracle's
view of the same seeded workload.  Holds no arithmetic of the method."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2308_15030_amd import workloads as wl


def to_dev(a: np.ndarray, device="cuda:0"):
    """numpy (fp32 / uint16 bf16 bits / int32) -> device tensor with the same bits."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def to_host(t: torch.Tensor) -> np.ndarray:
    a = t.detach().cpu().numpy()
    return a.view(np.uint16) if a.dtype == np.int16 else a


def values(a: np.ndarray, dtype: int) -> np.ndarray:
    """Storage array -> float64 values."""
    return wl.as_f32(a, dtype).astype(np.float64)


def max_abs_rel(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / max |ref| over the whole tensor."""
    if ref.size == 0:
        return 0.0
    scale = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (scale if scale > 0 else 1.0))


class Case:
    """One layer of a workload on both sides.

    resident: slot -> expert list (default: the config's initial set).  Only
    the experts in `bank_experts` (default: the resident ones) are generated.
    """

    def __init__(self, cfg: wl.MoEConfig, layer: int = 0, resident=None, bank_experts=None,
                 gate_mode=0, x=None, router_scale=1.0, device="cuda:0", spare_slots=0):
        from paper_2308_15030_amd import binding as b
        self.b = b
        self.cfg, self.layer_idx = cfg, layer
        self.Wr = (wl.router_weights(cfg, layer) * np.float32(router_scale)).astype(np.float32)
        s2e0, _ = wl.initial_resident(cfg)
        self.s2e = np.array(s2e0 if resident is None else resident, np.int32)
        self.e2s = np.full(cfg.E, -1, np.int32)
        self.e2s[self.s2e] = np.arange(cfg.K, dtype=np.int32)
        self.bank_ids = list(self.s2e) if bank_experts is None else list(bank_experts)
        W1, W2 = wl.expert_bank(cfg, layer, self.bank_ids)
        self.bank_pos = {int(e): i for i, e in enumerate(self.bank_ids)}
        self.W1_bank, self.W2_bank = W1, W2                   # host, bank layout, storage dtype
        self.x = wl.hidden_states(cfg, layer) if x is None else x
        self.T = self.x.shape[0]
        self.gate_mode = gate_mode
        self.dev = device
        self.d_W1 = to_dev(W1, device)
        self.d_W2 = to_dev(W2, device)
        self.d_x = to_dev(self.x, device) if self.T else torch.empty(0, cfg.d_model, device=device)
        # |E_i| for the experts we hold; 1.0 elsewhere (never used by the tests)
        self.en_oracle = np.ones(cfg.E, np.float64)
        self.en_oracle[self.bank_ids] = oracle.expert_norm(W1, W2)
        self.L = b.Layer(cfg.E, cfg.K, cfg.d_model, cfg.d_ff, max(self.T, 1), cfg.dtype, gate_mode,
                         router_w=torch.from_numpy(self.Wr), device=device, spare_slots=spare_slots)
        en_dev = self.L.expert_norm_of(self.d_W1, self.d_W2)
        full = torch.ones(cfg.E, dtype=torch.float32, device=device)
        full[torch.tensor(self.bank_ids, device=device)] = en_dev
        self.L.expert_norm.copy_(full)
        for s, e in enumerate(self.s2e):
            self.load(s, int(e))

    def load(self, slot: int, expert: int):
        i = self.bank_pos[expert]
        self.L.set_resident(slot, expert, self.d_W1[i], self.d_W2[i])

    def slot_weights_host(self):
        idx = [self.bank_pos[int(e)] for e in self.s2e]
        return self.W1_bank[idx], self.W2_bank[idx]

    def oracle_route(self):
        return oracle.route(self.x, self.Wr, self.e2s, self.gate_mode)
