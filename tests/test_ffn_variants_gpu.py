"""Every tile shape of the bf16 expert FFN against the oracle.

The library picks the tile shapes of the two products from the batch size; the
shapes that small test batches never select are forced here through
SMOE_FFN_VARIANT (read once, at smoe_create), so that each kernel instance a
caller can reach is compared with the oracle: teacher-forced smoe_expert_ffn on
the sorted rows, and the fused single-call layer (gather in the first product,
gate / residual scatter in the second).  Tolerances as in test_parity_gpu.py.
"""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2308_15030_amd import workloads as wl
from harness import Case, max_abs_rel, to_dev, to_host, values

pytestmark = pytest.mark.gpu

# indices of launch_variant in csrc/ffn_bf16.hip: (first product, second product).  (10, 10) and
# (8, 10) run the 256-row tile as the second product: its output turn handles more pieces per
# thread than fit one group, and the short last group once ran past the tile.
PAIRS = [(1, 1), (3, 3), (4, 4), (5, 5), (6, 6), (8, 8), (10, 1), (10, 8), (8, 3), (5, 6), (4, 6), (10, 10), (8, 10)]


@pytest.mark.parametrize("v1,v2", PAIRS)
# (d_model, d_ff): 160 makes the second product's reduction length no multiple of 64; 768 x 768 is the
# Switch-base reduction length (12 slices of 64) in both products
@pytest.mark.parametrize("d_model,d_ff", [(128, 256), (128, 160), (768, 768)])
def test_tile_variant(v1, v2, d_model, d_ff):
    cfg = wl.MoEConfig("variants", E=8, K=3, d_model=d_model, d_ff=d_ff, T=1000, dtype=wl.BF16, seed=31)
    os.environ["SMOE_FFN_VARIANT"] = f"{v1},{v2}"
    try:
        c = Case(cfg, resident=[5, 0, 6], router_scale=20.0)
    finally:
        del os.environ["SMOE_FFN_VARIANT"]
    L = c.L
    r = oracle.layer_forward(c.x, c.Wr, *c.slot_weights_host(), c.e2s)
    assert min(np.diff(r["offsets"])) > 0 and max(np.diff(r["offsets"])) > 256   # several row tiles and a ragged tail
    L.x_perm.copy_(to_dev(r["x_perm"])); L.offsets.copy_(to_dev(r["offsets"]))
    L.y_perm.fill_(0)
    L.expert_ffn(c.T)
    torch.cuda.synchronize()
    got = values(to_host(L.y_perm), cfg.dtype)
    for k in range(cfg.K):
        a, b_ = r["offsets"][k], r["offsets"][k + 1]
        assert max_abs_rel(got[a:b_], r["y_perm"][a:b_]) <= 2e-2, (v1, v2, k)
    ok = ~r["ambiguous"]
    out = L.forward_fused(c.d_x, c.T, accumulate=0)
    torch.cuda.synchronize()
    assert np.array_equal(to_host(L.perm), r["perm"]) or not ok.all()
    assert max_abs_rel(values(to_host(out), cfg.dtype)[ok], values(r["out"], cfg.dtype)[ok]) <= 2e-2
    # and with the residual stream: bit-identical to the separate calls under the same tile shapes
    res = to_dev(c.x)
    want = to_host(L.forward(c.d_x, c.T, accumulate=0, residual=res)).copy()
    L.out.fill_(0)
    got2 = to_host(L.forward_fused(c.d_x, c.T, accumulate=0, residual=res))
    torch.cuda.synchronize()
    assert np.array_equal(got2, want)
    L.close()
