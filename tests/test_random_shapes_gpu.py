"""Seeded sweep over layer shapes that no other test names: expert counts that
are not multiples of 32, widths that do not fill a workgroup tile, batches on
both sides of the 32-token boundary, both gate modes, with and without a
residual.  Each case checks the single-call path against the oracle (integers
exactly, the output within the bf16 bar) and against the five separate calls
(every output, bit for bit)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2308_15030_amd import workloads as wl
from harness import Case, max_abs_rel, to_dev, to_host, values

pytestmark = pytest.mark.gpu

NAMES = ("orig_expert", "orig_gate", "slot", "gate", "xnorm", "count", "gsum", "score", "perm", "inv_perm",
         "offsets", "out")


def _cases():
    rng = np.random.default_rng(20230815)
    Ts = [1, 17, 32, 33, 130, 700, 1500, 2049]
    out = []
    for i in range(16):
        E = int(rng.choice([4, 8, 16, 33, 64, 130, 200]))
        out.append(dict(E=E, K=int(rng.integers(1, min(E, 24) + 1)), d=int(rng.choice([32, 64, 96, 160, 256, 384])),
                        f=int(rng.choice([32, 96, 224, 512, 1024])), T=Ts[i % len(Ts)], gate_mode=int(rng.integers(0, 2)),
                        residual=bool(rng.integers(0, 2)), perm_seed=int(rng.integers(1 << 30)), seed=3000 + i))
    # more 32-token blocks than compute units: the router takes two blocks per workgroup
    out.append(dict(E=16, K=5, d=64, f=96, T=8300, gate_mode=0, residual=True, perm_seed=11, seed=3100))
    out.append(dict(E=100, K=9, d=96, f=64, T=8211, gate_mode=1, residual=False, perm_seed=12, seed=3101))
    return out


@pytest.mark.parametrize("p", _cases(), ids=lambda p: f"E{p['E']}-K{p['K']}-d{p['d']}-f{p['f']}-T{p['T']}")
def test_random_shape(p):
    cfg = wl.MoEConfig("rand", E=p["E"], K=p["K"], d_model=p["d"], d_ff=p["f"], T=p["T"], dtype=wl.BF16, seed=p["seed"])
    resident = list(map(int, np.random.default_rng(p["perm_seed"]).permutation(p["E"])[:p["K"]]))
    c = Case(cfg, resident=resident, router_scale=20.0, gate_mode=p["gate_mode"])
    L, T = c.L, c.T
    res_host = c.x if p["residual"] else None
    res_dev = to_dev(c.x) if p["residual"] else None
    ref = oracle.layer_forward(c.x, c.Wr, *c.slot_weights_host(), c.e2s, p["gate_mode"], residual=res_host)
    st = oracle.importance(ref["orig_expert"], ref["orig_gate"], ref["xnorm"], c.en_oracle)
    out = L.forward_fused(c.d_x, T, accumulate=0, residual=res_dev)
    torch.cuda.synchronize()
    ok = ~ref["ambiguous"]
    assert np.array_equal(to_host(L.orig_expert)[:T][ok], ref["orig_expert"][ok])
    assert np.array_equal(to_host(L.slot)[:T][ok], ref["slot"][ok])
    np.testing.assert_allclose(to_host(L.gate)[:T][ok], ref["gate"][ok], rtol=1e-5)
    np.testing.assert_allclose(to_host(L.xnorm)[:T], ref["xnorm"], rtol=1e-5)
    if ok.all():   # the permutation is unique only when every token's choice is
        assert np.array_equal(to_host(L.perm)[:T], ref["perm"])
        assert np.array_equal(to_host(L.inv_perm)[:T], ref["inv_perm"])
        assert np.array_equal(to_host(L.offsets), ref["offsets"])
        assert np.array_equal(to_host(L.count), st[0])
        np.testing.assert_allclose(to_host(L.score), st[2], rtol=1e-4, atol=1e-30)
    assert max_abs_rel(values(to_host(out)[:T], cfg.dtype)[ok], values(ref["out"], cfg.dtype)[ok]) <= 2e-2
    # the separate calls give the same bits
    got = {n: to_host(getattr(L, n)).copy() for n in NAMES}
    for n in NAMES:
        getattr(L, n).fill_(0)
    L.forward(c.d_x, T, accumulate=0, residual=res_dev)
    torch.cuda.synchronize()
    for n in NAMES:
        assert np.array_equal(to_host(getattr(L, n)), got[n]), n
    L.close()
