"""smoe_permute_static, the entry point for callers that cannot allocate: its
sort histograms live in a fixed device array inside the library instead of a
bound workspace.  Through the C ABI, against smoe_permute on the same inputs,
bit for bit (indices and row copies are integer / byte work), on two calls in a
row -- the second with a smaller input, so stale contents of the shared array
from the first call would show -- and against the oracle's stable sort.  The
handle used for the static call is never bound to a workspace."""
import numpy as np
import pytest
import torch

import oracle
from paper_2308_15030_amd import binding as b
from paper_2308_15030_amd import workloads as wl
from harness import to_dev, to_host

pytestmark = pytest.mark.gpu


def _run_both(cfg, T, seed, bound, unbound, dev="cuda:0"):
    rng = np.random.default_rng(seed)
    # skewed slot popularity, one slot left empty
    p = np.arange(1, cfg.K + 1, dtype=np.float64) ** -1.1
    p[cfg.K // 2] = 0.0
    slot = rng.choice(cfg.K, size=T, p=p / p.sum()).astype(np.int32)
    x = wl.hidden_states(cfg.scaled(seed=seed), T=T)
    d_x, d_slot = to_dev(x, dev), to_dev(slot, dev)
    outs = []
    for static in (False, True):
        x_perm = torch.full((T, cfg.d_model), -1, dtype=torch.int16, device=dev)
        perm = torch.full((T,), -1, dtype=torch.int32, device=dev)
        inv = torch.full((T,), -1, dtype=torch.int32, device=dev)
        offsets = torch.full((cfg.K + 1,), -1, dtype=torch.int32, device=dev)
        if static:
            print(f"[no-alloc] smoe_permute_static T={T} K={cfg.K}", flush=True)
            b.smoe_permute_static(unbound, d_x, d_slot, T, x_perm, perm, inv, offsets)
        else:
            b.smoe_permute(bound.handle, d_x, d_slot, T, x_perm, perm, inv, offsets)
        torch.cuda.synchronize()
        outs.append([to_host(t).copy() for t in (x_perm, perm, inv, offsets)])
    for a, s_ in zip(*outs):
        assert np.array_equal(a, s_)
    xp, perm, inv, offsets = oracle.permute(x, slot, cfg.K)
    for got, want in zip(outs[1], (xp, perm, inv, offsets)):
        assert np.array_equal(got, want)


def test_static_permute_matches_permute_twice():
    cfg = wl.MoEConfig("no-alloc", E=64, K=24, d_model=256, d_ff=64, T=9000, dtype=wl.BF16, clusters=8, seed=41)
    bound = b.Layer(cfg.E, cfg.K, cfg.d_model, cfg.d_ff, cfg.T, cfg.dtype)
    unbound = b.smoe_create(cfg.E, cfg.K, cfg.d_model, cfg.d_ff, cfg.T, cfg.dtype)   # never bound: no workspace
    _run_both(cfg, 9000, 1, bound, unbound)          # 9 sort blocks
    _run_both(cfg, 2500, 2, bound, unbound)          # 3 blocks: entries 3..8 of the shared array are stale
    _run_both(cfg, 700, 3, bound, unbound)           # single block: the array is not touched at all
    # an empty batch still writes offsets = 0
    offsets = torch.full((cfg.K + 1,), -1, dtype=torch.int32, device="cuda:0")
    b.smoe_permute_static(unbound, None, None, 0, None, None, None, offsets)
    torch.cuda.synchronize()
    assert to_host(offsets).tolist() == [0] * (cfg.K + 1)
    b.smoe_destroy(unbound)
    bound.close()


def test_static_permute_rejects_sizes_beyond_its_array():
    big = b.smoe_create(8, 4, 64, 64, 1 << 20, b.SMOE_BF16)
    fake = 0x10000
    with pytest.raises(b.SmoeError) as e:
        b._check(b._lib.smoe_permute_static(big, fake, fake, 65537, fake, fake, fake, fake, None))
    assert e.value.status == b.SMOE_EINVAL and "65536" in str(e.value)
    b.smoe_destroy(big)
