"""GPU edge cases of the C ABI: empty and tiny inputs, empty segments, one
slot, handle state rules, slot refresh and replacement -- each against the
oracle, same tolerances as test_parity_gpu.py."""
import numpy as np
import pytest
import torch

import oracle
from paper_2308_15030_amd import workloads as wl
from harness import Case, max_abs_rel, to_dev, to_host, values

pytestmark = pytest.mark.gpu


def cfg_of(**kw):
    base = dict(E=8, K=4, d_model=64, d_ff=96, T=100, dtype=wl.BF16, seed=21)
    base.update(kw)
    return wl.MoEConfig("edge", **base)


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_zero_and_one_token(dtype):
    c = Case(cfg_of(dtype=dtype, T=1), router_scale=20.0)
    L = c.L
    # T = 0: every call is a legal no-op; permute still writes offsets = 0
    L.offsets.fill_(-7)
    L.route(c.d_x, 0); L.importance(0, 0); L.permute(c.d_x, 0); L.expert_ffn(0); L.combine(0)
    torch.cuda.synchronize()
    assert to_host(L.offsets).tolist() == [0] * (c.cfg.K + 1)
    assert to_host(L.count).sum() == 0 and to_host(L.score).sum() == 0
    # T = 1
    ref = oracle.layer_forward(c.x, c.Wr, *c.slot_weights_host(), c.e2s)
    out = L.forward(c.d_x, 1, accumulate=0)
    torch.cuda.synchronize()
    assert to_host(L.slot)[0] == ref["slot"][0]
    assert to_host(L.perm).tolist() == [0] and to_host(L.inv_perm).tolist() == [0]
    assert np.array_equal(to_host(L.offsets), ref["offsets"])
    tol = 1e-4 if dtype == wl.F32 else 2e-2
    assert max_abs_rel(values(to_host(out), dtype), values(ref["out"], dtype)) <= tol
    L.close()


def test_empty_segments_and_single_busy_slot():
    """Slots that get no token at all, and every token in one slot, with the
    layer created for more tokens than are passed."""
    cfg = cfg_of(T=333, K=4)
    c = Case(cfg.scaled(T=400), router_scale=20.0)       # max_tokens = 400 > T used
    L, T = c.L, 333
    x = c.x[:T]
    W1s, W2s = c.slot_weights_host()
    for pattern in ("two-empty", "one-slot"):
        slot = np.zeros(T, np.int32)
        if pattern == "two-empty":
            slot[::3] = 2                                  # slots 1 and 3 stay empty
        else:
            slot[:] = 3
        xp, perm, inv, offsets = oracle.permute(x, slot, cfg.K)
        L.slot[:T].copy_(to_dev(slot))
        L.permute(c.d_x, T)
        torch.cuda.synchronize()
        assert np.array_equal(to_host(L.offsets), offsets)
        assert np.array_equal(to_host(L.perm)[:T], perm)
        assert np.array_equal(to_host(L.inv_perm)[:T], inv)
        assert np.array_equal(to_host(L.x_perm)[:T], xp)
        y = oracle.expert_ffn(xp, W1s, W2s, offsets)
        L.expert_ffn(T)
        torch.cuda.synchronize()
        assert max_abs_rel(values(to_host(L.y_perm)[:T], cfg.dtype), y) <= 2e-2
    L.close()


def test_state_rules_and_slot_replacement():
    from paper_2308_15030_amd import binding as b
    cfg = cfg_of(T=64, K=2, E=6)
    c = Case(cfg, bank_experts=range(cfg.E), router_scale=20.0)
    L = c.L
    # a fresh handle bound to real buffers refuses route until both slots are filled
    L2 = b.Layer(cfg.E, cfg.K, cfg.d_model, cfg.d_ff, cfg.T, cfg.dtype, router_w=torch.from_numpy(c.Wr))
    with pytest.raises(b.SmoeError) as e:
        L2.route(c.d_x, cfg.T)
    assert e.value.status == b.SMOE_ESTATE
    L2.set_resident(0, 4, c.d_W1[4], c.d_W2[4])
    with pytest.raises(b.SmoeError):
        L2.expert_ffn(cfg.T)
    with pytest.raises(b.SmoeError) as e:
        L2.set_resident(1, 4, c.d_W1[4], c.d_W2[4])        # already resident in slot 0
    assert e.value.status == b.SMOE_ESTATE
    L2.set_resident(1, 1, c.d_W1[1], c.d_W2[1])
    L2.set_resident(0, 4, c.d_W1[4], c.d_W2[4])            # refresh of the same slot is legal
    s2e, e2s = L2.maps()
    assert s2e.tolist() == [4, 1] and e2s.tolist() == [-1, 1, -1, -1, 0, -1]
    L2.expert_norm.copy_(L.expert_norm)
    ref = oracle.layer_forward(c.x, c.Wr, c.W1_bank[[4, 1]], c.W2_bank[[4, 1]], e2s)
    out = L2.forward(c.d_x, cfg.T, accumulate=0)
    torch.cuda.synchronize()
    ok = ~ref["ambiguous"]
    assert np.array_equal(to_host(L2.slot)[ok], ref["slot"][ok])
    assert max_abs_rel(values(to_host(out), cfg.dtype)[ok], values(ref["out"], cfg.dtype)[ok]) <= 2e-2
    # replace the occupant of slot 1: expert 1 leaves, expert 5 enters
    L2.set_resident(1, 5, c.d_W1[5], c.d_W2[5])
    s2e, e2s = L2.maps()
    assert s2e.tolist() == [4, 5] and e2s.tolist() == [-1, -1, -1, -1, 0, 1]
    ref = oracle.layer_forward(c.x, c.Wr, c.W1_bank[[4, 5]], c.W2_bank[[4, 5]], e2s)
    out = L2.forward(c.d_x, cfg.T, accumulate=0)
    torch.cuda.synchronize()
    ok = ~ref["ambiguous"]
    assert np.array_equal(to_host(L2.slot)[ok], ref["slot"][ok])
    assert np.array_equal(to_host(L2.orig_expert)[ok], ref["orig_expert"][ok])
    assert max_abs_rel(values(to_host(out), cfg.dtype)[ok], values(ref["out"], cfg.dtype)[ok]) <= 2e-2
    L2.close(); L.close()


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_route_exact_and_near_ties(dtype):
    """Planted ties.  Experts 2 and 7 have identical router rows, so every token's two logits
    are equal on both sides and the lower id must win (original choice and served slot alike);
    experts 4 and 9 differ by a few units in the last place, a near tie inside the margin,
    where either of the two is a correct answer and the slot must belong to the chosen pair."""
    cfg = cfg_of(E=12, K=5, T=257, d_model=128, d_ff=64, dtype=dtype)
    c = Case(cfg, resident=[2, 7, 4, 9, 0], router_scale=20.0)
    L = c.L
    c.Wr[7] = c.Wr[2]
    c.Wr[9] = c.Wr[4] * np.float32(1 + 2.0 ** -20)
    L.router_w.copy_(torch.from_numpy(c.Wr))
    L.rebind()                                               # the router changed: bind again, reload the slots
    for s_, e_ in enumerate(c.s2e):
        c.load(s_, int(e_))
    r = c.oracle_route()
    L.route(c.d_x, c.T)
    torch.cuda.synchronize()
    g_oe, g_slot = to_host(L.orig_expert), to_host(L.slot)
    lg = r["logits"]
    top = lg.max(axis=1)
    exact = (lg[:, 2] == lg[:, 7]) & (lg[:, 2] == top)
    near = (np.abs(lg[:, 4] - lg[:, 9]) < oracle.MARGIN) & (np.maximum(lg[:, 4], lg[:, 9]) == top)
    assert exact.sum() > 5 and near.sum() > 5, "the planted ties are not exercised"
    assert r["ambiguous"][exact].all() and r["ambiguous"][near].all()
    assert (g_oe[exact] == 2).all() and (g_slot[exact] == 0).all()
    assert np.array_equal(r["orig_expert"][exact], g_oe[exact])
    assert np.isin(g_oe[near], [4, 9]).all() and np.isin(g_slot[near], [2, 3]).all()
    # the same tie among the resident experts only (the token's own choice may be elsewhere)
    rtop = lg[:, c.e2s >= 0].max(axis=1)
    rexact = (lg[:, 2] == lg[:, 7]) & (lg[:, 2] == rtop)
    assert rexact.sum() > exact.sum() and (g_slot[rexact] == 0).all()
    ok = ~r["ambiguous"]
    assert np.array_equal(g_oe[ok], r["orig_expert"][ok]) and np.array_equal(g_slot[ok], r["slot"][ok])
    # the whole layer still serves every token from a resident slot
    out = L.forward(c.d_x, c.T, accumulate=0)
    torch.cuda.synchronize()
    assert int(to_host(L.offsets)[-1]) == c.T
    L.close()


def test_large_sampled_c5():
    """Switch-large-128 shape at full size (T = 16384, E = 128, K = 32): routing,
    sort and importance in full, the FFN and the layer output on sampled rows
    that the oracle computes one by one -- first through the five separate calls
    (teacher-forced), then through smoe_forward, free-running, with and without the
    residual stream."""
    cfg = wl.CONFIGS["c5"]
    c = Case(cfg)
    L, T = c.L, cfg.T
    r = c.oracle_route()
    L.route(c.d_x, T)
    torch.cuda.synchronize()
    ok = ~r["ambiguous"]
    assert ok.mean() > 0.98
    assert np.array_equal(to_host(L.orig_expert)[ok], r["orig_expert"][ok])
    assert np.array_equal(to_host(L.slot)[ok], r["slot"][ok])
    np.testing.assert_allclose(to_host(L.gate)[ok], r["gate"][ok], rtol=1e-5)
    np.testing.assert_allclose(to_host(L.xnorm), r["xnorm"], rtol=1e-5)
    # teacher-forced from here on
    L.slot.copy_(to_dev(r["slot"])); L.orig_expert.copy_(to_dev(r["orig_expert"]))
    L.orig_gate.copy_(to_dev(r["orig_gate"])); L.xnorm.copy_(to_dev(r["xnorm"])); L.gate.copy_(to_dev(r["gate"]))
    st = oracle.importance(r["orig_expert"], r["orig_gate"], r["xnorm"], c.en_oracle)
    L.importance(T, 0)
    xp, perm, inv, offsets = oracle.permute(c.x, r["slot"], cfg.K)
    L.permute(c.d_x, T)
    L.expert_ffn(T)
    L.combine(T)
    torch.cuda.synchronize()
    assert np.array_equal(to_host(L.count), st[0])
    np.testing.assert_allclose(to_host(L.score), st[2], rtol=1e-4)
    assert np.array_equal(to_host(L.offsets), offsets)
    assert np.array_equal(to_host(L.perm), perm)
    assert np.array_equal(to_host(L.x_perm), xp)
    rows = np.unique(np.concatenate([np.arange(0, T, 67), offsets[:-1].clip(0, T - 1),
                                     (offsets[1:] - 1).clip(0, T - 1)])).astype(np.int32)
    W1s, W2s = c.slot_weights_host()
    y = oracle.expert_ffn(xp, W1s, W2s, offsets, rows=rows)
    got = values(to_host(L.y_perm), cfg.dtype)
    assert max_abs_rel(got[rows], y[rows]) <= 2e-2
    # layer output for the tokens that own those rows
    toks = perm[rows]
    ref_out = r["gate"][toks].astype(np.float64)[:, None] * y[rows]
    got_out = values(to_host(L.out), cfg.dtype)[toks]
    assert max_abs_rel(got_out, ref_out) <= 2e-2

    # ---- the same layer through smoe_forward (the entry point the benchmark times), free-running:
    # the router's own choices feed the sort, so the oracle's sort and importance are given the
    # library's slot / original-choice arrays once those have been checked
    names = ("orig_expert", "orig_gate", "slot", "gate", "xnorm", "count", "gsum", "score", "perm", "inv_perm",
             "offsets", "out")
    for n in names:
        getattr(L, n).fill_(0)
    out = L.forward_fused(c.d_x, T, accumulate=0)
    torch.cuda.synchronize()
    g_oe, g_slot = to_host(L.orig_expert), to_host(L.slot)
    assert np.array_equal(g_oe[ok], r["orig_expert"][ok])
    assert np.array_equal(g_slot[ok], r["slot"][ok])
    resident = c.e2s >= 0
    for t in np.nonzero(~ok)[0]:                             # near ties: one of the tied experts
        lg = r["logits"][t]
        delta = oracle.MARGIN * max(1.0, np.abs(lg).max())
        assert lg[g_oe[t]] >= lg.max() - delta
        assert lg[c.s2e[g_slot[t]]] >= lg[resident].max() - delta
    np.testing.assert_allclose(to_host(L.orig_gate)[ok], r["orig_gate"][ok], rtol=1e-5)
    np.testing.assert_allclose(to_host(L.gate)[ok], r["gate"][ok], rtol=1e-5)
    np.testing.assert_allclose(to_host(L.xnorm), r["xnorm"], rtol=1e-5)
    xp2, perm2, inv2, offsets2 = oracle.permute(c.x, g_slot, cfg.K)
    assert np.array_equal(to_host(L.offsets), offsets2)
    assert np.array_equal(to_host(L.perm), perm2)
    assert np.array_equal(to_host(L.inv_perm), inv2)
    st2 = oracle.importance(g_oe, r["orig_gate"], r["xnorm"], c.en_oracle)
    assert np.array_equal(to_host(L.count), st2[0])
    np.testing.assert_allclose(to_host(L.gsum), st2[1], rtol=1e-4)
    np.testing.assert_allclose(to_host(L.score), st2[2], rtol=1e-4)
    rows2 = np.unique(np.concatenate([np.arange(3, T, 61), offsets2[:-1].clip(0, T - 1),
                                      (offsets2[1:] - 1).clip(0, T - 1)])).astype(np.int32)
    rows2 = rows2[ok[perm2[rows2]]]                          # a near-tie token's gate may be the other expert's
    y2 = oracle.expert_ffn(xp2, W1s, W2s, offsets2, rows=rows2)
    toks2 = perm2[rows2]
    ref2 = r["gate"][toks2].astype(np.float64)[:, None] * y2[rows2]
    assert max_abs_rel(values(to_host(out), cfg.dtype)[toks2], ref2) <= 2e-2
    # with the residual stream: out = x + gate * y, rounded once to bf16
    res = to_dev(c.x)
    out = L.forward_fused(c.d_x, T, accumulate=1, residual=res)
    torch.cuda.synchronize()
    assert np.array_equal(to_host(L.count), 2 * st2[0])      # accumulate = 1 added the same batch again
    xv = values(c.x, cfg.dtype)[toks2]
    got2 = values(to_host(out), cfg.dtype)[toks2]
    assert (np.abs(got2 - (xv + ref2)) <= 2.0 ** -8 * np.abs(xv + ref2) + 2e-2 * np.abs(ref2).max()).all()
    L.close()
