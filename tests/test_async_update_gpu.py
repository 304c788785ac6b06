"""Asynchronous, amortized resident-set update (Section 3.2 "Seamless update",
Figure 5(ii)): experts are packed into a spare physical slot on a second
stream while the forward pass keeps running, and the maps switch between two
steps once a load has arrived.

The library runs free on a decode-shaped stream; after every step the oracle
is given the same input and the resident set the library reported for that
step, so every output is checked while loads are in flight.  The schedule
itself is checked against the rule: each plan is the update rule applied to the
scores of its period (the oracle's select_resident on the maps the plan saw),
at most `spare_slots` loads are in flight, and every planned change is
committed within a bounded number of steps.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2308_15030_amd import binding as b
from paper_2308_15030_amd import workloads as wl
from harness import Case, max_abs_rel, to_dev, to_host, values

pytestmark = pytest.mark.gpu

STEPS = 64


def _bank(c, where):
    """All E experts contiguously, on the device or in pinned host memory."""
    assert c.bank_ids == list(range(c.cfg.E))
    if where == "device":
        return c.d_W1, c.d_W2
    w1 = torch.from_numpy(c.W1_bank.view(np.int16)).pin_memory()
    w2 = torch.from_numpy(c.W2_bank.view(np.int16)).pin_memory()
    return w1, w2


@pytest.mark.parametrize("where,spare", [("device", 1), ("pinned", 1), ("device", 3)])
def test_decode_with_asynchronous_updates(where, spare):
    cfg = wl.CONFIGS["c4"]
    c = Case(cfg, bank_experts=range(cfg.E), x=np.zeros((cfg.T, cfg.d_model), np.uint16), spare_slots=spare)
    L, T, K = c.L, cfg.T, cfg.K
    bank1, bank2 = _bank(c, where)
    load_stream = torch.cuda.Stream()
    xs = wl.decode_stream(cfg, STEPS)
    d_xs = to_dev(xs.reshape(STEPS * T, cfg.d_model)).view(STEPS, T, cfg.d_model)
    state, commits, plans, max_pending = None, 0, 0, 0
    since_plan = 0
    for step in range(STEPS):
        first = step % cfg.period == 0
        # between two steps: commit arrived loads, start the next ones (never waits)
        n = L.update_tick(bank1, bank2, load_stream)
        commits += n
        pend = L.update_pending()
        max_pending = max(max_pending, pend)
        s2e, e2s = L.maps()                                  # what this step will be served with
        assert sorted(e2s[e2s >= 0].tolist()) == list(range(K)) and np.array_equal(e2s[s2e], np.arange(K))
        out = L.forward_fused(d_xs[step], T, accumulate=0 if first else 1)
        # ---- oracle, same input, same resident set (no synchronisation before this point:
        # the load started by the tick above overlaps the forward pass)
        idx = [c.bank_pos[int(e)] for e in s2e]
        ref = oracle.layer_forward(xs[step], c.Wr, c.W1_bank[idx], c.W2_bank[idx], e2s)
        state = oracle.importance(ref["orig_expert"], ref["orig_gate"], ref["xnorm"], c.en_oracle,
                                  state=None if first else state)
        torch.cuda.current_stream().synchronize()
        ok = ~ref["ambiguous"]
        assert np.array_equal(to_host(L.slot)[ok], ref["slot"][ok]), step
        err = max_abs_rel(values(to_host(out), cfg.dtype)[ok], values(ref["out"], cfg.dtype)[ok])
        assert err <= 2e-2, (step, err)
        if pend:
            since_plan += 1
            assert since_plan <= 4 * K, "a planned change was never committed"
        # ---- end of a period: plan the next changes from the scores
        if (step + 1) % cfg.period == 0:
            score = to_host(L.score)
            if ok.all():
                np.testing.assert_allclose(score, state[2], rtol=1e-4, atol=1e-30)
            before = L.update_pending()
            n_plan = L.update_begin(score)
            plans += 1
            since_plan = 0
            # the plan is the update rule applied to the maps with the loads in flight taken as done;
            # with nothing in flight that is exactly the oracle's rule on the current maps
            if before == 0:
                _, _, ref_loads = oracle.select_resident(score.astype(np.float64), s2e, e2s)
                assert n_plan == len(ref_loads), (step, n_plan, ref_loads)
    assert commits > 0, "the stream never changed the resident set: the test exercises nothing"
    assert max_pending >= 1
    # drain: every planned change arrives
    for _ in range(8 * K):
        load_stream.synchronize()
        commits += L.update_tick(bank1, bank2, load_stream)
        if L.update_pending() == 0:
            break
    assert L.update_pending() == 0
    # after the drain the resident set is the one the last plan asked for
    s2e, e2s = L.maps()
    out = L.forward_fused(d_xs[STEPS - 1], T, accumulate=1)
    idx = [c.bank_pos[int(e)] for e in s2e]
    ref = oracle.layer_forward(xs[STEPS - 1], c.Wr, c.W1_bank[idx], c.W2_bank[idx], e2s)
    torch.cuda.synchronize()
    ok = ~ref["ambiguous"]
    assert max_abs_rel(values(to_host(out), cfg.dtype)[ok], values(ref["out"], cfg.dtype)[ok]) <= 2e-2
    print(f"async updates ({where} bank, {spare} spare): {plans} plans, {commits} commits, "
          f"at most {max_pending} changes outstanding", flush=True)
    L.close()


def test_asynchronous_update_state_rules():
    cfg = wl.MoEConfig("async-rules", E=8, K=3, d_model=64, d_ff=96, T=40, dtype=wl.BF16, seed=5)
    c = Case(cfg, bank_experts=range(cfg.E))                 # no spare slot
    score = np.arange(cfg.E, dtype=np.float32)
    with pytest.raises(b.SmoeError):
        c.L.update_begin(score)
    with pytest.raises(b.SmoeError):
        c.L.update_tick(c.d_W1, c.d_W2, torch.cuda.Stream())
    c.L.close()
    c = Case(cfg, bank_experts=range(cfg.E), spare_slots=1)
    assert c.L.update_pending() == 0
    n = c.L.update_begin(score)                              # wants experts 7, 6, 5; holds 0, 1, 2
    assert n == 3 and c.L.update_pending() == 3
    ls = torch.cuda.Stream()
    assert c.L.update_tick(c.d_W1, c.d_W2, ls) == 0          # nothing had been staged before this call
    # one spare slot: one load in flight, and its slot / expert cannot be set synchronously meanwhile
    with pytest.raises(b.SmoeError):
        c.L.set_resident(0, 7, c.d_W1[7], c.d_W2[7])
    total = 0
    for _ in range(10):
        ls.synchronize()
        total += c.L.update_tick(c.d_W1, c.d_W2, ls)
    assert total == 3 and c.L.update_pending() == 0
    s2e, e2s = c.L.maps()
    assert s2e.tolist() == [7, 6, 5]
    # the layer serves the new experts: whole layer against the oracle
    out = c.L.forward_fused(c.d_x, c.T, accumulate=0)
    ref = oracle.layer_forward(c.x, c.Wr, c.W1_bank[s2e], c.W2_bank[s2e], e2s)
    torch.cuda.synchronize()
    ok = ~ref["ambiguous"]
    assert max_abs_rel(values(to_host(out), cfg.dtype)[ok], values(ref["out"], cfg.dtype)[ok]) <= 2e-2
    # a second plan replaces what has not started; a no-change plan is empty
    assert c.L.update_begin(score) == 0
    c.L.close()


def test_new_plan_while_a_load_is_in_flight():
    """A second plan arrives while the first plan's load is still staged, and its ranking no
    longer wants the expert in flight: that slot's new occupant must not be lost -- it is loaded
    once the earlier load has been committed -- so the final resident set is the update rule
    (the oracle's select_resident) applied to the second plan's scores."""
    cfg = wl.MoEConfig("async-replan", E=8, K=4, d_model=64, d_ff=96, T=40, dtype=wl.BF16, seed=6)
    c = Case(cfg, bank_experts=range(cfg.E), spare_slots=1)
    L = c.L
    ls = torch.cuda.Stream()
    score1 = np.array([0, 5, 4, 3, 9, 0, 0, 0], np.float32)      # wants 4, 1, 2, 3: expert 4 into slot 0
    assert L.update_begin(score1) == 1
    assert L.update_tick(c.d_W1, c.d_W2, ls) == 0                # the load of expert 4 is now in flight
    assert L.update_pending() == 1
    score2 = np.array([0, 5, 4, 3, 0, 9, 0, 0], np.float32)      # now wants 5, 1, 2, 3: slot 0 again
    assert L.update_begin(score2) == 1                           # (slot 0, expert 5), behind the load in flight
    assert L.update_pending() == 2
    for _ in range(12):
        ls.synchronize()
        L.update_tick(c.d_W1, c.d_W2, ls)
        if L.update_pending() == 0:
            break
    assert L.update_pending() == 0
    s2e, e2s = L.maps()
    # the oracle's rule on the second scores, from the maps after the first load's commit
    s2e1 = np.array([4, 1, 2, 3], np.int32)
    e2s1 = np.full(cfg.E, -1, np.int32); e2s1[s2e1] = np.arange(cfg.K)
    want_s2e, want_e2s, _ = oracle.select_resident(score2.astype(np.float64), s2e1, e2s1)
    assert np.array_equal(s2e, want_s2e) and np.array_equal(e2s, want_e2s)
    assert s2e.tolist() == [5, 1, 2, 3]
    out = L.forward_fused(c.d_x, c.T, accumulate=0)
    ref = oracle.layer_forward(c.x, c.Wr, c.W1_bank[s2e], c.W2_bank[s2e], e2s)
    torch.cuda.synchronize()
    ok = ~ref["ambiguous"]
    assert np.array_equal(to_host(L.slot)[ok], ref["slot"][ok])
    assert max_abs_rel(values(to_host(out), cfg.dtype)[ok], values(ref["out"], cfg.dtype)[ok]) <= 2e-2
    L.close()


def test_device_side_update_after_slots_have_moved():
    """smoe_update_on_device on a layer whose virtual slots no longer sit in their own physical
    slots (asynchronous loads have been committed into the spare one): it must load into the
    physical slot each virtual slot is mapped to, refuse to run while an asynchronous update is
    pending, and leave maps that equal the oracle's rule.  Scores given by hand, small shape."""
    cfg = wl.MoEConfig("device-update", E=8, K=3, d_model=64, d_ff=96, T=40, dtype=wl.BF16, seed=7)
    c = Case(cfg, bank_experts=range(cfg.E), spare_slots=1)
    L = c.L
    ls = torch.cuda.Stream()
    score1 = np.array([9, 8, 0, 0, 7, 0, 0, 0], np.float32)      # wants 0, 1, 4: expert 4 into slot 2 via the spare
    assert L.update_begin(score1) == 1
    d_score = torch.zeros(cfg.E, dtype=torch.float32, device=c.dev)
    L.update_tick(c.d_W1, c.d_W2, ls)
    with pytest.raises(b.SmoeError):                             # a load is in flight
        b.smoe_update_on_device(L.handle, d_score, c.d_W1, c.d_W2)
    for _ in range(12):
        ls.synchronize()
        L.update_tick(c.d_W1, c.d_W2, ls)
        if L.update_pending() == 0:
            break
    assert L.update_pending() == 0 and L.maps()[0].tolist() == [0, 1, 4]
    # now the device's turn, twice: a change of two slots, then nothing to change
    score2 = np.array([0, 1, 0, 6, 5, 0, 0, 7], np.float32)      # wants 7, 3, 4: slots 0 and 1 go to 7 and 3
    d_score.copy_(torch.from_numpy(score2))
    s2e0, e2s0 = L.maps()
    b.smoe_update_on_device(L.handle, d_score, c.d_W1, c.d_W2)
    want_s2e, want_e2s, loads = oracle.select_resident(score2.astype(np.float64), s2e0, e2s0)
    s2e, e2s = L.maps()
    assert np.array_equal(s2e, want_s2e) and np.array_equal(e2s, want_e2s) and s2e.tolist() == [7, 3, 4]
    out = L.forward_fused(c.d_x, c.T, accumulate=0)
    ref = oracle.layer_forward(c.x, c.Wr, c.W1_bank[s2e], c.W2_bank[s2e], e2s)
    torch.cuda.synchronize()
    ok = ~ref["ambiguous"]
    assert np.array_equal(to_host(L.slot)[ok], ref["slot"][ok])
    assert max_abs_rel(values(to_host(out), cfg.dtype)[ok], values(ref["out"], cfg.dtype)[ok]) <= 2e-2
    b.smoe_update_on_device(L.handle, d_score, c.d_W1, c.d_W2)  # same scores: nothing moves
    assert L.maps()[0].tolist() == [7, 3, 4]
    # the host-side calls see the device's maps: expert 7 is resident in slot 0 now
    with pytest.raises(b.SmoeError):
        L.set_resident(1, 7, c.d_W1[7], c.d_W2[7])
    assert L.select_resident(score2) == []
    L.close()


def test_pageable_host_memory_is_refused_before_any_launch():
    """Weight sources and banks are read by kernels or by the copy engines: a numpy array
    (pageable host memory) must come back as SMOE_EINVAL from the host-side check, with no
    kernel launched; pinned host memory is accepted."""
    cfg = wl.MoEConfig("ptr-check", E=6, K=2, d_model=64, d_ff=96, T=16, dtype=wl.BF16, seed=7)
    c = Case(cfg, bank_experts=range(cfg.E), spare_slots=1)
    L = c.L
    w1, w2 = c.W1_bank, c.W2_bank                                # numpy, pageable
    with pytest.raises(b.SmoeError) as e:
        b.smoe_set_resident(L.handle, 0, 0, w1[0], w2[0])
    assert e.value.status == b.SMOE_EINVAL
    with pytest.raises(b.SmoeError) as e:
        b.smoe_set_resident(L.handle, 0, 0, c.d_W1[0], w2[0])    # one good, one bad
    assert e.value.status == b.SMOE_EINVAL
    with pytest.raises(b.SmoeError) as e:
        b.smoe_expert_norm(L.handle, w1, w2, cfg.E, L.expert_norm)
    assert e.value.status == b.SMOE_EINVAL
    L.update_begin(np.arange(cfg.E, dtype=np.float32))
    ls = torch.cuda.Stream()
    with pytest.raises(b.SmoeError) as e:
        b.smoe_update_tick(L.handle, w1, w2, ls)
    assert e.value.status == b.SMOE_EINVAL and L.update_pending() == 2       # nothing was started
    # the refusals left no error behind in the runtime and changed no state
    s2e, _ = L.maps()
    assert s2e.tolist() == [0, 1]
    p1 = torch.from_numpy(w1.view(np.int16)).pin_memory()
    p2 = torch.from_numpy(w2.view(np.int16)).pin_memory()
    L.set_resident(0, 0, p1[0], p2[0])                           # pinned host memory is a legal source
    for _ in range(12):
        ls.synchronize()
        L.update_tick(p1, p2, ls)
        if L.update_pending() == 0:
            break
    assert L.update_pending() == 0
    torch.cuda.synchronize()
    assert L.maps()[0].tolist() == [5, 4]
    L.close()
