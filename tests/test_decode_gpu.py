"""Decode-shaped run with resident-set updates (Switch-base-64 decode shape,
T = 32 tokens per step, E = 64, K = 16, update every 16 steps): the HIP path
runs free, the oracle is fed the same inputs and follows step by step.

Per step: original choices and slots bit-exact on the tokens without a near
tie (on the others: one of the near-tied experts); sort, offsets and token
counts bit-exact on EVERY step -- the oracle's sort and importance are fed the
library's own slot / original-choice arrays, which the previous line has just
checked -- importance sums within 1e-4; outputs within the bf16 tolerance.  Per update: importance scores
within 1e-4, and the new resident set and slot assignment must equal the
oracle's unless the K-th and (K+1)-th scores are within 1e-4 of each other, in
which case either set is right and the oracle adopts the library's choice."""
import numpy as np
import pytest
import torch

import oracle
from paper_2308_15030_amd import workloads as wl
from harness import Case, max_abs_rel, to_dev, to_host, values

pytestmark = pytest.mark.gpu

STEPS = wl.CONFIGS["c4"].steps        # all 256 steps of the workload, 16 updates


@pytest.mark.parametrize("fused", [False, True])
def test_decode_with_updates(fused):
    cfg = wl.CONFIGS["c4"]
    c = Case(cfg, bank_experts=range(cfg.E), x=np.zeros((cfg.T, cfg.d_model), np.uint16))
    L, T, K = c.L, cfg.T, cfg.K
    xs = wl.decode_stream(cfg, STEPS)                       # [steps, T, d]
    d_xs = to_dev(xs.reshape(STEPS * T, cfg.d_model)).view(STEPS, T, cfg.d_model)
    s2e, e2s = c.s2e.copy(), c.e2s.copy()
    state = None
    swaps = 0
    hits = []
    for step in range(STEPS):
        first = step % cfg.period == 0
        # ---- library, free-running
        fwd = L.forward_fused if fused else L.forward
        out = fwd(d_xs[step], T, accumulate=0 if first else 1)
        torch.cuda.synchronize()
        # ---- oracle on the same input and the same resident set
        idx = [c.bank_pos[int(e)] for e in s2e]
        ref = oracle.layer_forward(xs[step], c.Wr, c.W1_bank[idx], c.W2_bank[idx], e2s)
        ok = ~ref["ambiguous"]
        g_oe, g_slot = to_host(L.orig_expert), to_host(L.slot)
        assert np.array_equal(g_oe[ok], ref["orig_expert"][ok]), step
        assert np.array_equal(g_slot[ok], ref["slot"][ok]), step
        for t in np.nonzero(~ok)[0]:                         # near ties: one of the tied experts, resident for the slot
            lg = ref["logits"][t]
            delta = oracle.MARGIN * max(1.0, np.abs(lg).max())
            assert lg[g_oe[t]] >= lg.max() - delta, (step, t)
            assert e2s[s2e[g_slot[t]]] == g_slot[t] and lg[s2e[g_slot[t]]] >= lg[e2s >= 0].max() - delta, (step, t)
        hits.append(float((e2s[ref["orig_expert"]] >= 0).mean()))
        # integers on every step: the oracle's sort and importance take the library's (checked) choices
        _, o_perm, o_inv, o_off = oracle.permute(None, g_slot, K)
        assert np.array_equal(to_host(L.perm), o_perm), step
        assert np.array_equal(to_host(L.inv_perm), o_inv), step
        assert np.array_equal(to_host(L.offsets), o_off), step
        state = oracle.importance(g_oe, ref["orig_gate"], ref["xnorm"], c.en_oracle, state=None if first else state)
        assert np.array_equal(to_host(L.count), state[0]), step
        np.testing.assert_allclose(to_host(L.gsum), state[1], rtol=1e-4, atol=1e-30)
        np.testing.assert_allclose(to_host(L.score), state[2], rtol=1e-4, atol=1e-30)
        err = max_abs_rel(values(to_host(out), cfg.dtype)[ok], values(ref["out"], cfg.dtype)[ok])
        assert err <= 2e-2, (step, err)
        # ---- update at the end of a period
        if (step + 1) % cfg.period == 0:
            score = to_host(L.score)
            loads = L.select_resident(score)
            n_s2e, n_e2s, ref_loads = oracle.select_resident(state[2], s2e, e2s)
            if loads != ref_loads:
                order = np.sort(state[2])[::-1]
                gap = (order[K - 1] - order[K]) / max(order[K - 1], 1e-30)
                assert gap < 1e-4, (step, loads, ref_loads, gap)
            for sl, ex in loads:
                c.load(sl, ex)
            swaps += len(loads)
            s2e, e2s = L.maps()                              # the oracle follows the library's maps
            if loads == ref_loads:
                assert np.array_equal(s2e, n_s2e) and np.array_equal(e2s, n_e2s)
    assert swaps > 0, "the stream never changed the resident set: the test exercises nothing"
    # activation locality: after the first update most tokens find their own expert resident
    assert np.mean(hits[cfg.period:]) > np.mean(hits[:cfg.period])
    print(f"decode: {swaps} experts swapped over {STEPS // cfg.period} updates; "
          f"hit rate {np.mean(hits[:cfg.period]):.2f} -> {np.mean(hits[cfg.period:]):.2f}", flush=True)
    L.close()


def test_decode_with_updates_on_the_device():
    """The same run with the update rule and the slot loads done by the device
    (smoe_update_on_device): after every period the library's maps -- fetched
    from the device on demand -- must equal the oracle's update rule applied to
    the oracle's own scores (near ties at the K-th place aside), and every
    step's outputs must match the oracle on the set the device has chosen."""
    cfg = wl.CONFIGS["c4"]
    c = Case(cfg, bank_experts=range(cfg.E), x=np.zeros((cfg.T, cfg.d_model), np.uint16))
    L, T, K = c.L, cfg.T, cfg.K
    steps = 96                                               # six updates
    xs = wl.decode_stream(cfg, steps)
    d_xs = to_dev(xs.reshape(steps * T, cfg.d_model)).view(steps, T, cfg.d_model)
    s2e, e2s = c.s2e.copy(), c.e2s.copy()
    state, swaps = None, 0
    for step in range(steps):
        first = step % cfg.period == 0
        out = L.forward_fused(d_xs[step], T, accumulate=0 if first else 1)
        torch.cuda.synchronize()
        idx = [c.bank_pos[int(e)] for e in s2e]
        ref = oracle.layer_forward(xs[step], c.Wr, c.W1_bank[idx], c.W2_bank[idx], e2s)
        ok = ~ref["ambiguous"]
        g_oe, g_slot = to_host(L.orig_expert), to_host(L.slot)
        assert np.array_equal(g_oe[ok], ref["orig_expert"][ok]), step
        assert np.array_equal(g_slot[ok], ref["slot"][ok]), step
        state = oracle.importance(g_oe, ref["orig_gate"], ref["xnorm"], c.en_oracle, state=None if first else state)
        assert np.array_equal(to_host(L.count), state[0]), step
        np.testing.assert_allclose(to_host(L.score), state[2], rtol=1e-4, atol=1e-30)
        err = max_abs_rel(values(to_host(out), cfg.dtype)[ok], values(ref["out"], cfg.dtype)[ok])
        assert err <= 2e-2, (step, err)
        if (step + 1) % cfg.period == 0:
            L.update_on_device(c.d_W1, c.d_W2)               # ranks by L.score, on the device; no read-back here
            n_s2e, n_e2s, ref_loads = oracle.select_resident(state[2], s2e, e2s)
            g_s2e, g_e2s = L.maps()                          # waits for the update and fetches the device's maps
            if not (np.array_equal(g_s2e, n_s2e) and np.array_equal(g_e2s, n_e2s)):
                order = np.sort(state[2])[::-1]
                gap = (order[K - 1] - order[K]) / max(order[K - 1], 1e-30)
                assert gap < 1e-4, (step, g_s2e, n_s2e, gap)
            # the maps are a consistent pair, whichever way a near tie went
            assert sorted(g_s2e.tolist()) == sorted(np.nonzero(g_e2s >= 0)[0].tolist())
            assert all(g_e2s[g_s2e[k]] == k for k in range(K))
            swaps += int((g_s2e != s2e).sum())
            s2e, e2s = g_s2e, g_e2s                          # the oracle follows the library's maps
    assert swaps > 0, "the stream never changed the resident set: the test exercises nothing"
    # pageable host memory is refused before any launch
    from paper_2308_15030_amd import binding as b
    with pytest.raises(b.SmoeError):
        b.smoe_update_on_device(L.handle, L.score, np.zeros(4096, np.uint16), np.zeros(4096, np.uint16))
    print(f"device-side updates: {swaps} experts swapped over {steps // cfg.period} updates", flush=True)
    L.close()


def test_decode_streaming_loads_same_bits():
    """Once the expert slots of the live layers outgrow the Infinity Cache the decode kernels
    read their weights with non-temporal loads (other kernel instances, same arithmetic): the
    step's outputs, choices and sums must keep their bits."""
    cfg = wl.CONFIGS["c4"]
    from paper_2308_15030_amd import binding as b
    c = Case(cfg, bank_experts=range(cfg.K), x=np.zeros((cfg.T, cfg.d_model), np.uint16))
    L, T = c.L, cfg.T
    xs = wl.decode_stream(cfg, 4)
    d_xs = to_dev(xs.reshape(4 * T, cfg.d_model)).view(4, T, cfg.d_model)

    def run():
        got = []
        for step in range(4):
            out = L.forward_fused(d_xs[step], T, accumulate=0 if step == 0 else 1, residual=d_xs[step])
            torch.cuda.synchronize()
            got.append([to_host(out).copy(), to_host(L.slot).copy(), to_host(L.perm).copy(), to_host(L.offsets).copy(),
                        to_host(L.count).copy(), to_host(L.gsum).copy(), to_host(L.score).copy()])
        return got

    assert "_stream" not in b.smoe_describe_ffn(L.handle, T, True)
    cached = run()
    ballast = []
    while "_stream" not in b.smoe_describe_ffn(L.handle, T, True):
        assert len(ballast) < 4, "four more layers of this shape are 600 MB: the switch should have happened"
        ballast.append(b.Layer(cfg.E, cfg.K, cfg.d_model, cfg.d_ff, T, cfg.dtype, 0,
                               router_w=torch.from_numpy(c.Wr), device=c.dev))
    streamed = run()
    for step, (a, s) in enumerate(zip(cached, streamed)):
        for u, v in zip(a, s):
            assert np.array_equal(u, v), step
    # and against the oracle, on the last step
    ref = oracle.layer_forward(xs[3], c.Wr, *c.slot_weights_host(), c.e2s, residual=xs[3])
    ok = ~ref["ambiguous"]
    assert max_abs_rel(values(streamed[3][0], cfg.dtype)[ok], values(ref["out"], cfg.dtype)[ok]) <= 2e-2
    for lay in ballast:
        lay.close()
    assert "_stream" not in b.smoe_describe_ffn(L.handle, T, True)
    L.close()
