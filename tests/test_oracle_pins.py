"""Pins of the CPU oracle against what the paper and mathematics fix.

None of these tests touch the HIP path.  Each pins a part of oracle.cpp to
something other than the oracle itself: a hand-worked example, a closed form,
an invariant, a special case that reduces to a library routine (PyTorch CPU in
fp64), or brute force with a deliberately different formulation.
"""
import json
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2308_15030_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_layer(seed, E, K, d, f, T, dtype=wl.F32, resident=None):
    cfg = wl.MoEConfig("t", E=E, K=K, d_model=d, d_ff=f, T=T, dtype=dtype, seed=seed)
    Wr = wl.router_weights(cfg)
    # larger router weights than the workloads use, so routing is spread out
    Wr = (Wr * 25).astype(np.float32)
    W1, W2 = wl.expert_bank(cfg)
    x = wl.hidden_states(cfg)
    if resident is None:
        s2e, e2s = wl.initial_resident(cfg)
    else:
        s2e = np.array(resident, np.int32)
        e2s = np.full(E, -1, np.int32)
        e2s[s2e] = np.arange(K, dtype=np.int32)
    return cfg, x, Wr, W1, W2, s2e, e2s


def _dense_switch_torch(x, Wr, W1, W2):
    """Standard Switch top-1 layer with library tensor ops in fp64:
    out = sum_e 1[e = argmax] * p_e * FFN_e(x)."""
    xt = torch.from_numpy(np.asarray(x, np.float64))
    logits = xt @ torch.from_numpy(Wr.astype(np.float64)).T
    p = torch.softmax(logits, dim=-1)
    top = torch.argmax(logits, dim=-1)
    W1t = torch.from_numpy(np.asarray(W1, np.float64))
    W2t = torch.from_numpy(np.asarray(W2, np.float64))
    h = torch.relu(torch.einsum("td,edf->etf", xt, W1t))
    y_all = torch.einsum("etf,efd->etd", h, W2t)                     # [E,T,d]
    onehot = torch.nn.functional.one_hot(top, Wr.shape[0]).to(torch.float64)   # [T,E]
    out = torch.einsum("te,te,etd->td", onehot, p, y_all)
    return out.numpy(), top.numpy(), p.numpy()


# --------------------------------------------------------------------- P9a
def test_hand_worked_example():
    """Every step on a 4-token example small enough to do on paper."""
    g = json.load(open(os.path.join(GOLDEN, "tiny_layer.json")))
    E, K = g["E"], g["K"]
    x = np.array(g["x"], np.float32)
    Wr = np.array(g["router_w"], np.float32)
    W1 = np.array(g["W1"], np.float32)
    W2 = np.array(g["W2"], np.float32)
    s2e = np.array(g["slot_to_expert"], np.int32)
    e2s = np.full(E, -1, np.int32)
    e2s[s2e] = np.arange(K)
    r = oracle.layer_forward(x, Wr, W1[s2e], W2[s2e], e2s, out_dtype=oracle.F64)

    assert np.array_equal(r["logits"], np.array(g["logits"], np.float64))
    assert r["orig_expert"].tolist() == g["orig_expert"]
    assert r["slot"].tolist() == g["slot"]
    assert s2e[r["slot"]].tolist() == g["served_expert"]
    assert r["offsets"].tolist() == g["offsets"]
    assert r["perm"].tolist() == g["perm"]
    assert r["inv_perm"].tolist() == g["inv_perm"]
    assert not r["ambiguous"].any()

    # softmax closed forms, from the integer logits
    def p(t, e):
        lg = g["logits"][t]
        return math.exp(lg[e]) / sum(math.exp(v) for v in lg)
    e1, e2, e3, e4, e5, e6 = (math.exp(-k) for k in range(1, 7))
    assert p(0, 0) == pytest.approx(1 / (1 + e2 + e4), rel=1e-15)
    exp_orig_gate = [1 / (1 + e2 + e4), 1 / (1 + e3 + e6), 1 / (1 + 2 * e3), 1 / (1 + e1 + e5)]
    exp_gate = [1 / (1 + e2 + e4), e3 / (1 + e3 + e6), 1 / (1 + 2 * e3), e1 / (1 + e1 + e5)]
    np.testing.assert_allclose(r["orig_gate"], exp_orig_gate, rtol=2e-7)
    np.testing.assert_allclose(r["gate"], exp_gate, rtol=2e-7)
    np.testing.assert_allclose(r["xnorm"], np.sqrt(g["xnorm_squared"]), rtol=2e-7)

    # FFN rows are integers; y_perm is in sorted order
    ffn = np.array(g["ffn_of_token"], np.float64)
    assert np.array_equal(r["y_perm"], ffn[g["perm"]])
    # out = gate * FFN in token order (gate is an fp32 value at the interface)
    np.testing.assert_allclose(r["out"], r["gate"].astype(np.float64)[:, None] * ffn, rtol=1e-15)
    np.testing.assert_allclose(r["out"], np.array(exp_gate)[:, None] * ffn, rtol=2e-7)

    # importance (Eq. 1) with the Frobenius norm of each expert
    en = oracle.expert_norm(W1, W2)
    np.testing.assert_allclose(en, np.sqrt(g["expert_norm_squared"]), rtol=1e-15)
    count, gsum, score = oracle.importance(r["orig_expert"], r["orig_gate"], r["xnorm"], en)
    assert count.tolist() == g["count"]
    og = exp_orig_gate
    np.testing.assert_allclose(gsum, [og[0], og[1] + og[3], og[2]], rtol=3e-7)
    exp_score = [math.sqrt(11) * 2 * og[0],
                 math.sqrt(12) * (3 * og[1] + math.sqrt(5) * og[3]),
                 math.sqrt(22) * math.sqrt(2) * og[2]]
    np.testing.assert_allclose(score, exp_score, rtol=5e-7)

    # RENORM gate mode: divide by the resident experts' total probability
    rr = oracle.route(x, Wr, e2s, oracle.GATE_RENORM)
    exp_renorm = [p(t, s2e[g["slot"][t]]) / (p(t, 0) + p(t, 2)) for t in range(4)]
    np.testing.assert_allclose(rr["gate"], exp_renorm, rtol=2e-7)


# --------------------------------------------------------------------- P1
@pytest.mark.parametrize("seed,E,d,f,T", [(0, 8, 64, 256, 256), (3, 5, 24, 40, 97)])
def test_all_resident_is_switch_layer(seed, E, d, f, T):
    """K = E with the identity map reduces to the standard Switch top-1 layer
    (the paper's "original MoE" baseline), written with PyTorch CPU ops."""
    cfg, x, Wr, W1, W2, s2e, e2s = _rand_layer(seed, E, E, d, f, T)
    r = oracle.layer_forward(x, Wr, W1, W2, e2s, out_dtype=oracle.F64)
    ref, top, p = _dense_switch_torch(x, Wr, W1, W2)
    assert np.array_equal(r["orig_expert"], top)
    assert np.array_equal(r["slot"], top)
    np.testing.assert_allclose(r["orig_gate"], p[np.arange(T), top], rtol=2e-7)
    assert np.array_equal(r["gate"], r["orig_gate"])
    scale = np.abs(ref).max()
    # gates are fp32 at the interface: 6e-8 relative
    assert np.abs(r["out"] - ref).max() <= 2e-7 * scale
    assert len(set(top.tolist())) > 1           # the case does exercise several experts


def test_all_resident_permuted_slots():
    """K = E but a scrambled slot assignment: output unchanged, slots follow the map."""
    E = 6
    perm_slots = [4, 2, 5, 0, 1, 3]            # slot -> expert
    cfg, x, Wr, W1, W2, s2e, e2s = _rand_layer(7, E, E, 16, 24, 61, resident=perm_slots)
    r = oracle.layer_forward(x, Wr, W1[s2e], W2[s2e], e2s, out_dtype=oracle.F64)
    ref, top, _ = _dense_switch_torch(x, Wr, W1, W2)
    assert np.array_equal(s2e[r["slot"]], top)
    assert np.abs(r["out"] - ref).max() <= 2e-7 * np.abs(ref).max()


# --------------------------------------------------------------------- P2
def test_resident_choices_untouched():
    """Tokens whose own top-1 expert is resident get exactly the full layer's
    output; the others get a resident expert."""
    E, K = 8, 3
    cfg, x, Wr, W1, W2, s2e, e2s = _rand_layer(11, E, K, 32, 48, 200, resident=[5, 1, 6])
    r = oracle.layer_forward(x, Wr, W1[s2e], W2[s2e], e2s, out_dtype=oracle.F64)
    _, e2s_full = wl.initial_resident(cfg.scaled(K=E))
    full = oracle.layer_forward(x, Wr, W1, W2, e2s_full, out_dtype=oracle.F64)
    hit = e2s[full["orig_expert"]] >= 0
    assert 0 < hit.sum() < cfg.T
    assert np.array_equal(r["orig_expert"], full["orig_expert"])
    assert np.array_equal(r["orig_gate"], full["orig_gate"])
    assert np.array_equal(r["out"][hit], full["out"][hit])
    assert np.array_equal(s2e[r["slot"]][hit], full["orig_expert"][hit])
    assert np.isin(s2e[r["slot"]], s2e).all()
    # a redirected token goes to the best resident expert by logit
    lg = r["logits"]
    masked = np.where(e2s[None, :] >= 0, lg, -np.inf)
    assert np.array_equal(s2e[r["slot"]], masked.argmax(1))
    assert (r["gate"][~hit] < r["orig_gate"][~hit]).all()


# --------------------------------------------------------------------- P3
@pytest.mark.parametrize("only", [0, 3])
def test_single_resident_closed_form(only):
    """K = 1: every token is served by the one resident expert r with gate
    softmax(logits)[r]: out = p[:, r] * FFN_r(x), two dense matrix products."""
    E = 5
    cfg, x, Wr, W1, W2, s2e, e2s = _rand_layer(5, E, 1, 20, 36, 77, resident=[only])
    r = oracle.layer_forward(x, Wr, W1[s2e], W2[s2e], e2s, out_dtype=oracle.F64)
    xt = torch.from_numpy(x.astype(np.float64))
    p = torch.softmax(xt @ torch.from_numpy(Wr.astype(np.float64)).T, -1)[:, only]
    ffn = torch.relu(xt @ torch.from_numpy(W1[only].astype(np.float64))) @ \
        torch.from_numpy(W2[only].astype(np.float64))
    ref = (p[:, None] * ffn).numpy()
    assert (r["slot"] == 0).all()
    assert r["perm"].tolist() == list(range(cfg.T))
    assert np.abs(r["out"] - ref).max() <= 2e-7 * np.abs(ref).max()


# --------------------------------------------------------------------- P4
def test_importance_invariants():
    E, K, T = 16, 4, 1000
    cfg, x, Wr, W1, W2, s2e, e2s = _rand_layer(2, E, K, 32, 16, T)
    r = oracle.route(x, Wr, e2s)
    en = oracle.expert_norm(W1, W2)
    count, gsum, score = oracle.importance(r["orig_expert"], r["orig_gate"], r["xnorm"], en)
    assert count.sum() == T
    assert np.array_equal(count, np.bincount(r["orig_expert"], minlength=E))
    assert gsum.sum() == pytest.approx(r["orig_gate"].astype(np.float64).sum(), rel=1e-12)
    # Eq. 1 written with a different routine: weighted bincount
    raw = np.bincount(r["orig_expert"], minlength=E,
                      weights=r["xnorm"].astype(np.float64) * r["orig_gate"].astype(np.float64))
    np.testing.assert_allclose(score, en * raw, rtol=1e-12)
    # counts include experts that are NOT resident (they must be able to earn a slot)
    assert count[K:].sum() > 0 and score[K:].sum() > 0
    # accumulate = add
    c2, g2, s2 = oracle.importance(r["orig_expert"], r["orig_gate"], r["xnorm"], en,
                                   state=(count, gsum, score))
    assert np.array_equal(c2, 2 * count)
    np.testing.assert_allclose(g2, 2 * gsum, rtol=1e-15)
    np.testing.assert_allclose(s2, 2 * score, rtol=1e-15)
    # segment lengths sum to T
    _, _, _, offsets = oracle.permute(None, r["slot"], K)
    assert offsets[0] == 0 and offsets[-1] == T and (np.diff(offsets) >= 0).all()


def test_unit_norm_tokens_score_equals_gsum():
    """With |x| = 1 for every token and |E_i| = 1, Eq. 1 collapses to the
    summed gate probability."""
    E, T, d = 8, 300, 16
    cfg, x, Wr, *_ = _rand_layer(9, E, 2, d, 8, T)
    x64 = x.astype(np.float64)
    x = (x64 / np.linalg.norm(x64, axis=1, keepdims=True)).astype(np.float32)
    _, e2s = wl.initial_resident(cfg)
    r = oracle.route(x, Wr, e2s)
    np.testing.assert_allclose(r["xnorm"], 1.0, rtol=3e-7)
    count, gsum, score = oracle.importance(r["orig_expert"], r["orig_gate"], r["xnorm"], np.ones(E))
    np.testing.assert_allclose(score, gsum, rtol=1e-6)


def test_xnorm_and_expert_norm_match_library():
    cfg, x, Wr, W1, W2, s2e, e2s = _rand_layer(4, 4, 2, 50, 30, 40, dtype=wl.BF16)
    r = oracle.route(x, Wr, e2s)
    xf = wl.bf16_bits_to_f32(x).astype(np.float64)
    np.testing.assert_allclose(r["xnorm"], np.linalg.norm(xf, axis=1), rtol=2e-7)
    w1 = wl.bf16_bits_to_f32(W1).astype(np.float64)
    w2 = wl.bf16_bits_to_f32(W2).astype(np.float64)
    ref = np.sqrt((w1 ** 2).sum((1, 2)) + (w2 ** 2).sum((1, 2)))
    np.testing.assert_allclose(oracle.expert_norm(W1, W2), ref, rtol=1e-12)


# --------------------------------------------------------------------- P5
@pytest.mark.parametrize("T,K", [(0, 3), (1, 1), (257, 4), (1000, 32)])
def test_permute_is_stable_sort(T, K):
    rng = np.random.default_rng(T + K)
    slot = rng.integers(0, K, size=T).astype(np.int32)
    if T > 10:
        slot[slot == 1] = 0                      # an empty segment
    x = rng.standard_normal((T, 6)).astype(np.float32)
    xp, perm, inv, offsets = oracle.permute(x, slot, K)
    assert sorted(perm.tolist()) == list(range(T))
    assert np.array_equal(perm, np.argsort(slot, kind="stable"))
    assert np.array_equal(inv[perm], np.arange(T))
    assert np.array_equal(offsets, np.concatenate([[0], np.cumsum(np.bincount(slot, minlength=K))]))
    assert np.array_equal(xp, x[perm])
    assert np.array_equal(xp[inv], x)


# --------------------------------------------------------------------- P6
def test_identity_ffn_plumbing():
    """W1 = [I | 0], W2 = [I ; 0], x >= 0: the FFN is the identity, so the layer
    returns gate * x exactly; catches any mix-up of permute / slot / combine."""
    E, K, d, f, T = 6, 3, 8, 12, 90
    cfg, x, Wr, W1, W2, s2e, e2s = _rand_layer(21, E, K, d, f, T, resident=[4, 0, 3])
    x = np.abs(x)
    W1 = np.zeros((E, d, f), np.float32); W2 = np.zeros((E, f, d), np.float32)
    for e in range(E):
        W1[e, :, :d] = np.eye(d) * (e + 1)       # expert e scales by (e+1)
        W2[e, :d, :] = np.eye(d)
    r = oracle.layer_forward(x, Wr, W1[s2e], W2[s2e], e2s, out_dtype=oracle.F64)
    served = s2e[r["slot"]]
    ref = r["gate"].astype(np.float64)[:, None] * (served + 1)[:, None] * x.astype(np.float64)
    assert np.array_equal(r["out"], ref)
    assert len(set(served.tolist())) == K


# --------------------------------------------------------------------- P7
def test_ffn_positive_homogeneity():
    cfg, x, Wr, W1, W2, s2e, e2s = _rand_layer(13, 4, 2, 24, 40, 50)
    offsets = np.array([0, 20, 50], np.int32)
    y1 = oracle.expert_ffn(x, W1[:2], W2[:2], offsets)
    y8 = oracle.expert_ffn((x * 8).astype(np.float32), W1[:2], W2[:2], offsets)
    assert np.array_equal(y8, 8 * y1)
    # and ReLU really clips: negating x does not negate y
    yn = oracle.expert_ffn(-x, W1[:2], W2[:2], offsets)
    assert not np.allclose(yn, -y1)


def test_ffn_matches_library_matmul_per_segment():
    """Each segment against torch fp64 matmul, fp32 and bf16 storage, with an
    empty segment and the `rows` subset option."""
    for dtype in (wl.F32, wl.BF16):
        cfg, x, Wr, W1, W2, s2e, e2s = _rand_layer(17, 5, 4, 40, 72, 120, dtype=dtype)
        offsets = np.array([0, 33, 33, 100, 120], np.int32)
        y = oracle.expert_ffn(x, W1[:4], W2[:4], offsets)
        xf = torch.from_numpy(wl.as_f32(x, dtype).astype(np.float64))
        for k in range(4):
            a, b = offsets[k], offsets[k + 1]
            w1 = torch.from_numpy(wl.as_f32(W1[k], dtype).astype(np.float64))
            w2 = torch.from_numpy(wl.as_f32(W2[k], dtype).astype(np.float64))
            ref = (torch.relu(xf[a:b] @ w1) @ w2).numpy()
            if b > a:
                assert np.abs(y[a:b] - ref).max() <= 1e-12 * max(1.0, np.abs(ref).max())
        rows = np.array([119, 0, 33, 57], np.int32)
        ys = oracle.expert_ffn(x, W1[:4], W2[:4], offsets, rows=rows)
        assert np.array_equal(ys[rows], y[rows])
        assert np.isnan(ys[1]).all()


# --------------------------------------------------------------------- P8
def test_token_shuffle_equivariance():
    cfg, x, Wr, W1, W2, s2e, e2s = _rand_layer(19, 8, 3, 16, 24, 128)
    r = oracle.layer_forward(x, Wr, W1[s2e], W2[s2e], e2s, out_dtype=oracle.F64)
    sh = np.random.default_rng(0).permutation(cfg.T)
    rs = oracle.layer_forward(x[sh], Wr, W1[s2e], W2[s2e], e2s, out_dtype=oracle.F64)
    assert np.array_equal(rs["out"], r["out"][sh])
    assert np.array_equal(rs["slot"], r["slot"][sh])


# --------------------------------------------------------------------- P9b
@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("mode", [oracle.GATE_FULL, oracle.GATE_RENORM])
def test_brute_force_dense_then_select(seed, mode):
    """Different formulation: run EVERY expert on EVERY token with numpy,
    then pick per token; Python loops, tiny shapes."""
    rng = np.random.default_rng(100 + seed)
    E = int(rng.integers(2, 7)); K = int(rng.integers(1, E + 1))
    d = int(rng.integers(1, 6)); f = int(rng.integers(1, 7)); T = int(rng.integers(1, 12))
    resident = rng.permutation(E)[:K]
    cfg, x, Wr, W1, W2, s2e, e2s = _rand_layer(seed, E, K, d, f, T, resident=resident)
    r = oracle.layer_forward(x, Wr, W1[s2e], W2[s2e], e2s, gate_mode=mode, out_dtype=oracle.F64)
    x64, Wr64 = x.astype(np.float64), Wr.astype(np.float64)
    for t in range(T):
        logits = [sum(x64[t, j] * Wr64[e, j] for j in range(d)) for e in range(E)]
        z = sum(math.exp(v - max(logits)) for v in logits)
        p = [math.exp(v - max(logits)) / z for v in logits]
        ys = []
        for e in range(E):
            h = np.maximum(x64[t] @ W1[e].astype(np.float64), 0)
            ys.append(h @ W2[e].astype(np.float64))
        cand = sorted(resident.tolist(), key=lambda e: (-logits[e], e))
        s = cand[0]
        gate = p[s] / sum(p[e] for e in resident) if mode == oracle.GATE_RENORM else p[s]
        assert s2e[r["slot"][t]] == s
        assert r["orig_expert"][t] == sorted(range(E), key=lambda e: (-logits[e], e))[0]
        np.testing.assert_allclose(r["out"][t], gate * ys[s], rtol=3e-7, atol=1e-300)


def test_exact_tie_goes_to_lowest_index():
    Wr = np.array([[1, 0], [1, 0], [0, 1], [1, 0]], np.float32)
    x = np.array([[2, 1], [0, 0]], np.float32)
    e2s = np.array([-1, 1, -1, 0], np.int32)     # experts 1 and 3 resident (tie between them)
    r = oracle.route(x, Wr, e2s)
    assert r["orig_expert"].tolist() == [0, 0]
    assert r["slot"].tolist() == [1, 1]          # expert 1 (lower id) wins the resident tie
    assert r["ambiguous"].all()
    np.testing.assert_allclose(r["orig_gate"][1], 0.25)


def test_ambiguous_mask_written_out_by_hand():
    """The near-tie mask: a token is ambiguous when the gap between the largest and the
    second largest logit -- over all experts, or over the resident experts only -- is below
    1e-4 * max(1, max_e |logit_e|).  The router is the identity here, so a token's logits
    are its own coordinates, and the expected mask is worked out by hand for each row.
    Experts 0 and 2 are resident."""
    E = 4
    Wr = np.eye(E, dtype=np.float32)
    e2s = np.array([0, -1, 1, -1], np.int32)
    rows = [
        # logits                         ambiguous  why
        ([0.5, 0.1, 0.2, 0.0],           False),  # every gap is large
        ([0.5, 0.49993, 0.2, 0.0],       True),   # |logit| < 1 so the margin is 1e-4 (not 1e-4 * 0.5): global gap 7e-5
        ([0.5, 0.49985, 0.2, 0.0],       False),  # global gap 1.5e-4 > 1e-4; resident gap 0.3
        ([100.0, 99.995, 3.0, 2.0],      True),   # margin scales with max|logit|: 1e-2 > gap 5e-3
        ([100.0, 99.98, 3.0, 2.0],       False),  # gap 2e-2 > 1e-2
        ([0.5, 0.497, 0.1, -50.0],       True),   # the scale is max |logit| (here from a negative one): margin 5e-3 > gap 3e-3
        ([0.5, 0.2, 0.1, -50.0],         False),
        ([0.3, 0.9, 0.29996, 0.0],       True),   # only the resident pair (experts 0 and 2) is close: gap 4e-5
        ([0.3, 0.29996, 0.1, 0.9],       False),  # a non-resident expert next to the resident best does not count;
                                                  # the resident runner-up is expert 2, 0.2 away
        ([0.9, 0.3, 0.1, 0.29996],       False),  # two close non-resident runners-up are no tie for the top
        ([0.2, 0.9, 0.1, 0.89995],       True),   # only the global pair (both non-resident) is close
    ]
    x = np.array([r[0] for r in rows], np.float32)
    want = np.array([r[1] for r in rows])
    r = oracle.route(x, Wr, e2s)
    assert r["ambiguous"].tolist() == want.tolist()
    # the choices themselves are the plain arg-maxes (no near-tie changes them)
    assert r["orig_expert"].tolist() == [0, 0, 0, 0, 0, 0, 0, 1, 3, 0, 1]
    assert r["slot"].tolist() == [0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0]
    # a custom margin is honoured: ten times wider flags row 2 (gap 1.5e-4 < 1e-3) as well
    wide = oracle.route(x, Wr, e2s, margin=1e-3)["ambiguous"]
    assert wide[2] and not wide[0]
    # one resident expert: there is no resident runner-up, so only the global gap decides
    one = np.array([-1, -1, 0, -1], np.int32)
    r1 = oracle.route(x, Wr, one)
    assert r1["ambiguous"].tolist() == [False, True, False, True, False, True, False, False, False, False, True]
    # a single expert can never tie
    r2 = oracle.route(x[:, :1].copy(), np.ones((1, 1), np.float32), np.array([0], np.int32))
    assert not r2["ambiguous"].any()


# --------------------------------------------------------------------- rounding
def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(1)
    a = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-30, 30, 20000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895313892515355e38, 1e-40,
                         9.18e-41, -2.5e-45]])
    ref = torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.round_bf16(a.astype(np.float32).astype(np.float64))
    assert np.array_equal(got, ref)
    # the workload generator's own formatter agrees too
    assert np.array_equal(wl.f32_to_bf16_bits(a.astype(np.float32)), ref)
    # exact ties between two bf16 neighbours go to the even one
    assert oracle.round_bf16(np.array([1.00390625]))[0] == 0x3F80      # 1 + 2^-8  -> 1.0
    assert oracle.round_bf16(np.array([1.01171875]))[0] == 0x3F82      # 1 + 3*2^-8 -> 1 + 2^-6


def test_combine_rounds_once_and_adds_residual():
    rng = np.random.default_rng(3)
    T, d = 50, 8
    y = rng.standard_normal((T, d))
    inv = rng.permutation(T).astype(np.int32)
    gate = rng.random(T).astype(np.float32)
    res = wl.f32_to_bf16_bits(rng.standard_normal((T, d)).astype(np.float32))
    out = oracle.combine(y, inv, gate, oracle.F64, residual=res)
    ref = gate.astype(np.float64)[:, None] * y[inv] + wl.bf16_bits_to_f32(res).astype(np.float64)
    assert np.array_equal(out, ref)
    out16 = oracle.combine(y, inv, gate, oracle.BF16, residual=res)
    assert np.array_equal(out16, oracle.round_bf16(ref))


# --------------------------------------------------------------------- P10 + update rule
def test_select_resident_against_argsort():
    rng = np.random.default_rng(5)
    for _ in range(50):
        E = int(rng.integers(2, 20)); K = int(rng.integers(1, E + 1))
        score = rng.random(E)
        score[rng.integers(0, E, 3)] = 0.5       # some exact ties
        s2e = rng.permutation(E)[:K].astype(np.int32)
        e2s = np.full(E, -1, np.int32); e2s[s2e] = np.arange(K)
        n2e, n_e2s, loads = oracle.select_resident(score, s2e, e2s)
        want = sorted(range(E), key=lambda e: (-score[e], e))[:K]
        assert sorted(n2e.tolist()) == sorted(want)
        for s in range(K):                        # stayers keep their slot
            if s2e[s] in want:
                assert n2e[s] == s2e[s]
        assert all(n_e2s[n2e[s]] == s for s in range(K))
        assert (n_e2s >= 0).sum() == K
        assert [s for s, _ in loads] == sorted(s for s, _ in loads)
        assert [e for _, e in loads] == sorted((e for _, e in loads), key=lambda e: (-score[e], e))
        assert {e for _, e in loads} == set(want) - set(s2e.tolist())


def test_update_brings_in_the_preferred_expert():
    """All tokens come from one cluster whose favourite expert is not resident:
    after one update it is, and those tokens then get the full layer's output."""
    E, K, d, f, T = 8, 2, 32, 16, 64
    cfg, x, Wr, W1, W2, s2e, e2s = _rand_layer(23, E, K, d, f, T)
    rng = np.random.default_rng(0)
    j = 6
    centre = Wr[j] / np.linalg.norm(Wr[j]) * 4
    x = (centre[None, :] + 0.05 * rng.standard_normal((T, d))).astype(np.float32)
    r = oracle.layer_forward(x, Wr, W1[s2e], W2[s2e], e2s, out_dtype=oracle.F64)
    assert (r["orig_expert"] == j).all() and e2s[j] < 0
    en = oracle.expert_norm(W1, W2)
    _, _, score = oracle.importance(r["orig_expert"], r["orig_gate"], r["xnorm"], en)
    n2e, n_e2s, loads = oracle.select_resident(score, s2e, e2s)
    assert n_e2s[j] >= 0 and (n_e2s[j], j) in loads
    r2 = oracle.layer_forward(x, Wr, W1[n2e], W2[n2e], n_e2s, out_dtype=oracle.F64)
    _, e2s_full = wl.initial_resident(cfg.scaled(K=E))
    full = oracle.layer_forward(x, Wr, W1, W2, e2s_full, out_dtype=oracle.F64)
    assert np.array_equal(r2["out"], full["out"])
    assert not np.array_equal(r["out"], full["out"])


# --------------------------------------------------------------------- policies
def test_policy_rankings_and_update_rule_by_hand():
    """The three rankings the evaluation compares feed the same update rule: Eq. 1 score
    (SwapMoE), token count ("simple scheduling", Section 4.5) and expert magnitude (the
    "Pruning" baseline, Section 4.1).  Expected resident sets written out by hand."""
    count = np.array([5, 0, 9, 9, 1, 2], np.int32)
    score = np.array([0.5, 0.0, 2.0, 0.1, 3.0, 0.2])
    en = np.array([1.0, 6.0, 2.0, 5.0, 3.0, 4.0])
    s2e = np.array([0, 1, 2], np.int32)
    e2s = np.array([0, 1, 2, -1, -1, -1], np.int32)
    want = {
        oracle.POLICY_IMPORTANCE: (score, [0, 4, 2], [(1, 4)]),             # top 3 by score: 4, 2, 0
        oracle.POLICY_COUNT: (count.astype(np.float64), [0, 3, 2], [(1, 3)]),   # 2 and 3 tie at 9, then 0
        oracle.POLICY_MAGNITUDE: (en, [3, 1, 5], [(0, 3), (2, 5)]),          # 1, 3, 5; newcomers by magnitude
    }
    for policy, (rank_want, s2e_want, loads_want) in want.items():
        rank = oracle.policy_scores(policy, count, score, en)
        assert np.array_equal(rank, rank_want)
        n_s2e, n_e2s, loads = oracle.select_resident(rank, s2e, e2s)
        assert n_s2e.tolist() == s2e_want and loads == loads_want, policy
        assert np.array_equal(n_e2s[n_s2e], np.arange(3))
    with pytest.raises(ValueError):
        oracle.policy_scores(7, count, score, en)


def test_on_demand_least_recently_used_by_hand():
    """Load-on-miss with least-recently-used replacement over four batches, every plan worked
    out by hand (K = 2 slots, E = 5 experts, slots start with experts 0 and 1)."""
    K, E = 2, 5
    s2e = np.array([0, 1], np.int32)
    e2s = np.array([0, 1, -1, -1, -1], np.int32)
    od = oracle.OnDemand(K)
    script = [
        # batch's original choices, expected loads, why
        ([0, 2, 2, 3], [(1, 2)]),          # slot 0 is used now; 2 (asked twice) beats 3; only slot 1 is free to evict
        ([1, 1, 4],    [(0, 1), (1, 4)]),  # no hit; both slots equally stale -> lower slot first; 1 (twice) before 4
        ([1, 0, 0, 2], [(1, 0)]),          # expert 1 (slot 0) is hit; 0 (twice) replaces the stale slot 1; 2 finds no slot
        ([3],          [(0, 3)]),          # both stamped in batch 3: the lower slot goes
        ([],           []),                # an empty batch asks for nothing
    ]
    for choices, loads_want in script:
        loads = od.plan(np.array(choices, np.int32), e2s)
        assert loads == loads_want, (choices, loads)
        for sl, ex in loads:
            e2s[s2e[sl]] = -1
            s2e[sl] = ex
            e2s[ex] = sl
    assert s2e.tolist() == [3, 0] and int(od.clock[0]) == 5
    # a resident expert is never loaded, and no slot is evicted twice in one batch
    od2 = oracle.OnDemand(3)
    e2s3 = np.array([0, 1, 2, -1, -1, -1, -1], np.int32)
    loads = od2.plan(np.array([3, 4, 5, 6, 6], np.int32), e2s3)
    assert loads == [(0, 6), (1, 3), (2, 4)]
