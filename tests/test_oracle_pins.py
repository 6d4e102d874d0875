"""Pins for the fp64 CPU oracle: closed forms, invariants, library special cases, autodiff and
finite differences.  None of these re-uses the oracle's own loops: each expected value comes
from mathematics (a closed form), from a stock library routine (torch's cross-entropy and
autograd in fp64), or from numerical differentiation of the oracle's *loss value*.

The paper prints no worked numeric example of the objective, so every pin is analytic.
"""
import math

import numpy as np
import pytest
import torch

import oracle

RNG = np.random.RandomState(20250727)


def softmax_from_oracle(z, y):
    """q = onehot - dz for g = 1 (uses only the oracle's gradient entry point)."""
    lse, _, _ = oracle.row_stats(z, y)
    dz = oracle.dlogits(z, y, lse, np.ones(z.shape[0]))
    onehot = np.zeros_like(dz)
    onehot[np.arange(z.shape[0]), y] = 1.0
    return onehot - dz


# ----------------------------------------------------------------------------- softmax / entropy

def test_probabilities_sum_to_one():
    z = RNG.normal(0, 3, size=(37, 1000))
    y = RNG.randint(0, 1000, size=37)
    q = softmax_from_oracle(z, y)
    assert np.all(q >= 0)
    np.testing.assert_allclose(q.sum(1), 1.0, rtol=0, atol=1e-12)


@pytest.mark.parametrize("V", [4096, 151936])
def test_uniform_row_has_entropy_log_V(V):
    for level in (0.0, -7.25, 11.0):
        z = np.full((2, V), level, dtype=np.float32)
        lse, logp, H = oracle.row_stats(z, np.array([0, V - 1]))
        np.testing.assert_allclose(H, math.log(V), rtol=1e-11)   # V sequential adds
        np.testing.assert_allclose(logp, -math.log(V), rtol=1e-13)
        np.testing.assert_allclose(lse, level + math.log(V), rtol=1e-13)


def test_masked_vocabulary_entries_have_probability_zero():
    """A logit of -infinity is a masked vocabulary entry: with k equal finite logits and the rest
    masked the row is uniform over k entries (H = ln k), and a masked column gets a zero gradient."""
    V, k = 1000, 37
    z = np.full((1, V), -np.inf, dtype=np.float32)
    keep = np.arange(0, V, 27)[:k]
    z[0, keep] = 2.5
    lse, logp, H = oracle.row_stats(z, np.array([keep[3]]))
    np.testing.assert_allclose(H, math.log(k), rtol=1e-12)
    np.testing.assert_allclose(logp, -math.log(k), rtol=1e-12)
    np.testing.assert_allclose(lse, 2.5 + math.log(k), rtol=1e-12)
    dz = oracle.dlogits(z, np.array([keep[3]]), lse, np.array([0.7]))
    masked = np.ones(V, dtype=bool)
    masked[keep] = False
    assert np.all(dz[0, masked] == 0.0)
    np.testing.assert_allclose(dz[0, keep].sum(), 0.0, atol=1e-15)


def spike_closed_form(V, a):
    """One logit at a, the other V-1 at 0:  p = e^a / (e^a + V - 1),
    H = -p ln p - (1-p) ln((1-p)/(V-1))."""
    p = math.exp(a) / (math.exp(a) + V - 1)
    H = -p * math.log(p) - (1 - p) * math.log((1 - p) / (V - 1))
    return p, H


@pytest.mark.parametrize("V,a,p_ref,H_ref", [
    (4096, 12.0, 0.975457, 0.319366),     # rounded values of the closed form, kept as a
    (4096, 15.0, 0.998749, 0.020018),     # guard against an error in spike_closed_form itself
    (151936, 15.0, 0.955587, 0.711626),
])
def test_spike_row_closed_form(V, a, p_ref, H_ref):
    p, H = spike_closed_form(V, a)
    assert abs(p - p_ref) < 1e-6 and abs(H - H_ref) < 1e-6
    z = np.zeros((1, V))
    z[0, 1234] = a
    lse, logp, Hor = oracle.row_stats(z, np.array([1234]))
    np.testing.assert_allclose(np.exp(logp[0]), p, rtol=1e-10)    # V sequential adds
    np.testing.assert_allclose(Hor[0], H, rtol=1e-10)  # 1-p cancels in the closed form
    # a non-chosen token of the same row: p' = (1-p)/(V-1)
    _, logp2, _ = oracle.row_stats(z, np.array([7]))
    np.testing.assert_allclose(np.exp(logp2[0]), (1 - p) / (V - 1), rtol=1e-9)


def test_one_hot_dominant_row_has_entropy_near_zero():
    z = np.zeros((1, 4096), dtype=np.float32)
    z[0, 5] = 60.0
    _, logp, H = oracle.row_stats(z, np.array([5]))
    assert 0 <= H[0] < 1e-20
    assert abs(logp[0]) < 1e-20


def test_shift_and_permutation_invariance():
    z = RNG.normal(0, 2, size=(5, 257))
    y = RNG.randint(0, 257, size=5)
    lse, logp, H = oracle.row_stats(z, y)
    lse2, logp2, H2 = oracle.row_stats(z + 3.5, y)
    np.testing.assert_allclose(logp2, logp, atol=1e-13)
    np.testing.assert_allclose(H2, H, atol=1e-12)
    np.testing.assert_allclose(lse2, lse + 3.5, atol=1e-13)
    perm = RNG.permutation(257)
    inv = np.argsort(perm)
    lse3, logp3, H3 = oracle.row_stats(np.ascontiguousarray(z[:, perm]), inv[y])
    np.testing.assert_allclose(logp3, logp, atol=1e-13)
    np.testing.assert_allclose(H3, H, atol=1e-12)


def test_bf16_storage_decodes_like_the_library():
    t = torch.randn(3, 64, dtype=torch.float32).mul(5).to(torch.bfloat16)
    raw = t.view(torch.int16).numpy().view(np.uint16)
    y = np.array([1, 2, 3])
    a = oracle.row_stats(raw, y)
    b = oracle.row_stats(t.to(torch.float64).numpy(), y)
    for u, v in zip(a, b):
        np.testing.assert_array_equal(u, v)


def test_row_stride_is_honoured():
    big = RNG.normal(size=(4, 100)).astype(np.float32)
    view = big[:, :60]
    a = oracle.row_stats(view, np.array([0, 1, 2, 59]))
    b = oracle.row_stats(np.ascontiguousarray(view), np.array([0, 1, 2, 59]))
    for u, v in zip(a, b):
        np.testing.assert_array_equal(u, v)


def test_sentinel_logit_pins_token_indexing():
    z = RNG.normal(size=(6, 50))
    y = np.array([0, 49, 7, 7, 23, 1])
    lse, logp, _ = oracle.row_stats(z, y)
    for t in range(6):
        z2 = z.copy()
        z2[t, y[t]] = -1e9      # removing exactly the chosen logit must drive only row t to -inf-ish
        _, lp2, _ = oracle.row_stats(z2, y)
        assert lp2[t] < -1e8
        others = np.arange(6) != t
        np.testing.assert_array_equal(lp2[others], logp[others])


def test_out_of_range_token_is_rejected():
    z = np.zeros((2, 8))
    with pytest.raises(ValueError):
        oracle.row_stats(z, np.array([0, 8]))


# ----------------------------------------------------------------------------- library special case

def test_reduces_to_library_cross_entropy():
    """A = 1, ratio = 1 (POIS), no mask  =>  loss = mean NLL, dz = (softmax - onehot)/N."""
    N, V = 24, 300
    z = RNG.normal(0, 2, size=(N, V))
    y = RNG.randint(0, V, size=N)
    zt = torch.tensor(z, dtype=torch.float64, requires_grad=True)
    ce = torch.nn.functional.cross_entropy(zt, torch.tensor(y), reduction="mean")
    ce.backward()
    lse, logp, H = oracle.row_stats(z, y)
    tt = oracle.token_terms(logp, H, [0, 10, N], np.ones(N), None, is_mode=oracle.IS_POIS,
                            gate_mode=oracle.GATE_NEVER)
    # POIS value of the surrogate is sum(A)/D = 1, the NLL appears through the gradient
    assert tt.loss == -1.0
    dz = oracle.dlogits(z, y, lse, tt.gcoef)
    np.testing.assert_allclose(dz, zt.grad.numpy(), rtol=1e-10, atol=1e-16)
    np.testing.assert_allclose(-logp.mean(), ce.item(), rtol=1e-12)


# ----------------------------------------------------------------------------- ratio, clip, mask

def test_ratio_is_exactly_one_when_old_equals_current():
    N, V = 64, 128
    z = RNG.normal(0, 3, size=(N, V))
    z[::3, 5] += 14
    y = np.where(np.arange(N) % 3 == 0, 5, RNG.randint(0, V, size=N))
    lse, logp, H = oracle.row_stats(z, y)
    adv = np.where(np.arange(N) < 40, 1.0, -1.0)
    tt = oracle.token_terms(logp, H, [0, 40, N], adv, logp.copy(), gate_mode=oracle.GATE_ALWAYS)
    assert np.all(tt.ratio == 1.0)
    assert tt.n_clip_inactive == 0
    p = np.exp(logp)
    expect_mask = (adv > 0) & (p >= 0.99)
    assert expect_mask.sum() > 0
    np.testing.assert_array_equal(tt.mask, expect_mask.astype(np.uint8))
    # +-1 advantages: the loss is an integer count over D
    count = int((adv[~expect_mask] > 0).sum()) - int((adv[~expect_mask] < 0).sum())
    assert tt.loss == -count / N
    pois = oracle.token_terms(logp, H, [0, 40, N], adv, None, is_mode=oracle.IS_POIS,
                              gate_mode=oracle.GATE_ALWAYS)
    assert pois.loss == tt.loss
    np.testing.assert_array_equal(pois.gcoef, tt.gcoef)


@pytest.mark.parametrize("r,A,s_ref,active", [
    (1.5, +1.0, 1.2, False),
    (0.5, +1.0, 0.5, True),
    (1.5, -1.0, -1.5, True),
    (0.5, -1.0, -0.8, False),
    (1.0, +1.0, 1.0, True),
    (1.1, -2.0, -2.2, True),
])
def test_clip_quadrants_by_hand(r, A, s_ref, active):
    logp = np.array([-1.0])
    old = logp - math.log(r)
    tt = oracle.token_terms(logp, np.array([5.0]), [0, 1], np.array([A]), old,
                            gate_mode=oracle.GATE_NEVER, denominator=1.0)
    np.testing.assert_allclose(tt.ratio[0], r, rtol=1e-14)
    np.testing.assert_allclose(tt.surrogate[0], s_ref, rtol=1e-14)
    np.testing.assert_allclose(tt.loss, -s_ref, rtol=1e-14)
    assert tt.n_clip_inactive == (0 if active else 1)
    if active:
        np.testing.assert_allclose(tt.gcoef[0], -r * A, rtol=1e-14)
    else:
        assert tt.gcoef[0] == 0.0


def test_asymmetric_clip_range():
    logp = np.zeros(2)
    old = logp - np.log([1.25, 0.85])
    tt = oracle.token_terms(logp, np.ones(2), [0, 2], np.array([1.0, -1.0]), old, eps_low=0.1,
                            eps_high=0.28, gate_mode=oracle.GATE_NEVER, denominator=1.0)
    # r=1.25 < 1.28 with A>0: unclipped; r=0.85 < 0.9 with A<0: clipped at 0.9
    np.testing.assert_allclose(tt.surrogate, [1.25, -0.9], rtol=1e-14)
    assert tt.n_clip_inactive == 1


def test_threshold_boundary_of_the_mpt_set():
    V = 4096
    a_star = math.log(99 * (V - 1))          # p = 0.99 exactly in exact arithmetic
    assert abs(a_star - 12.912642) < 1e-6
    z = np.zeros((3, V))
    z[0, 9] = a_star + 1e-6
    z[1, 9] = a_star - 1e-6
    z[2, 9] = a_star + 1e-6
    y = np.array([9, 9, 9])
    lse, logp, H = oracle.row_stats(z, y)
    adv = np.array([1.0, 1.0, -1.0])
    tt = oracle.token_terms(logp, H, [0, 3], adv, logp, gate_mode=oracle.GATE_ALWAYS)
    # above the threshold & positive -> masked; below -> kept; negative advantage -> never masked
    np.testing.assert_array_equal(tt.mask, [1, 0, 0])
    assert tt.gcoef[0] == 0.0 and tt.gcoef[1] != 0.0 and tt.gcoef[2] != 0.0
    assert tt.n_masked == 1 and tt.n_pos == 2
    # the masked token's whole gradient row is exactly zero
    dz = oracle.dlogits(z, y, lse, tt.gcoef)
    assert np.all(dz[0] == 0.0) and np.any(dz[1] != 0.0)
    # it also contributes exactly nothing to the loss: D stays N=3 (all tokens counted)
    assert tt.loss == -(1.0 - 1.0) / 3.0 or tt.loss == 0.0
    # zero advantage is not "positive"
    t0 = oracle.token_terms(logp[:1], H[:1], [0, 1], np.array([0.0]), logp[:1],
                            gate_mode=oracle.GATE_ALWAYS)
    assert t0.mask[0] == 0


def test_gate_modes_and_strictness():
    V = 512
    p_spike, H_spike = spike_closed_form(V, 14.0)
    z = np.zeros((6, V))
    z[3:, 2] = 14.0                               # response 1: three peaked rows
    y = np.array([0, 1, 2, 2, 2, 2])
    lse, logp, H = oracle.row_stats(z, y)
    adv = np.ones(6)
    cu = [0, 3, 6]
    sigma = 0.5 * (math.log(V) + H_spike)
    tt = oracle.token_terms(logp, H, cu, adv, logp, sigma=sigma)
    np.testing.assert_allclose(tt.resp_entropy, [math.log(V), H_spike], rtol=1e-11)
    np.testing.assert_array_equal(tt.resp_gate, [0, 1])
    assert p_spike > 0.99
    np.testing.assert_array_equal(tt.mask, [0, 0, 0, 1, 1, 1])
    # sigma far above both: both responses gated, but uniform rows are not MPTs
    tt2 = oracle.token_terms(logp, H, cu, adv, logp, sigma=100.0)
    np.testing.assert_array_equal(tt2.resp_gate, [1, 1])
    np.testing.assert_array_equal(tt2.mask, [0, 0, 0, 1, 1, 1])
    # the paper's sigma = 0.2 lies above the peaked response's mean entropy only if H_spike < .2
    assert H_spike < 0.2
    tt3 = oracle.token_terms(logp, H, cu, adv, logp)       # defaults tau=.99 sigma=.2
    np.testing.assert_array_equal(tt3.resp_gate, [0, 1])
    # strict inequality: H-bar == sigma does not gate, the next double above does
    hb = tt.resp_entropy[1]
    eq = oracle.token_terms(logp, H, cu, adv, logp, sigma=hb)
    up = oracle.token_terms(logp, H, cu, adv, logp, sigma=np.nextafter(hb, np.inf))
    assert eq.resp_gate[1] == 0 and up.resp_gate[1] == 1
    # never / always / global
    assert oracle.token_terms(logp, H, cu, adv, logp, gate_mode=oracle.GATE_NEVER).mask.sum() == 0
    al = oracle.token_terms(logp, H, cu, adv, logp, gate_mode=oracle.GATE_ALWAYS, sigma=-1.0)
    np.testing.assert_array_equal(al.mask, [0, 0, 0, 1, 1, 1])
    hglob = H.mean()
    lo = oracle.token_terms(logp, H, cu, adv, logp, gate_mode=oracle.GATE_GLOBAL, sigma=hglob * 0.99)
    hi = oracle.token_terms(logp, H, cu, adv, logp, gate_mode=oracle.GATE_GLOBAL, sigma=hglob * 1.01)
    assert lo.mask.sum() == 0 and list(hi.resp_gate) == [1, 1] and hi.mask.sum() == 3


def test_mean_entropy_spans_the_whole_response_not_a_segment():
    H = np.array([1.0, 1.0, 0.0, 0.0, 0.0, 0.0])
    logp = np.full(6, -1e-4)
    tt = oracle.token_terms(logp, H, [0, 6], np.ones(6), logp, seg_len=2, sigma=0.34)
    np.testing.assert_allclose(tt.resp_entropy, [1.0 / 3.0])
    assert tt.resp_gate[0] == 1 and tt.mask.sum() == 6
    np.testing.assert_array_equal(tt.seg, [0, 0, 1, 1, 2, 2])


def test_denominator_counts_all_tokens_and_can_be_overridden():
    logp = np.full(8, -0.001)
    H = np.full(8, 0.01)
    adv = np.array([1, 1, 1, 1, -1, -1, -1, -1.0])
    tt = oracle.token_terms(logp, H, [0, 4, 8], adv, logp, gate_mode=oracle.GATE_ALWAYS)
    assert tt.n_masked == 4
    # 4 masked positive tokens vanish, 4 negative ones stay: J = -4/8 (not -4/4)
    assert tt.loss == 0.5
    np.testing.assert_array_equal(tt.gcoef[:4], 0.0)
    np.testing.assert_allclose(tt.gcoef[4:], 1.0 / 8.0)
    tt2 = oracle.token_terms(logp, H, [0, 4, 8], adv, logp, gate_mode=oracle.GATE_ALWAYS,
                             denominator=32.0)
    assert tt2.loss == 4.0 / 32.0


def test_segment_ids_from_offsets_brute_force():
    lengths = [5, 1, 12, 7]
    cu = np.concatenate([[0], np.cumsum(lengths)])
    N = cu[-1]
    seg_len = 4
    expect = []
    for L in lengths:
        k, c = 0, 0
        for _ in range(L):
            expect.append(k)
            c += 1
            if c == seg_len:
                k, c = k + 1, 0
    logp = np.full(N, -1.0)
    tt = oracle.token_terms(logp, np.ones(N), cu, np.ones(N), logp, seg_len=seg_len)
    np.testing.assert_array_equal(tt.seg, expect)
    explicit = np.arange(N, dtype=np.int32)[::-1].copy()
    tt2 = oracle.token_terms(logp, np.ones(N), cu, np.ones(N), logp, segment_ids=explicit)
    np.testing.assert_array_equal(tt2.seg, explicit)


def test_malformed_cu_seqlens_is_rejected():
    logp = np.zeros(4)
    with pytest.raises(ValueError):
        oracle.token_terms(logp, logp, [0, 3, 2, 4], np.ones(4), logp)
    with pytest.raises(ValueError):
        oracle.token_terms(logp, logp, [0, 3], np.ones(4), logp)


# ----------------------------------------------------------------------------- gradients

def _oracle_loss_and_grad(z, y, cu, adv, old, **kw):
    lse, logp, H = oracle.row_stats(z, y)
    tt = oracle.token_terms(logp, H, cu, adv, old, **kw)
    return tt, oracle.dlogits(z, y, lse, tt.gcoef), logp


def _smooth_case(V, N, seed):
    """Inputs kept away from every kink of the objective (clip edges, tau, sigma)."""
    rs = np.random.RandomState(seed)
    while True:
        z = rs.normal(0, 1.5, size=(N, V))
        y = rs.randint(0, V, size=N)
        adv = rs.choice([-1.0, 1.0, 0.5, -2.0], size=N)
        lse, logp, H = oracle.row_stats(z, y)
        old = logp + rs.normal(0, 0.25, size=N)      # wide enough that some tokens clip
        r = np.exp(logp - old)
        ok = (np.abs(r - 0.8) > 1e-2).all() and (np.abs(r - 1.2) > 1e-2).all()
        ok = ok and (np.abs(np.exp(logp) - 0.6) > 1e-2).all()
        if ok:
            return z, y, adv, old


@pytest.mark.parametrize("V", [4, 8, 16])
def test_dlogits_matches_central_finite_differences(V):
    N = 8
    cu = [0, 3, N]
    for seed in range(1000):
        # draw until the case exercises both branches of the min, the mask and the gate
        z, y, adv, old = _smooth_case(V, N, seed=1000 * V + seed)
        lse, logp, H = oracle.row_stats(z, y)
        hbar = [H[:3].mean(), H[3:].mean()]
        sigma = 0.5 * (hbar[0] + hbar[1])           # exactly one response gated
        kw = dict(tau=0.6, sigma=sigma, seg_len=2)
        tt, dz, _ = _oracle_loss_and_grad(z, y, cu, adv, old, **kw)
        if abs(hbar[0] - hbar[1]) > 2e-3 and 0 < tt.n_clip_inactive < N and tt.n_masked > 0:
            break
    else:
        raise AssertionError("no suitable case drawn")
    assert tt.resp_gate.sum() == 1
    h = 1e-6
    fd = np.zeros_like(z)
    for t in range(N):
        for j in range(V):
            zp, zm = z.copy(), z.copy()
            zp[t, j] += h
            zm[t, j] -= h
            lp = _oracle_loss_and_grad(zp, y, cu, adv, old, **kw)[0].loss
            lm = _oracle_loss_and_grad(zm, y, cu, adv, old, **kw)[0].loss
            fd[t, j] = (lp - lm) / (2 * h)
    np.testing.assert_allclose(dz, fd, rtol=1e-6, atol=1e-9)
    np.testing.assert_allclose(dz.sum(1), 0.0, atol=1e-15)
    nz = tt.gcoef != 0
    assert np.all(np.sign(dz[np.arange(N), y])[nz] == np.sign(tt.gcoef)[nz])
    # grad_out scales linearly
    dz3 = oracle.dlogits(z, y, lse, tt.gcoef, grad_out=-3.0)
    np.testing.assert_allclose(dz3, -3.0 * dz, rtol=1e-15)


def test_pois_gradient_is_the_on_policy_limit_of_sais():
    """POIS keeps the value r = 1 but differentiates the numerator: its gradient equals the
    finite-difference gradient of the SAIS loss evaluated at old_logp = current logp."""
    N, V = 6, 8
    z, y, adv, _ = _smooth_case(V, N, seed=99)
    cu = [0, N]
    lse, logp, H = oracle.row_stats(z, y)
    tt = oracle.token_terms(logp, H, cu, adv, None, is_mode=oracle.IS_POIS,
                            gate_mode=oracle.GATE_NEVER)
    dz = oracle.dlogits(z, y, lse, tt.gcoef)
    h = 1e-6
    fd = np.zeros_like(z)
    for t in range(N):
        for j in range(V):
            vals = []
            for sgn in (+1, -1):
                z2 = z.copy()
                z2[t, j] += sgn * h
                l2, lp2, H2 = oracle.row_stats(z2, y)
                vals.append(oracle.token_terms(lp2, H2, cu, adv, logp,
                                               gate_mode=oracle.GATE_NEVER).loss)
            fd[t, j] = (vals[0] - vals[1]) / (2 * h)
    np.testing.assert_allclose(dz, fd, rtol=1e-6, atol=1e-9)
    assert tt.loss == -adv.sum() / N and np.all(tt.ratio == 1.0) and tt.n_clip_inactive == 0


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_whole_objective_against_autograd(seed):
    """The objective of Sec. 3.2.2 assembled from stock torch ops in fp64 and differentiated by
    autograd; the oracle's loss and analytic logits gradient must agree."""
    rs = np.random.RandomState(seed)
    lengths = [7, 1, 12]
    N, V = sum(lengths), 33
    cu = np.concatenate([[0], np.cumsum(lengths)])
    z = rs.normal(0, 2.0, size=(N, V))
    z[::2, 3] += 9.0
    y = np.where(np.arange(N) % 2 == 0, 3, rs.randint(0, V, size=N))
    adv = np.repeat([1.0, -1.0, 0.7], lengths)
    tau, eps_lo, eps_hi = 0.9, 0.2, 0.28

    zt = torch.tensor(z, requires_grad=True)
    logq = torch.log_softmax(zt, dim=-1)
    logp_t = logq.gather(1, torch.tensor(y).unsqueeze(1)).squeeze(1)
    ent_t = torch.distributions.Categorical(logits=zt).entropy()
    old = logp_t.detach().numpy() + rs.normal(0, 0.2, size=N)
    hbar = torch.stack([ent_t[cu[i]:cu[i + 1]].mean() for i in range(3)])
    srt = np.sort(hbar.detach().numpy())
    sigma = 0.5 * (srt[1] + srt[2])                  # two of three responses gated
    gate = (hbar < sigma)[torch.tensor(np.repeat(np.arange(3), lengths))]
    A = torch.tensor(adv)
    mpt = (A > 0) & (logp_t.exp() >= tau)
    keep = (~(gate & mpt)).to(torch.float64)
    r = torch.exp(logp_t - torch.tensor(old))
    sur = torch.minimum(r * A, torch.clamp(r, 1 - eps_lo, 1 + eps_hi) * A)
    loss = -(keep.detach() * sur).sum() / N
    loss.backward()

    tt, dz, logp = _oracle_loss_and_grad(z, y, cu, adv, old, tau=tau, sigma=sigma,
                                         eps_low=eps_lo, eps_high=eps_hi)
    np.testing.assert_allclose(logp, logp_t.detach().numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(tt.resp_entropy, hbar.detach().numpy(), rtol=1e-11)
    np.testing.assert_array_equal(tt.mask, (gate & mpt).numpy().astype(np.uint8))
    assert 0 < tt.n_masked < N
    np.testing.assert_allclose(tt.loss, loss.item(), rtol=1e-12)
    np.testing.assert_allclose(dz, zt.grad.numpy(), rtol=1e-9, atol=1e-15)


# ----------------------------------------------------------------------------- lm_head variant

def _raw_bf16(t: torch.Tensor) -> np.ndarray:
    return t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def test_lmhead_logits_and_grads_against_loops_and_autograd():
    rs = np.random.RandomState(5)
    N, Hd, V = 7, 8, 24
    h = torch.tensor(rs.normal(size=(N, Hd))).to(torch.bfloat16)
    w = torch.tensor(rs.normal(0, 0.5, size=(Hd, V))).to(torch.bfloat16)
    hr, wr = _raw_bf16(h), _raw_bf16(w)
    z = oracle.lmhead_logits(hr, wr)
    # brute force triple loop on the exactly decoded operands
    hd, wd = h.double().numpy(), w.double().numpy()
    ref = np.zeros((N, V))
    for t in range(N):
        for v in range(V):
            for k in range(Hd):
                ref[t, v] += hd[t, k] * wd[k, v]
    np.testing.assert_allclose(z, ref, rtol=1e-13, atol=1e-15)
    # one-hot hidden rows pick rows of W exactly
    e = torch.zeros(3, Hd)
    e[0, 2] = e[1, 5] = e[2, 7] = 1.0
    np.testing.assert_array_equal(oracle.lmhead_logits(_raw_bf16(e), wr), wd[[2, 5, 7]])

    # the whole lm_head objective differentiated by autograd (fp64) vs the oracle's chain rule
    y = rs.randint(0, V, size=N)
    adv = rs.choice([-1.0, 1.0], size=N)
    ht = h.double().requires_grad_(True)
    wt = w.double().requires_grad_(True)
    logq = torch.log_softmax(ht @ wt, -1)
    lp = logq.gather(1, torch.tensor(y)[:, None])[:, 0]
    old = lp.detach().numpy() + rs.normal(0, 0.15, size=N)
    r = torch.exp(lp - torch.tensor(old))
    A = torch.tensor(adv)
    loss = -torch.minimum(r * A, torch.clamp(r, 0.8, 1.2) * A).sum() / N
    loss.backward()
    lse, logp, H = oracle.row_stats(z, y)
    tt = oracle.token_terms(logp, H, [0, 3, N], adv, old, gate_mode=oracle.GATE_NEVER)
    np.testing.assert_allclose(tt.loss, loss.item(), rtol=1e-12)
    dz = oracle.dlogits(z, y, lse, tt.gcoef)
    dh, dw = oracle.lmhead_grads(hr, wr, dz)
    np.testing.assert_allclose(dh, ht.grad.numpy(), rtol=1e-9, atol=1e-14)
    np.testing.assert_allclose(dw, wt.grad.numpy(), rtol=1e-9, atol=1e-14)


# ----------------------------------------------------------------------------- neighbours of the hot path

def test_group_advantages_closed_forms():
    # G = 4 with binary rewards: k correct of 4 -> mean k/4, population std sqrt(k(4-k))/4
    cu = np.arange(0, 9 * 3, 3)[:9]            # 8 responses of 3 tokens
    cu = np.concatenate([[0], np.cumsum([3, 1, 2, 4, 3, 3, 3, 3])])
    rewards = [1, 0, 0, 0,   1, 1, 1, 1]
    resp, keep, tok, kept = oracle.advantages(rewards, cu, 4, eps=0.0)
    sd = math.sqrt(3) / 4
    np.testing.assert_allclose(resp[:4], [0.75 / sd, -0.25 / sd, -0.25 / sd, -0.25 / sd], rtol=1e-14)
    assert list(keep) == [1, 0] and np.all(resp[4:] == 0.0)          # all-correct group is filtered
    assert kept == 3 + 1 + 2 + 4
    np.testing.assert_array_equal(tok[:3], resp[0])
    np.testing.assert_array_equal(tok[3:4], resp[1])
    assert np.all(tok[10:] == 0.0)
    # advantages of a kept group sum to zero and have unit population variance
    assert abs(resp[:4].sum()) < 1e-14 and abs((resp[:4] ** 2).mean() - 1.0) < 1e-14
    # with {0,1} rewards in a mixed group: reward 1 <=> positive advantage (Sec. 3.3)
    assert np.all((resp[:4] > 0) == (np.array(rewards[:4]) > 0))
    # the library's group normalisation: torch.std unbiased / population
    r = np.array([1.0, 0.0, 1.0, 0.0, 0.0, 0.0, 1.0, 0.0])
    cu8 = np.arange(9)
    for unbiased in (False, True):
        a, k, _, _ = oracle.advantages(r, cu8, 8, eps=1e-6, unbiased=unbiased)
        t = torch.tensor(r)
        ref = (t - t.mean()) / (t.std(unbiased=unbiased) + 1e-6)
        np.testing.assert_allclose(a, ref.numpy(), rtol=1e-13)
    # overlong samples are scored as wrong: a correct but truncated answer gets the negative side
    a, k, _, _ = oracle.advantages([1, 1, 0, 0], np.arange(5), 4, truncated=[1, 0, 0, 0], eps=0.0)
    b, _, _, _ = oracle.advantages([0, 1, 0, 0], np.arange(5), 4, eps=0.0)
    np.testing.assert_array_equal(a, b)
    # all wrong after truncation -> group dropped
    a, k, _, kept = oracle.advantages([1, 0], np.arange(3), 2, truncated=[1, 0], eps=0.0)
    assert list(k) == [0] and kept == 0 and np.all(a == 0)
    with pytest.raises(ValueError):
        oracle.advantages([1, 0, 1], np.arange(4), 2)


def test_segment_diagnostics_against_masks_and_library_sums():
    rs = np.random.RandomState(8)
    N, K = 500, 5
    seg = rs.randint(-1, K + 1, size=N)
    logp = -rs.exponential(1.0, size=N)
    old = logp + rs.normal(0, 0.2, size=N)
    ratio = np.exp(logp - old)
    ent = rs.uniform(0, 5, size=N)
    mask = rs.randint(0, 2, size=N)
    adv = rs.choice([-1.0, 1.0], size=N)
    d = oracle.segment_diagnostics(seg, ratio, logp, old, ent, mask, adv, K)
    assert d["out_of_range"] == int(((seg < 0) | (seg >= K)).sum())
    inactive = ((adv > 0) & (ratio > 1.2)) | ((adv < 0) & (ratio < 0.8))
    for k in range(K):
        m = seg == k
        assert d["count"][k] == m.sum()
        np.testing.assert_allclose(d["ratio_sum"][k], math.fsum(ratio[m]), rtol=1e-13)
        assert d["ratio_max"][k] == ratio[m].max()
        assert d["clipped"][k] == inactive[m].sum()
        np.testing.assert_allclose(d["kl_sum"][k], math.fsum((old - logp)[m]), rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(d["ent_sum"][k], math.fsum(ent[m]), rtol=1e-13)
        assert d["masked"][k] == mask[m].sum()
    # on-policy data: every ratio is 1, nothing clipped, the KL estimate vanishes
    d0 = oracle.segment_diagnostics(np.zeros(N, int), np.ones(N), logp, logp, ent, mask, adv, 1)
    assert d0["ratio_sum"][0] == N and d0["clipped"][0] == 0 and d0["kl_sum"][0] == 0.0
