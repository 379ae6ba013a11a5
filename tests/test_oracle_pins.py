"""Pins of the CPU oracle against what the paper and the mathematics fix.

The paper prints no worked example, so every pin is a hand-worked fixture, a
closed form, an invariant, brute force or autograd.  Each test is chosen so a
plausible mistake in the oracle (dropped term, wrong sign or index,
transposed operand, missing 1/n) fails it.
"""
import json
import os

import numpy as np
import pytest
import torch

from oracle import isopo_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_layer(rng, lengths, d_in, d_out, sx=1.0, sd=0.1):
    n = int(np.sum(lengths))
    X = rng.standard_normal((n, d_in)) * sx
    D = rng.standard_normal((n, d_out)) * sd
    off = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    return X, D, off


def test_hand_worked_fixture():
    """Hand-derived 2-sequence example: G, K, Fisher norms, both coefficient
    variants, dW and the REINFORCE gradient."""
    with open(os.path.join(GOLDEN, "hand_worked_two_sequences.json")) as f:
        g = json.load(f)
    X, D, off = np.array(g["X"], float), np.array(g["Delta"], float), g["seq_offsets"]
    A = np.array(g["A"], float)
    G = orc.seq_logprob_grads(X, D, off)
    np.testing.assert_array_equal(G, np.array(g["G"], float))
    K = orc.ntk_from_seq_grads(G)
    np.testing.assert_array_equal(K, np.array(g["K"], float))
    np.testing.assert_allclose(orc.fisher_norm_sq(K), g["fisher_norm_sq"], rtol=1e-15)
    np.testing.assert_allclose(orc.coeff_fisher(K, A, g["fisher_reg"]), g["c_fisher"], rtol=1e-13)
    c, info = orc.coeff_interacting(K, A, g["interacting_reg"])
    assert info == 0
    np.testing.assert_allclose(c * 69, g["c_interacting_times_69"], rtol=1e-13)
    np.testing.assert_allclose(orc.weighted_grad(G, c) * 69, g["dW_interacting_times_69"], rtol=1e-13)
    np.testing.assert_allclose(orc.weighted_grad(G, A), g["dW_reinforce"], rtol=1e-15)
    step = orc.layer_step(X, D, off, A, "interacting", g["interacting_reg"])
    np.testing.assert_allclose(step["dW"] * 69, g["dW_interacting_times_69"], rtol=1e-13)
    np.testing.assert_allclose(step["dW_reinforce"], g["dW_reinforce"], rtol=1e-15)


def test_p1_autograd_brute_force():
    """A tiny softmax policy logits = W x_t: autograd's d/dW of each sequence's
    summed log-prob equals Delta_i^T X_i with Delta_t = onehot(y_t) - softmax.
    Pins the per-sequence gradient and its d_out x d_in orientation, then K and
    the interacting update via autograd Jacobian rows."""
    torch.manual_seed(0)
    d_in, d_out = 5, 7
    lengths = [3, 1, 4]
    n = sum(lengths)
    W = torch.randn(d_out, d_in, dtype=torch.float64, requires_grad=True)
    X = torch.randn(n, d_in, dtype=torch.float64)
    y = torch.randint(0, d_out, (n,))
    off = np.concatenate([[0], np.cumsum(lengths)])
    J = []
    for i in range(len(lengths)):
        s, e = off[i], off[i + 1]
        logp = torch.log_softmax(X[s:e] @ W.T, dim=1)
        obj = logp[torch.arange(e - s), y[s:e]].sum()
        (gW,) = torch.autograd.grad(obj, W)
        J.append(gW.numpy().copy())
    J = np.stack(J)
    with torch.no_grad():
        Delta = (torch.nn.functional.one_hot(y, d_out).double() - torch.softmax(X @ W.T, dim=1)).numpy()
    G = orc.seq_logprob_grads(X.numpy(), Delta, off)
    np.testing.assert_allclose(G, J, rtol=1e-12, atol=1e-14)
    Jm = J.reshape(len(lengths), -1)
    K = orc.layer_ntk(X.numpy(), Delta, off)
    np.testing.assert_allclose(K, Jm @ Jm.T, rtol=1e-12)
    A = np.array([0.5, -1.0, 2.0])
    lam = 0.3
    v = Jm.T @ np.linalg.solve(K + lam * np.eye(3), A)      # v = J^T (K + cI)^-1 A
    step = orc.layer_step(X.numpy(), Delta, off, A, "interacting", lam)
    np.testing.assert_allclose(step["dW"].ravel(), v, rtol=1e-11)


def test_p2_two_formulas_one_K():
    """Frobenius definition and ghost double sum agree (independent code)."""
    rng = np.random.default_rng(1)
    X, D, off = _rand_layer(rng, [5, 1, 9, 0, 3], 11, 6)
    K1 = orc.layer_ntk(X, D, off)
    K2 = orc.ntk_ghost(X, D, off)
    np.testing.assert_allclose(K1, K2, rtol=1e-11, atol=1e-13 * np.abs(K1).max())
    # chunked accumulation equals the unchunked one
    np.testing.assert_allclose(orc.layer_ntk(X, D, off, chunk_rows=4), K1, rtol=1e-12)
    for (i, j) in [(0, 0), (0, 2), (4, 1), (3, 3)]:
        np.testing.assert_allclose(orc.ntk_entry(X, D, off, i, j), K1[i, j], rtol=1e-12, atol=1e-18)


def test_p3_symmetry_psd_diagonal():
    rng = np.random.default_rng(2)
    X, D, off = _rand_layer(rng, [4, 7, 2, 6, 3, 5], 8, 9)
    G = orc.seq_logprob_grads(X, D, off)
    K = orc.ntk_from_seq_grads(G)
    assert np.array_equal(K, K.T)
    assert np.linalg.eigvalsh(K).min() >= -1e-12 * np.trace(K)
    np.testing.assert_allclose(np.diag(K), [np.sum(g * g) for g in G], rtol=1e-14)
    # more sequences than parameters: K is rank-deficient but still PSD
    X, D, off = _rand_layer(rng, [2] * 8, 2, 3)
    K = orc.layer_ntk(X, D, off)
    ev = np.linalg.eigvalsh(K)
    assert ev.min() >= -1e-12 * np.trace(K) and (ev < 1e-10 * ev.max()).sum() >= 2


def test_p4_rank_one_closed_form():
    """Every sequence one token long: K_ij = (x_i . x_j)(delta_i . delta_j)."""
    rng = np.random.default_rng(3)
    X, D, off = _rand_layer(rng, [1] * 6, 5, 4)
    K = orc.layer_ntk(X, D, off)
    np.testing.assert_allclose(K, (X @ X.T) * (D @ D.T), rtol=1e-12)


def test_p5_unit_fisher_norm():
    """With reg = 0 each rescaled sequence gradient w_i = G_i / F_i has
    (1/m) sum_j <w_i, G_j>^2 = 1."""
    rng = np.random.default_rng(4)
    X, D, off = _rand_layer(rng, [6, 3, 8, 5], 7, 5)
    G = orc.seq_logprob_grads(X, D, off)
    K = orc.ntk_from_seq_grads(G)
    c = orc.coeff_fisher(K, np.ones(4), 0.0)
    for i in range(4):
        w = c[i] * G[i]
        fn = np.mean([np.sum(w * G[j]) ** 2 for j in range(4)])
        assert abs(fn - 1.0) < 1e-12
    # the regulariser enters under the square root, added to the squared norm
    c_reg = orc.coeff_fisher(K, np.ones(4), 2.5)
    np.testing.assert_allclose(1.0 / c_reg ** 2 - 1.0 / c ** 2, 2.5, rtol=1e-10)


def test_p6_orthogonal_reduction():
    """Exactly orthogonal G_i (each sequence owns a disjoint block of input
    channels): K is diagonal; at reg 0 c_fisher = sqrt(m) c_interacting; for
    reg > 0 the interacting coefficients are A_i / (k_i + reg)."""
    rng = np.random.default_rng(5)
    m, blk, d_out = 4, 3, 5
    lengths = [3, 5, 2, 4]
    X, D, off = _rand_layer(rng, lengths, m * blk, d_out)
    for i in range(m):
        mask = np.zeros(m * blk)
        mask[i * blk:(i + 1) * blk] = 1.0
        X[off[i]:off[i + 1]] *= mask
    K = orc.layer_ntk(X, D, off)
    assert np.abs(K - np.diag(np.diag(K))).max() == 0.0
    A = rng.standard_normal(m)
    cf = orc.coeff_fisher(K, A, 0.0)
    ci, info = orc.coeff_interacting(K, A, 0.0)
    assert info == 0
    np.testing.assert_allclose(cf, np.sqrt(m) * ci, rtol=1e-12)
    lam = 0.7
    ci, _ = orc.coeff_interacting(K, A, lam)
    np.testing.assert_allclose(ci, A / (np.diag(K) + lam), rtol=1e-12)
    np.testing.assert_allclose(orc.coeff_fisher(K, A, lam), A / np.sqrt(np.diag(K) ** 2 / m + lam), rtol=1e-12)
    # for reg > 0 the interacting coefficients match the r = -2 re-scaling ("Alternative sequence
    # re-scalings"): rel_F_norm^2 = (k_i^2/m)/k_i = k_i/m, so A_i/(k_i/m + reg) = m A_i/(k_i + m reg), i.e.
    # interacting(lam) = (1/m) alt(reg = lam/m); the listing's 1e-8 moves it by under 1e-8 relative here
    alt = orc.coeff_rescaled(orc.fisher_norm_sq(K), np.diag(K), A, 0, 0, -2, reg=(0, 0, lam / m), expectation=(None, None, 1.0))
    np.testing.assert_allclose(alt / m, ci, rtol=1e-7)


def test_p7_solve_residual_and_eigh_route():
    rng = np.random.default_rng(6)
    X, D, off = _rand_layer(rng, [4, 6, 3, 7, 5], 6, 6)
    K = orc.layer_ntk(X, D, off)
    A = rng.standard_normal(5)
    for lam, mode in [(1e-3, orc.REG_ABSOLUTE), (0.5, orc.REG_REL_TRACE)]:
        c, info = orc.coeff_interacting(K, A, lam, mode)
        assert info == 0
        le = orc.effective_reg(K, lam, mode)
        r = (K + le * np.eye(5)) @ c - A
        assert np.linalg.norm(r) <= 1e-12 * np.linalg.norm(A) * np.linalg.cond(K + le * np.eye(5))
        np.testing.assert_allclose(c, orc.coeff_interacting_eigh(K, A, lam, mode), rtol=1e-9)
    assert orc.effective_reg(K, 0.5, orc.REG_REL_TRACE) == pytest.approx(0.5 * np.trace(K) / 5)


def test_relative_regulariser_is_scale_free_in_both_variants():
    """A relative regulariser has the dimension of what it is added to: under
    Delta -> a Delta (K -> a^2 K, Fisher norms -> a^4) the interacting
    coefficients scale by a^-2 and so do the non-interacting ones, for any
    lambda.  Also pinned by value: reg = lam * mean_i F_i^2 (non-interacting,
    the typical value of ||.||_F^2) and lam * tr(K)/m (interacting)."""
    rng = np.random.default_rng(61)
    X, D, off = _rand_layer(rng, [4, 6, 3, 7, 5], 6, 6)
    A = rng.standard_normal(5)
    K = orc.layer_ntk(X, D, off)
    f2 = np.sum(K * K, axis=1) / 5
    assert orc.effective_reg(K, 0.3, orc.REG_REL_TRACE, "fisher") == pytest.approx(0.3 * f2.mean(), rel=1e-14)
    assert orc.effective_reg(K, 0.3, orc.REG_REL_TRACE, "interacting") == pytest.approx(0.3 * np.trace(K) / 5, rel=1e-14)
    np.testing.assert_allclose(orc.coeff_fisher(K, A, 0.3, orc.REG_REL_TRACE), A / np.sqrt(f2 + 0.3 * f2.mean()), rtol=1e-13)
    for a in (0.01, 7.0):
        Ka = orc.layer_ntk(X, a * D, off)
        for lam in (1e-3, 0.5, 4.0):
            np.testing.assert_allclose(orc.coeff_fisher(Ka, A, lam, orc.REG_REL_TRACE) * a ** 2,
                                       orc.coeff_fisher(K, A, lam, orc.REG_REL_TRACE), rtol=1e-11)
            np.testing.assert_allclose(orc.coeff_interacting(Ka, A, lam, orc.REG_REL_TRACE)[0] * a ** 2,
                                       orc.coeff_interacting(K, A, lam, orc.REG_REL_TRACE)[0], rtol=1e-9)
    step = orc.layer_step(X, D, off, A, "fisher", 0.3, orc.REG_REL_TRACE)
    assert step["reg_eff"] == pytest.approx(0.3 * f2.mean(), rel=1e-14)


def test_p8_minsr_property():
    """<dW, G_i> = (K c)_i = A_i - reg c_i."""
    rng = np.random.default_rng(7)
    X, D, off = _rand_layer(rng, [5, 4, 6], 9, 8)
    A = rng.standard_normal(3)
    lam = 0.01
    step = orc.layer_step(X, D, off, A, "interacting", lam)
    G = orc.seq_logprob_grads(X, D, off)
    lhs = np.array([np.sum(step["dW"] * G[i]) for i in range(3)])
    np.testing.assert_allclose(lhs, A - lam * step["c"], rtol=1e-10)


def test_p9_large_reg_limit_is_reinforce():
    rng = np.random.default_rng(8)
    X, D, off = _rand_layer(rng, [5, 4, 6, 2], 7, 6)
    A = rng.standard_normal(4)
    K = orc.layer_ntk(X, D, off)
    lam = 1e9 * np.linalg.norm(K, 2)
    step = orc.layer_step(X, D, off, A, "interacting", lam)
    np.testing.assert_allclose(lam * step["dW"], step["dW_reinforce"], rtol=1e-8)
    G = orc.seq_logprob_grads(X, D, off)
    np.testing.assert_allclose(step["dW_reinforce"], sum(A[i] * G[i] for i in range(4)), rtol=1e-13)


def test_p10_equivariances():
    rng = np.random.default_rng(9)
    lengths = [4, 6, 3, 5]
    X, D, off = _rand_layer(rng, lengths, 6, 5)
    A = rng.standard_normal(4)
    base = {v: orc.layer_step(X, D, off, A, v, 0.05) for v in ("fisher", "interacting")}
    # permute sequences
    perm = [2, 0, 3, 1]
    Xp = np.concatenate([X[off[i]:off[i + 1]] for i in perm])
    Dp = np.concatenate([D[off[i]:off[i + 1]] for i in perm])
    offp = np.concatenate([[0], np.cumsum([lengths[i] for i in perm])])
    for v in base:
        s = orc.layer_step(Xp, Dp, offp, A[perm], v, 0.05)
        np.testing.assert_allclose(s["K"], base[v]["K"][np.ix_(perm, perm)], rtol=1e-12)
        np.testing.assert_allclose(s["c"], base[v]["c"][perm], rtol=1e-10)
        np.testing.assert_allclose(s["dW"], base[v]["dW"], rtol=1e-10, atol=1e-14)
    # permute tokens inside a sequence
    Xq, Dq = X.copy(), D.copy()
    idx = off[1] + rng.permutation(lengths[1])
    Xq[off[1]:off[2]], Dq[off[1]:off[2]] = X[idx], D[idx]
    np.testing.assert_allclose(orc.layer_ntk(Xq, Dq, off), base["fisher"]["K"], rtol=1e-12)
    # scaling Delta by alpha: K scales by alpha^2, dW by 1/alpha (reg 0)
    alpha = 3.0
    for v in base:
        s0 = orc.layer_step(X, D, off, A, v, 0.0)
        s1 = orc.layer_step(X, alpha * D, off, A, v, 0.0)
        np.testing.assert_allclose(s1["K"], alpha ** 2 * s0["K"], rtol=1e-12)
        np.testing.assert_allclose(s1["dW"], s0["dW"] / alpha, rtol=1e-9, atol=1e-13)
    # splitting a sequence: G_i = G_i' + G_i''
    off_split = np.array([0, 4, 7, 10, 13, 18])
    Ks = orc.layer_ntk(X, D, off_split)
    K = base["fisher"]["K"]
    assert Ks[1, 1] + 2 * Ks[1, 2] + Ks[2, 2] == pytest.approx(K[1, 1], rel=1e-12)
    assert Ks[0, 1] + Ks[0, 2] == pytest.approx(K[0, 1], rel=1e-10)


def test_p11_single_sequence_closed_form():
    rng = np.random.default_rng(10)
    X, D, off = _rand_layer(rng, [7], 5, 4)
    G = D.T @ X
    g2 = np.sum(G * G)
    a, lam = -1.3, 0.2
    s = orc.layer_step(X, D, off, np.array([a]), "interacting", lam)
    np.testing.assert_allclose(s["dW"], a * G / (g2 + lam), rtol=1e-12)
    s = orc.layer_step(X, D, off, np.array([a]), "fisher", lam)
    np.testing.assert_allclose(s["dW"], a * G / np.sqrt(g2 ** 2 + lam), rtol=1e-12)


def test_p12_weighted_grad_two_ways():
    rng = np.random.default_rng(11)
    X, D, off = _rand_layer(rng, [3, 0, 5, 4], 6, 7)
    c = rng.standard_normal(4)
    G = orc.seq_logprob_grads(X, D, off)
    dW = orc.weighted_grad(G, c)
    np.testing.assert_allclose(orc.weighted_grad_tokens(X, D, off, c), dW, rtol=1e-12, atol=1e-15)
    brute = np.zeros((7, 6))
    for i in range(4):
        for t in range(off[i], off[i + 1]):
            brute += c[i] * np.outer(D[t], X[t])
    np.testing.assert_allclose(dW, brute, rtol=1e-12, atol=1e-15)
    val, mag = orc.weighted_grad_entry(X, D, off, c, 2, 3)
    assert val == pytest.approx(dW[2, 3], rel=1e-12)
    assert mag == pytest.approx(sum(abs(c[i] * D[t, 2] * X[t, 3]) for i in range(4) for t in range(off[i], off[i + 1])))
    S = orc.weighted_grad_abs(G, c)
    assert np.all(S >= np.abs(dW) - 1e-15)
    np.testing.assert_allclose(orc.weighted_grad_abs(np.abs(G), np.abs(c)), orc.weighted_grad(np.abs(G), np.abs(c)))
    np.testing.assert_allclose(orc.weighted_grad_tokens(X, D, off, c, rows=(2, 5)), dW[2:5], rtol=1e-12, atol=1e-15)
    dW0 = rng.standard_normal((7, 6))
    np.testing.assert_allclose(orc.weighted_grad(G, c, dW0, 0.5), dW + 0.5 * dW0, rtol=1e-13)


def test_p13_interacting_listing_in_torch():
    """The interacting hook restated with torch fp64 ops (per-sequence
    grad_out.T @ act_in, pairwise sums, eigh, stack @ coefficients) and the
    non-interacting update with the reduced-gradient Fisher estimate."""
    rng = np.random.default_rng(12)
    lengths = [32] * 4
    X, D, off = _rand_layer(rng, lengths, 64, 128, sd=1e-2)
    A = rng.standard_normal(4)
    reg = 1e-3
    Xt, Dt, At = torch.from_numpy(X), torch.from_numpy(D), torch.from_numpy(A)
    grads = [Dt[off[i]:off[i + 1]].T @ Xt[off[i]:off[i + 1]] for i in range(4)]
    ntk = torch.tensor([[torch.sum(gi * gj).item() for gj in grads] for gi in grads], dtype=torch.float64)
    ev, U = torch.linalg.eigh(ntk)
    coef = U @ ((1.0 / (ev + reg)) * (U.T @ At))
    upd = torch.stack(grads, dim=-1) @ coef
    s = orc.layer_step(X, D, off, A, "interacting", reg)
    np.testing.assert_allclose(s["K"], ntk.numpy(), rtol=1e-12)
    np.testing.assert_allclose(s["dW"], upd.numpy(), rtol=1e-8, atol=1e-12)
    upd = sum(At[i] * grads[i] / torch.sqrt(torch.mean(ntk[i] ** 2) + reg) for i in range(4))
    s = orc.layer_step(X, D, off, A, "fisher", reg)
    np.testing.assert_allclose(s["dW"], upd.numpy(), rtol=1e-11, atol=1e-14)


def test_p14_duplicate_sequences_and_not_pd():
    rng = np.random.default_rng(13)
    X, D, off = _rand_layer(rng, [4, 4, 5], 6, 5)
    X[4:8], D[4:8] = X[0:4], D[0:4]
    K = orc.layer_ntk(X, D, off)
    A = np.array([1.0, -0.5, 0.3])
    lam = 0.1
    c, info = orc.coeff_interacting(K, A, lam)
    assert info == 0 and np.all(np.isfinite(c))
    assert c[0] - c[1] == pytest.approx((A[0] - A[1]) / lam, rel=1e-9)
    # singular K with reg 0: the second pivot is not positive -> reported, not clamped
    Kd = np.array([[4.0, 2.0, 0.0], [2.0, 1.0, 0.0], [0.0, 0.0, 1.0]])
    c, info = orc.coeff_interacting(Kd, A, 0.0)
    assert info == 2 and np.all(np.isnan(c))
    c, info = orc.coeff_interacting(-np.eye(3), A, 0.5)
    assert info == 1
    # an empty sequence with reg 0 in the fisher variant gives c_i = 0, not inf
    X, D, off = _rand_layer(rng, [3, 0, 4], 5, 4)
    K = orc.layer_ntk(X, D, off)
    assert np.all(K[1] == 0) and np.all(K[:, 1] == 0)
    c = orc.coeff_fisher(K, np.ones(3), 0.0)
    assert c[1] == 0.0 and np.all(np.isfinite(c))


def test_widen_bf16_bits_exact():
    x = torch.randn(257, dtype=torch.float32).to(torch.bfloat16)
    bits = x.view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(orc.widen(bits), x.to(torch.float64).numpy())
    with pytest.raises(TypeError):
        orc.widen(np.zeros(3, dtype=np.int32))
    with pytest.raises(ValueError):
        orc.check_offsets([0, 3, 2, 5], 5)
    with pytest.raises(ValueError):
        orc.check_offsets([1, 5], 5)


def test_token_sample_fisher_estimate():
    """The token-position-sample Fisher norm: the oracle (materialised rank-one
    sample gradients) against the non-interacting listing's own expression in
    torch, and against closed forms."""
    rng = np.random.default_rng(20)
    X, D, off = _rand_layer(rng, [5, 3, 6, 2], 7, 6)
    idx = rng.permutation(16)[:9]
    f2 = orc.fisher_norm_sq_token_samples(X, D, off, idx)
    # the fast forms the paper derives for rank-one sample gradients: eq. (one), v . g^(j) = g0_j^T V a0_j,
    # and eq. (two), ||g^(j)||^2 = ||g0_j||^2 ||a0_j||^2 (the oracle materialises every g^(j) instead)
    a0, g0 = X[idx], D[idx]
    den = np.sum(np.sum(g0 ** 2, axis=1) * np.sum(a0 ** 2, axis=1))
    for i in range(4):
        V = D[off[i]:off[i + 1]].T @ X[off[i]:off[i + 1]]
        proj = np.einsum("jo,ok,jk->j", g0, V, a0)
        assert f2[i] == pytest.approx(float(np.sum(proj ** 2) / den), rel=1e-12)
    # one sample equal to the only token of a one-token sequence: v = g^(j), so
    # ||v||_F^2 = (v.v)^2 / (v.v) = ||x||^2 ||delta||^2 (eq. (two))
    X1, D1, off1 = _rand_layer(rng, [1, 4], 5, 4)
    f2 = orc.fisher_norm_sq_token_samples(X1, D1, off1, [0])
    assert f2[0] == pytest.approx(np.dot(X1[0], X1[0]) * np.dot(D1[0], D1[0]), rel=1e-12)
    # scaling: Delta -> 2 Delta scales numerator by 2^4 and denominator by 2^2
    f2a = orc.fisher_norm_sq_token_samples(X, D, off, idx)
    f2b = orc.fisher_norm_sq_token_samples(X, 2 * D, off, idx)
    np.testing.assert_allclose(f2b, 4 * f2a, rtol=1e-12)
    # sample order and repetition-free permutation do not matter; coefficients follow the update formula
    np.testing.assert_allclose(orc.fisher_norm_sq_token_samples(X, D, off, idx[::-1]), f2a, rtol=1e-12)
    A = rng.standard_normal(4)
    c, f2c = orc.coeff_fisher_token_samples(X, D, off, idx, A, 0.3)
    np.testing.assert_allclose(c, A / np.sqrt(f2a + 0.3), rtol=1e-12)
    c, _ = orc.coeff_fisher_token_samples(X, D, off, idx, A, 0.5, orc.REG_REL_TRACE)
    np.testing.assert_allclose(c, A / np.sqrt(f2a + 0.5 * f2a.mean()), rtol=1e-12)
    # trailing-mean regulariser over three minibatches of different scale, iterated by hand
    state, means = None, []
    for scale in (1.0, 3.0, 0.5):
        c, f2s, state = orc.coeff_fisher_token_samples_ema(X, scale * D, off, idx, A, 0.7, state, 0.9)
        means.append(float(np.mean(f2s)))
        np.testing.assert_allclose(f2s, scale ** 2 * f2a, rtol=1e-12)
        want = means[0] if len(means) == 1 else (0.9 * means[0] + 0.1 * means[1] if len(means) == 2
                                                 else 0.81 * means[0] + 0.09 * means[1] + 0.1 * means[2])
        assert state == pytest.approx(want, rel=1e-12)
        np.testing.assert_allclose(c, A / np.sqrt(f2s + 0.7 * want), rtol=1e-12)
    # an empty sequence has zero Fisher norm; with reg 0 its coefficient is 0
    X2, D2, off2 = _rand_layer(rng, [3, 0, 4], 5, 4)
    c, f2 = orc.coeff_fisher_token_samples(X2, D2, off2, [0, 5], np.ones(3), 0.0)
    assert f2[1] == 0.0 and c[1] == 0.0


def test_token_sample_estimate_restricted_to_some_sequences():
    """seqs= evaluates only the named sequences (the form the full-size checks
    use): their entries equal the unrestricted call's, the others are NaN; an
    empty named sequence gives 0; bf16 bit patterns are widened per sequence."""
    rng = np.random.default_rng(21)
    X, D, off = _rand_layer(rng, [5, 0, 6, 2, 7], 9, 6)
    idx = rng.permutation(20)[:7]
    full = orc.fisher_norm_sq_token_samples(X, D, off, idx)
    for seqs in ([2], [4, 0], [1, 3], np.array([0, 1, 2, 3, 4])):
        part = orc.fisher_norm_sq_token_samples(X, D, off, idx, seqs=seqs)
        named = np.zeros(5, bool)
        named[np.asarray(seqs)] = True
        np.testing.assert_array_equal(part[named], full[named])
        assert np.all(np.isnan(part[~named]))
    assert full[1] == 0.0
    Xb = torch.from_numpy(X).to(torch.bfloat16)
    Db = torch.from_numpy(D).to(torch.bfloat16)
    bits = lambda t: t.view(torch.int16).numpy().view(np.uint16)
    part = orc.fisher_norm_sq_token_samples(bits(Xb), bits(Db), off, idx, seqs=[3])
    full_b = orc.fisher_norm_sq_token_samples(Xb.double().numpy(), Db.double().numpy(), off, idx)
    assert part[3] == pytest.approx(full_b[3], rel=1e-13)


def test_ntk_as_one_matrix_product():
    """K = J J^T (interacting-variant section) formed as one matrix product:
    the hand-worked K, the listing's double loop on random gradients, and the
    chunked accumulation over output rows."""
    with open(os.path.join(GOLDEN, "hand_worked_two_sequences.json")) as f:
        g = json.load(f)
    G = orc.seq_logprob_grads(np.array(g["X"], float), np.array(g["Delta"], float), g["seq_offsets"])
    np.testing.assert_array_equal(orc.ntk_as_matrix_product(G), np.array(g["K"], float))
    rng = np.random.default_rng(22)
    X, D, off = _rand_layer(rng, [4, 1, 0, 6, 3], 8, 10)
    G = orc.seq_logprob_grads(X, D, off)
    K_loop = orc.ntk_from_seq_grads(G)
    K_mat = orc.ntk_as_matrix_product(G)
    np.testing.assert_allclose(K_mat, K_loop, rtol=1e-13, atol=1e-13 * np.abs(K_loop).max())
    assert np.array_equal(K_mat, K_mat.T) and np.all(K_mat[2] == 0)
    for chunk in (3, 4, 10):
        np.testing.assert_allclose(orc.layer_ntk(X, D, off, chunk_rows=chunk, matrix_product=True), K_loop,
                                   rtol=1e-13, atol=1e-13 * np.abs(K_loop).max())
    np.testing.assert_allclose(orc.layer_ntk(X, D, off, matrix_product=True), K_loop, rtol=1e-13,
                               atol=1e-13 * np.abs(K_loop).max())


def test_generalised_rescaling_fixture():
    """Hand-worked values of the generalised re-scaling (alternative re-scalings
    listing), including regularisation with batch-mean and caller-supplied
    expectations."""
    fx = json.load(open(os.path.join(GOLDEN, "hand_worked_rescaling.json")))
    f2, g2 = fx["fisher_sq"], fx["grad_sq"]
    for case in ("headline", "fisher_reg", "mixed"):
        c = fx[case]
        got = orc.rescaling_general(f2, g2, c["p"], c["q"], c["r"], tuple(c.get("reg", (0, 0, 0))),
                                    tuple(c.get("expectation", (None, None, None))))
        np.testing.assert_allclose(got, c["scaling"], rtol=c["rel_tol"], err_msg=case)


def test_generalised_rescaling_properties():
    """What the paper fixes about the (p, q, r) family: p = -1 is the
    KL-bounding re-scaling (unit Fisher norm), q = -1 gives unit Euclidean norm,
    r = -2 is the minimiser of ||lambda v - F^-1 g||_F over lambda for an
    explicit Fisher matrix, and the exponents compose multiplicatively."""
    rng = np.random.default_rng(31)
    X, D, off = _rand_layer(rng, [5, 3, 6, 4, 7], 6, 5)
    G = orc.seq_logprob_grads(X, D, off)
    K = orc.ntk_from_seq_grads(G)
    m = K.shape[0]
    f2, g2 = orc.fisher_norm_sq(K), np.diag(K).copy()
    # p = -1 reproduces the non-interacting coefficients with reg = 1e-8 (absolute)
    A = rng.standard_normal(m)
    np.testing.assert_allclose(orc.coeff_rescaled(f2, g2, A), orc.coeff_fisher(K, A, 1e-8), rtol=1e-12)
    # ... and with a regularisation factor on E[F^2] given by the caller
    np.testing.assert_allclose(orc.coeff_rescaled(f2, g2, A, reg=(0.3, 0, 0), expectation=(2.0, None, None)),
                               orc.coeff_fisher(K, A, 0.6 + 1e-8), rtol=1e-12)
    # q = -1: every scaled gradient has Euclidean norm 1
    s = orc.rescaling_general(f2, g2, 0, -1, 0)
    for i in range(m):
        assert np.linalg.norm(s[i] * G[i]) == pytest.approx(1.0, rel=1e-7)
    # r = -2 against an explicit Fisher matrix: F = (1/m) sum_j g_j g_j^T + small ridge (so F^-1 exists);
    # the best scalar multiple of v = g_i approximating F^-1 (A v) in the F metric, found by
    # fitting the quadratic objective at three points, is A ||v||^2 / (v.F v)
    J = G.reshape(m, -1)
    Fm = J.T @ J / m + 1e-3 * np.eye(J.shape[1])
    Finv = np.linalg.inv(Fm)
    for i in range(m):
        v = J[i]
        a = 1.7
        target = Finv @ (a * v)
        obj = lambda lam: (lam * v - target) @ Fm @ (lam * v - target)
        y0, y1, y2 = obj(0.0), obj(1.0), obj(2.0)      # exact quadratic in lam
        qa = (y2 - 2 * y1 + y0) / 2
        qb = y1 - y0 - qa
        lam_star = -qb / (2 * qa)
        vFv = v @ Fm @ v
        s_i = orc.rescaling_general([vFv], [v @ v], 0, 0, -2)[0]
        assert a * s_i == pytest.approx(lam_star, rel=1e-6)
    # exponents compose: scaling(p,q,r) = scaling(p,0,0) * scaling(0,q,0) * scaling(0,0,r); scaling(0,0,0) = 1
    full = orc.rescaling_general(f2, g2, -0.5, 0.7, -1.3, (0.1, 0.2, 0.3))
    parts = (orc.rescaling_general(f2, g2, -0.5, 0, 0, (0.1, 0.2, 0.3)) * orc.rescaling_general(f2, g2, 0, 0.7, 0, (0.1, 0.2, 0.3))
             * orc.rescaling_general(f2, g2, 0, 0, -1.3, (0.1, 0.2, 0.3)))
    np.testing.assert_allclose(full, parts, rtol=1e-12)
    np.testing.assert_array_equal(orc.rescaling_general(f2, g2, 0, 0, 0), np.ones(m))
    # homogeneity (no regularisation): G -> 3 G scales F by 9 (F is quadratic in g), ||G|| by 3, rel by 3
    s1 = orc.rescaling_general(f2, g2, -1, -1, -2)
    s3 = orc.rescaling_general(81 * f2, 9 * g2, -1, -1, -2)
    np.testing.assert_allclose(s3, s1 * 9.0 ** -1 * 3.0 ** -1 * 3.0 ** -2, rtol=1e-6)
    # a zero gradient: finite scaling, zero coefficient contribution c_i * G_i
    s0 = orc.rescaling_general([0.0, 1.0], [0.0, 2.0], 0, -1, -2)
    assert np.isfinite(s0).all()


def test_eigh_route_and_ema():
    """D, U = eigh(K) once, any number of regularisers: equals the Cholesky
    solve for each; the trailing mean iterated by hand."""
    rng = np.random.default_rng(41)
    X, D_, off = _rand_layer(rng, [4, 6, 3, 5], 6, 5)
    K = orc.layer_ntk(X, D_, off)
    A = rng.standard_normal(4)
    D, U = orc.ntk_eigh(K)
    np.testing.assert_allclose(U @ np.diag(D) @ U.T, K, atol=1e-10 * np.trace(K))
    np.testing.assert_allclose(U.T @ U, np.eye(4), atol=1e-12)
    assert np.mean(D) == pytest.approx(np.trace(K) / 4, rel=1e-12)
    for lam in (1e-4, 1e-3, 1e-2):
        c_ref, info = orc.coeff_interacting(K, A, lam, orc.REG_REL_TRACE)
        np.testing.assert_allclose(orc.coeff_from_eigh(D, U, A, lam * np.mean(D)), c_ref, rtol=1e-8)
    # EMA with decay 0.9 over three minibatches, by hand: s1 = m1; s2 = 0.9 m1 + 0.1 m2; s3 = 0.9 s2 + 0.1 m3
    state = None
    means, states = [], []
    for scale in (1.0, 4.0, 0.25):
        c, state = orc.coeff_interacting_ema(scale * K, A, 1.0, state)
        means.append(scale * np.trace(K) / 4)
        states.append(state)
        c_ref, _ = orc.coeff_interacting(scale * K, A, state, orc.REG_ABSOLUTE)
        np.testing.assert_allclose(c, c_ref, rtol=1e-8)
    assert states[0] == pytest.approx(means[0], rel=1e-12)
    assert states[1] == pytest.approx(0.9 * means[0] + 0.1 * means[1], rel=1e-12)
    assert states[2] == pytest.approx(0.81 * means[0] + 0.09 * means[1] + 0.1 * means[2], rel=1e-12)
