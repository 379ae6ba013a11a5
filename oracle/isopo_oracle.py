"""CPU fp64 oracle for the ISOPO layer step.  TEST INFRASTRUCTURE ONLY.

This module is the slow, plain definition of what the layer step computes.
It is imported by the tests, by the smoke check and by the benchmark's
cpu_baseline leg, and by nothing else: the product path (the HIP library and
its binding) never calls it and shares no code with it.

Everything is numpy float64.  Every per-sequence gradient is materialised
explicitly; there is no blocking, fusion or reordering beyond what the paper's
definitions state.  Notation follows the paper:

    X      act_in   [N, d_in]     token activations of one linear layer
    Delta  grad_out [N, d_out]    back-propagated gradient of sum(log_prob)
    G_i    seq_logprob_grad       = Delta_i^T X_i, shape [d_out, d_in]
    K      ntk      [m, m]        K = J J^T, J_i = vec(G_i)
    A      advantages [m]
    c      per-sequence coefficients applied to the G_i

Pins (tests/test_oracle_pins.py): autograd brute force, the ghost double sum,
rank-one closed form, unit Fisher norm, the orthogonal-gradient reduction,
solve residual and the eigendecomposition route, the MinSR property, the
large-regulariser limit, equivariances, the one-sequence closed form, the
token-by-token contraction, duplicate sequences, (token-sample Fisher
estimate) the listing's own formula in torch plus a one-token closed form,
(generalised re-scaling) a hand-worked fixture, the explicit-Fisher minimiser
for r = -2 and unit norms for p = -1 / q = -1, and (eigh route) agreement with
the Cholesky solve plus a hand-iterated EMA, (K = J J^T as one matrix product)
the double loop and the hand-worked fixture, (the seqs= restriction of the
token-sample estimate) the unrestricted call.  Every public function
below is pinned by at least one of them; none is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

REG_ABSOLUTE = 0
REG_REL_TRACE = 1


def widen(a) -> np.ndarray:
    """Exact widening of an input buffer to float64.

    uint16 arrays are taken as bfloat16 bit patterns (the upper half of an
    IEEE float32); float32/float64 arrays are widened as they are.  No value
    changes, so input quantisation is never part of an error budget.
    """
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if a.dtype in (np.float32, np.float64):
        return a.astype(np.float64)
    raise TypeError(f"unsupported input dtype {a.dtype}")


def check_offsets(seq_offsets, n_tokens: int) -> np.ndarray:
    off = np.asarray(seq_offsets, dtype=np.int64)
    if off.ndim != 1 or off.size < 2:
        raise ValueError("seq_offsets needs at least two entries")
    if off[0] != 0 or off[-1] != n_tokens or np.any(np.diff(off) < 0):
        raise ValueError("seq_offsets must start at 0, end at N and be non-decreasing")
    return off


def seq_logprob_grads(X, Delta, seq_offsets, rows=None) -> np.ndarray:
    """G_i = Delta_i^T X_i for every sequence (non-interacting and interacting
    listings: `seq_logprob_grad = grad_out.T @ act_in` over one sequence's rows).

    Returns [m, d_out, d_in]; with rows=(r0, r1) only output rows r0:r1 of each
    G_i are formed, [m, r1-r0, d_in] (used to bound memory on large layers).
    An empty sequence gives G_i = 0.
    """
    X = widen(X)
    Delta = widen(Delta)
    off = check_offsets(seq_offsets, X.shape[0])
    if Delta.shape[0] != X.shape[0]:
        raise ValueError("X and Delta must have the same number of token rows")
    r0, r1 = (0, Delta.shape[1]) if rows is None else rows
    m = off.size - 1
    G = np.zeros((m, r1 - r0, X.shape[1]), dtype=np.float64)
    for i in range(m):
        s, e = off[i], off[i + 1]
        if e > s:
            G[i] = Delta[s:e, r0:r1].T @ X[s:e]
    return G


def ntk_from_seq_grads(G) -> np.ndarray:
    """K_ij = sum(G_i * G_j) for i <= j, mirrored (interacting listing's
    double loop; K = J J^T of the interacting-variant section)."""
    m = G.shape[0]
    K = np.empty((m, m), dtype=np.float64)
    for i in range(m):
        for j in range(i, m):
            K[i, j] = np.sum(G[i] * G[j])
            K[j, i] = K[i, j]
    return K


def ntk_as_matrix_product(G) -> np.ndarray:
    """The same K as the printed definition K = J J^T (interacting-variant
    section), J being the m x P matrix whose row i is G_i flattened: one
    library matrix product instead of the listing's double loop, so that K of a
    wide layer at full size takes seconds.  Pinned against the double loop and
    the hand-worked fixture."""
    J = G.reshape(G.shape[0], -1)
    K = J @ J.T
    return 0.5 * (K + K.T)          # the product is symmetric up to summation order; make it exactly so


def ntk_ghost(X, Delta, seq_offsets) -> np.ndarray:
    """The same K from the rank-one structure of token gradients
    (efficient-implementation paragraph: each token gradient is the outer
    product grad_out[t] act_in[t]^T, so <g^(t), g^(s)> = (x_t.x_s)(d_t.d_s)):

        K_ij = sum_{t in i} sum_{s in j} (x_t . x_s) (delta_t . delta_s).

    No G_i is formed.  Quadratic in N: small inputs only.
    """
    X = widen(X)
    Delta = widen(Delta)
    off = check_offsets(seq_offsets, X.shape[0])
    H = (X @ X.T) * (Delta @ Delta.T)
    m = off.size - 1
    K = np.zeros((m, m), dtype=np.float64)
    for i in range(m):
        for j in range(m):
            K[i, j] = np.sum(H[off[i]:off[i + 1], off[j]:off[j + 1]])
    return K


def layer_ntk(X, Delta, seq_offsets, chunk_rows=None, matrix_product=False) -> np.ndarray:
    """K for one layer.  For large layers the G_i are held d_out-rows-chunk by
    chunk (all sequences at once) and K accumulates over the chunks; every
    chunk of every G_i is still materialised.  matrix_product: form each
    chunk's K as J J^T (ntk_as_matrix_product) instead of the double loop."""
    d_out = np.asarray(Delta).shape[1]
    gram = ntk_as_matrix_product if matrix_product else ntk_from_seq_grads
    if chunk_rows is None or chunk_rows >= d_out:
        return gram(seq_logprob_grads(X, Delta, seq_offsets))
    Xw, Dw = widen(X), widen(Delta)
    m = len(seq_offsets) - 1
    K = np.zeros((m, m), dtype=np.float64)
    for r0 in range(0, d_out, chunk_rows):
        r1 = min(d_out, r0 + chunk_rows)
        K += gram(seq_logprob_grads(Xw, Dw, seq_offsets, rows=(r0, r1)))
    return K


def ntk_entry(X, Delta, seq_offsets, i: int, j: int) -> float:
    """One entry K_ij = <G_i, G_j>_F, forming only G_i and G_j (only the rows
    of the two sequences are widened)."""
    X = np.asarray(X)
    Delta = np.asarray(Delta)
    off = check_offsets(seq_offsets, X.shape[0])
    Gi = widen(Delta[off[i]:off[i + 1]]).T @ widen(X[off[i]:off[i + 1]])
    Gj = Gi if j == i else widen(Delta[off[j]:off[j + 1]]).T @ widen(X[off[j]:off[j + 1]])
    return float(np.sum(Gi * Gj))


def effective_reg(K, lam: float, reg_mode: int = REG_ABSOLUTE, variant: str = "interacting") -> float:
    """The regulariser actually added.  ABSOLUTE: lam itself (the Tikhonov c of
    v = J^T (K + cI)^-1 A; reg_l of the update u_l).  REL_TRACE scales lam by
    this batch's typical value of the quantity it is added to, the current
    batch standing in for the trailing mean over minibatches:
      interacting  lam * tr(K)/m, the mean eigenvalue of K (the interacting
                   experiment's regulariser = factor * E[mean(D)]);
      fisher       lam * mean_i ||g_i||_F^2 (the non-interacting derivation
                   compares reg_l with the typical value of ||.||_F^2)."""
    K = np.asarray(K, dtype=np.float64)
    if reg_mode == REG_ABSOLUTE:
        return float(lam)
    if reg_mode == REG_REL_TRACE:
        if variant == "fisher":
            return float(lam) * float(np.mean(fisher_norm_sq(K)))
        if variant != "interacting":
            raise ValueError("variant must be 'fisher' or 'interacting'")
        return float(lam) * float(np.trace(K)) / K.shape[0]
    raise ValueError("unknown reg_mode")


def fisher_norm_sq(K) -> np.ndarray:
    """||g_i||_F^2 ~= (1/n) sum_j (g_i . g_j)^2 = (1/m) sum_j K_ij^2
    (eq. F-norm-basic with v = g_i and the batch's reduced gradients as the
    samples, j = i included)."""
    K = np.asarray(K, dtype=np.float64)
    return np.sum(K * K, axis=1) / K.shape[0]


def coeff_fisher(K, A, lam: float, reg_mode: int = REG_ABSOLUTE) -> np.ndarray:
    """Non-interacting update's coefficients:
    c_i = A_i / sqrt(||g_i||_F^2 + reg)   (layer-wise update u_l; rescaling()
    of the non-interacting listing).  A zero denominator (empty sequence with
    reg = 0) gives c_i = 0 by convention."""
    A = np.asarray(A, dtype=np.float64)
    den = fisher_norm_sq(K) + effective_reg(K, lam, reg_mode, "fisher")
    c = np.zeros_like(A)
    nz = den > 0
    c[nz] = A[nz] / np.sqrt(den[nz])
    return c


def fisher_norm_sq_token_samples(X, Delta, seq_offsets, sample_idx, seqs=None) -> np.ndarray:
    """The non-interacting listing's Fisher-norm estimate per sequence, squared
    (eq. formal-F-norm):

        ||v||_F^2 ~= sum_j (v . g^(j))^2 / sum_j ||g^(j)||^2

    with v = G_i and g^(j) = grad_out[j] act_in[j]^T the un-reduced gradients at
    the sampled token rows j (`a0 = act_in[samples]`, `g0 = grad_out[samples]`,
    samples drawn from the whole microbatch).  Written with G_i and every
    rank-one g^(j) materialised; the listing's `sum((g0 @ G) * a0, dim=1)` and
    `norm(g0) * norm(a0)` are eq. (one) and eq. (two) applied to the same sums.

    seqs: only these sequences are evaluated (the others' entries are NaN); rows
    are widened one sequence at a time, so a large layer can be checked on a few
    short sequences.
    """
    off = check_offsets(seq_offsets, X.shape[0])
    idx = np.asarray(sample_idx, dtype=np.int64)
    m = off.size - 1
    which = range(m) if seqs is None else [int(i) for i in seqs]
    g0, a0 = widen(Delta[idx]), widen(X[idx])
    den = 0.0
    for j in range(idx.size):
        gj = np.outer(g0[j], a0[j])                   # g^(j), [d_out, d_in]
        den += np.sum(gj * gj)
    num = np.full(m, np.nan)
    for i in which:
        s, e = off[i], off[i + 1]
        G_i = widen(Delta[s:e]).T @ widen(X[s:e])     # zero for an empty sequence
        num[i] = 0.0
        for j in range(idx.size):
            num[i] += np.sum(G_i * np.outer(g0[j], a0[j])) ** 2
    return num / den if den > 0 else np.where(np.isnan(num), num, 0.0)


def coeff_fisher_token_samples(X, Delta, seq_offsets, sample_idx, A, lam: float,
                               reg_mode: int = REG_ABSOLUTE):
    """c_i = A_i / sqrt(F_norm_i^2 + reg) with the token-sample estimate
    (`rescaling()` of the non-interacting listing).  REL mode: reg = lam times
    the batch mean of F_norm^2 (the listing's "trailing minibatch means", with
    the current batch standing in).  Returns (c, F_norm^2)."""
    A = np.asarray(A, dtype=np.float64)
    f2 = fisher_norm_sq_token_samples(X, Delta, seq_offsets, sample_idx)
    reg = float(lam) if reg_mode == REG_ABSOLUTE else float(lam) * float(np.mean(f2))
    den = f2 + reg
    c = np.zeros_like(A)
    nz = den > 0
    c[nz] = A[nz] / np.sqrt(den[nz])
    return c, f2


def coeff_fisher_token_samples_ema(X, Delta, seq_offsets, sample_idx, A, factor: float, ema_state, decay: float = 0.9):
    """The same coefficients with the regulariser the listing suggests: factor
    times the trailing mean over minibatches (this one included) of the batch
    mean of F_norm^2.  Returns (c, F_norm^2, new_state)."""
    A = np.asarray(A, dtype=np.float64)
    f2 = fisher_norm_sq_token_samples(X, Delta, seq_offsets, sample_idx)
    state = ema_update(ema_state, float(np.mean(f2)), decay)
    den = f2 + float(factor) * state
    c = np.zeros_like(A)
    nz = den > 0
    c[nz] = A[nz] / np.sqrt(den[nz])
    return c, f2, state


RESCALE_EPS = 1e-8     # the additive constant of reg() in the generalised re-scaling listing


def reg2_squared(val_sq, regularization: float = 0.0, expectation=None) -> np.ndarray:
    """reg2(val)^2 of the generalised re-scaling listing, from val^2:
    reg(val^2) = val^2 + regularization * E[val^2] + 1e-8  (reg2 is its square
    root).  `expectation` is E[val^2]; None takes the batch mean of val_sq (the
    listing suggests an EMA of trailing minibatch means; the caller carries it)."""
    v = np.asarray(val_sq, dtype=np.float64)
    e = float(np.mean(v)) if expectation is None else float(expectation)
    return v + float(regularization) * e + RESCALE_EPS


def rescaling_general(fisher_sq, grad_sq, p: float = -1.0, q: float = 0.0, r: float = 0.0,
                      reg=(0.0, 0.0, 0.0), expectation=(None, None, None)) -> np.ndarray:
    """Per-sequence scale factors of the generalised re-scaling (the alternative
    re-scalings listing):

        rel_F_norm = F_norm / ||G||
        scaling = reg2(F_norm)^p * reg2(||G||)^q * reg2(rel_F_norm)^r

    fisher_sq = F_norm^2 and grad_sq = ||G_i||^2 (= K_ii) per sequence.  reg and
    expectation hold the regularisation factor and E[val^2] for the three
    regularised quantities in the order (F_norm, ||G||, rel_F_norm).
    p = -1: the KL-bounding re-scaling; r = -2: the closest-to-natural-gradient
    one; q = -1, r = -2: the headline experiment's setting.

    A sequence with G_i = 0 (empty, or all-zero rows) has no direction to scale:
    rel_F_norm is taken as 0 there (the listing's 0/0), which leaves
    reg2(rel)^r finite because of the 1e-8.
    """
    f2 = np.asarray(fisher_sq, dtype=np.float64)
    g2 = np.asarray(grad_sq, dtype=np.float64)
    rel2 = np.zeros_like(f2)
    nz = g2 > 0
    rel2[nz] = f2[nz] / g2[nz]
    sF = np.sqrt(reg2_squared(f2, reg[0], expectation[0]))
    sG = np.sqrt(reg2_squared(g2, reg[1], expectation[1]))
    sR = np.sqrt(reg2_squared(rel2, reg[2], expectation[2]))
    return sF ** float(p) * sG ** float(q) * sR ** float(r)


def coeff_rescaled(fisher_sq, grad_sq, A, p=-1.0, q=0.0, r=0.0, reg=(0.0, 0.0, 0.0),
                   expectation=(None, None, None)) -> np.ndarray:
    """c_i = A_i * scaling_i: the coefficient with which G_i enters the layer's
    update (`grad += advantages[seq_id] * rescaling(seq_logprob_grad, F_norm)`)."""
    return np.asarray(A, dtype=np.float64) * rescaling_general(fisher_sq, grad_sq, p, q, r, reg, expectation)


def ema_update(state, value: float, decay: float = 0.9):
    """Trailing mean over minibatches with exponential decay (the interacting
    experiment's E[mean(D)], decay 0.9).  state None: first minibatch, the mean
    is the value itself.  Returns the new state (a float)."""
    return float(value) if state is None else float(decay) * float(state) + (1.0 - float(decay)) * float(value)


def ntk_eigh(K):
    """D, U = eigh(K) of the interacting listing (ascending eigenvalues,
    orthonormal columns)."""
    return np.linalg.eigh(np.asarray(K, dtype=np.float64))


def coeff_from_eigh(D, U, A, reg: float) -> np.ndarray:
    """advantages_preconditioned = U ((1 / (D + regularization)) * (U^T A)) of
    the interacting listing, for one decomposition and any number of
    regularisers."""
    A = np.asarray(A, dtype=np.float64)
    return U @ ((1.0 / (D + float(reg))) * (U.T @ A))


def coeff_interacting_ema(K, A, factor: float, ema_state, decay: float = 0.9):
    """Interacting coefficients with the regulariser factor * E[mean(D)], the
    expectation being the trailing mean over minibatches INCLUDING the current
    one (so that the first minibatch is defined).  Returns (c, new_state)."""
    D, U = ntk_eigh(K)
    state = ema_update(ema_state, float(np.mean(D)), decay)
    return coeff_from_eigh(D, U, A, float(factor) * state), state


def coeff_interacting(K, A, lam: float, reg_mode: int = REG_ABSOLUTE):
    """Interacting update's coefficients c = (K + reg I)^-1 A, so that
    v = J^T c (interacting-variant section).  Returns (c, info): info = 0 on
    success, k > 0 if the k-th leading minor of K + reg I is not positive
    (no pseudo-inverse, no clamping; c is then NaN)."""
    K = np.asarray(K, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    m = K.shape[0]
    M = K + effective_reg(K, lam, reg_mode) * np.eye(m)
    # Cholesky by the textbook column recurrence, so the failing pivot is known.
    L = np.zeros_like(M)
    for k in range(m):
        d = M[k, k] - np.dot(L[k, :k], L[k, :k])
        if not d > 0.0:
            return np.full(m, np.nan), k + 1
        L[k, k] = np.sqrt(d)
        for r in range(k + 1, m):
            L[r, k] = (M[r, k] - np.dot(L[r, :k], L[k, :k])) / L[k, k]
    y = np.zeros(m)
    for k in range(m):
        y[k] = (A[k] - np.dot(L[k, :k], y[:k])) / L[k, k]
    c = np.zeros(m)
    for k in range(m - 1, -1, -1):
        c[k] = (y[k] - np.dot(L[k + 1:, k], c[k + 1:])) / L[k, k]
    return c, 0


def coeff_interacting_eigh(K, A, lam: float, reg_mode: int = REG_ABSOLUTE) -> np.ndarray:
    """The same coefficients by the route the interacting listing takes:
    D, U = eigh(K); c = U ((1/(D + reg)) * (U^T A))."""
    K = np.asarray(K, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    D, U = np.linalg.eigh(K)
    pre = 1.0 / (D + effective_reg(K, lam, reg_mode))
    return U @ (pre * (U.T @ A))


def weighted_grad(G, c, dW_in=None, beta: float = 0.0) -> np.ndarray:
    """dW = beta * dW_in + sum_i c_i G_i   (`grad += advantages[i] * scale_i *
    seq_logprob_grad`; `stack(seq_grads, -1) @ advantages_preconditioned`;
    `mod.grad += grad`)."""
    c = np.asarray(c, dtype=np.float64)
    dW = np.zeros(G.shape[1:], dtype=np.float64)
    for i in range(G.shape[0]):
        dW += c[i] * G[i]
    if dW_in is not None and beta != 0.0:
        dW += beta * np.asarray(dW_in, dtype=np.float64)
    return dW


def weighted_grad_abs(G, c) -> np.ndarray:
    """sum_i |c_i| |G_i|, element-wise: the scale against which rounding of the
    terms of dW = sum_i c_i G_i is measured when they cancel."""
    c = np.abs(np.asarray(c, dtype=np.float64))
    S = np.zeros(G.shape[1:], dtype=np.float64)
    for i in range(G.shape[0]):
        S += c[i] * np.abs(G[i])
    return S


def weighted_grad_tokens(X, Delta, seq_offsets, c, rows=None) -> np.ndarray:
    """The same contraction written over token rows:
    dW = Delta^T diag(c_tok) X with c_tok[t] = c_{seq(t)}."""
    X = widen(X)
    Delta = widen(Delta)
    off = check_offsets(seq_offsets, X.shape[0])
    c = np.asarray(c, dtype=np.float64)
    c_tok = np.repeat(c, np.diff(off))
    r0, r1 = (0, Delta.shape[1]) if rows is None else rows
    return (Delta[:, r0:r1] * c_tok[:, None]).T @ X


def weighted_grad_entry(X, Delta, seq_offsets, c, o: int, k: int):
    """One element dW[o, k] = sum_t c_tok[t] Delta[t, o] X[t, k], and the sum of
    the absolute values of its terms."""
    off = check_offsets(seq_offsets, np.asarray(X).shape[0])
    c_tok = np.repeat(np.asarray(c, dtype=np.float64), np.diff(off))
    terms = c_tok * widen(np.asarray(Delta)[:, o]) * widen(np.asarray(X)[:, k])
    return float(np.sum(terms)), float(np.sum(np.abs(terms)))


def layer_step(X, Delta, seq_offsets, A, variant: str, lam: float,
               reg_mode: int = REG_ABSOLUTE, dW_in=None, beta: float = 0.0,
               chunk_rows=None) -> dict:
    """The whole layer step: K, c, dW and the plain REINFORCE gradient
    dW_R = sum_i A_i G_i that ISOPO is compared with.

    variant: "fisher" (non-interacting) or "interacting".
    With chunk_rows the G_i are held chunk_rows output rows at a time: one
    sweep accumulates K, a second sweep (after c is known) forms dW.
    """
    Xw, Dw = widen(X), widen(Delta)
    off = check_offsets(seq_offsets, Xw.shape[0])
    A = np.asarray(A, dtype=np.float64)
    d_out = Dw.shape[1]
    step = d_out if chunk_rows is None else int(chunk_rows)
    K = layer_ntk(Xw, Dw, off, chunk_rows=chunk_rows)
    info = 0
    if variant == "fisher":
        c = coeff_fisher(K, A, lam, reg_mode)
    elif variant == "interacting":
        c, info = coeff_interacting(K, A, lam, reg_mode)
    else:
        raise ValueError("variant must be 'fisher' or 'interacting'")
    dW = np.zeros((d_out, Xw.shape[1]), dtype=np.float64)
    dW_R = np.zeros_like(dW)
    dW_abs = np.zeros_like(dW)
    if info == 0:
        for r0 in range(0, d_out, step):
            r1 = min(d_out, r0 + step)
            G = seq_logprob_grads(Xw, Dw, off, rows=(r0, r1))
            dW[r0:r1] = weighted_grad(G, c)
            dW_R[r0:r1] = weighted_grad(G, A)
            dW_abs[r0:r1] = weighted_grad_abs(G, c)
        if dW_in is not None and beta != 0.0:
            dW += beta * np.asarray(dW_in, dtype=np.float64)
    else:
        dW[:] = np.nan
    return {"K": K, "c": c, "info": info, "dW": dW, "dW_reinforce": dW_R, "dW_abs": dW_abs,
            "reg_eff": effective_reg(K, lam, reg_mode, variant)}
