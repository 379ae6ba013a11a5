"""Parity of the generalised (p, q, r) re-scaling and of the eigendecomposition
route of the interacting variant with the oracle."""
import numpy as np
import pytest
import torch

from oracle import isopo_oracle as orc
from paper_2512_23353_amd import isopo
from paper_2512_23353_amd import workloads as wl

from helpers import TOL, assert_c_close, rel_err, to_device

pytestmark = pytest.mark.gpu


def _random_gram(rng, m, rank=None, scale=1.0):
    """A Gram matrix with a spread spectrum, rounded to fp32 and exactly symmetric."""
    r = rank or 4 * m
    J = rng.standard_normal((m, r)) * np.logspace(0, -2, r)[None, :]
    K = (scale * (J @ J.T)).astype(np.float32)
    return ((K + K.T) / 2).astype(np.float32)


PQR = [(-1.0, 0.0, 0.0), (0.0, -1.0, 0.0), (0.0, 0.0, -2.0), (0.0, -1.0, -2.0), (-0.5, 0.7, -1.3)]


@pytest.mark.parametrize("pqr", PQR)
@pytest.mark.parametrize("m", [1, 4, 32, 257, 1024])
def test_rescale_from_gram(gpu_device, pqr, m):
    rng = np.random.default_rng(m)
    K = _random_gram(rng, m, scale=1e-3)
    A = rng.standard_normal(m).astype(np.float32)
    Kd, Ad = torch.from_numpy(K).to(gpu_device), torch.from_numpy(A).to(gpu_device)
    f2, g2 = isopo.gram_norms(Kd)
    f2_ref, g2_ref = orc.fisher_norm_sq(K), np.diag(K).astype(np.float64)
    np.testing.assert_allclose(f2.cpu().numpy(), f2_ref, rtol=1e-6)
    np.testing.assert_array_equal(g2.cpu().numpy(), np.diag(K))
    means = torch.zeros(3, dtype=torch.float32, device=gpu_device)
    for reg, expect in (((0, 0, 0), (None, None, None)), ((0.5, 0.1, 2.0), (None, None, None)),
                        ((0.5, 0.1, 2.0), (3e-6, None, 0.7))):
        # the kernel takes fisher_sq as gram_norms left it (fp32) and reads the diagonal in place from K;
        # the reference is the oracle's chain from K alone
        c = isopo.rescale(f2, Kd, Ad, *pqr, reg=reg, expectation=expect, batch_means=means)
        torch.cuda.synchronize()
        c_ref = orc.coeff_rescaled(f2_ref, g2_ref, A, *pqr, reg=reg, expectation=expect)
        np.testing.assert_allclose(c.cpu().numpy(), c_ref, rtol=5e-6, atol=0)
        rel2 = np.where(g2_ref > 0, f2_ref / np.where(g2_ref > 0, g2_ref, 1), 0)
        np.testing.assert_allclose(means.cpu().numpy(), [f2_ref.mean(), g2_ref.mean(), rel2.mean()], rtol=2e-6)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_rescaled_layer_update(gpu_device, dtype):
    """The headline setting (q = -1, r = -2) end to end on a ragged layer with an
    empty sequence: K from the layer, norms, re-scaled coefficients, dW from the
    stash, against the oracle's chain."""
    prob = wl.custom_layer(256, 320, [100, 37, 0, 250, 64, 1], dtype=dtype, seed=77, sigma_delta=1e-2)
    tol = TOL[dtype]
    layer, A = to_device(prob, gpu_device)
    K, ws = isopo.layer_gram(layer, "materialised", keep_stash=True)
    f2, g2 = isopo.gram_norms(K)
    c = isopo.rescale(f2, g2, A, 0.0, -1.0, -2.0)
    dW = isopo.weighted_grad(layer, c, ws)
    torch.cuda.synchronize()
    Xo, Do = wl.to_oracle(prob.X), wl.to_oracle(prob.Delta)
    G = orc.seq_logprob_grads(Xo, Do, prob.seq_offsets)
    K_ref = orc.ntk_from_seq_grads(G)
    c_ref = orc.coeff_rescaled(orc.fisher_norm_sq(K_ref), np.diag(K_ref), prob.A, 0.0, -1.0, -2.0)
    ch = c.cpu().numpy()
    live = np.diff(prob.seq_offsets) > 0       # the empty sequence's coefficient is huge (1e-8 floors) and multiplies G = 0
    assert_c_close(ch[live], c_ref[live], tol, "rescaled c")
    np.testing.assert_allclose(ch[~live], c_ref[~live], rtol=1e-5)
    dW_ref, mag = orc.weighted_grad(G, c_ref), orc.weighted_grad_abs(G, c_ref)
    from helpers import assert_dW_close
    assert_dW_close(dW.cpu().numpy(), dW_ref, tol, "rescaled dW", mag)


@pytest.mark.parametrize("m", [1, 2, 3, 4, 16, 31, 32, 64, 65, 94, 95, 96, 128, 135, 200, 256, 511, 1024])
def test_eigh_sizes(gpu_device, m):
    """Both routes (Jacobi in LDS with 256 or 1024 threads up to 94 sequences, tridiagonalisation
    and implicit QL in global scratch from 95), odd sizes (one idle index in the Jacobi pairing),
    the degenerate m = 1 and the library's limit of 1024 sequences."""
    rng = np.random.default_rng(1000 + m)
    K = _random_gram(rng, m)
    A = rng.standard_normal(m).astype(np.float32)
    Kd, Ad = torch.from_numpy(K).to(gpu_device), torch.from_numpy(A).to(gpu_device)
    D, U, info = isopo.ntk_eigh(Kd)
    lambdas = [1e-4, 1e-3, 1e-2]
    c, sinfo = isopo.transform_eigh(D, U, Ad, lambdas, isopo.REG_REL_TRACE)
    c_chol = torch.stack([isopo.transform(Kd, Ad, "interacting", lam, isopo.REG_REL_TRACE)[0] for lam in lambdas])
    torch.cuda.synchronize()
    assert info.item() == 0 and sinfo.item() == 0
    Dh, Uh = D.cpu().numpy(), U.cpu().numpy()
    K64 = K.astype(np.float64)
    D_ref, _ = orc.ntk_eigh(K64)
    scale = np.abs(D_ref).max()
    assert np.all(np.diff(Dh) >= 0)
    np.testing.assert_allclose(Dh, D_ref, atol=1e-12 * scale, rtol=0)
    np.testing.assert_allclose(Uh.T @ Uh, np.eye(m), atol=1e-12)
    np.testing.assert_allclose(Uh @ np.diag(Dh) @ Uh.T, K64, atol=1e-12 * scale)
    for l, lam in enumerate(lambdas):
        c_ref = orc.coeff_interacting_eigh(K64, A, lam, orc.REG_REL_TRACE)
        assert rel_err(c[l].cpu().numpy(), c_ref) <= 1e-5, f"m={m} lambda={lam}"
        assert rel_err(c_chol[l].cpu().numpy(), c_ref) <= 1e-5


@pytest.mark.parametrize("m,batch", [(5, 3), (64, 7), (96, 4), (200, 2)])
def test_eigh_batch_of_problems(gpu_device, m, batch):
    """The projections of a block in one launch (one workgroup per problem), in
    every storage regime: each problem's D, U and its lambda sweep must equal
    what a launch of its own gives (bit for bit: the same arithmetic), the
    trailing-mean state is kept per problem, and the coefficients match the
    oracle's eigendecomposition route."""
    rng = np.random.default_rng(2000 + m)
    Ks = np.stack([_random_gram(rng, m, scale=10.0 ** b) for b in range(batch)])
    A = rng.standard_normal((batch, m)).astype(np.float32)
    Kd, Ad = torch.from_numpy(Ks).to(gpu_device), torch.from_numpy(A).to(gpu_device)
    D, U, info = isopo.ntk_eigh(Kd)
    lambdas = [1e-3, 1e-1]
    ema = torch.zeros((batch, 2), dtype=torch.float32, device=gpu_device)
    c, sinfo = isopo.transform_eigh(D, U, Ad, lambdas, isopo.REG_EMA_TRACE, ema_state=ema, ema_decay=0.9)
    torch.cuda.synchronize()
    assert D.shape == (batch, m) and U.shape == (batch, m, m) and c.shape == (batch, 2, m)
    assert not info.any() and not sinfo.any()
    for b in range(batch):
        D1, U1, _ = isopo.ntk_eigh(Kd[b])
        e1 = torch.zeros(2, dtype=torch.float32, device=gpu_device)
        c1, _ = isopo.transform_eigh(D1, U1, Ad[b], lambdas, isopo.REG_EMA_TRACE, ema_state=e1, ema_decay=0.9)
        torch.cuda.synchronize()
        assert torch.equal(D[b], D1) and torch.equal(U[b], U1) and torch.equal(c[b], c1)
        assert torch.equal(ema[b], e1) and ema[b, 1].item() == 1.0
        K64 = Ks[b].astype(np.float64)
        for l, lam in enumerate(lambdas):
            c_ref = orc.coeff_interacting_eigh(K64, A[b], lam, orc.REG_REL_TRACE)      # first minibatch: E = mean(D)
            assert rel_err(c[b, l].cpu().numpy(), c_ref) <= 1e-5, f"problem {b} lambda={lam}"


def test_eigh_on_a_layer_and_lambda_sweep(gpu_device):
    """Config-2-shaped projection: K from the layer, one decomposition, the
    lambda sweep of the 28-layer configuration, against the oracle's
    eigendecomposition route on the oracle's own K."""
    w = wl.CONFIGS["config2"]
    prob = wl.make_block(w)[2]            # k projection
    layer, A = to_device(prob, gpu_device)
    K, _ = isopo.layer_gram(layer, "auto")
    D, U, info = isopo.ntk_eigh(K)
    lambdas = [1e-4, 1e-3, 1e-2]
    c, _ = isopo.transform_eigh(D, U, A, lambdas, isopo.REG_REL_TRACE)
    torch.cuda.synchronize()
    assert info.item() == 0
    K_ref = orc.layer_ntk(wl.to_oracle(prob.X), wl.to_oracle(prob.Delta), prob.seq_offsets, chunk_rows=1024)
    for l, lam in enumerate(lambdas):
        c_ref = orc.coeff_interacting_eigh(K_ref, prob.A, lam, orc.REG_REL_TRACE)
        assert_c_close(c[l].cpu().numpy(), c_ref, TOL["bf16"], f"lambda={lam}")


def test_trailing_mean_regulariser(gpu_device):
    """factor * E[mean(D)] with the trailing mean carried on the device over
    three minibatches of different scale."""
    rng = np.random.default_rng(9)
    m = 24
    K0 = _random_gram(rng, m)
    A = rng.standard_normal(m).astype(np.float32)
    Ad = torch.from_numpy(A).to(gpu_device)
    ema = torch.zeros(2, dtype=torch.float32, device=gpu_device)
    state = None
    for scale in (1.0, 4.0, 0.25):
        K = (scale * K0).astype(np.float32)
        D, U, _ = isopo.ntk_eigh(torch.from_numpy(K).to(gpu_device))
        c, info = isopo.transform_eigh(D, U, Ad, [1.0], isopo.REG_EMA_TRACE, ema_state=ema, ema_decay=0.9)
        torch.cuda.synchronize()
        c_ref, state = orc.coeff_interacting_ema(K.astype(np.float64), A, 1.0, state, 0.9)
        assert info.item() == 0
        assert ema[0].item() == pytest.approx(state, rel=1e-6)
        assert rel_err(c[0].cpu().numpy(), c_ref) <= 1e-5
    assert ema[1].item() == 3.0


@pytest.mark.parametrize("m", [24, 160])
def test_trailing_mean_regulariser_on_the_factorisation_route(gpu_device, m):
    """isopo_transform_ema: the same regulariser without a decomposition (the mean
    eigenvalue is tr(K)/m), for a batch of two problems with states of their
    own, both variants, over three minibatches; LDS and global-scratch sizes."""
    rng = np.random.default_rng(19 + m)
    K0 = np.stack([_random_gram(rng, m), _random_gram(rng, m, scale=50.0)])
    A = rng.standard_normal((2, m)).astype(np.float32)
    Ad = torch.from_numpy(A).to(gpu_device)
    for variant in ("interacting", "fisher"):
        ema = torch.zeros((2, 2), dtype=torch.float32, device=gpu_device)
        states = [None, None]
        for scale in (1.0, 4.0, 0.25):
            K = (scale * K0).astype(np.float32)
            c, info = isopo.transform_ema(torch.from_numpy(K).to(gpu_device), Ad, variant, 0.5, ema, 0.9)
            torch.cuda.synchronize()
            assert not info.any()
            for b in range(2):
                K64 = K[b].astype(np.float64)
                if variant == "interacting":
                    c_ref, states[b] = orc.coeff_interacting_ema(K64, A[b], 0.5, states[b], 0.9)
                else:
                    states[b] = orc.ema_update(states[b], float(np.mean(orc.fisher_norm_sq(K64))), 0.9)
                    c_ref = orc.coeff_fisher(K64, A[b], 0.5 * states[b], orc.REG_ABSOLUTE)
                assert ema[b, 0].item() == pytest.approx(states[b], rel=1e-6)
                assert rel_err(c[b].cpu().numpy(), c_ref) <= 1e-5, (variant, scale, b)
        assert ema[:, 1].tolist() == [3.0, 3.0]
    with pytest.raises(isopo.IsopoError):
        isopo.transform_ema(torch.from_numpy(K0).to(gpu_device), Ad, "interacting", 0.5, ema, 1.0)     # decay < 1
    with pytest.raises(isopo.IsopoError):
        isopo.transform_ema(torch.from_numpy(K0).to(gpu_device), Ad, "interacting", -1.0, ema, 0.9)


@pytest.mark.parametrize("kind", ["rank_deficient", "diagonal", "tridiagonal", "zero", "clustered", "scaled"])
def test_eigh_large_route_on_special_matrices(gpu_device, kind):
    """The tridiagonal route on matrices that exercise its special paths: a Gram matrix of rank 40 (eighty
    eigenvalues at rounding level), a diagonal and a tridiagonal matrix (nothing to reduce: every reflector is
    skipped), the zero matrix, a cluster of nearly equal eigenvalues, and entries of order 1e12 and 1e-12 (the
    power-of-two scaling)."""
    rng = np.random.default_rng(77)
    m = 120
    if kind == "rank_deficient":
        J = rng.standard_normal((m, 40))
        K = J @ J.T
    elif kind == "diagonal":
        K = np.diag(rng.uniform(0.5, 3.0, m))
    elif kind == "tridiagonal":
        K = np.diag(rng.uniform(2.0, 3.0, m)) + np.diag(rng.uniform(-1, 1, m - 1), 1)
        K = K + np.triu(K, 1).T
    elif kind == "zero":
        K = np.zeros((m, m))
    elif kind == "clustered":
        Q, _ = np.linalg.qr(rng.standard_normal((m, m)))
        K = (Q * (1.0 + 1e-9 * rng.standard_normal(m))) @ Q.T
    else:
        J = rng.standard_normal((m, 300))
        K = J @ J.T
    for scale in ((1e12, 1e-12) if kind == "scaled" else (1.0,)):
        K32 = (scale * K).astype(np.float32)
        D, U, info = isopo.ntk_eigh(torch.from_numpy(K32).to(gpu_device))
        torch.cuda.synchronize()
        assert info.item() == 0
        Dh, Uh = D.cpu().numpy(), U.cpu().numpy()
        K64 = 0.5 * (K32.astype(np.float64) + K32.astype(np.float64).T)
        D_ref, _ = orc.ntk_eigh(K64)
        size = max(np.abs(D_ref).max(), 1e-300)
        assert np.all(np.diff(Dh) >= 0)
        np.testing.assert_allclose(Dh, D_ref, atol=1e-12 * size, rtol=0)
        np.testing.assert_allclose(Uh.T @ Uh, np.eye(m), atol=1e-12)
        np.testing.assert_allclose(Uh @ np.diag(Dh) @ Uh.T, K64, atol=1e-12 * size)


def test_eigh_semidefinite_and_bad_arguments(gpu_device):
    """Duplicate sequences make K singular: with reg = 0 the null components are
    reported and left out; with reg > 0 the result matches the oracle."""
    rng = np.random.default_rng(5)
    J = rng.standard_normal((6, 40))
    J[3] = J[1]
    K = (J @ J.T).astype(np.float32)
    K = ((K + K.T) / 2).astype(np.float32)
    A = rng.standard_normal(6).astype(np.float32)
    Kd, Ad = torch.from_numpy(K).to(gpu_device), torch.from_numpy(A).to(gpu_device)
    D, U, info = isopo.ntk_eigh(Kd)
    c, sinfo = isopo.transform_eigh(D, U, Ad, [1e-2], isopo.REG_REL_TRACE)
    torch.cuda.synchronize()
    assert info.item() == 0 and sinfo.item() == 0
    assert abs(D[0].item()) <= 1e-6 * D[-1].item()
    c_ref = orc.coeff_interacting_eigh(K.astype(np.float64), A, 1e-2, orc.REG_REL_TRACE)
    assert rel_err(c[0].cpu().numpy(), c_ref) <= 1e-5
    Dz = D.clone()
    Dz[0] = -1e-9
    _, sinfo = isopo.transform_eigh(Dz, U, Ad, [0.0, 1e-2], isopo.REG_ABSOLUTE)
    assert sinfo.item() == 1
    with pytest.raises(isopo.IsopoError):
        isopo.transform_eigh(D, U, Ad, [], isopo.REG_ABSOLUTE)
    with pytest.raises(isopo.IsopoError):
        isopo.transform_eigh(D, U, Ad, [-1.0], isopo.REG_ABSOLUTE)
    with pytest.raises(isopo.IsopoError):
        isopo.transform_eigh(D, U, Ad, [1.0], isopo.REG_EMA_TRACE)          # no state
    with pytest.raises(isopo.IsopoError):
        isopo.ntk_eigh(Kd, workspace=torch.empty(256, dtype=torch.uint8, device=gpu_device)[:0])
    with pytest.raises(isopo.IsopoError):
        isopo.rescale(D.float(), D.float(), Ad, reg=(-1.0, 0, 0))
