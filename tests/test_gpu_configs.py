"""Parity at the benchmark's configurations.

config1 and config2 are compared in full (config1 in test_gpu_parity.py).  At
the larger configurations the HIP path runs at full size, in the launch
configuration the benchmark times (isopo_layer_gram keeping the stash in the
library's preferred layout, one batched transform, the stash-weighted sum), and
is compared with the oracle on

  * the WHOLE Gram matrix K and both variants' coefficients c for every
    projection of configs 3 and 4 (the oracle forms every G_i in chunks of
    output rows and K = J J^T chunk by chunk: seconds per projection),
  * sampled off-diagonal and diagonal K entries at config 5 (the 256-sequence
    layer's whole K would take the oracle minutes), the 256 x 256 solve against
    the oracle's own factorisation of the same matrix,
  * sampled dW elements, each summed token by token in fp64,

plus properties that hold at any size (bit symmetry, positive diagonal,
positive semi-definiteness within rounding, the solve's residual).
"""
import numpy as np
import pytest
import torch

from oracle import isopo_oracle as orc
from paper_2512_23353_amd import isopo
from paper_2512_23353_amd import workloads as wl

from helpers import TOL, assert_K_close, assert_c_close, assert_dW_close, oracle_step, rel_err, to_device

pytestmark = pytest.mark.gpu

LAMBDAS = (1e-4, 1e-3, 1e-2)          # the sweep the 28-layer configuration names


@pytest.mark.parametrize("rho", [0.0, 0.5])
def test_config2_block_full(gpu_device, rho):
    """All 7 projections of the 1.5B-class block, both variants, against the
    oracle in full.  rho > 0 adds the per-prompt shared component."""
    w = wl.CONFIGS["config2"]
    block = wl.make_block(w, rho=rho)
    tol = TOL["bf16"]
    for prob in block:
        print(f"config2 rho={rho} {prob.name} N={prob.n_tokens}", flush=True)
        layer, A = to_device(prob, gpu_device)
        assert isopo.gram_plan(layer)[0] == "materialised"
        out = isopo.layer_step(layer, A, "interacting", 1e-3, isopo.REG_REL_TRACE, "auto")
        cf, _ = isopo.transform(out["K"], A, "fisher", 1e-3, isopo.REG_REL_TRACE)
        dWf = isopo.weighted_grad(layer, cf, out["workspace"], layout=out["stash_layout"])
        torch.cuda.synchronize()
        ref = oracle_step(prob, "interacting", 1e-3, isopo.REG_REL_TRACE, chunk_rows=2048)
        assert_K_close(out["K"].cpu().numpy(), ref["K"], tol, prob.name)
        assert_c_close(out["c"].cpu().numpy(), ref["c"], tol, prob.name)
        assert_dW_close(out["dW"].cpu().numpy(), ref["dW"], tol, prob.name, ref["dW_abs"])
        cf_ref = orc.coeff_fisher(ref["K"], prob.A, 1e-3, isopo.REG_REL_TRACE)
        assert_c_close(cf.cpu().numpy(), cf_ref, tol, prob.name + "/fisher")
        # fisher dW checked on a band of output rows
        rows = (0, min(256, prob.d_out))
        band = orc.weighted_grad_tokens(wl.to_oracle(prob.X), wl.to_oracle(prob.Delta), prob.seq_offsets, cf_ref, rows)
        mag = orc.weighted_grad_tokens(np.abs(orc.widen(wl.to_oracle(prob.X))), np.abs(orc.widen(wl.to_oracle(prob.Delta))),
                                       prob.seq_offsets, np.abs(cf_ref), rows)
        assert_dW_close(dWf[rows[0]:rows[1]].cpu().numpy(), band, tol, prob.name + "/fisher dW band", mag)


def _sampled_pairs(rng, n_seq, n_pairs, pool=None, must=()):
    """n_pairs distinct off-diagonal (i, j) from `pool` (default: all sequences), after the pairs in `must`."""
    pool = np.arange(n_seq) if pool is None else np.asarray(pool)
    pairs = [tuple(int(v) for v in p) for p in must]
    while len(pairs) < len(must) + n_pairs:
        i, j = (int(v) for v in rng.choice(pool, 2, replace=False))
        if (i, j) not in pairs and (j, i) not in pairs:
            pairs.append((i, j))
    return pairs


def _assert_dW_samples(prob, Xo, Do, c_host, dWs, rng, tol, n=24):
    """Sampled elements of dW = Delta^T diag(c_tok) X against the token-by-token fp64 sum; the guard is
    relative to the sum of the terms' absolute values (rounding of the terms is relative to the terms)."""
    os_ = rng.integers(0, prob.d_out, n)
    ks = rng.integers(0, prob.d_in, n)
    pairs_ref = [orc.weighted_grad_entry(Xo, Do, prob.seq_offsets, c_host, int(o), int(k)) for o, k in zip(os_, ks)]
    ref = np.array([p[0] for p in pairs_ref])
    mag = np.array([p[1] for p in pairs_ref])
    for name, dW in dWs.items():
        got = dW[torch.from_numpy(os_).to(dW.device), torch.from_numpy(ks).to(dW.device)].cpu().numpy()
        assert np.all(np.abs(got - ref) <= tol * mag), f"{prob.name}: dW samples ({name})"
        assert rel_err(got, ref) <= tol, f"{prob.name}: dW samples ({name}) rel {rel_err(got, ref)}"


def _full_size_checks(prob, gpu_device, rng, *, full_k, k_pairs=(), lams=(1e-3,), reg_modes=(isopo.REG_REL_TRACE,)):
    """One layer at full size through the three calls of the layer step, in the launch configuration the
    benchmark times; K, c (both variants, every lambda and regulariser mode asked for) and dW against the
    oracle.  full_k: the whole K and c from the oracle's K; otherwise the sampled `k_pairs` entries of K
    against the oracle, and for c the defining property on the device's own K (the residual of the linear
    system, the normalisation by the Fisher norms): no device value goes into the oracle, and the transform
    itself is compared with the oracle at these sizes on synthetic matrices in test_transform_sizes."""
    tol = TOL[prob.dtype]
    layer, A = to_device(prob, gpu_device)
    chosen, _, _ = isopo.gram_plan(layer)
    assert chosen == "materialised"
    layout = isopo.stash_layout(layer)[0]
    K, ws = isopo.layer_gram(layer, "auto", keep_stash=isopo.KEEP_FAST)
    cs = {}
    for variant in ("fisher", "interacting"):
        for mode in reg_modes:
            for lam in lams:
                c, info = isopo.transform(K, A, variant, lam, mode)
                cs[(variant, mode, lam)] = (c, info)
    c_int = cs[("interacting", reg_modes[0], lams[len(lams) // 2])][0]
    dW_stash = isopo.weighted_grad(layer, c_int, ws, layout=layout)          # the step's own dW
    c_rand = torch.from_numpy(rng.standard_normal(prob.n_seq).astype(np.float32)).to(gpu_device)
    dW_stash_r = isopo.weighted_grad(layer, c_rand, ws, layout=layout)
    dW_re = isopo.weighted_grad(layer, c_rand)                                # from X and Delta, no stash
    if prob.dtype == "bf16":
        # the bf16 gradient buffer: the fp32 sums above, rounded once (so the oracle checks of dW_stash below cover it)
        dW_half = isopo.weighted_grad_stash_bf16(layer, c_int, ws, layout)
        torch.cuda.synchronize()
        assert torch.equal(dW_half, dW_stash.to(torch.bfloat16)), f"{prob.name}: bf16 dW"
        del dW_half
    torch.cuda.synchronize()
    del ws
    Kh = K.cpu().numpy().astype(np.float64)
    m = prob.n_seq
    # properties that hold at any size
    assert np.array_equal(Kh, Kh.T) and np.all(np.diag(Kh) > 0)
    assert np.linalg.eigvalsh(Kh).min() > -tol * np.trace(Kh) / m
    assert all(int(info.item()) == 0 for _, info in cs.values())
    Xo, Do = wl.to_oracle(prob.X), wl.to_oracle(prob.Delta)
    if full_k:
        K_ref = orc.layer_ntk(Xo, Do, prob.seq_offsets, chunk_rows=1024, matrix_product=True)
        assert_K_close(Kh, K_ref, tol, prob.name)
        off_diag = ~np.eye(m, dtype=bool)
        print(f"{prob.name}: K rel err {rel_err(Kh, K_ref):.2e}, off-diagonal part alone "
              f"{rel_err(Kh[off_diag], K_ref[off_diag]):.2e}, max |K_ij|/sqrt(K_ii K_jj) off the diagonal "
              f"{np.max(np.abs(K_ref[off_diag]) / np.sqrt(np.outer(np.diag(K_ref), np.diag(K_ref))[off_diag])):.2e}",
              flush=True)
        # the off-diagonal part on its own scale, so that a mistake there is not hidden behind the diagonal
        assert rel_err(Kh[off_diag], K_ref[off_diag]) <= tol, f"{prob.name}: off-diagonal K"
    else:
        K_ref = None
        for (i, j) in k_pairs:
            ref = orc.ntk_entry(Xo, Do, prob.seq_offsets, i, j)
            guard = tol * np.sqrt(Kh[i, i] * Kh[j, j])
            assert abs(Kh[i, j] - ref) <= guard, f"{prob.name}: K[{i},{j}] {Kh[i, j]} vs {ref}"
            if i != j:
                # the entry on its own scale, not the diagonal's: |<G_i, G_j>| of unrelated gradients is about
                # sqrt(K_ii K_jj / P_eff), P_eff the number of parameters that carry the energy (a few per
                # cent of d_out * d_in with the outlier channels); an entry may also be near zero by chance
                typical = np.sqrt(Kh[i, i] * Kh[j, j] / (prob.d_in * prob.d_out))
                assert abs(Kh[i, j] - ref) <= tol * (abs(ref) + 10.0 * typical), \
                    f"{prob.name}: K[{i},{j}] {Kh[i, j]} vs {ref} (typical {typical})"
    for (variant, mode, lam), (c, _) in cs.items():
        what = f"{prob.name}/{variant}/mode{mode}/lam{lam}"
        ch = c.cpu().numpy().astype(np.float64)
        A64 = prob.A.astype(np.float64)
        # the coefficients' defining property on the matrix the device produced, at any size
        f2 = np.mean(Kh * Kh, axis=1)
        if variant == "fisher":
            reg = lam * f2.mean() if mode == isopo.REG_REL_TRACE else lam
            assert np.linalg.norm(ch * np.sqrt(f2 + reg) - A64) <= 1e-4 * np.linalg.norm(A64), what
        else:
            reg = lam * np.trace(Kh) / m if mode == isopo.REG_REL_TRACE else lam
            resid = (Kh + reg * np.eye(m)) @ ch - A64
            assert np.linalg.norm(resid) <= 1e-4 * np.linalg.norm(A64), what
        if full_k:
            if variant == "fisher":
                c_ref = orc.coeff_fisher(K_ref, prob.A, lam, mode)
            else:
                c_ref, info_ref = orc.coeff_interacting(K_ref, prob.A, lam, mode)
                assert info_ref == 0
            assert_c_close(ch, c_ref, tol, what)
    # sampled dW elements: the step's own update (interacting coefficients, from the stash), and a random
    # coefficient vector from the stash and from X, Delta
    _assert_dW_samples(prob, Xo, Do, c_int.cpu().numpy(), {"step": dW_stash}, rng, tol)
    _assert_dW_samples(prob, Xo, Do, c_rand.cpu().numpy(), {"stash": dW_stash_r, "recompute": dW_re}, rng, tol)


# rho = 0.12: rollouts of one prompt correlate at a few tenths; rho = 0.5: they are nearly parallel (0.99),
# so K + reg I is close to singular within each group of eight
CONFIG3_CASES = [(p.name, 0.0) for p in wl.CONFIGS["config3"].projections] + [("gate", 0.12), ("k", 0.5)]


@pytest.mark.parametrize("name,rho", CONFIG3_CASES, ids=[f"{n}-rho{r}" for n, r in CONFIG3_CASES])
def test_config3_full_size(gpu_device, name, rho):
    """Every projection of the 7B-class block at full size (B = 32, lengths in
    [512, 4096], about 7e4 tokens): whole K, both variants' coefficients and
    sampled dW elements against the oracle.  The last two cases add the
    per-prompt shared component: the widest projection with off-diagonal
    entries of a few tenths of the diagonal (what the interacting update exists
    for), and a narrow one with nearly parallel rollouts."""
    w = wl.CONFIGS["config3"]
    lengths = wl.draw_lengths(w)
    proj = {p.name: p for p in w.projections}[name]
    rng = np.random.default_rng(33 + sum(map(ord, name)))
    prob = wl.make_layer(w, proj, lengths, device=gpu_device, rho=rho)
    print(f"config3 {name} rho={rho} N={prob.n_tokens}", flush=True)
    _full_size_checks(prob, gpu_device, rng, full_k=True)
    del prob
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name", ["v", "up"])
def test_config4_one_layer_full_k_and_lambda_sweep(gpu_device, name):
    """One layer of the 28-layer sweep (B = 64 sequences of 2048 tokens): whole
    K, then both variants' coefficients at every lambda of the sweep, with the
    relative and the absolute regulariser, against the oracle."""
    w = wl.CONFIGS["config4"]
    lengths = wl.draw_lengths(w)
    proj = {p.name: p for p in w.projections}[name]
    rng = np.random.default_rng(44 + sum(map(ord, name)))
    prob = wl.make_layer(w, proj, lengths, device=gpu_device, layer=27)
    print(f"config4 {name} N={prob.n_tokens}", flush=True)
    _full_size_checks(prob, gpu_device, rng, full_k=True, lams=LAMBDAS,
                      reg_modes=(isopo.REG_REL_TRACE, isopo.REG_ABSOLUTE))
    del prob
    torch.cuda.empty_cache()


@pytest.mark.parametrize("n_short", [4, 8, 16])
def test_config5_ghost_on_shortest_sequences(gpu_device, n_short):
    """Sub-microbatches of the stress layer's shortest sequences: few tokens on
    a 5120 -> 27648 layer is where the ghost form is the cheaper one."""
    w = wl.CONFIGS["config5"]
    lengths = np.sort(wl.draw_lengths(w))[:n_short]
    prob = wl.make_layer(w, w.projections[0], lengths, device=gpu_device)
    layer, A = to_device(prob, gpu_device)
    assert isopo.gram_plan(layer)[0] == "ghost"
    out = isopo.layer_step(layer, A, "interacting", 1e-3, isopo.REG_REL_TRACE, "auto")
    Km, _ = isopo.layer_gram(layer, "materialised")
    torch.cuda.synchronize()
    K_ref = orc.layer_ntk(wl.to_oracle(prob.X), wl.to_oracle(prob.Delta), prob.seq_offsets, chunk_rows=2048)
    assert_K_close(out["K"].cpu().numpy(), K_ref, TOL["bf16"], "config5 ghost")
    assert_K_close(Km.cpu().numpy(), K_ref, TOL["bf16"], "config5 materialised")
    c_ref, _ = orc.coeff_interacting(K_ref, prob.A, 1e-3, isopo.REG_REL_TRACE)
    assert_c_close(out["c"].cpu().numpy(), c_ref, TOL["bf16"], "config5 c")


def test_config5_full_size_sampled(gpu_device):
    """The stress layer at full size: 5120 -> 27648, B = 256 sequences with
    clipped log-normal lengths (about 4e5 tokens, a 67 GiB bf16 stash).  AUTO
    must choose the materialised path.  K: ten off-diagonal entries among the
    forty shortest sequences, two entries that pair the longest sequence with
    short ones, two diagonal entries.  c: the residual of the 256 x 256 system
    and the Fisher normalisation on the device's K (the oracle's own K would
    take it minutes).  dW: sampled elements."""
    w = wl.CONFIGS["config5"]
    lengths = wl.draw_lengths(w)
    assert lengths.min() >= 128 and lengths.max() <= 16384
    rng = np.random.default_rng(55)
    prob = wl.make_layer(w, w.projections[0], lengths, device=gpu_device)
    print(f"config5 gate N={prob.n_tokens}", flush=True)
    order = np.argsort(lengths, kind="stable")
    longest = int(order[-1])
    pairs = _sampled_pairs(rng, prob.n_seq, 10, pool=order[:40],
                           must=[(longest, int(order[0])), (int(order[1]), longest), (int(order[0]), int(order[0])),
                                 (int(order[7]), int(order[7]))])
    _full_size_checks(prob, gpu_device, rng, full_k=False, k_pairs=pairs)
    # the token-sample Fisher coefficients at the same size (256 sequences, 64 samples): the two
    # shortest sequences against the oracle, finiteness and positivity for the rest
    layer, A = to_device(prob, gpu_device)
    idx = rng.permutation(prob.n_tokens)[:64].astype(np.int32)
    c, f2 = isopo.fisher_samples(layer, torch.from_numpy(idx).to(gpu_device), A, 1e-3, isopo.REG_REL_TRACE)
    torch.cuda.synchronize()
    f2h = f2.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(f2h)) and np.all(f2h > 0) and np.all(np.isfinite(c.cpu().numpy()))
    short = order[:2]
    ref = orc.fisher_norm_sq_token_samples(wl.to_oracle(prob.X), wl.to_oracle(prob.Delta), prob.seq_offsets, idx, seqs=short)
    for i in short:
        assert abs(f2h[i] - ref[i]) <= TOL["bf16"] * ref[i], f"config5 F^2[{i}] {f2h[i]} vs {ref[i]}"
