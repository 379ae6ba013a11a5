"""Parity at the benchmark's configurations.

config1 and config2 are compared in full.  At the larger configurations the
oracle cannot form everything in reasonable time, so the HIP path runs at full
size, in the launch configuration the benchmark times, and is checked on what
the oracle can compute one by one: whole K for the narrow projections, sampled
K entries and sampled dW elements for the wide ones, and properties that hold
at any size (symmetry, positive diagonal, the solve's residual).
"""
import numpy as np
import pytest
import torch

from oracle import isopo_oracle as orc
from paper_2512_23353_amd import isopo
from paper_2512_23353_amd import workloads as wl

from helpers import TOL, assert_K_close, assert_c_close, assert_dW_close, oracle_step, rel_err, to_device

pytestmark = pytest.mark.gpu


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


def _sampled_checks(prob, gpu_device, rng, n_k_entries, full_k=False):
    tol = TOL[prob.dtype]
    layer, A = to_device(prob, gpu_device)
    chosen, full, _ = isopo.gram_plan(layer)
    # the stash in the layout the benchmark's step uses (tile order for these shapes)
    K, ws = isopo.layer_gram(layer, "auto", keep_stash=isopo.KEEP_FAST if chosen == "materialised" else 0)
    c_rand = torch.from_numpy(rng.standard_normal(prob.n_seq).astype(np.float32)).to(gpu_device)
    dW_stash = (isopo.weighted_grad(layer, c_rand, ws, layout=isopo.stash_layout(layer)[0])
                if chosen == "materialised" else None)
    dW_re = isopo.weighted_grad(layer, c_rand)
    c_int, info = isopo.transform(K, A, "interacting", 1e-3, isopo.REG_REL_TRACE)
    torch.cuda.synchronize()
    Kh = K.cpu().numpy().astype(np.float64)
    Xo, Do = wl.to_oracle(prob.X), wl.to_oracle(prob.Delta)
    # properties that hold at any size
    assert np.array_equal(Kh, Kh.T) and np.all(np.diag(Kh) > 0)
    assert np.linalg.eigvalsh(Kh).min() > -tol * np.trace(Kh) / prob.n_seq
    assert info.item() == 0
    reg = 1e-3 * np.trace(Kh) / prob.n_seq
    resid = (Kh + reg * np.eye(prob.n_seq)) @ c_int.cpu().numpy().astype(np.float64) - prob.A
    assert np.linalg.norm(resid) <= 1e-4 * np.linalg.norm(prob.A)
    # K against the oracle
    if full_k:
        K_ref = orc.layer_ntk(Xo, Do, prob.seq_offsets, chunk_rows=1024)
        assert_K_close(Kh, K_ref, tol, prob.name)
        c_ref, _ = orc.coeff_interacting(K_ref, prob.A, 1e-3, isopo.REG_REL_TRACE)
        assert_c_close(c_int.cpu().numpy(), c_ref, tol, prob.name)
    pairs = [(0, 0), (prob.n_seq - 1, prob.n_seq - 1)]
    pairs += [tuple(rng.integers(0, prob.n_seq, 2)) for _ in range(n_k_entries)]
    for (i, j) in pairs[: n_k_entries]:
        ref = orc.ntk_entry(Xo, Do, prob.seq_offsets, int(i), int(j))
        guard = tol * np.sqrt(Kh[i, i] * Kh[j, j])
        assert abs(Kh[i, j] - ref) <= guard, f"{prob.name}: K[{i},{j}] {Kh[i, j]} vs {ref}"
    # sampled dW elements for a random coefficient vector
    c_host = c_rand.cpu().numpy()
    os_ = rng.integers(0, prob.d_out, 24)
    ks = rng.integers(0, prob.d_in, 24)
    pairs_ref = [orc.weighted_grad_entry(Xo, Do, prob.seq_offsets, c_host, int(o), int(k)) for o, k in zip(os_, ks)]
    ref = np.array([p[0] for p in pairs_ref])
    mag = np.array([p[1] for p in pairs_ref])     # sum of |terms|: the scale rounding is relative to
    for name, dW in (("stash", dW_stash), ("recompute", dW_re)):
        if dW is None:
            continue
        got = dW[torch.from_numpy(os_).to(gpu_device), torch.from_numpy(ks).to(gpu_device)].cpu().numpy()
        assert np.all(np.abs(got - ref) <= tol * mag), f"{prob.name}: dW samples ({name})"
        assert rel_err(got, ref) <= tol, f"{prob.name}: dW samples ({name}) rel {rel_err(got, ref)}"


def test_config3_full_size_sampled(gpu_device):
    """7B-class block at full size (B=32, lengths in [512, 4096]), generated on
    the device: whole K for the k projection, sampled K entries for gate and
    down, sampled dW elements for all three."""
    w = wl.CONFIGS["config3"]
    lengths = wl.draw_lengths(w)
    rng = np.random.default_rng(33)
    by_name = {p.name: p for p in w.projections}
    for name, n_entries, full_k in (("k", 3, True), ("gate", 2, False), ("down", 2, False)):
        print(f"config3 {name}", flush=True)
        prob = wl.make_layer(w, by_name[name], lengths, device=gpu_device)
        _sampled_checks(prob, gpu_device, rng, n_entries, full_k)
        del prob
        torch.cuda.empty_cache()


def test_config4_one_layer_sampled(gpu_device):
    """One layer of the 28-layer sweep: B=64 sequences of 2048 tokens."""
    w = wl.CONFIGS["config4"]
    lengths = wl.draw_lengths(w)
    rng = np.random.default_rng(44)
    by_name = {p.name: p for p in w.projections}
    for name, n_entries, full_k in (("v", 3, True), ("up", 2, False)):
        print(f"config4 {name}", flush=True)
        prob = wl.make_layer(w, by_name[name], lengths, device=gpu_device, layer=27)
        _sampled_checks(prob, gpu_device, rng, n_entries, full_k)
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
    must choose the materialised path; K entries, the solve's residual and dW
    elements are checked where the oracle can form them one by one."""
    w = wl.CONFIGS["config5"]
    lengths = wl.draw_lengths(w)
    assert lengths.min() >= 128 and lengths.max() <= 16384
    rng = np.random.default_rng(55)
    prob = wl.make_layer(w, w.projections[0], lengths, device=gpu_device)
    print(f"config5 gate N={prob.n_tokens}", flush=True)
    layer, _ = to_device(prob, gpu_device)
    assert isopo.gram_plan(layer)[0] == "materialised"
    del layer
    _sampled_checks(prob, gpu_device, rng, 3, full_k=False)
    # the token-sample Fisher coefficients at the same size (256 sequences, 64 samples): the two
    # shortest sequences against the oracle, finiteness and positivity for the rest
    layer, A = to_device(prob, gpu_device)
    idx = rng.permutation(prob.n_tokens)[:64].astype(np.int32)
    c, f2 = isopo.fisher_samples(layer, torch.from_numpy(idx).to(gpu_device), A, 1e-3, isopo.REG_REL_TRACE)
    torch.cuda.synchronize()
    f2h = f2.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(f2h)) and np.all(f2h > 0) and np.all(np.isfinite(c.cpu().numpy()))
    short = np.argsort(lengths)[:2]
    ref = orc.fisher_norm_sq_token_samples(wl.to_oracle(prob.X), wl.to_oracle(prob.Delta), prob.seq_offsets, idx, seqs=short)
    for i in short:
        assert abs(f2h[i] - ref[i]) <= TOL["bf16"] * ref[i], f"config5 F^2[{i}] {f2h[i]} vs {ref[i]}"
