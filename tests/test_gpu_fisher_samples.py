"""Parity of the token-position-sample Fisher coefficients (the non-interacting
listing's F_norm estimate, evaluated in ghost form on the GPU) with the oracle,
which forms every G_i and every rank-one g^(j) explicitly."""
import numpy as np
import pytest
import torch

from oracle import isopo_oracle as orc
from paper_2512_23353_amd import isopo
from paper_2512_23353_amd import workloads as wl

from helpers import TOL, assert_c_close, assert_dW_close, rel_err, to_device

pytestmark = pytest.mark.gpu


def _draw_samples(rng, n_tokens, n_s, replace=False):
    if replace or n_s > n_tokens:
        return rng.integers(0, n_tokens, n_s).astype(np.int32)
    return rng.permutation(n_tokens)[:n_s].astype(np.int32)


def _check(prob, device, idx, lam, reg_mode, what):
    tol = TOL[prob.dtype]
    layer, A = to_device(prob, device)
    c, f2 = isopo.fisher_samples(layer, torch.from_numpy(idx).to(device), A, lam, reg_mode)
    torch.cuda.synchronize()
    c_ref, f2_ref = orc.coeff_fisher_token_samples(wl.to_oracle(prob.X), wl.to_oracle(prob.Delta), prob.seq_offsets,
                                                   idx, prob.A, lam, reg_mode)
    f2h = f2.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(f2h)) and np.all(f2h >= 0)
    assert rel_err(f2h, f2_ref) <= tol, f"{what}: F^2 rel {rel_err(f2h, f2_ref)}"
    assert np.all(np.abs(f2h - f2_ref) <= tol * (f2_ref + f2_ref.mean())), f"{what}: F^2 element guard"
    assert_c_close(c.cpu().numpy(), c_ref, tol, what)
    return layer, c, c_ref


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n_s", [1, 8, 31, 32, 33, 64, 100, 128])
def test_sample_counts(gpu_device, dtype, n_s):
    """Every sample-block count (1..4 blocks of 32) with ragged last blocks, on a
    microbatch spanning several 128-token workgroups and a ragged tail."""
    rng = np.random.default_rng(100 + n_s)
    lengths = [100, 37, 1, 0, 250, 64, 190]
    prob = wl.custom_layer(256, 384, lengths, dtype=dtype, seed=5, sigma_delta=1e-2)
    idx = _draw_samples(rng, prob.n_tokens, n_s)
    _check(prob, gpu_device, idx, 1e-3, isopo.REG_REL_TRACE, f"{dtype}/n_s={n_s}")


CASES = [
    ("all_single_tokens", 64, 128, [1] * 40),
    ("one_huge_many_tiny", 128, 256, [3, 1, 700, 2, 5, 1, 1, 9]),
    ("one_sequence", 256, 128, [333]),
    ("narrow_dims", 72, 200, [31, 32, 33, 65]),
    ("empty_first_and_last", 128, 128, [0, 50, 0, 0, 70, 0]),
    ("boundaries_inside_a_wave", 136, 88, [5, 7, 11, 13, 17, 19, 23, 29, 31, 2, 3]),
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("reg", [(0.0, isopo.REG_ABSOLUTE), (1e-6, isopo.REG_ABSOLUTE), (1e-2, isopo.REG_REL_TRACE)])
def test_ragged_edge_cases(gpu_device, dtype, case, reg):
    name, d_in, d_out, lengths = case
    rng = np.random.default_rng(7)
    prob = wl.custom_layer(d_in, d_out, lengths, dtype=dtype, seed=13, sigma_delta=1e-2)
    idx = _draw_samples(rng, prob.n_tokens, 16)
    _check(prob, gpu_device, idx, reg[0], reg[1], f"{name}/{dtype}")


def test_repeated_and_clustered_samples(gpu_device):
    """Samples drawn with replacement, and samples all taken from one sequence:
    the estimate is defined for both."""
    rng = np.random.default_rng(3)
    prob = wl.custom_layer(192, 320, [60, 90, 30, 120], dtype="bf16", seed=17, sigma_delta=1e-2, rho=0.5)
    _check(prob, gpu_device, _draw_samples(rng, prob.n_tokens, 48, replace=True), 1e-3, isopo.REG_REL_TRACE, "replace")
    idx = (60 + rng.permutation(90)[:24]).astype(np.int32)
    _check(prob, gpu_device, idx, 1e-3, isopo.REG_REL_TRACE, "clustered")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_whole_non_interacting_update(gpu_device, dtype):
    """rescaling() followed by the weighted accumulation (non-interacting
    listing): coefficients from the token samples, then one contraction with
    pre-scaled rows, against the oracle's sum_i c_i G_i."""
    rng = np.random.default_rng(23)
    prob = wl.custom_layer(320, 256, [130, 70, 1, 200, 45], dtype=dtype, seed=29, sigma_delta=1e-2)
    idx = _draw_samples(rng, prob.n_tokens, 32)
    layer, c, c_ref = _check(prob, gpu_device, idx, 1e-3, isopo.REG_REL_TRACE, "update")
    dW = isopo.weighted_grad_prescaled(layer, c)
    torch.cuda.synchronize()
    Xo, Do = wl.to_oracle(prob.X), wl.to_oracle(prob.Delta)
    G = orc.seq_logprob_grads(Xo, Do, prob.seq_offsets)
    ref = orc.weighted_grad(G, c_ref)
    mag = orc.weighted_grad_abs(G, c_ref)
    assert_dW_close(dW.cpu().numpy(), ref, TOL[dtype], "token-sample update", mag)


def test_config3_full_size_sampled_sequences(gpu_device):
    """The 7B-class gate projection at full size (4096 -> 14336, B = 32, lengths
    in [512, 4096]) with the listing's default of 32 samples: F^2 of the three
    shortest sequences against the oracle, and properties of the rest."""
    w = wl.CONFIGS["config3"]
    lengths = wl.draw_lengths(w)
    proj = {p.name: p for p in w.projections}["gate"]
    prob = wl.make_layer(w, proj, lengths, device=gpu_device)
    rng = np.random.default_rng(303)
    idx = _draw_samples(rng, prob.n_tokens, 32)
    layer, A = to_device(prob, gpu_device)
    c, f2 = isopo.fisher_samples(layer, torch.from_numpy(idx).to(gpu_device), A, 1e-3, isopo.REG_REL_TRACE)
    torch.cuda.synchronize()
    f2h = f2.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(f2h)) and np.all(f2h > 0)
    ch = c.cpu().numpy().astype(np.float64)
    assert np.allclose(ch, prob.A / np.sqrt(f2h + 1e-3 * f2h.mean()), rtol=1e-5, atol=0)
    short = np.argsort(lengths)[:3]
    Xo, Do = wl.to_oracle(prob.X), wl.to_oracle(prob.Delta)
    ref = orc.fisher_norm_sq_token_samples(Xo, Do, prob.seq_offsets, idx, seqs=short)
    for i in short:
        print(f"config3 gate seq {i} len {lengths[i]}: F^2 {f2h[i]:.6e} vs {ref[i]:.6e}", flush=True)
        assert abs(f2h[i] - ref[i]) <= TOL["bf16"] * ref[i]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_group_sharing_the_input(gpu_device, dtype):
    """q/k/v-like layers on one input: the group call (X streamed once) against
    the oracle layer by layer and against the single-layer calls."""
    rng = np.random.default_rng(91)
    lengths = [130, 70, 1, 0, 200, 45]
    base = wl.custom_layer(256, 320, lengths, dtype=dtype, seed=60, sigma_delta=1e-2)
    d_outs = [320, 64, 136, 512]
    X = base.X.to(gpu_device)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    g = torch.Generator().manual_seed(61)
    Deltas = [(torch.randn(base.n_tokens, d, generator=g) * 1e-2).to(tdt).to(gpu_device) for d in d_outs]
    first = isopo.Layer(X, Deltas[0], base.seq_offsets)
    layers = [first] + [isopo.Layer(X, D, base.seq_offsets, seq_offsets_dev=first.off_dev) for D in Deltas[1:]]
    A = torch.from_numpy(base.A).to(gpu_device)
    idx = _draw_samples(rng, base.n_tokens, 40)
    idx_d = torch.from_numpy(idx).to(gpu_device)
    for n in (1, 2, 4):
        c, f2 = isopo.fisher_samples_group(layers[:n], idx_d, A, 1e-3, isopo.REG_REL_TRACE)
        torch.cuda.synchronize()
        for l in range(n):
            c_ref, f2_ref = orc.coeff_fisher_token_samples(wl.to_oracle(X), wl.to_oracle(Deltas[l]), base.seq_offsets,
                                                           idx, base.A, 1e-3, isopo.REG_REL_TRACE)
            assert rel_err(f2[l].cpu().numpy(), f2_ref) <= TOL[dtype], f"group of {n}, layer {l}"
            assert_c_close(c[l].cpu().numpy(), c_ref, TOL[dtype], f"group of {n}, layer {l}")
            c1, f1 = isopo.fisher_samples(layers[l], idx_d, A, 1e-3, isopo.REG_REL_TRACE)
            assert torch.allclose(f1, f2[l], rtol=1e-5, atol=0)
    other = isopo.Layer(X.clone(), Deltas[1], base.seq_offsets, seq_offsets_dev=first.off_dev)
    with pytest.raises(isopo.IsopoError):
        isopo.fisher_samples_group([first, other], idx_d, A)           # not the same input
    with pytest.raises(isopo.IsopoError):
        isopo.fisher_samples_group(layers + [layers[0]], idx_d, A)      # more than ISOPO_MAX_GROUP


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_block_of_groups_in_one_launch(gpu_device, dtype):
    """A transformer block's groups ({three layers on one input}, {one}, {two}, {one}, with different
    input widths) in one launch: every layer against the oracle and against the group-by-group calls;
    token counts that do and do not fill the last workgroup; the trailing-mean state kept per layer."""
    rng = np.random.default_rng(95)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    # the first three microbatches are short enough for the launch to make every layer a group of its own; the
    # last one (175 token tiles x 7 layers) keeps the groups
    for lengths in ([130, 70, 1, 0, 200, 45], [128] * 9, [3, 0, 0, 2], [2800] * 8 + [13]):
        seq_offsets = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
        n_tok, m = int(seq_offsets[-1]), len(lengths)
        g = torch.Generator().manual_seed(62)
        shapes = [(256, [320, 64, 136]), (320, [256]), (72, [512, 8]), (512, [72])]
        groups, Xs, Ds = [], [], []
        first = None
        for d_in, d_outs in shapes:
            X = torch.randn(n_tok, d_in, generator=g).to(tdt).to(gpu_device)
            grp = []
            for d in d_outs:
                D = (torch.randn(n_tok, d, generator=g) * 1e-2).to(tdt).to(gpu_device)
                lay = isopo.Layer(X, D, seq_offsets) if first is None else isopo.Layer(X, D, seq_offsets, seq_offsets_dev=first.off_dev)
                first = first or lay
                grp.append(lay)
                Xs.append(X)
                Ds.append(D)
            groups.append(grp)
        A_h = rng.standard_normal(m).astype(np.float32)
        A = torch.from_numpy(A_h).to(gpu_device)
        idx = _draw_samples(rng, n_tok, min(24, n_tok))
        idx_d = torch.from_numpy(idx).to(gpu_device)
        c, f2 = isopo.fisher_samples_block(groups, idx_d, A, 1e-3, isopo.REG_REL_TRACE)
        torch.cuda.synchronize()
        l = 0
        for grp in groups:
            cg, fg = isopo.fisher_samples_group(grp, idx_d, A, 1e-3, isopo.REG_REL_TRACE)
            torch.cuda.synchronize()
            for k in range(len(grp)):
                c_ref, f2_ref = orc.coeff_fisher_token_samples(wl.to_oracle(Xs[l]), wl.to_oracle(Ds[l]), seq_offsets, idx,
                                                               A_h, 1e-3, isopo.REG_REL_TRACE)
                what = f"lengths {lengths[:3]}.., layer {l}"
                assert rel_err(f2[l].cpu().numpy(), f2_ref) <= TOL[dtype], what
                assert_c_close(c[l].cpu().numpy(), c_ref, TOL[dtype], what)
                assert torch.allclose(fg[k], f2[l], rtol=1e-5, atol=0) and torch.allclose(cg[k], c[l], rtol=1e-5, atol=0), what
                l += 1
        assert l == 7
    # one trailing mean per layer, in the order of the layers
    ema = torch.zeros((7, 2), dtype=torch.float32, device=gpu_device)
    c1, f1 = isopo.fisher_samples_block(groups, idx_d, A, 0.5, isopo.REG_EMA_TRACE, ema_state=ema, ema_decay=0.9)
    torch.cuda.synchronize()
    assert torch.allclose(ema[:, 0], f1.mean(dim=1), rtol=1e-5) and bool((ema[:, 1] == 1).all())
    with pytest.raises(isopo.IsopoError):
        isopo.fisher_samples_block([groups[0] + groups[1]], idx_d, A)          # a group on two inputs
    with pytest.raises(isopo.IsopoError):
        isopo.fisher_samples_block([[l_] for l_ in (groups[0] * 3)], idx_d, A)  # more than ISOPO_MAX_GROUPS groups


def test_trailing_mean_regulariser(gpu_device):
    """reg = factor * E[mean F^2] with the trailing mean kept on the device over
    three minibatches of different scale."""
    rng = np.random.default_rng(71)
    ema = torch.zeros(2, dtype=torch.float32, device=gpu_device)
    state = None
    for k, scale in enumerate((1e-2, 3e-2, 5e-3)):
        prob = wl.custom_layer(192, 256, [60, 90, 30, 120, 11], dtype="bf16", seed=80 + k, sigma_delta=scale)
        idx = _draw_samples(rng, prob.n_tokens, 24)
        layer, A = to_device(prob, gpu_device)
        c, f2 = isopo.fisher_samples(layer, torch.from_numpy(idx).to(gpu_device), A, 0.7, isopo.REG_EMA_TRACE,
                                     ema_state=ema, ema_decay=0.9)
        torch.cuda.synchronize()
        c_ref, f2_ref, state = orc.coeff_fisher_token_samples_ema(wl.to_oracle(prob.X), wl.to_oracle(prob.Delta),
                                                                  prob.seq_offsets, idx, prob.A, 0.7, state, 0.9)
        assert ema[0].item() == pytest.approx(state, rel=TOL["bf16"])
        assert ema[1].item() == k + 1
        assert_c_close(c.cpu().numpy(), c_ref, TOL["bf16"], f"minibatch {k}")
    with pytest.raises(isopo.IsopoError):
        isopo.fisher_samples(layer, torch.from_numpy(idx).to(gpu_device), A, 0.7, isopo.REG_EMA_TRACE)   # no state


def test_bad_arguments(gpu_device):
    prob = wl.custom_layer(64, 64, [10, 20], dtype="f32", seed=1)
    layer, A = to_device(prob, gpu_device)
    idx = torch.zeros(200, dtype=torch.int32, device=gpu_device)
    with pytest.raises(isopo.IsopoError):
        isopo.fisher_samples(layer, idx[:0], A)
    with pytest.raises(isopo.IsopoError):
        isopo.fisher_samples(layer, idx[:129], A)
    with pytest.raises(isopo.IsopoError):
        isopo.fisher_samples(layer, idx[:8], A, lam=-1.0)
    with pytest.raises(isopo.IsopoError):
        isopo.fisher_samples(layer, idx[:8], A, workspace=torch.empty(256, dtype=torch.uint8, device=gpu_device))
