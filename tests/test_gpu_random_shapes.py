"""Seeded random shapes through every route of the HIP path against the oracle:
dimensions that are not multiples of any tile size, sequences of length 0 and
1 mixed with long ones, both dtypes, both Gram paths, both transforms, the
stash-free update and the token-sample coefficients.  Four families: small
layers, layers wide enough for the 256x256 tiles, wide layers on few tokens, and
more than 128 short sequences on layers whose stash is kept in tile order (the
Gram kernels and the transform for many sequences, the bf16 gradient buffer)."""
import numpy as np
import pytest
import torch

from oracle import isopo_oracle as orc
from paper_2512_23353_amd import isopo
from paper_2512_23353_amd import workloads as wl

from helpers import TOL, assert_K_close, assert_c_close, assert_dW_close, oracle_step, rel_err, to_device

pytestmark = pytest.mark.gpu


def _draw_case(seed):
    rng = np.random.default_rng(seed)
    if seed >= 300:
        # many short sequences, dimensions that are multiples of 256: tile-order stash, the Gram kernels for 129 - 256
        # and for more than 256 sequences, the transform's panels in global scratch
        dtype = "bf16"
        d_in = 256
        d_out = int(rng.integers(1, 3)) * 256
        n_seq = int(rng.integers(129, 257)) if seed % 2 == 0 else int(rng.integers(257, 330))
        lengths = [int(rng.integers(0, 2)) if rng.random() < 0.1 else int(rng.integers(2, 48)) for _ in range(n_seq)]
        return dtype, d_in, d_out, lengths
    if seed >= 200:
        # few tokens on a wide layer: the ghost launch cuts the features into ranges (64-feature tails included)
        dtype = "bf16"
        d_in = int(rng.integers(128, 400)) * 8
        d_out = int(rng.integers(128, 400)) * 8
        n_seq = int(rng.integers(1, 7))
        lengths = [int(rng.integers(0, 2)) if rng.random() < 0.2 else int(rng.integers(2, 150)) for _ in range(n_seq)]
        if sum(lengths) == 0:
            lengths[0] = int(rng.integers(1, 50))
        return dtype, d_in, d_out, lengths
    if seed >= 100:
        # wide enough for the 256x256 tiles with ragged edge tiles, enough sequences to fill the chip
        dtype = "bf16"
        d_in = int(rng.integers(33, 110)) * 8
        d_out = int(rng.integers(33, 110)) * 8
        n_seq = int(rng.integers(24, 48))
        lengths = [int(rng.integers(0, 3)) if rng.random() < 0.15 else int(rng.integers(3, 260)) for _ in range(n_seq)]
        return dtype, d_in, d_out, lengths
    dtype = "bf16" if seed % 2 else "f32"
    unit = 8 if dtype == "bf16" else 4
    d_in = int(rng.integers(1, 80)) * unit
    d_out = int(rng.integers(1, 80)) * unit
    n_seq = int(rng.integers(1, 12))
    kinds = rng.integers(0, 4, n_seq)
    lengths = [int({0: 0, 1: 1, 2: rng.integers(2, 40), 3: rng.integers(40, 400)}[k]) for k in kinds]
    if sum(lengths) == 0:
        lengths[0] = int(rng.integers(1, 50))
    return dtype, d_in, d_out, lengths


@pytest.mark.parametrize("seed", list(range(32)) + list(range(100, 112)) + list(range(200, 210)) + list(range(300, 306)))
def test_random_shape(gpu_device, seed):
    dtype, d_in, d_out, lengths = _draw_case(seed)
    print(f"seed {seed}: {dtype} d_in={d_in} d_out={d_out} lengths={lengths}", flush=True)
    prob = wl.custom_layer(d_in, d_out, lengths, dtype=dtype, seed=1000 + seed, sigma_delta=1e-2, rho=0.3 * (seed % 3))
    tol = TOL[dtype]
    layer, A = to_device(prob, gpu_device)
    ref = oracle_step(prob, "interacting", 1e-2, isopo.REG_REL_TRACE)
    ref_f = oracle_step(prob, "fisher", 1e-2, isopo.REG_REL_TRACE)
    for path in ("materialised", "ghost"):
        out = isopo.layer_step(layer, A, "interacting", 1e-2, isopo.REG_REL_TRACE, path)
        torch.cuda.synchronize()
        what = f"seed {seed}/{path}"
        assert int(out["info"].item()) == 0
        Kh = out["K"].cpu().numpy()
        assert np.array_equal(Kh, Kh.T)
        assert_K_close(Kh, ref["K"], tol, what)
        assert_c_close(out["c"].cpu().numpy(), ref["c"], tol, what)
        assert_dW_close(out["dW"].cpu().numpy(), ref["dW"], tol, what, ref["dW_abs"])
        cf, _ = isopo.transform(out["K"], A, "fisher", 1e-2, isopo.REG_REL_TRACE)
        assert_c_close(cf.cpu().numpy(), ref_f["c"], tol, what + "/fisher")
        if path == "materialised" and dtype == "bf16":
            # the bf16 gradient buffer from the same stash: the fp32 result rounded once
            half = isopo.weighted_grad_stash_bf16(layer, out["c"], out["workspace"], out["stash_layout"])
            torch.cuda.synchronize()
            assert torch.equal(half, out["dW"].to(torch.bfloat16)), what + "/bf16 dW"
    # the stash-free routes with the oracle's own coefficients
    c_dev = torch.from_numpy(ref["c"].astype(np.float32)).to(gpu_device)
    c32 = c_dev.cpu().numpy().astype(np.float64)
    G = orc.seq_logprob_grads(wl.to_oracle(prob.X), wl.to_oracle(prob.Delta), prob.seq_offsets)
    want, mag = orc.weighted_grad(G, c32), orc.weighted_grad_abs(G, c32)
    for name, dW in (("weighted", isopo.weighted_grad(layer, c_dev)), ("prescaled", isopo.weighted_grad_prescaled(layer, c_dev))):
        assert_dW_close(dW.cpu().numpy(), want, tol, f"seed {seed}/{name}", mag)
    plain = isopo.weighted_grad(layer, None)
    ones = np.ones(prob.n_seq)
    assert_dW_close(plain.cpu().numpy(), orc.weighted_grad(G, ones), tol, f"seed {seed}/plain", orc.weighted_grad_abs(G, ones))
    # token-sample coefficients
    rng = np.random.default_rng(seed)
    n_s = int(rng.integers(1, min(prob.n_tokens, 128) + 1))
    idx = rng.permutation(prob.n_tokens)[:n_s].astype(np.int32)
    c_ts, f2 = isopo.fisher_samples(layer, torch.from_numpy(idx).to(gpu_device), A, 1e-2, isopo.REG_REL_TRACE)
    torch.cuda.synchronize()
    c_ref, f2_ref = orc.coeff_fisher_token_samples(wl.to_oracle(prob.X), wl.to_oracle(prob.Delta), prob.seq_offsets,
                                                   idx, prob.A, 1e-2, isopo.REG_REL_TRACE)
    assert rel_err(f2.cpu().numpy(), f2_ref) <= tol, f"seed {seed}: F^2"
    assert_c_close(c_ts.cpu().numpy(), c_ref, tol, f"seed {seed}/token samples")
