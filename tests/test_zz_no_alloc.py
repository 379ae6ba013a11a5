"""isopo_transform_noalloc: the transform for callers that cannot allocate.

Its scratch is an array the library holds on the GPU; every buffer the call
touches besides it comes from the caller.  Checked against isopo_transform
(same kernels, caller-provided workspace) on two calls in a row, the second
on a smaller problem, so that what the first call left in the shared array
is shown not to matter.  This file sorts last on purpose.
"""
import numpy as np
import pytest
import torch

from oracle import isopo_oracle as orc
from paper_2512_23353_amd import isopo

from helpers import assert_c_close

pytestmark = pytest.mark.gpu


def _random_gram(rng, m, scale=1.0):
    J = rng.standard_normal((m, m + 8)) * scale
    J += 0.5 * scale * rng.standard_normal((1, m + 8))
    return (J @ J.T).astype(np.float32)


def _problem(rng, m, batch, dev, singular=None):
    K = np.stack([_random_gram(rng, m, 1.0 + b) for b in range(batch)])
    if singular is not None:
        K[singular] = 0.0
        K[singular, :3, :3] = np.array([[4, 2, 0], [2, 1, 0], [0, 0, 1]], np.float32)   # second pivot fails
    A = rng.standard_normal((batch, m)).astype(np.float32)
    return K, A, torch.from_numpy(K).to(dev), torch.from_numpy(A).to(dev)


def test_two_calls_in_a_row_match_the_workspace_entry_point(gpu_device):
    lib = isopo.load()
    rng = np.random.default_rng(777)
    # both sizes are above 128 sequences, where the scratch is used; the second is smaller and has one problem
    # that is not positive definite
    for m, batch, singular in ((256, 3, None), (160, 2, 1)):
        K, A, Kd, Ad = _problem(rng, m, batch, gpu_device, singular)
        for variant, lam, mode in (("interacting", 1e-2, isopo.REG_REL_TRACE), ("interacting", 0.0, isopo.REG_ABSOLUTE),
                                   ("fisher", 1e-2, isopo.REG_REL_TRACE)):
            if lam == 0.0 and singular is None:
                continue
            c_ws, info_ws = isopo.transform(Kd, Ad, variant, lam, mode)
            c = torch.full_like(Ad, 7.0)
            info = torch.full((batch,), -1, dtype=torch.int32, device=gpu_device)
            # the count of allocation requests, not the bytes in use: those may drop under the call when Python
            # collects what earlier tests left behind
            before = torch.cuda.memory_stats(gpu_device)["allocation.all.allocated"]
            isopo.transform_noalloc(Kd, Ad, variant, lam, mode, c, info)
            assert torch.cuda.memory_stats(gpu_device)["allocation.all.allocated"] == before
            torch.cuda.synchronize()
            assert info.cpu().tolist() == info_ws.cpu().tolist()
            # the same kernels on the same inputs: identical bits, NaN fill of a failed problem included
            assert torch.equal(c.view(torch.int32), c_ws.view(torch.int32)), (m, variant, lam)
            for b in range(batch):
                if variant == "fisher":
                    ref = orc.coeff_fisher(K[b], A[b], lam, mode)
                else:
                    ref, oinfo = orc.coeff_interacting(K[b], A[b], lam, mode)
                    assert oinfo == int(info[b].item())
                    if oinfo:
                        assert torch.isnan(c[b]).all()
                        continue
                assert_c_close(c[b].cpu().numpy(), ref, 1e-5, f"noalloc m={m} {variant} lam={lam} b={b}")
    # small problems need no scratch at all
    K, A, Kd, Ad = _problem(rng, 32, 7, gpu_device)
    c = torch.empty_like(Ad)
    isopo.transform_noalloc(Kd, Ad, "interacting", 1e-3, isopo.REG_REL_TRACE, c)
    c_ws, _ = isopo.transform(Kd, Ad, "interacting", 1e-3, isopo.REG_REL_TRACE)
    torch.cuda.synchronize()
    assert torch.equal(c, c_ws)


def test_replays_from_a_hip_graph(gpu_device):
    """The callers this entry point is for: captured once, replayed on the buffers' current contents, with
    eager calls of the workspace entry point in between (they do not touch the library's array)."""
    rng = np.random.default_rng(778)
    m, batch = 200, 2
    K, A, Kd, Ad = _problem(rng, m, batch, gpu_device)
    c = torch.empty_like(Ad)
    info = torch.zeros(batch, dtype=torch.int32, device=gpu_device)
    isopo.transform_noalloc(Kd, Ad, "interacting", 1e-2, isopo.REG_REL_TRACE, c, info)     # resolves the array's address
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        isopo.transform_noalloc(Kd, Ad, "interacting", 1e-2, isopo.REG_REL_TRACE, c, info,
                                stream=torch.cuda.current_stream())
    A0 = Ad.clone()
    for rep in range(3):
        Ad.copy_(A0 * (1.0 + rep))
        c.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        want, winfo = isopo.transform(Kd, Ad, "interacting", 1e-2, isopo.REG_REL_TRACE)
        torch.cuda.synchronize()
        assert torch.equal(c, want) and info.cpu().tolist() == winfo.cpu().tolist() == [0, 0], rep


def test_limit_and_bad_arguments(gpu_device):
    lib = isopo.load()
    dev = gpu_device
    m = 1024
    assert isopo.transform_workspace(m, 1) <= isopo.NOALLOC_SCRATCH_BYTES < isopo.transform_workspace(m, 2)
    K = torch.eye(m, device=dev).repeat(2, 1, 1).contiguous()
    A = torch.ones((2, m), device=dev)
    c = torch.zeros((2, m), device=dev)
    with pytest.raises(isopo.IsopoError) as e:
        isopo.transform_noalloc(K, A, "interacting", 0.0, isopo.REG_ABSOLUTE, c)
    assert e.value.status == 6 and "static scratch" in str(e.value)
    torch.cuda.synchronize()
    assert not c.any()                                   # nothing was enqueued
    isopo.transform_noalloc(K, A, "fisher", 0.0, isopo.REG_ABSOLUTE, c)      # no scratch needed for this variant
    isopo.transform_noalloc(K[0], A[0], "interacting", 1.0, isopo.REG_ABSOLUTE, c[0])   # one problem fits
    torch.cuda.synchronize()
    assert torch.allclose(c[0], torch.full((m,), 0.5, device=dev)) and torch.allclose(c[1], torch.full((m,), m ** 0.5, device=dev))
    assert lib.isopo_transform_noalloc(None, None, 4, 1, 0, 0.0, 0, None, None, None) == 1
    assert lib.isopo_transform_noalloc(K.data_ptr(), A.data_ptr(), 4, 1, 5, 0.0, 0, c.data_ptr(), None, None) == 1
