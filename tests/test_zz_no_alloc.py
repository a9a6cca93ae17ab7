"""The entry point that allocates nothing (ppo_solve_static, for callers that cannot allocate device memory):
through the C ABI, bit for bit against ppo_solve, on two calls in a row of which the second is smaller."""
import ctypes as C

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_2210_12219_amd import workloads as W


def test_static_scratch_entry_point_matches_ppo_solve():
    import torch
    assert torch.cuda.is_available(), "this test needs the GPU"
    from paper_2210_12219_amd import binding as ppo
    lib = ppo.load()
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    big, small = W.headline().take(24), W.resnet50_shaped(n_inst=40)
    assert ppo.ppo_workspace_bytes(big.L, big.k, big.n_inst) > ppo.ppo_workspace_bytes(small.L, small.k, small.n_inst)
    for w in (big, small):          # the second call finds the first one's tables in the array
        t, m, M, B = ppo.to_device(w)
        ref = ppo.alloc_outputs(w.n_inst, w.k)
        got = ppo.alloc_outputs(w.n_inst, w.k)
        for o in got:
            o.fill_(-7)
        ptr = lambda x: C.c_void_p(x.data_ptr())
        args = (ptr(t), ptr(m), w.L, ptr(M), ptr(B), w.k, w.n_inst)
        assert lib.ppo_solve(*args, *(ptr(o) for o in ref), stream) == ppo.PPO_OK
        assert lib.ppo_solve_static(*args, *(ptr(o) for o in got), stream) == ppo.PPO_OK
        torch.cuda.synchronize()
        assert np.array_equal(got[0].cpu().numpy().view(np.uint32), ref[0].cpu().numpy().view(np.uint32)), w.name
        assert np.array_equal(got[1].cpu().numpy(), ref[1].cpu().numpy()), w.name
        assert np.array_equal(got[2].cpu().numpy(), ref[2].cpu().numpy()), w.name
        assert np.isfinite(ref[0].cpu().numpy()).any()
    # a batch beyond the array is refused, and nothing is written
    w = W.headline()
    n_over = 113
    assert ppo.ppo_workspace_bytes(w.L, w.k, n_over) > ppo.PPO_STATIC_SCRATCH_BYTES
    p = C.c_void_p(0x1000)
    assert lib.ppo_solve_static(p, p, w.L, p, p, w.k, n_over, p, p, p, stream) == ppo.PPO_ENOSPC


def test_static_scratch_entry_point_under_graph_capture():
    """What the entry point is for: a caller that records its work into a HIP graph.  The call is captured once
    (after one eager call, which looks up the array's address and raises the kernels' LDS limits) and replayed
    on new inputs, with eager work and synchronisations in between; every replay is compared with ppo_solve."""
    import torch
    from paper_2210_12219_amd import binding as ppo
    lib = ppo.load()
    ptr = lambda x: C.c_void_p(x.data_ptr())
    first = W.random_instances(3100, 24, 40, 7, capacity_factor=1.3)
    t, m, M, B = ppo.to_device(first)
    got = ppo.alloc_outputs(first.n_inst, first.k)
    args = lambda s: (ptr(t), ptr(m), first.L, ptr(M), ptr(B), first.k, first.n_inst, *(ptr(o) for o in got), s)
    assert lib.ppo_solve_static(*args(C.c_void_p(torch.cuda.current_stream().cuda_stream))) == ppo.PPO_OK
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        rc = lib.ppo_solve_static(*args(C.c_void_p(torch.cuda.current_stream().cuda_stream)))
    assert rc == ppo.PPO_OK
    for trial in range(3):
        w = W.random_instances(3101 + trial, 24, 40, 7, capacity_factor=1.2 + 0.2 * trial, quantised=trial == 1)
        for dst, src in zip((t, m, M, B), ppo.to_device(w)):
            dst.copy_(src)
        for o in got:
            o.fill_(-7)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ref = ppo.ppo_solve(t, m, M, B)
        torch.cuda.synchronize()
        assert np.array_equal(got[0].cpu().numpy().view(np.uint32), ref[0].cpu().numpy().view(np.uint32)), trial
        assert np.array_equal(got[1].cpu().numpy(), ref[1].cpu().numpy()), trial
        assert np.array_equal(got[2].cpu().numpy(), ref[2].cpu().numpy()), trial
