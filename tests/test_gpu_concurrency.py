"""Calls from two host threads on streams of their own (include/ppo.h allows them when outputs and workspaces are
distinct): each thread's results must be what the same call gives alone."""
import threading

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_2210_12219_amd import workloads as W


def test_two_threads_two_streams():
    import torch
    assert torch.cuda.is_available(), "this test needs the GPU"
    from paper_2210_12219_amd import binding as ppo
    ppo.load()
    jobs = [W.headline().take(6), W.resnet50_shaped(n_inst=200), W.random_instances(4100, 30, 24, 7, capacity_factor=1.3),
            W.tiny()]
    alone = []
    for w in jobs:
        out = ppo.ppo_solve(*ppo.to_device(w))
        torch.cuda.synchronize()
        alone.append(tuple(x.cpu().numpy() for x in out))
    results, errors = {}, []

    def worker(which):
        try:
            stream = torch.cuda.Stream()          # default priority
            with torch.cuda.stream(stream):
                for rep in range(3):
                    for idx in which:
                        w = jobs[idx]
                        dev = ppo.to_device(w)
                        out = ppo.ppo_solve(*dev, stream=stream)
                        stream.synchronize()
                        results[(idx, rep, which[0])] = tuple(x.cpu().numpy() for x in out)
        except Exception as exc:                  # surfaces in the main thread
            errors.append(exc)

    threads = [threading.Thread(target=worker, args=([0, 1, 2, 3],)), threading.Thread(target=worker, args=([3, 2, 1, 0],))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    assert len(results) == 24
    for (idx, rep, first), got in results.items():
        ref = alone[idx]
        assert np.array_equal(got[0].view(np.uint32), ref[0].view(np.uint32)), (idx, rep, first)
        assert np.array_equal(got[1], ref[1]) and np.array_equal(got[2], ref[2]), (idx, rep, first)
