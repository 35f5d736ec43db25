"""Host threads calling the library at once, each on its own stream.

The C ABI promises thread safety: the only shared host state is the workspace table of
dconv_general and a few cached launch parameters.  ctypes releases the interpreter lock during a
call, so Python threads do overlap inside the library.
"""
import threading

import numpy as np
import pytest
import torch

import oracle
import workloads as wl
import paper_1705_10591_amd as dconv
from helpers import assert_within_bound

pytestmark = pytest.mark.gpu


def test_two_threads_different_shapes_shared_tiles_and_single_channel():
    shared = dconv.VARIANT_TILED_CFG0 + 2 * 3          # + tile shape: tiles cut over channels
    # per thread: a list of (kind, device inputs, variant); shapes differ between the threads so
    # that cached launch parameters of one are wrong for the other
    specs = [
        [("g", (3, 16, 28, 28, 130, 3), shared + 1), ("g", (2, 8, 30, 30, 70, 3), dconv.VARIANT_AUTO),
         ("s", (1, 1, 60, 300, 40, 5), dconv.VARIANT_AUTO)],
        [("g", (2, 37, 14, 14, 70, 3), shared + 0), ("g", (7, 24, 9, 35, 96, 3), shared + 2),
         ("s", (1, 1, 33, 131, 16, 3), dconv.VARIANT_AUTO)],
    ]
    work, refs = [], []
    for t, lst in enumerate(specs):
        w, r = [], []
        for i, (kind, shp, variant) in enumerate(lst):
            x, f = wl.random_case(1200 + 10 * t + i, *shp)
            if kind == "s":
                xd, fd = torch.from_numpy(x[0, 0]).cuda(), torch.from_numpy(f[:, 0]).cuda()
                acc, mag, _ = oracle.single_channel(x[0, 0], f[:, 0])
            else:
                xd, fd = torch.from_numpy(x).cuda(), torch.from_numpy(f).cuda()
                acc, mag, _ = oracle.general(x, f)
            w.append((kind, xd, fd, variant))
            r.append((acc, mag))
        work.append(w)
        refs.append(r)
    torch.cuda.synchronize()
    results = [[], []]
    errors = []

    def worker(t):
        try:
            torch.cuda.set_device(0)
            s = torch.cuda.Stream()
            with torch.cuda.stream(s):
                for rep in range(40):
                    for kind, xd, fd, variant in work[t]:
                        fn = dconv.dconv_single_channel if kind == "s" else dconv.dconv_general
                        out = fn(xd, fd, variant=variant)
                        if rep in (0, 39):
                            results[t].append(out)
            s.synchronize()
        except Exception as e:          # surfaced below: an exception in a thread is not a test failure by itself
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(2)]
    print("two threads, 120 calls each", flush=True)
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for t in range(2):
        n = len(work[t])
        assert len(results[t]) == 2 * n
        for i in range(n):
            acc, mag = refs[t][i]
            assert_within_bound(results[t][i].cpu().numpy(), acc, mag, f"thread {t} call {i}")
            assert torch.equal(results[t][i], results[t][n + i]), f"thread {t} call {i}: repeat differs"
