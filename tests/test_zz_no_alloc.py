"""gemm_mp_run_static, the entry point for callers that cannot allocate: the same C as
gemm_mp_run bit for bit, on two calls in a row that share the GPU's static scratch, the second on
a smaller problem; and its refusals."""
import numpy as np
import pytest

import workloads as W
from paper_2508_14848_amd import gemm_mp as G
from tests.harness import gpu_problem


def _say(*a):
    print(*a, flush=True)


def test_static_scratch_limit_is_refused_before_anything_else():
    """More tile products than the static table holds: ETOOBIG, on the host, whatever the state."""
    nb = 128
    g = G.GemmMP(41 * nb, 41 * nb, 41 * nb, nb)             # 41^3 = 68 921 > 65 536 products
    with pytest.raises(G.GemmMPError) as e:
        g.run_static(1.0, 0.0, None)
    assert e.value.status == G.ETOOBIG and "static scratch" in str(e.value)
    g.destroy()
    g = G.GemmMP(40 * nb, 40 * nb, 40 * nb, nb)             # 64 000: allowed, but nothing is set up
    with pytest.raises(G.GemmMPError) as e:
        g.run_static(1.0, 0.0, None)
    assert e.value.status == G.ESTATE
    g.destroy()


@pytest.mark.gpu
def test_run_static_equals_run_bit_for_bit_on_two_calls_sharing_the_scratch():
    import torch
    big = W.random_maps(M=1536, N=1024, K=1280, nb=256, name="static-a")                   # 6 x 4 x 5 tiles, FP64 / FP32 / FP16
    small = W.decay_rect(M=512, N=768, K=256, nb=128, eps=1e-4, name="static-b")           # rule maps down to FP8, FP32 C
    results = []
    problems = []
    for w in (big, small):
        A, B = w.dense("A"), w.dense("B")
        C0 = w.dense("C") if w.beta != 0.0 else None
        d, dev = gpu_problem(w, A, B, C0)
        d.run(w.alpha, w.beta)
        ref = d.unpack_tiles("C").cpu().numpy()
        torch.cuda.synchronize()
        if dev["C"] is not None:
            d.pack_tiles("C", dev["C"])                     # beta != 0: the run overwrote the C it read
        else:
            d.storage["C"].zero_()
        problems.append((w, d, dev, ref))
    # set-up done for both; now the two calls in a row, the second on the smaller problem
    for w, d, dev, ref in problems:
        d.ctx.set_policy(1 - w.policy)                      # the policy changed (and changed back): the schedule
        d.ctx.set_policy(w.policy)                          # on the device is no longer known to be current
        with pytest.raises(G.GemmMPError) as e:
            d.run_static(w.alpha, w.beta)
        assert e.value.status == G.ESTATE
        d.prepare()
    allocs = [d.ctx.host_counters() for _, d, _, _ in problems]
    for w, d, dev, ref in problems:
        _say("run_static", w.name, (w.M, w.N, w.K, w.nb))
        d.run_static(w.alpha, w.beta)
    assert [d.ctx.host_counters() for _, d, _, _ in problems] == allocs      # no allocation, no wait
    for w, d, dev, ref in problems:
        got = d.unpack_tiles("C").cpu().numpy()
        torch.cuda.synchronize()
        assert np.array_equal(got, ref), "gemm_mp_run_static differs from gemm_mp_run on %s" % w.name
        results.append(got)
    # once more in the other order, after ordinary runs have used their own tables in between
    for w, d, dev, ref in reversed(problems):
        if dev["C"] is not None:
            d.pack_tiles("C", dev["C"])
        d.run_static(w.alpha, w.beta)
        got = d.unpack_tiles("C").cpu().numpy()
        torch.cuda.synchronize()
        assert np.array_equal(got, ref)
