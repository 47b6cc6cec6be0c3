"""cocod_consensus_distance_noalloc (static scratch, device result, no allocation) against
cocod_consensus_distance, through the C ABI: same bits, on two calls in a row of which the second
works on a smaller model (the shared scratch still holds the first call's partials), flat and packed,
and the size limit is refused on the host."""
import gc

import numpy as np
import pytest
import torch

import paper_1906_12043_amd as P
import synth_inputs
from oracle import cocod_oracle as orc
from tests.gpu_harness import GpuWorkers

pytestmark = pytest.mark.gpu


def make(W, d, seed, sizes=None, weights=None):
    hyper = dict(lr=0.05, momentum=0.9, weight_decay=5e-4, noise_sigma=0.01, seed=seed, weights=weights)
    h, c = synth_inputs.quadratic_data(seed, W, d)
    g = GpuWorkers(W, d, h=h, c=c, tensor_numel=sizes, **hyper)
    o = orc.QuadraticOracle(h, c, **hyper)
    for _ in range(2):
        g.ctx.round(3); o.round(3)
    g.ctx.local_steps(2); o.local_steps(2)               # workers apart from each other
    return g, o


def test_no_alloc_consensus_distance_matches_the_allocating_call():
    big, o_big = make(6, 300_011, 51)                                            # 293 chunks + ragged tail
    sizes = [7, 1024, 2050, 3, 1021, 4097]
    small, o_small = make(5, sum(sizes), 52, sizes=sizes, weights=[0.1, 0.2, 0.3, 0.15, 0.25])   # 9 chunks, packed, weighted
    out = torch.full((2,), float("nan"), dtype=torch.float64, device=big.dev)    # allocated before the calls under test
    gc.collect()                                    # tensors of earlier tests go now, not in the middle of the measurement
    torch.cuda.synchronize()
    free_before, torch_before = torch.cuda.mem_get_info()[0], torch.cuda.memory_allocated()
    big.ctx.consensus_distance_noalloc(out[0:1])
    big.ctx.sync()
    small.ctx.consensus_distance_noalloc(out[1:2])                               # second call, smaller input, same scratch
    small.ctx.sync()
    # the device's free memory sees every allocation, the library's own hipMalloc included
    assert torch.cuda.mem_get_info()[0] >= free_before and torch.cuda.memory_allocated() <= torch_before
    got = out.cpu().numpy()
    want_big, want_small = big.ctx.consensus_distance(), small.ctx.consensus_distance()
    assert got[0] == want_big and got[1] == want_small                           # same kernels, fixed order: same bits
    for value, o in ((got[0], o_big), (got[1], o_small)):
        want = o.consensus_distance()
        assert want > 0 and abs(value - want) <= 1e-5 * want, (value, want)
    # again in the other order, and twice on one stream without a wait in between
    out.fill_(float("nan"))
    torch.cuda.synchronize()
    small.ctx.consensus_distance_noalloc(out[1:2])
    small.ctx.consensus_distance_noalloc(out[1:2])
    small.ctx.sync()
    big.ctx.consensus_distance_noalloc(out[0:1])
    big.ctx.sync()
    got = out.cpu().numpy()
    assert got[0] == want_big and got[1] == want_small
    big.close(); small.close()


def test_no_alloc_call_refuses_bad_arguments_on_the_host():
    g, _ = make(2, 5000, 53)
    with pytest.raises(P.CocodError) as e:
        g.ctx.consensus_distance_noalloc(None)
    assert e.value.status == P.ERR_INVALID
    with pytest.raises(P.CocodError) as e:
        g.ctx.consensus_distance_noalloc(g.mean.data_ptr() + 4)                  # misaligned for a double
    assert e.value.status == P.ERR_INVALID
    g.close()
