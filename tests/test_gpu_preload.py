"""Layer-wise preloading runtime (Algorithm 2) on the GPU: data arrives before it is used, a slot of
the read buffer is not overwritten while its layer is still being computed, and copies are asked
for in the order the algorithm prescribes."""
import numpy as np
import pytest
import torch

from oracle import cachecraft_oracle as O

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n_layers,depth,n_slots", [(8, 2, 3), (6, 1, 2), (5, 3, 5), (3, 5, 3), (1, 1, 1)])
def test_preloaded_layers_arrive_in_time_and_slots_are_not_clobbered(n_layers, depth, n_slots):
    import paper_2502_15734_amd as P
    n = 4 * 1024 * 1024                                            # 16 MiB of int32 per layer
    host = [torch.full((n,), 3 * l + 1, dtype=torch.int32).pin_memory() for l in range(n_layers)]
    for l in range(n_layers):
        host[l][::4096] += l                                       # not a constant fill
    slots = [torch.zeros(n, dtype=torch.int32, device="cuda") for _ in range(n_slots)]
    results = torch.zeros(n_layers, dtype=torch.int64, device="cuda")
    pre = P.Preloader(n_layers, depth, n_slots)
    for l in range(n_layers):
        pre.set_layer(l, host[l], slots[l % n_slots])
    issued_before = []
    for l in range(n_layers):
        pre.acquire(l)
        issued_before.append(pre.issued())
        buf = slots[l % n_slots]
        acc = torch.zeros((), dtype=torch.int64, device="cuda")
        for k in range(12):                                        # slow enough for the copies to run ahead
            acc = acc + (buf.to(torch.int64) * (k + 1)).sum()
        results[l] = acc
        pre.release(l)
    torch.cuda.synchronize()
    want = [int(host[l].to(torch.int64).sum()) * sum(range(1, 13)) for l in range(n_layers)]
    assert results.cpu().tolist() == want
    # the order of the copies is Algorithm 2's
    steps = O.preload_schedule(n_layers, depth)
    flat, expect = [], []
    for s in steps:
        flat += s
        expect.append(list(flat))
    assert issued_before == expect
    pre.close()


def test_preloader_rejects_bad_arguments():
    import paper_2502_15734_amd as P
    with pytest.raises(P.CacheCraftError):
        P.Preloader(4, 2, 2)                                       # ring shorter than depth + 1
    with pytest.raises(P.CacheCraftError):
        P.Preloader(0, 1, 1)
    pre = P.Preloader(3, 1, 2)
    with pytest.raises(P.CacheCraftError):
        pre.release(0)                                             # nothing enqueued yet
    h = torch.zeros(16, dtype=torch.int32).pin_memory(); d = torch.zeros(16, dtype=torch.int32, device="cuda")
    for l in range(3):
        pre.set_layer(l, h, d)
    pre.acquire(0)
    with pytest.raises(P.CacheCraftError):
        pre.set_layer(0, h, d)                                     # its copy is already on its way
    torch.cuda.synchronize()
    pre.close()
