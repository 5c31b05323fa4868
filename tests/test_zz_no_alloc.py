"""The entry point that allocates nothing (pulsecol_select_noalloc) against pulsecol_select on a
context of the same shape: same kernels, same inputs, so the column sets must be identical.  Two
calls in a row share the static scratch; the second is smaller, so whatever the first left behind
lies beyond and inside what the second uses."""

import sys

import pytest
import torch

from paper_2605_20813_amd import pulsecol as pc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def rand_qk(B, H, n, d, dtype, seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    Q, K = (torch.randn(B, H, n, d, generator=g, dtype=torch.float32) for _ in range(2))
    K[:, :, ::13] *= 2.5
    return Q.to(dtype).to(DEV), K.to(dtype).to(DEV)


CALLS = [
    # the largest shape the static scratch holds, then smaller ones; other dtypes / group sizes over
    # the same scratch
    (1, 32, 65536, 128, torch.bfloat16, 0, 0.10),
    (1, 4, 3000, 128, torch.bfloat16, 0, 0.10),
    (1, 2, 1100, 128, torch.bfloat16, 0, 0.25),
    (2, 3, 777, 64, torch.bfloat16, 256, 0.10),
    (1, 2, 256, 64, torch.float32, 0, 0.25),
    (1, 2, 640, 128, torch.bfloat16, 64, 0.05),
]


def test_noalloc_select_equals_select_on_a_context():
    torch.cuda.set_device(0)
    for call, (B, H, n, d, dtype, G, keep) in enumerate(CALLS):
        say(f"noalloc case B={B} H={H} n={n} d={d} {dtype} G={G} keep={keep}")
        Q, K = rand_qk(B, H, n, d, dtype, seed=n + d)
        with pc.Context(B, H, n, d, dtype, group_size=G) as ctx:
            want = ctx.select(Q, K, keep)
            torch.cuda.synchronize()
            U = ctx.groups
        k = pc.num_keep(n, keep)
        got = torch.full((B, H, U, k), -1, dtype=torch.int32, device=DEV)
        # free device memory as the driver sees it (torch's own caching does not move it): the first call on
        # a device may make the runtime place the library's static array, later calls change nothing
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        pc.select_noalloc(pc.make_shape(B, H, n, d, dtype, group_size=G), Q, K, keep, got)
        torch.cuda.synchronize()
        if call > 0:
            assert torch.cuda.mem_get_info()[0] == free_before
        assert torch.equal(got, want), f"B={B} H={H} n={n} G={G}"


def test_noalloc_select_rejects_what_does_not_fit():
    n = 65536
    shape = pc.make_shape(1, 33, n, 128, torch.bfloat16)              # one head more than the scratch holds
    Q = torch.zeros(16, dtype=torch.bfloat16, device=DEV)            # never read: the call fails on the host
    idx = torch.zeros(16, dtype=torch.int32, device=DEV)
    with pytest.raises(pc.PulseColError) as e:
        pc.select_noalloc(shape, Q, Q, 0.1, idx)
    assert e.value.status == pc.ERR_UNSUPPORTED and "static scratch" in str(e.value)
    with pytest.raises(pc.PulseColError) as e:
        pc.select_noalloc(pc.make_shape(1, 2, 256, 64, torch.float32), Q, Q, 1.5, idx)
    assert e.value.status == pc.ERR_INVALID_ARG
