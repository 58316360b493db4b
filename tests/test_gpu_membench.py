"""The measurement kernels of include/hps_membench.h move what they say they move: the gather
equals a plain index of the rows, its read-only half writes nothing, its write-only half writes
exactly the rows of the given positions, and the streaming copy copies."""
import numpy as np
import pytest
import torch

from paper_2210_08804_amd import binding as B

pytestmark = pytest.mark.gpu
NONE = 0xFFFFFFFF


@pytest.mark.parametrize("d,n", [(128, 5000), (128, 106496), (32, 3000), (320, 700)])
def test_gather_equals_indexing(d, n):
    rng = np.random.Generator(np.random.PCG64(d + n))
    n_rows = 20000
    rows = torch.from_numpy(rng.integers(0, 1 << 32, size=(n_rows, d), dtype=np.uint32).view(np.int32)).cuda()
    slot = rng.integers(0, n_rows, size=n, dtype=np.int64).astype(np.uint32)
    slot[rng.random(n) < 0.1] = NONE                                     # positions without a row
    d_slot = torch.from_numpy(slot.view(np.int32)).cuda()
    out = torch.full((n, d), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    B.hps_membench_gather(rows.view(torch.float32), d_slot, n, d, out.view(torch.float32))
    torch.cuda.synchronize()
    exp = np.full((n, d), 0x5A5A5A5A, dtype=np.uint32)
    has = slot != NONE
    exp[has] = rows.cpu().numpy().view(np.uint32)[slot[has]]
    assert (out.cpu().numpy().view(np.uint32) == exp).all()


def test_halves_of_the_gather():
    d, n, n_rows = 128, 30000, 50000
    rng = np.random.Generator(np.random.PCG64(3))
    rows = torch.from_numpy(rng.integers(0, 1 << 30, size=(n_rows, d), dtype=np.int32)).cuda()
    slot = rng.integers(0, n_rows, size=n, dtype=np.int64).astype(np.uint32)
    slot[::7] = NONE
    d_slot = torch.from_numpy(slot.view(np.int32)).cuda()
    out = torch.full((n, d), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    B.hps_membench_gather_half(rows.view(torch.float32), d_slot, n, out.view(torch.float32), True)
    torch.cuda.synchronize()
    assert (out == 0x5A5A5A5A).all()                                     # the read-only half stores nothing
    B.hps_membench_gather_half(rows.view(torch.float32), d_slot, n, out.view(torch.float32), False)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    has = slot != NONE
    assert (got[~has] == 0x5A5A5A5A).all()                               # positions without a row stay as they were
    assert (got[has] != 0x5A5A5A5A).all(axis=1).all()                    # every row of a position with one was written whole
    with pytest.raises(B.HpsError):
        B.hps_membench_gather_half(None, d_slot, n, out.view(torch.float32), True)


@pytest.mark.parametrize("nt", [False, True])
def test_streaming_copy(nt):
    n = (1 << 22) + 4096
    src = torch.arange(n, dtype=torch.int32, device="cuda")
    dst = torch.zeros(n, dtype=torch.int32, device="cuda")
    B.hps_membench_copy(src, dst, n * 4, nt)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    with pytest.raises(B.HpsError):
        B.hps_membench_copy(src, dst, 24, nt)                            # not a multiple of 16
