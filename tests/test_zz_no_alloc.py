"""hps_dedup_noalloc (the entry point for callers that cannot allocate: its hash table is a static
device array) against hps_dedup on the same inputs, through the C ABI.

What dedup leaves unique is compared exactly between the two entry points and with the oracle
(the number of distinct keys, the set of distinct keys); the rest (the order of the list, which
is the order in which tiles arrive) is checked for validity: no key twice,
unique[inverse[i]] == keys[i] everywhere, nothing written behind n_unique.  Two calls in a row,
the second with a smaller input, so that whatever the first call left in the array would show.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2210_08804_amd import binding as B
from paper_2210_08804_amd import inputs

pytestmark = pytest.mark.gpu

GUARD = -0x1234567


def run(entry, keys, session=None):
    n = len(keys)
    dk = torch.from_numpy(keys).cuda() if n else torch.empty(0, dtype=torch.int64, device="cuda")
    uk = torch.full((max(n, 1),), GUARD, dtype=torch.int64, device="cuda")
    inv = torch.full((max(n, 1),), -1, dtype=torch.int32, device="cuda")
    nu = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    if session is None:
        entry(dk, n, uk, inv, nu)
    else:
        entry(session, dk, n, uk, inv, nu)
    torch.cuda.synchronize()
    u = int(nu.item())
    return uk.cpu().numpy(), inv.cpu().numpy().view(np.uint32)[:n], u


def check_pair(keys, session):
    a_uk, a_inv, a_u = run(B.hps_dedup_noalloc, keys)
    b_uk, b_inv, b_u = run(B.hps_dedup, keys, session)
    ou, _ = oracle.dedup(keys) if len(keys) <= 20000 else (np.unique(keys), None)
    assert a_u == b_u == len(ou)
    assert (np.sort(a_uk[:a_u]) == np.sort(b_uk[:b_u])).all() and (np.sort(a_uk[:a_u]) == np.sort(ou)).all()
    assert len(np.unique(a_uk[:a_u])) == a_u                       # no key twice
    if len(keys):
        assert (a_uk[a_inv] == keys).all()                         # the map leads back to every position's key
        assert a_inv.max() < a_u
        assert (a_uk[a_u:] == GUARD).all()                         # nothing written behind the list


def test_no_alloc_dedup_matches_the_session_entry_point_twice_in_a_row():
    session = B.hps_dedup_create(B.HPS_DEDUP_NOALLOC_MAX)
    try:
        big = inputs.zipf_keys(4096 * 26, 10 ** 8, 1.05, 1)        # the hot-cache batch: several tiles and a ragged tail
        check_pair(big, session)
        small = inputs.zipf_keys(3001, 500, 1.1, 2)                # smaller, other keys, many repeats
        small[::97] = -(1 << 63)                                   # the value that marks a free slot is a key like any other
        check_pair(small, session)
        check_pair(np.arange(B.HPS_DEDUP_NOALLOC_MAX, dtype=np.int64)[::-1].copy(), session)   # the largest call, all distinct
        check_pair(np.full(777, 42, dtype=np.int64), session)     # one key
        check_pair(np.empty(0, dtype=np.int64), session)
    finally:
        B.hps_dedup_destroy(session)


def test_no_alloc_dedup_rejects_what_does_not_fit():
    n = B.HPS_DEDUP_NOALLOC_MAX + 1
    dk = torch.zeros(n, dtype=torch.int64, device="cuda")
    uk = torch.full((n,), GUARD, dtype=torch.int64, device="cuda")
    inv = torch.zeros(n, dtype=torch.int32, device="cuda")
    nu = torch.full((1,), -5, dtype=torch.int32, device="cuda")
    with pytest.raises(B.HpsError) as e:
        B.hps_dedup_noalloc(dk, n, uk, inv, nu)
    assert e.value.status == B.HPS_ERR_INVALID_ARG and "at most" in str(e.value)
    torch.cuda.synchronize()
    assert int(nu.item()) == -5 and (uk == GUARD).all()            # nothing was launched


def test_no_alloc_dedup_inside_a_graph():
    """The caller it is for: captured once, replayed on new keys; every replay is checked."""
    n = 20000
    dk = torch.zeros(n, dtype=torch.int64, device="cuda")
    uk = torch.empty(n, dtype=torch.int64, device="cuda")
    inv = torch.empty(n, dtype=torch.int32, device="cuda")
    nu = torch.zeros(1, dtype=torch.int32, device="cuda")
    g = torch.cuda.CUDAGraph()
    cs = torch.cuda.Stream()
    cs.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(cs):
        g.capture_begin()
        B.hps_dedup_noalloc(dk, n, uk, inv, nu, cs)
        g.capture_end()
    torch.cuda.synchronize()
    for replay in range(4):
        keys = inputs.zipf_keys(n, 3000 * (replay + 1), 1.1, 40 + replay)
        dk.copy_(torch.from_numpy(keys))
        uk.fill_(GUARD)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        u = int(nu.item())
        ou, _ = oracle.dedup(keys)
        h_uk, h_inv = uk.cpu().numpy(), inv.cpu().numpy().view(np.uint32)
        assert u == len(ou) and (np.sort(h_uk[:u]) == np.sort(ou)).all()
        assert (h_uk[h_inv] == keys).all() and (h_uk[u:] == GUARD).all()
