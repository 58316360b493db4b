"""GPU parity of the dedup operator (Sec. 2.2, Q* = dedup(Q)) and the row expansion, through the
C ABI, against the CPU oracle.

The order of Q* is not unique (the operator lists distinct keys in the order tiles finish), so
what is compared with the oracle is what is unique - the number of distinct keys and their set -
and the rest is checked for validity: no key listed twice, unique[inverse[i]] == keys[i] at every
position, nothing written past n_unique.  The expansion is a pure gather and is compared bit by
bit.
"""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
from oracle import EMPTY_KEY, RESERVED_KEY, OracleCache
from paper_2210_08804_amd import binding as B
from paper_2210_08804_amd import inputs
from harness import DeviceCache, SENTINEL

pytestmark = pytest.mark.gpu

KEY_FILL = 0x5A5A5A5A5A5A5A5A
IDX_FILL = 0x7EADBEEF


class Dedup:
    def __init__(self, max_n):
        self.h = B.hps_dedup_create(max_n)

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        torch.cuda.synchronize()
        B.hps_dedup_destroy(self.h)

    def run(self, keys):
        keys = np.ascontiguousarray(keys, dtype=np.int64)
        n = len(keys)
        dk = torch.from_numpy(keys).cuda() if n else torch.empty(0, dtype=torch.int64, device="cuda")
        uk = torch.full((max(n, 1),), KEY_FILL, dtype=torch.int64, device="cuda")
        inv = torch.full((max(n, 1),), IDX_FILL, dtype=torch.int32, device="cuda")
        nu = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        B.hps_dedup(self.h, dk, n, uk, inv, nu)
        torch.cuda.synchronize()
        return uk.cpu().numpy(), inv.cpu().numpy().view(np.uint32), int(nu.item())


def check_against_oracle(keys, uk, inv, u, exact_oracle=True):
    keys = np.asarray(keys, dtype=np.int64)
    n = len(keys)
    if exact_oracle:
        ou, oinv = oracle.dedup(keys)
        assert u == len(ou), f"n_unique {u} != {len(ou)}"
        assert (np.sort(uk[:u]) == np.sort(ou)).all(), "the sets of distinct keys differ"
    else:                                          # sizes the oracle's quadratic search cannot finish
        assert u == len(np.unique(keys))
    assert len(np.unique(uk[:u])) == u, "a key is listed twice"
    assert (uk[u:] == KEY_FILL).all(), "unique_keys written past n_unique"
    if n:
        assert int(inv[:n].max()) < u
        assert (uk[inv[:n]] == keys).all(), "inverse does not lead back to the key"
    assert (inv[n:] == IDX_FILL).all()


@pytest.mark.parametrize("n", [0, 1, 2, 63, 64, 65, 1023, 1024, 1025, 5000])
def test_sizes_around_tiles(n):
    keys = inputs.zipf_keys(n, 3000, 1.05, n + 1) if n else np.zeros(0, dtype=np.int64)
    with Dedup(max(n, 1)) as dd:
        check_against_oracle(keys, *dd.run(keys))


def test_degenerate_batches_and_reserved_values():
    with Dedup(20000) as dd:
        same = np.full(20000, 77, dtype=np.int64)
        uk, inv, u = dd.run(same)
        assert u == 1 and uk[0] == 77 and (inv == 0).all()
        distinct = np.random.Generator(np.random.PCG64(3)).permutation(20000).astype(np.int64) - 10000
        check_against_oracle(distinct, *dd.run(distinct))
        # INT64_MIN is the table's own free-slot marker: it must still be an ordinary key here
        special = np.array([EMPTY_KEY, RESERVED_KEY, 0, (1 << 63) - 1, -1], dtype=np.int64)
        keys = special[np.random.Generator(np.random.PCG64(4)).integers(0, 5, size=7000)]
        check_against_oracle(keys, *dd.run(keys))
        only_marker = np.full(3000, EMPTY_KEY, dtype=np.int64)
        uk, inv, u = dd.run(only_marker)
        assert u == 1 and uk[0] == EMPTY_KEY and (inv == 0).all()
        keys = np.concatenate([only_marker[:10], inputs.uniform_keys(5000, 900, 5)])
        check_against_oracle(keys, *dd.run(keys))


def test_session_reuse_with_shrinking_and_growing_batches():
    """The table keeps the previous call's keys until the next call clears it: a smaller batch
    after a larger one (and back) must not see them."""
    with Dedup(60000) as dd:
        for i, n in enumerate([60000, 300, 17, 40000, 1, 60000, 0, 2048]):
            keys = inputs.zipf_keys(n, 50000, 1.1, 10 + i) if n else np.zeros(0, dtype=np.int64)
            check_against_oracle(keys, *dd.run(keys), exact_oracle=n <= 40000)


@pytest.mark.parametrize("n,space,alpha,seed", [(4096 * 26, 10 ** 8, 1.05, 1), (16384 * 26, 10 ** 8, 1.1, 1)])
def test_full_size_batches(n, space, alpha, seed):
    keys = inputs.zipf_keys(n, space, alpha, seed)
    with Dedup(n) as dd:
        uk, inv, u = dd.run(keys)
        check_against_oracle(keys, uk, inv, u, exact_oracle=n <= 4096 * 26)
        # sampled positions against the definition, one by one
        pos = np.random.Generator(np.random.PCG64(seed)).choice(n, 2000, replace=False)
        for p in pos.tolist():
            assert uk[inv[p]] == keys[p]


@pytest.mark.parametrize("d", [4, 16, 100, 128, 132, 256, 320, 516])
def test_expand_rows_matches_oracle(d):
    rng = np.random.Generator(np.random.PCG64(d))
    for u, n in [(1, 1), (37, 500), (1000, 4099), (3, 70)]:
        rows = rng.integers(0, 1 << 32, size=(u, d), dtype=np.uint64).astype(np.uint32)
        inv = rng.integers(0, u, size=n).astype(np.uint32)
        drows = torch.from_numpy(rows.view(np.float32)).cuda()
        dinv = torch.from_numpy(inv.view(np.int32)).cuda()
        out = torch.full((n + 3, d), SENTINEL, dtype=torch.int32, device="cuda").view(torch.float32)
        B.hps_expand_rows(drows, dinv, n, d, out)
        torch.cuda.synchronize()
        got = out.view(torch.int32).cpu().numpy().view(np.uint32)
        assert (got[:n] == oracle.expand(rows, inv)).all()
        assert (got[n:] == SENTINEL).all(), "rows past n were written"
    B.hps_expand_rows(drows, dinv, 0, d, out)                            # n = 0: nothing happens


def test_dedup_query_fill_expand_equals_direct_lookup():
    """Sec. 2.2 in front of the cache: dedup, query Q*, fetch the missing distinct rows, expand.
    Every position must get what the direct query + fill gives it, and the miss list of Q* is the
    deduplicated miss list of Q."""
    S, W, d, n = 1 << 12, 8, 128, 30000
    keys = inputs.zipf_keys(n, 200000, 1.05, 3)
    resident = np.unique(inputs.zipf_keys(20000, 200000, 1.05, 4))
    oc = OracleCache(S * W, W, d)
    with DeviceCache(S * W, W, d) as gc, Dedup(n) as dd:
        oc.insert(resident, inputs.backing_rows(resident, d).view(np.uint32))
        gc.load(np.array(oc.keys), np.array(oc.ctr), np.array(oc.vals))
        # oracle pipeline
        ou, oinv = oracle.dedup(keys)
        ourows = np.zeros((len(ou), d), dtype=np.uint32)
        _, omi, omk = oc.query(ou, ourows)
        ourows[omi] = inputs.backing_rows(omk, d).view(np.uint32)
        expect = oracle.expand(ourows, oinv)
        assert (expect == inputs.backing_rows(keys, d).view(np.uint32)).all()
        # device pipeline
        dk = torch.from_numpy(keys).cuda()
        uk = torch.empty(n, dtype=torch.int64, device="cuda")
        inv = torch.empty(n, dtype=torch.int32, device="cuda")
        nu = torch.zeros(1, dtype=torch.int32, device="cuda")
        B.hps_dedup(dd.h, dk, n, uk, inv, nu)
        u = int(nu.item())
        urows = torch.full((n, d), SENTINEL, dtype=torch.int32, device="cuda").view(torch.float32)
        mi = torch.empty(n, dtype=torch.int32, device="cuda")
        mk = torch.empty(n, dtype=torch.int64, device="cuda")
        nm = torch.zeros(1, dtype=torch.int32, device="cuda")
        B.hps_cache_query(gc.h, uk, u, urows, mi, mk, nm)
        B.hps_backing_fetch(mk, n, d, version=0, rows=None, n_dev=nm, scatter_idx=mi, scatter_out=urows)
        out = torch.full((n, d), SENTINEL, dtype=torch.int32, device="cuda").view(torch.float32)
        B.hps_expand_rows(urows, inv, n, d, out)
        torch.cuda.synchronize()
        assert u == len(ou)
        assert (out.view(torch.int32).cpu().numpy().view(np.uint32) == expect).all()
        m = int(nm.item())
        assert sorted(mk[:m].cpu().tolist()) == sorted(omk.tolist())


def test_bad_arguments():
    with Dedup(100) as dd:
        k = torch.zeros(200, dtype=torch.int64, device="cuda")
        uk = torch.zeros(200, dtype=torch.int64, device="cuda")
        inv = torch.zeros(200, dtype=torch.int32, device="cuda")
        nu = torch.zeros(1, dtype=torch.int32, device="cuda")
        with pytest.raises(B.HpsError, match="max_n"):
            B.hps_dedup(dd.h, k, 101, uk, inv, nu)
        lib = B.load_library()
        assert lib.hps_dedup(dd.h, k.data_ptr() + 4, 10, uk.data_ptr(), inv.data_ptr(), nu.data_ptr(), None) == -1
        assert "aligned" in B.hps_dedup_last_error()
        assert lib.hps_dedup(dd.h, k.data_ptr(), 10, uk.data_ptr(), inv.data_ptr(), None, None) == -1
        assert lib.hps_dedup(dd.h, None, 10, uk.data_ptr(), inv.data_ptr(), nu.data_ptr(), None) == -1
        B.hps_dedup(dd.h, k, 100, uk, inv, nu)                            # still usable
        torch.cuda.synchronize()
        assert int(nu.item()) == 1
