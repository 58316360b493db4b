"""Query, insert and update captured into a HIP graph: the library records no memset nodes (the
miss counter resets itself), so replays must keep giving the eager results.  Each replay is
checked, with eager work and synchronisations in between."""
import numpy as np
import pytest
import torch

from oracle import OracleCache
from paper_2210_08804_amd import binding as B
from paper_2210_08804_amd import inputs
from harness import (DeviceCache, SENTINEL, assert_same_state, check_state_invariants,
                     insert_is_order_independent)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("checked", [False, True])
def test_graph_replays_match_eager_results(checked):
    S, W, d, n = 1 << 10, 8, 64, 5000
    with DeviceCache(S * W, W, d, concurrent_writers=checked) as gc:
        oc = OracleCache(S * W, W, d)
        ids = np.arange(4000, dtype=np.int64)
        for ck in np.array_split(ids, 8):
            gc.insert(ck, inputs.backing_rows(ck, d))
        oc.load_state(*gc.export())
        batches = [inputs.zipf_keys(n, 9000, 1.05, 50 + b) for b in range(3)]
        dk = [torch.from_numpy(k).cuda() for k in batches]
        outs = [torch.empty(n, d, dtype=torch.float32, device="cuda") for _ in batches]
        mi = [torch.empty(n, dtype=torch.int32, device="cuda") for _ in batches]
        mk = [torch.empty(n, dtype=torch.int64, device="cuda") for _ in batches]
        nm = torch.zeros(3, dtype=torch.int32, device="cuda")
        upd_keys = torch.from_numpy(ids[:512].copy()).cuda()
        upd_rows = torch.empty(512, d, dtype=torch.float32, device="cuda")

        g = torch.cuda.CUDAGraph()
        cs = torch.cuda.Stream()
        cs.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(cs):
            g.capture_begin()
            for b in range(3):
                B.hps_cache_query(gc.h, dk[b], n, outs[b], mi[b], mk[b], nm[b:b + 1], cs)
            B.hps_cache_update(gc.h, upd_keys, upd_rows, 512, cs)       # takes effect after the three queries
            g.capture_end()
        torch.cuda.synchronize()

        for replay in range(4):
            # eager work between replays: new rows for the update, scribble over the outputs
            version = replay + 1
            B.hps_backing_fetch(upd_keys, 512, d, version=version, rows=upd_rows)
            for o in outs:
                o.view(torch.int32).fill_(SENTINEL)
            nm.fill_(-7)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            for b in range(3):
                exp = np.full((n, d), SENTINEL, dtype=np.uint32)
                _, omi, omk = oc.query(batches[b], exp)
                m = int(nm[b].item())
                order = np.argsort(mi[b][:m].cpu().numpy().view(np.uint32))
                assert m == len(omi), f"replay {replay}, batch {b}"
                assert (mi[b][:m].cpu().numpy().view(np.uint32)[order] == omi).all()
                assert (mk[b][:m].cpu().numpy()[order] == omk).all()
                got = outs[b].view(torch.int32).cpu().numpy().view(np.uint32)
                bad = np.nonzero((got != exp).any(axis=1))[0]
                assert bad.size == 0, (f"replay {replay}, batch {b}: {bad.size} rows differ, first at position {bad[:5]}, "
                                       f"keys {batches[b][bad[:5]]}, got {got[bad[0], :3]} expected {exp[bad[0], :3]}")
            oc.update(ids[:512], inputs.backing_rows(ids[:512], d, version))
            # an eager query in between sees the update of the replay
            got, gmi, _ = gc.query(ids[:512])
            exp = np.full((512, d), SENTINEL, dtype=np.uint32)
            _, omi, _ = oc.query(ids[:512], exp)
            assert (gmi == omi).all() and (got == exp).all() and len(omi) < 100


def test_dedup_query_fill_insert_expand_as_one_graph():
    """Sec. 2.2 + Alg. 1 without a host round trip, captured once and replayed on new key batches:
    dedup -> query of the distinct keys (count read on the device) -> fetch of the missing distinct
    rows -> insert of them -> expansion to the positions.  Every replay is checked against the
    same steps on the oracle; the cache warms up from replay to replay."""
    import oracle
    S, W, d, n = 1 << 12, 8, 32, 6000
    with DeviceCache(S * W, W, d, concurrent_writers=False) as gc:
        oc = OracleCache(S * W, W, d)
        dd = B.hps_dedup_create(n)
        try:
            dk = torch.zeros(n, dtype=torch.int64, device="cuda")
            uk = torch.empty(n, dtype=torch.int64, device="cuda")
            inv = torch.empty(n, dtype=torch.int32, device="cuda")
            nu = torch.zeros(1, dtype=torch.int32, device="cuda")
            urows = torch.empty(n, d, dtype=torch.float32, device="cuda")
            mrows = torch.empty(n, d, dtype=torch.float32, device="cuda")
            mi = torch.empty(n, dtype=torch.int32, device="cuda")
            mk = torch.empty(n, dtype=torch.int64, device="cuda")
            nm = torch.zeros(1, dtype=torch.int32, device="cuda")
            out = torch.empty(n, d, dtype=torch.float32, device="cuda")
            g = torch.cuda.CUDAGraph()
            cs = torch.cuda.Stream()
            cs.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(cs):
                g.capture_begin()
                B.hps_dedup(dd, dk, n, uk, inv, nu, cs)
                B.hps_cache_query_dn(gc.h, uk, n, nu, urows, mi, mk, nm, cs)
                B.hps_backing_fetch(mk, n, d, version=0, rows=mrows, n_dev=nm, scatter_idx=mi, scatter_out=urows, stream=cs)
                B.hps_cache_insert_dn(gc.h, mk, mrows, n, nm, cs)
                B.hps_expand_rows(urows, inv, n, d, out, cs)
                g.capture_end()
            torch.cuda.synchronize()
            misses = []
            for replay in range(5):
                keys = inputs.zipf_keys(n, 20000, 1.1, 70 + replay)
                dk.copy_(torch.from_numpy(keys))
                out.view(torch.int32).fill_(SENTINEL)
                urows.view(torch.int32).fill_(SENTINEL)
                torch.cuda.synchronize()
                g.replay()
                torch.cuda.synchronize()
                ou, _ = oracle.dedup(keys)
                _, omi, omk = oc.query(ou, np.zeros((len(ou), d), dtype=np.uint32))
                assert int(nu.item()) == len(ou) and int(nm.item()) == len(omi)
                assert sorted(mk[:len(omi)].cpu().tolist()) == sorted(omk.tolist())
                assert (out.view(torch.int32).cpu().numpy().view(np.uint32)
                        == inputs.backing_rows(keys, d).view(np.uint32)).all()
                exact = insert_is_order_independent(oc, omk)
                oc.insert(omk, inputs.backing_rows(omk, d).view(np.uint32))
                state = gc.export()
                if exact:
                    assert_same_state(state, oc)
                else:
                    check_state_invariants(*state, oc.set_of)
                oc.load_state(*state)
                misses.append(len(omi))
            assert misses[-1] < misses[0]
        finally:
            torch.cuda.synchronize()
            B.hps_dedup_destroy(dd)


def test_lru_iteration_count_advances_on_every_graph_replay():
    """The paper's LRU rule under graph replay: query -> fetch of the missing rows -> insert,
    captured once on an LRU cache.  The global iteration count g of Alg. 2 is a device word that
    the query kernel advances, so every replay stamps with a new g; with a g frozen at capture
    time all ages would tie and replacement would degenerate to 'lowest way'.  After every replay
    the stamps, g, keys, counters and rows equal the oracle's (policy 1)."""
    import test_gpu_lru as L
    S, W, d, n = 512, 8, 16, 3000             # most sets fill and evict within the ten replays
    with DeviceCache(S * W, W, d, concurrent_writers=False, policy=L.LRU) as gc:
        oc = OracleCache(S * W, W, d, policy=L.LRU)
        dk = torch.zeros(n, dtype=torch.int64, device="cuda")
        out = torch.empty(n, d, dtype=torch.float32, device="cuda")
        mrows = torch.empty(n, d, dtype=torch.float32, device="cuda")
        mi = torch.empty(n, dtype=torch.int32, device="cuda")
        mk = torch.empty(n, dtype=torch.int64, device="cuda")
        nm = torch.zeros(1, dtype=torch.int32, device="cuda")
        g = torch.cuda.CUDAGraph()
        cs = torch.cuda.Stream()
        cs.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(cs):
            g.capture_begin()
            B.hps_cache_query(gc.h, dk, n, out, mi, mk, nm, cs)
            B.hps_backing_fetch(mk, n, d, version=0, rows=mrows, n_dev=nm, stream=cs)
            B.hps_cache_insert_dn(gc.h, mk, mrows, n, nm, cs)
            g.capture_end()
        torch.cuda.synchronize()
        n_exact = 0
        for replay in range(10):
            keys = inputs.zipf_keys(n, 20000, 1.05, 300 + replay)
            dk.copy_(torch.from_numpy(keys))
            out.view(torch.int32).fill_(SENTINEL)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            exp = np.full((n, d), SENTINEL, dtype=np.uint32)
            _, omi, omk = oc.query(keys, exp)
            assert oc.g == replay + 1
            m = int(nm.item())
            order = np.argsort(mi[:m].cpu().numpy().view(np.uint32))
            assert m == len(omi) and (mi[:m].cpu().numpy().view(np.uint32)[order] == omi).all()
            assert (mk[:m].cpu().numpy()[order] == omk).all()
            assert (out.view(torch.int32).cpu().numpy().view(np.uint32) == exp).all()
            exact = L.lru_insert_is_order_independent(oc, omk)
            oc.insert(omk, L.rows_u32(omk, d))
            if exact:
                gk, gctr, gv, gt = L.assert_same(gc, oc)           # stamps and g included
                n_exact += 1
            else:
                gk, gctr, gv = gc.export()
                gt, gg = gc.export_lru()
                assert gg == oc.g
                check_state_invariants(gk, gctr, gv, oc.set_of)
            oc.load_state(gk, gctr, gv, stamps=gt)
            # stamps of this replay are the new g, not the g of capture time
            assert gt.max() == replay + 1
        assert n_exact >= 5, n_exact
        assert (np.array(oc.ctr) > W).sum() > S // 2           # the LRU rule chose victims in most sets
