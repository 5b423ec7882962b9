"""GPU parity of table growth and eviction (des_table_migrate and the least-recently-seen helpers)
against the CPU oracle's migration, inside a short training run so that every state array holds
distinct values and the migrated table is used again afterwards."""
import numpy as np
import pytest

from paper_1909_04823_amd import synth
from _harness import Pair, assert_close, assert_equal, dev, host_u64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def des():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_1909_04823_amd import des as d
    return d


def train_step(p, w, step, last_seen_o=None, last_seen_g=None, oracle=None, des=None, insert=True):
    batch = synth.gen_batch(w, step)
    p.find(batch, insert=insert)
    if last_seen_o is not None:
        oracle.mark_seen(last_seen_o, p.rows_o, step + 1)
        des.mark_seen(p.rows_g, step + 1, last_seen_g)
    A_sum = p.forward(batch)
    g_lr, g_fm, g_pool = synth.upstream_gradients(w, step)
    p.backward(batch, g_lr, g_fm, A_sum, g_pool, lr=w.lr, eps=1e-8)
    p.check_weights(f"step {step}")
    return batch


@pytest.mark.parametrize("roomy", [True, False])
def test_evict_least_recently_seen_then_keep_training(oracle, des, roomy):
    import torch
    w = synth.workload(1, scale=1 / 16)
    p = Pair(oracle, des, w.D, w.capacity, w.K, 0, des.OPT_ADAGRAD, seed=w.seed, init_scale=w.init_std, max_n=1 << 17)
    keys0 = synth.preinsert_keys(w)
    p.ot.insert(keys0); p.gt.insert(dev(keys0, torch))
    ls_o = np.zeros(w.capacity, np.uint32)
    ls_g = torch.zeros(w.capacity, dtype=torch.int32, device="cuda")
    for step in range(3):
        train_step(p, w, step, ls_o, ls_g, oracle, des)
        p.sync_weights()
    n = p.check_table("before migration")
    assert_equal(ls_g[:n].cpu().numpy().view(np.uint32), ls_o[:n], "last_seen")
    # keep what was seen in the last two steps (stamps 2 and 3)
    keep_o = oracle.select_recent(ls_o, n, 2)
    keep_g = des.select_recent(ls_g, n, 2)
    torch.cuda.synchronize()
    assert_equal(keep_g.cpu().numpy(), keep_o, "keep flags")
    kept = int(keep_o.sum())
    assert 0 < kept < n
    cap2 = 2 * kept if roomy else kept          # a larger table that keeps growing, or an exact fit (lookups only)
    ot2 = p.ot.migrate(keep_o, cap2)
    gt2 = des.Table(w.D, cap2, num_shards=w.K, opt=des.OPT_ADAGRAD, init_seed=w.seed, init_scale=w.init_std,
                    max_n=max(1 << 17, n))
    ls_g2 = torch.full((cap2,), -1, dtype=torch.int32, device="cuda")
    print(f"migrate {n} -> {kept} rows, capacity {w.capacity} -> {cap2}", flush=True)
    assert p.gt.migrate_into(gt2, keep_g, ls_g, ls_g2) == kept
    # the move is a copy: bit-exact against the source rows, and the keys are the oracle's
    sel = torch.from_numpy(np.flatnonzero(keep_o)).cuda()
    for name in ("emb", "w", "acc_emb", "acc_w", "row_keys"):
        assert torch.equal(getattr(gt2, name)[:kept], getattr(p.gt, name)[sel]), name
    assert torch.equal(ls_g2[:kept], ls_g[sel])
    assert gt2.size() == ot2.n_rows == kept and gt2.status() == 0
    assert_equal(host_u64(gt2.row_keys[:kept]), ot2.row_keys, "migrated row_keys")
    assert p.gt.size() == n                                           # the source is untouched
    # train on: dropped IDs come back as fresh rows, surviving ones keep their state
    old_ot, old_gt = p.ot, p.gt
    p.ot, p.gt = ot2, gt2
    try:
        train_step(p, w, 3, insert=roomy)
        p.check_table("after post-migration step")
    finally:
        old_gt.close(); old_ot.close(); p.close()


def test_growth_keeps_everything_and_errors(oracle, des):
    import torch
    w = synth.workload(0)
    p = Pair(oracle, des, w.D, w.capacity, w.K, 0, des.OPT_SGD, seed=w.seed, init_scale=w.init_std)
    keys0 = synth.preinsert_keys(w)
    vals0 = synth.host_values(w, keys0.shape[0])
    p.ot.insert(keys0, vals0); p.gt.insert(dev(keys0, torch), dev(vals0, torch))
    n = p.check_table()
    mk = lambda cap, D=w.D: des.Table(D, cap, num_shards=w.K, opt=des.OPT_SGD, init_seed=w.seed,
                                      init_scale=w.init_std, max_n=1 << 16)
    small, other_dim, big = mk(n - 1), mk(4 * n, D=2 * w.D), mk(4 * n)
    try:
        with pytest.raises(des.DesError) as e:
            p.gt.migrate_into(small)
        assert e.value.code == des.ERR_FULL and small.size() == 0 and small.status() == 0
        with pytest.raises(des.DesError) as e:
            p.gt.migrate_into(other_dim)
        assert e.value.code == des.ERR_INVALID_ARG
        assert p.gt.migrate_into(big) == n
        assert torch.equal(big.emb[:n], p.gt.emb[:n]) and torch.equal(big.w[:n], p.gt.w[:n])
        assert torch.equal(big.row_keys[:n], p.gt.row_keys[:n])
        probe = np.concatenate([keys0[::7], np.array([12345, 999], np.uint64)])
        rows = big.find(dev(probe, torch))
        torch.cuda.synchronize()
        assert_equal(rows.cpu().numpy(), p.ot.find(probe), "find after growth")
        with pytest.raises(des.DesError) as e:                         # target no longer empty
            p.gt.migrate_into(big)
        assert e.value.code == des.ERR_INVALID_ARG
        # an empty source migrates to an empty target
        a, b = mk(16), mk(16)
        assert a.migrate_into(b) == 0 and b.size() == 0
        a.close(); b.close()
    finally:
        small.close(); other_dim.close(); big.close(); p.close()


@pytest.mark.parametrize("staging_rows", [4096, 1 << 20])
def test_compact_in_place_equals_migration_into_the_same_capacity(oracle, des, staging_rows):
    """Eviction inside one table (des_table_compact), walked in many chunks or in one: the table afterwards
    is the oracle's migration into a table of the same capacity, bit for bit, and training goes on in it."""
    import torch
    w = synth.workload(1, scale=1 / 16)
    p = Pair(oracle, des, w.D, w.capacity, w.K, 0, des.OPT_ADAGRAD, seed=w.seed, init_scale=w.init_std, max_n=1 << 17)
    keys0 = synth.preinsert_keys(w)
    p.ot.insert(keys0); p.gt.insert(dev(keys0, torch))
    ls_o = np.zeros(w.capacity, np.uint32)
    ls_g = torch.zeros(w.capacity, dtype=torch.int32, device="cuda")
    for step in range(3):
        train_step(p, w, step, ls_o, ls_g, oracle, des)
        p.sync_weights()
    n = p.check_table("before compaction")
    keep_o = oracle.select_recent(ls_o, n, 2)
    keep_g = des.select_recent(ls_g, n, 2)
    kept = int(keep_o.sum())
    assert 0 < kept < n and n > 3 * 4096                       # several chunks with the small staging buffer
    before = {name: getattr(p.gt, name)[:n].clone() for name in ("emb", "w", "acc_emb", "acc_w", "row_keys")}
    ls_before = ls_g[:n].clone()
    ot2 = p.ot.migrate(keep_o, w.capacity)
    staging = torch.empty(staging_rows * w.D * 4, dtype=torch.uint8, device="cuda")
    assert p.gt.compact(keep_g, staging, aux=ls_g) == kept
    sel = torch.from_numpy(np.flatnonzero(keep_o)).cuda()
    for name, old in before.items():
        assert torch.equal(getattr(p.gt, name)[:kept], old[sel]), name
    assert torch.equal(ls_g[:kept], ls_before[sel])
    assert p.gt.size() == ot2.n_rows == kept and p.gt.status() == 0
    assert_equal(host_u64(p.gt.row_keys[:kept]), ot2.row_keys, "row_keys after compaction")
    # every kept key is found at its new row, every dropped key is absent
    rows = p.gt.find(dev(p.ot.row_keys, torch), des.MISS_ZERO)
    assert_equal(rows.cpu().numpy(), ot2.find(p.ot.row_keys), "lookups after compaction")
    # keep == None is a no-op
    assert p.gt.compact(None, staging) == kept
    old_ot = p.ot
    p.ot = ot2
    try:
        train_step(p, w, 3, insert=True)                         # dropped IDs come back as fresh rows
        p.check_table("after post-compaction step")
    finally:
        old_ot.close(); p.close()
    with pytest.raises(des.DesError) as e:                       # staging buffer too small
        q = des.Table(8, 64, 1, opt=des.OPT_SGD, max_n=1024)
        q.insert(torch.arange(1, 11, dtype=torch.int64, device="cuda"))
        try:
            q.compact(torch.ones(10, dtype=torch.uint8, device="cuda"), torch.empty(1024, dtype=torch.uint8, device="cuda"))
        finally:
            q.close()
    assert e.value.code == des.ERR_WORKSPACE


def test_compact_keep_all_and_keep_none(des):
    """Degenerate flag sets: everything kept (rows, keys and lookups unchanged) and nothing kept (an empty table
    that takes new rows from 0 again)."""
    import torch
    t = des.Table(8, 20000, 2, opt=des.OPT_ADAGRAD, init_seed=3, max_n=1 << 15)
    keys = torch.arange(1, 10001, dtype=torch.int64, device="cuda") * 7919
    t.insert(keys)
    n = t.size()
    assert n == 10000
    emb, rk = t.emb[:n].clone(), t.row_keys[:n].clone()
    staging = torch.empty(4096 * 8 * 4, dtype=torch.uint8, device="cuda")
    assert t.compact(torch.ones(n, dtype=torch.uint8, device="cuda"), staging) == n
    assert torch.equal(t.emb[:n], emb) and torch.equal(t.row_keys[:n], rk)
    found = t.find(keys, des.MISS_ZERO)
    assert torch.equal(found, torch.arange(n, dtype=torch.int32, device="cuda"))
    assert t.compact(torch.zeros(n, dtype=torch.uint8, device="cuda"), staging) == 0
    assert t.size() == 0 and t.status() == 0
    assert int((t.find(keys, des.MISS_ZERO) >= 0).sum()) == 0
    again = t.find(keys[:100], des.MISS_INSERT)
    assert torch.equal(again, torch.arange(100, dtype=torch.int32, device="cuda")) and t.size() == 100
    t.close()
