"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

The CPU oracle cannot mirror a table of 2*10^7 .. 3*10^8 rows cheaply, so at these sizes
  * every integer output is checked in full against its plain definition (numpy): rows against
    the sequential-insert rule, the merged order against the sorted distinct rows, counts
    against a bincount, the row -> key map against the keys;
  * fp32 outputs are checked against the oracle on samples it can compute one by one: the
    forward partials of randomly chosen samples (the oracle table holds just their IDs; the
    initialiser is a pure function of the ID, and outputs do not depend on row numbers), and the
    updated weights / Adagrad state of chosen IDs, hottest ones included, from all their
    occurrences in the batch.
Upstream gradients and the aggregated FM vector fed to the backward pass are seeded arrays given
to both sides.
"""
import os
import sys
import time

import numpy as np
import pytest

from paper_1909_04823_amd import synth
from _harness import assert_close, assert_equal, dev, host_u64

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def progress(msg):
    """Long set-ups stay visibly alive: one line per stage on stderr (not captured per line by pytest's
    default capture once the test ends) and, when DES_PROGRESS_DIR names a folder, in a log file there."""
    line = f"{time.strftime('%H:%M:%S')} {msg}"
    d = os.environ.get("DES_PROGRESS_DIR", "")
    if d and os.path.isdir(d):
        with open(os.path.join(d, "full_size_progress.log"), "a") as f:
            f.write(line + "\n")
    print(line, file=sys.stderr, flush=True)


@pytest.fixture(scope="module")
def des():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_1909_04823_amd import des as d
    return d


def expected_rows(keys, known_keys):
    """Rows under the sequential-insert rule: known IDs keep their row (index in known_keys),
    unseen distinct IDs get the next rows in order of first occurrence."""
    order = np.argsort(known_keys, kind="stable")
    sk = known_keys[order]
    pos = np.minimum(np.searchsorted(sk, keys), sk.size - 1)
    hit = sk[pos] == keys
    rows = np.where(hit, order[pos], -1).astype(np.int64)
    miss = np.flatnonzero(~hit)
    if miss.size:
        uk, first, inv = np.unique(keys[miss], return_index=True, return_inverse=True)
        rank = np.empty(uk.size, np.int64)
        rank[np.argsort(first, kind="stable")] = np.arange(uk.size)
        rows[miss] = known_keys.size + rank[inv]
        new_keys = uk[np.argsort(first, kind="stable")]
    else:
        new_keys = np.empty(0, np.uint64)
    return rows.astype(np.int32), new_keys


def run_full_size(oracle, des, index, n_fwd_samples, n_bwd_keys, grown_rows=None, p_new=None):
    """`grown_rows`: streaming workload only, the table holds that many rows before the checked step (the stream's
    later state; the rows beyond the initial ones are the generator's seeded random IDs, inserted in bulk).
    `p_new`: probability of a brand-new ID per entry in the checked step (default: the workload's)."""
    import torch
    w = synth.workload(index)
    tag = f"workload {index}" + (f" at {grown_rows} rows" if grown_rows else "") + (f", p_new {p_new}" if p_new else "")
    progress(f"{tag}: generating batch")
    n_known = w.preinsert
    if w.p_new:
        gen = synth.StreamingGenerator(w)
        if grown_rows:
            gen.grow_to(grown_rows)
        known = gen.initial_keys()
        n_known = known.size
        batch = gen.next_batch(p_new)
    else:
        known = None
        batch = synth.gen_batch(w, 0)
    B, F, D, K, nnz = w.B, w.F, w.D, w.K, batch.nnz
    free, _ = torch.cuda.mem_get_info()
    need = w.capacity * (2 * D + 6) * 4 + nnz * (60 + 2 * D) + 2 * B * F * D * 4 + K * B * (D + 2) * 4
    if free < 1.15 * need:
        pytest.skip(f"needs about {need / 2**30:.0f} GiB of free HBM")

    progress(f"{tag}: building the table ({n_known} rows)")
    chunk = 1 << 22
    t = des.Table(D, w.capacity, K, des.SHARD_KEY_HASH, des.OPT_ADAGRAD, init_seed=w.seed, init_scale=w.init_std,
                  max_n=max(nnz, min(chunk, n_known)))
    if known is not None:
        for lo in range(0, n_known, chunk):
            t.insert(dev(known[lo:lo + chunk], torch))
    else:
        for lo in range(0, w.preinsert, chunk):
            t.insert(dev(synth.preinsert_keys(w, lo, min(w.preinsert, lo + chunk)), torch))
    assert t.status() == 0 and t.size() == n_known

    # ---- find: all integers ------------------------------------------------------------------
    progress(f"{tag}: find + integer checks")
    gb = des.Batch.from_numpy(batch)
    grows = w.preinsert < w.key_space or bool(w.p_new)
    rows_g = t.find(gb.keys, des.MISS_INSERT if grows else des.MISS_ZERO)
    rows_h = rows_g.cpu().numpy()
    if known is not None:
        exp_rows, new_keys = expected_rows(batch.keys, known)
    else:
        # pre-inserted rank r sits in row r-1; unseen ranks follow in order of first occurrence
        exp_rows = (batch.ranks - 1).astype(np.int64)
        miss = np.flatnonzero(batch.ranks > w.preinsert)
        new_keys = np.empty(0, np.uint64)
        if miss.size:
            uk, first, inv = np.unique(batch.keys[miss], return_index=True, return_inverse=True)
            o = np.argsort(first, kind="stable")
            rank = np.empty(uk.size, np.int64); rank[o] = np.arange(uk.size)
            exp_rows[miss] = w.preinsert + rank[inv]
            new_keys = uk[o]
        exp_rows = exp_rows.astype(np.int32)
    assert_equal(rows_h, exp_rows, "rows")
    n_rows = t.size()
    assert n_rows == n_known + new_keys.size and t.status() == 0
    assert_equal(host_u64(t.row_keys[n_known:n_rows]), new_keys, "row_keys of the new rows")
    if p_new:
        assert abs(new_keys.size / nnz - p_new) < 0.01, "the step does not insert the intended share of new IDs"
    sel = np.random.default_rng(7).integers(0, nnz, 4096)
    assert_equal(host_u64(t.row_keys[torch.from_numpy(rows_h[sel].astype(np.int64)).cuda()]), batch.keys[sel], "row_keys[rows]")

    # ---- forward: sampled against the oracle ---------------------------------------------------
    progress(f"{tag}: forward")
    z = lambda *s: torch.empty(s, dtype=torch.float32, device="cuda")
    P_lr, P_sum, P_sq, pool = z(K, B), z(K, B, D), z(K, B), z(B, F, D)
    t.partial_forward(gb, rows_g, P_lr, P_sum, P_sq, pool)
    A_lr, A_sum, A_sq = des.aggregate_partials(P_lr), des.aggregate_partials(P_sum), des.aggregate_partials(P_sq)
    fm2 = des.fm_finalize(A_sum, A_sq)
    torch.cuda.synchronize()
    rng = np.random.default_rng(11)
    S = np.sort(rng.choice(B, size=min(n_fwd_samples, B), replace=False))
    off = batch.offsets.astype(np.int64)
    ent = np.concatenate([np.arange(off[b * F], off[(b + 1) * F]) for b in S])
    sub_off = np.zeros(S.size * F + 1, np.int32)
    sub_off[1:] = np.cumsum(np.concatenate([np.diff(off[b * F:(b + 1) * F + 1]) for b in S]))
    sub_keys = batch.keys[ent]
    ot = oracle.Table(D, np.unique(sub_keys).size + 8, seed=w.seed, init_scale=w.init_std)
    o_rows = ot.insert(sub_keys)
    P = ot.partial_forward(S.size, F, sub_keys, sub_off, o_rows, K, oracle.SHARD_KEY_HASH, None, pool=False)
    o_pool = ot.partial_forward(S.size, F, sub_keys, sub_off, o_rows, 1, 0, None, lr=False, fm=False, pool=True)["P_pool"][0]
    Sd = torch.from_numpy(S).cuda()
    assert_close(P_lr[:, Sd].cpu().numpy(), P["P_lr"], "P_lr (sampled)")
    assert_close(P_sum[:, Sd].cpu().numpy(), P["P_sum"], "P_sum (sampled)")
    assert_close(P_sq[:, Sd].cpu().numpy(), P["P_sq"], "P_sq (sampled)")
    assert_close(pool[Sd].cpu().numpy(), o_pool, "pool (sampled)")
    oA_sum, oA_sq = oracle.aggregate(P["P_sum"]), oracle.aggregate(P["P_sq"])
    assert_close(A_lr[Sd].cpu().numpy(), oracle.aggregate(P["P_lr"]), "A_lr (sampled)")
    assert_close(A_sum[Sd].cpu().numpy(), oA_sum, "A_sum (sampled)")
    assert_close(fm2[Sd].cpu().numpy(), oracle.fm_finalize(oA_sum, oA_sq), "fm2 (sampled)")
    ot.close()
    del P_lr, P_sum, P_sq, pool

    # ---- backward: integers in full, chosen IDs against the oracle -----------------------------
    progress(f"{tag}: backward")
    g_lr, g_fm, g_pool = synth.upstream_gradients(w, 0)
    A_in = (np.random.default_rng(13).standard_normal((B, D)) * 0.1).astype(np.float32)
    dbg = {"uniq_rows": torch.empty(nnz, dtype=torch.int32, device="cuda"),
           "uniq_keys": torch.empty(nnz, dtype=torch.int64, device="cuda"),
           "counts": torch.empty(nnz, dtype=torch.int32, device="cuda"),
           "n_uniq": torch.zeros(1, dtype=torch.int64, device="cuda")}
    t.backward_update_adagrad(gb, rows_g, w.lr, w.eps, dev(g_lr, torch), dev(g_fm, torch), dev(A_in, torch),
                              dev(g_pool, torch), dbg=dbg)
    torch.cuda.synchronize()
    assert t.status() == 0
    uniq, counts = np.unique(rows_h, return_counts=True)
    U = int(dbg["n_uniq"].item())
    assert U == uniq.size
    assert_equal(dbg["uniq_rows"][:U].cpu().numpy(), uniq, "uniq_rows")
    assert_equal(dbg["counts"][:U].cpu().numpy(), counts.astype(np.int32), "counts")
    all_keys = host_u64(t.row_keys[:n_rows])
    assert_equal(host_u64(dbg["uniq_keys"][:U]), all_keys[uniq], "uniq_keys")

    progress(f"{tag}: oracle on chosen IDs")
    hot = uniq[np.argsort(counts)[-10:]]
    some = rng.choice(uniq, size=min(n_bwd_keys, uniq.size), replace=False)
    chosen_rows = np.unique(np.concatenate([hot, some]))
    chosen_keys = all_keys[chosen_rows]
    mask = np.isin(rows_h, chosen_rows)
    bag_of = np.repeat(np.arange(B * F, dtype=np.int64), np.diff(off))
    sub_off = np.zeros(B * F + 1, np.int64)
    np.cumsum(np.bincount(bag_of[mask], minlength=B * F), out=sub_off[1:])
    sub_keys = batch.keys[mask]
    ot = oracle.Table(D, chosen_keys.size + 8, seed=w.seed, init_scale=w.init_std)
    ot.insert(chosen_keys)                          # oracle row i <-> chosen_rows[i]
    o_rows = ot.find(sub_keys)
    ref = ot.backward_update(B, F, sub_off.astype(np.int32), o_rows, g_lr, g_fm, A_in, g_pool, oracle.OPT_ADAGRAD,
                             w.lr, w.eps)
    assert_equal(ref["counts"], counts[np.searchsorted(uniq, chosen_rows)].astype(np.int32), "counts of chosen IDs")
    idx = torch.from_numpy(chosen_rows.astype(np.int64)).cuda()
    assert_close(t.emb[idx].cpu().numpy(), ot.emb, "updated emb (chosen IDs)")
    assert_close(t.w[idx].cpu().numpy(), ot.w, "updated w (chosen IDs)")
    assert_close(t.acc_emb[idx].cpu().numpy(), ot.acc_emb, "updated acc_emb (chosen IDs)")
    assert_close(t.acc_w[idx].cpu().numpy(), ot.acc_w, "updated acc_w (chosen IDs)")
    # rows the batch did not touch keep their initial weights and zero state
    untouched = np.setdiff1d(rng.integers(0, n_rows, 2000), uniq)[:500]
    if untouched.size:
        uidx = torch.from_numpy(untouched.astype(np.int64)).cuda()
        assert not bool(t.acc_emb[uidx].any()) and not bool(t.acc_w[uidx].any())
        k0 = int(all_keys[untouched[0]])
        assert float(t.emb[int(untouched[0]), 1]) == np.float32(oracle.init_value(k0, 1, w.seed, w.init_std))
    ot.close()
    t.close()
    progress(f"{tag}: done (nnz={nnz}, U={U}, new rows={new_keys.size}, rows={n_rows}, hottest count={int(counts.max())})")


def test_full_size_deepfm(oracle, des):
    run_full_size(oracle, des, 2, n_fwd_samples=256, n_bwd_keys=3000)


def test_full_size_streaming_first_step(oracle, des):
    run_full_size(oracle, des, 3, n_fwd_samples=256, n_bwd_keys=3000)


def test_full_size_streaming_grown_table(oracle, des):
    """The streaming workload in the state it is about (Section 5, dynamic hash table; Section 1, dynamic
    features): 4.9e7 of the 5.2e7 rows in use (slot load 0.73), one step that looks up, inserts ~245,000 unseen
    IDs and updates with Adagrad.  Row numbers, the new rows' keys, the table size and the merged order are
    checked in full, the fp32 results on samples."""
    run_full_size(oracle, des, 3, n_fwd_samples=256, n_bwd_keys=3000, grown_rows=49_000_000)


def test_full_size_streaming_insert_heavy_step(oracle, des):
    """The same grown table with a step in which 30 % of the entries are brand-new IDs (2.4e6 inserts in one
    call: the literal reading of the workload's description, which cannot be kept up for 200 steps inside
    5e7 rows but can for one)."""
    run_full_size(oracle, des, 3, n_fwd_samples=128, n_bwd_keys=2000, grown_rows=49_000_000, p_new=0.30)


def test_full_size_large_table(oracle, des):
    run_full_size(oracle, des, 4, n_fwd_samples=48, n_bwd_keys=3000)


@pytest.mark.parametrize("index", [2, 4])
def test_dnn_layer_full_size_sampled(oracle, des, index):
    """First fully-connected layer (Section 4.3) at the benchmark shapes, H = 256, in the launch
    configuration bench.py times.  The oracle computes whole output rows for sampled samples
    (every shard's partial and g_pool) and, for the weight gradient, whole rows of sampled fields
    over a subset of the hidden units, each summed over the full batch."""
    import torch
    w = synth.workload(index)
    B, F, D, K, H = w.B, w.F, w.D, w.K, 256
    progress(f"dnn full size: workload {index} B={B} F={F} D={D} K={K} H={H}")
    gen = torch.Generator(device="cuda"); gen.manual_seed(100 + index)
    pool = torch.randn((B, F, D), device="cuda", generator=gen) * 0.05
    W = torch.randn((F * D, H), device="cuda", generator=gen) / float(np.sqrt(F * D))
    dY = torch.randn((B, H), device="cuda", generator=gen) * 0.01
    Yp = des.dnn_partial_forward(pool, W, K)
    Y = des.aggregate_partials(Yp)
    g_pool = torch.empty((B, F, D), device="cuda"); dW = torch.empty((F * D, H), device="cuda")
    ws = torch.empty(des.dnn_backward_bytes(B, F, D, H), dtype=torch.uint8, device="cuda")
    des.dnn_backward(pool, W, dY, g_pool, dW, ws)
    torch.cuda.synchronize()
    progress("dnn full size: kernels done")
    rng = np.random.default_rng(index)
    bsel = np.unique(np.concatenate([[0, 127, 128, B - 1], rng.integers(0, B, 12)]))
    bt = torch.from_numpy(bsel).cuda()
    pool_s, dY_s, W_h = pool[bt].cpu().numpy(), dY[bt].cpu().numpy(), W.cpu().numpy()
    Y_ref = oracle.dnn_partial_forward(pool_s, W_h, K)
    assert_close(Yp[:, bt].cpu().numpy(), Y_ref, "Y_partial rows")
    assert_close(Y[bt].cpu().numpy(), oracle.aggregate(Y_ref), "Y rows")
    g_ref, _ = oracle.dnn_backward(pool_s, W_h, dY_s, want_dW=False)
    assert_close(g_pool[bt].cpu().numpy(), g_ref, "g_pool rows")
    progress("dnn full size: forward and g_pool rows checked")
    fsel = np.array([0, F - 1])
    hsel = np.unique(np.concatenate([[0, 127, 128, H - 1], rng.integers(0, H, 28)]))
    ht = torch.from_numpy(hsel).cuda()
    pool_f = pool[:, torch.from_numpy(fsel).cuda(), :].cpu().numpy()
    jsel = np.concatenate([np.arange(f * D, (f + 1) * D) for f in fsel])
    _, dW_ref = oracle.dnn_backward(pool_f, W_h[jsel][:, hsel], dY[:, ht].cpu().numpy(), want_g_pool=False)
    assert_close(dW[torch.from_numpy(jsel).cuda()][:, ht].cpu().numpy(), dW_ref, "dW rows of sampled fields")
    progress("dnn full size: dW rows checked")
