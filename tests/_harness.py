"""Shared helpers of the GPU parity tests: run the same seeded inputs through the CPU oracle and
through the HIP library (via its C interface) and compare element by element.

Tolerance (fp32 outputs, gradients, updated weights):  |gpu - ref| <= max(1e-5*|ref|, 1e-6).
Integers (rows, row->key map, merged order, counts, sizes) must be equal.
"""
from __future__ import annotations

import numpy as np

RTOL, ATOL = 1e-5, 1e-6


def assert_close(gpu, ref, what=""):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    err = np.abs(gpu - ref)
    tol = np.maximum(RTOL * np.abs(ref), ATOL)
    bad = err > tol
    if bad.any():
        i = np.unravel_index(np.argmax(err - tol), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} of {bad.size} outside tolerance; worst at {i}: "
                             f"gpu={gpu[i]!r} ref={ref[i]!r} err={err[i]:.3e} tol={tol[i]:.3e}")


def assert_equal(gpu, ref, what=""):
    gpu, ref = np.asarray(gpu), np.asarray(ref)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    if not np.array_equal(gpu, ref):
        i = int(np.flatnonzero(gpu.ravel() != ref.ravel())[0])
        raise AssertionError(f"{what}: first mismatch at flat index {i}: gpu={gpu.ravel()[i]} ref={ref.ravel()[i]}")


def dev(a, torch):
    if a is None:
        return None
    if a.dtype == np.uint64:
        a = a.view(np.int64)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host_u64(t):
    return t.cpu().numpy().view(np.uint64)


class Pair:
    """An oracle table and a library table built from the same description."""

    def __init__(self, oracle, des, D, capacity, K, policy, opt, seed=1234, init_scale=0.01, max_n=1 << 16,
                 state_arrays=None):
        self.oracle, self.des = oracle, des
        self.D, self.K, self.policy, self.opt = D, K, policy, opt
        self.ot = oracle.Table(D, capacity, seed=seed, init_scale=init_scale)
        self.gt = des.Table(D, capacity, num_shards=K, shard_policy=policy, opt=opt, init_seed=seed,
                            init_scale=init_scale, max_n=max_n, state_arrays=state_arrays)

    def close(self):
        self.gt.close()
        self.ot.close()

    def check_table(self, what="table"):
        import torch
        torch.cuda.synchronize()
        n = self.ot.n_rows
        assert self.gt.status() == 0, what
        assert self.gt.size() == n, (what, self.gt.size(), n)
        assert_equal(host_u64(self.gt.row_keys[:n]), self.ot.row_keys, what + " row_keys")
        return n

    def check_weights(self, what="weights", exact=False):
        n = self.ot.n_rows
        cmp = assert_equal if exact else assert_close
        cmp(self.gt.emb[:n].cpu().numpy(), self.ot.emb, what + " emb")
        cmp(self.gt.w[:n].cpu().numpy(), self.ot.w, what + " w")
        for name in ("acc_emb", "acc_w", "acc2_emb", "acc2_w"):
            g = getattr(self.gt, name)
            if g is not None:
                cmp(g[:n].cpu().numpy(), getattr(self.ot, name), what + " " + name)

    def sync_weights(self):
        """Overwrite the library's weights and state with the oracle's, so that a test of several
        steps checks each step's arithmetic from a common state instead of the drift of two fp32
        trajectories (differences within tolerance are amplified by sums over hundreds of terms and
        by the first Adagrad / Adam step of a row)."""
        import torch
        n = self.ot.n_rows
        for name in ("emb", "w", "acc_emb", "acc_w", "acc2_emb", "acc2_w"):
            g = getattr(self.gt, name)
            if g is not None:
                g[:n].copy_(torch.from_numpy(np.ascontiguousarray(getattr(self.ot, name))))

    # ---- one batch through both sides ---------------------------------------------------------
    def find(self, batch, insert=True):
        import torch
        rows_o = self.ot.find(batch.keys, insert_missing=insert)
        self.gb = self.des.Batch.from_numpy(batch)
        self.rows_g = self.gt.find(self.gb.keys, self.des.MISS_INSERT if insert else self.des.MISS_ZERO)
        torch.cuda.synchronize()
        assert_equal(self.rows_g.cpu().numpy(), rows_o, "rows")
        self.rows_o = rows_o
        return rows_o

    def forward(self, batch, dense_pool=False, separate_calls=False):
        """Returns the oracle's fp32 aggregated A_sum (the backward input of both sides)."""
        import torch
        o, d = self.oracle, self.des
        B, F, D, K = batch.B, batch.F, self.D, self.K
        P = self.ot.partial_forward(B, F, batch.keys, batch.offsets, self.rows_o, K, self.policy, batch.vals,
                                    pool=dense_pool)
        pool_ref = self.ot.partial_forward(B, F, batch.keys, batch.offsets, self.rows_o, 1, self.policy, batch.vals,
                                           lr=False, fm=False, pool=True)["P_pool"][0]
        A_lr, A_sum, A_sq = o.aggregate(P["P_lr"]), o.aggregate(P["P_sum"]), o.aggregate(P["P_sq"])
        fm2 = o.fm_finalize(A_sum, A_sq)

        z = lambda *s: torch.full(s, float("nan"), dtype=torch.float32, device="cuda")
        P_lr, P_sum, P_sq, pool = z(K, B), z(K, B, D), z(K, B), z(B, F, D)
        if separate_calls:
            self.gt.partial_forward_lr(self.gb, self.rows_g, P_lr)
            self.gt.partial_forward_fm(self.gb, self.rows_g, P_sum, P_sq)
            self.gt.partial_forward_pool(self.gb, self.rows_g, pool, dense_k=False)
        else:
            self.gt.partial_forward(self.gb, self.rows_g, P_lr, P_sum, P_sq, pool)
        gA_lr, gA_sum, gA_sq = d.aggregate_partials(P_lr), d.aggregate_partials(P_sum), d.aggregate_partials(P_sq)
        g_fm2 = d.fm_finalize(gA_sum, gA_sq)
        torch.cuda.synchronize()
        assert_close(P_lr.cpu().numpy(), P["P_lr"], "P_lr")
        assert_close(P_sum.cpu().numpy(), P["P_sum"], "P_sum")
        assert_close(P_sq.cpu().numpy(), P["P_sq"], "P_sq")
        assert_close(pool.cpu().numpy(), pool_ref, "pool")
        assert_close(gA_lr.cpu().numpy(), A_lr, "A_lr")
        assert_close(gA_sum.cpu().numpy(), A_sum, "A_sum")
        assert_close(gA_sq.cpu().numpy(), A_sq, "A_sq")
        assert_close(g_fm2.cpu().numpy(), fm2, "fm2")
        # the same four results from the single fused launch
        fA_lr, fA_sum, fA_sq, f_fm2 = z(B), z(B, D), z(B), z(B)
        d.aggregate_forward(P_lr, P_sum, P_sq, fA_lr, fA_sum, fA_sq, f_fm2)
        torch.cuda.synchronize()
        assert torch.equal(fA_lr, gA_lr) and torch.equal(fA_sum, gA_sum) and torch.equal(fA_sq, gA_sq)
        assert_close(f_fm2.cpu().numpy(), fm2, "fm2 (fused aggregation)")
        if dense_pool:
            Pp = z(K, B, F, D)
            self.gt.partial_forward_pool(self.gb, self.rows_g, Pp, dense_k=True)
            torch.cuda.synchronize()
            assert_close(Pp.cpu().numpy(), P["P_pool"], "P_pool dense")
            assert_close(d.aggregate_partials(Pp).cpu().numpy(), pool_ref, "aggregated dense pool")
        self.fwd = {"A_lr": A_lr, "A_sum": A_sum, "fm2": fm2, "pool": pool_ref}
        return A_sum.astype(np.float32)

    def backward(self, batch, g_lr, g_fm, A_sum, g_pool, lr=0.05, eps=1e-8, opt=None, optimizer=None,
                 prepare_stream=None):
        """`optimizer`: dict of des_optimizer_t fields (separate optimizers for latent vectors and
        LR weights); otherwise `opt`, `lr`, `eps` for both.  `prepare_stream`: run the row-sorting
        half (des_backward_prepare) on that stream first, ordered by events."""
        import torch
        if prepare_stream is not None:
            main = torch.cuda.current_stream()
            found, sorted_ = torch.cuda.Event(), torch.cuda.Event()
            found.record(main)
            prepare_stream.wait_event(found)
            with torch.cuda.stream(prepare_stream):
                self.gt.backward_prepare(self.gb, self.rows_g)
                sorted_.record(prepare_stream)
            main.wait_event(sorted_)
        o, d = self.oracle, self.des
        opt = self.opt if opt is None else opt
        B, F = batch.B, batch.F
        o_opt = None if optimizer is None else o.Optimizer(**optimizer)
        ref = self.ot.backward_update(B, F, batch.offsets, self.rows_o, g_lr, g_fm, A_sum, g_pool, opt, lr, eps,
                                      vals=batch.vals, optimizer=o_opt)
        dbg = self.gt.debug_buffers(max(batch.nnz, 1))
        args = dict(g_lr=dev(g_lr, torch), g_fm=dev(g_fm, torch), A_sum=dev(A_sum, torch), g_pool=dev(g_pool, torch),
                    dbg=dbg)
        if optimizer is not None:
            self.gt.backward_update(self.gb, self.rows_g, d.Optimizer(**optimizer), **args)
        elif opt == d.OPT_SGD:
            self.gt.backward_update_sgd(self.gb, self.rows_g, lr, **args)
        elif opt == d.OPT_ADAGRAD:
            self.gt.backward_update_adagrad(self.gb, self.rows_g, lr, eps, **args)
        else:
            self.gt.backward_merge(self.gb, self.rows_g, **args)
        torch.cuda.synchronize()
        U = int(dbg["n_uniq"].item())
        assert U == ref["uniq_rows"].shape[0], ("n_uniq", U, ref["uniq_rows"].shape[0])
        assert_equal(dbg["uniq_rows"][:U].cpu().numpy(), ref["uniq_rows"], "uniq_rows")
        assert_equal(host_u64(dbg["uniq_keys"][:U]), ref["uniq_keys"], "uniq_keys")
        assert_equal(dbg["counts"][:U].cpu().numpy(), ref["counts"], "counts")
        assert_close(dbg["merged"][:U].cpu().numpy(), ref["merged"], "merged")
        return ref
