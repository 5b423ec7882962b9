"""GPU parity of the dense remainder of a model step (tower epilogue, output unit, dense optimizer)
and of whole training steps of LR / FM / W&D / DeepFM chained from library calls, against the CPU
oracle chained the same way from the same seeded inputs."""
import numpy as np
import pytest

from paper_1909_04823_amd import synth
from _harness import assert_close, assert_equal, dev, host_u64

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def des():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_1909_04823_amd import des as d
    return d


def ws_for(des, H):
    import torch
    return torch.empty(des.dense_workspace_bytes(H), dtype=torch.uint8, device="cuda")


@pytest.mark.parametrize("K,B,H,relu,with_bias", [(1, 1, 4, True, True), (3, 300, 20, True, True),
                                                  (8, 1000, 256, False, True), (2, 77, 132, True, False)])
def test_aggregate_bias_act_and_backward(oracle, des, K, B, H, relu, with_bias):
    import torch
    rng = np.random.default_rng(K * 1000 + B)
    P = rng.standard_normal((K, B, H)).astype(np.float32)
    bias = rng.standard_normal(H).astype(np.float32) if with_bias else None
    dA = rng.standard_normal((B, H)).astype(np.float32)
    A_ref = oracle.bias_act(oracle.aggregate(P), bias, relu)
    A = des.aggregate_bias_act(dev(P, torch), dev(bias, torch), relu)
    torch.cuda.synchronize()
    assert_close(A.cpu().numpy(), A_ref, "A")
    A32 = A_ref.astype(np.float32)
    dZ_ref, db_ref = oracle.bias_act_backward(A32, dA, relu)
    dZ = torch.full((B, H), float("nan"), device="cuda"); db = torch.full((H,), float("nan"), device="cuda")
    des.bias_act_backward(dev(A32, torch), dev(dA, torch), relu, dZ, db, ws_for(des, H))
    torch.cuda.synchronize()
    assert_close(dZ.cpu().numpy(), dZ_ref, "dZ")
    assert_close(db.cpu().numpy(), db_ref, "dbias")
    # in place: dZ written over dA
    dA_g = dev(dA, torch); db2 = torch.empty_like(db)
    des.bias_act_backward(dev(A32, torch), dA_g, relu, dA_g, db2, ws_for(des, H))
    torch.cuda.synchronize()
    assert torch.equal(dA_g, dZ) and torch.equal(db2, db)


@pytest.mark.parametrize("B,H,parts", [(1, 4, "lfa"), (5, 3, "lfa"), (1000, 128, "lfa"), (70000, 36, "la"),
                                       (333, 0, "lf"), (64, 0, "l"), (100, 8, "a")])
def test_output_unit(oracle, des, B, H, parts):
    import torch
    rng = np.random.default_rng(B + H)
    y = (rng.random(B) < 0.3).astype(np.float32)
    A_lr = (2 * rng.standard_normal(B)).astype(np.float32) if "l" in parts else None
    fm2 = rng.standard_normal(B).astype(np.float32) if "f" in parts else None
    if A_lr is not None and B >= 5:
        A_lr[:4] = [90.0, -90.0, 700.0, -700.0]                   # saturated units must stay finite
    a = rng.standard_normal((B, H)).astype(np.float32) if "a" in parts else None
    wv = rng.standard_normal(H).astype(np.float32) if "a" in parts else None
    b0 = np.array([0.25], np.float32)
    ref = oracle.head(y, A_lr, fm2, a, wv, float(b0[0]))
    nan = lambda *s: torch.full(s, float("nan"), dtype=torch.float32, device="cuda")
    out = {k: nan(B) for k in ("logit", "p", "g_logit")}
    loss, db0 = nan(1), nan(1)
    da = nan(B, H) if a is not None else None
    dw = nan(H) if a is not None else None
    des.head(dev(y, torch), out["g_logit"], ws_for(des, max(H, 4)), A_lr=dev(A_lr, torch), fm2=dev(fm2, torch),
             a=dev(a, torch), w_out=dev(wv, torch), b0=dev(b0, torch), logit=out["logit"], p=out["p"], loss=loss,
             da=da, dw_out=dw, db0=db0)
    torch.cuda.synchronize()
    for k in ("logit", "p", "g_logit"):
        assert_close(out[k].cpu().numpy(), ref[k], k)
    assert_close(loss.cpu().numpy(), [ref["loss"]], "loss")
    assert_close(db0.cpu().numpy(), [ref["db0"]], "db0")
    if a is not None:
        assert_close(da.cpu().numpy(), ref["da"], "da")
        assert_close(dw.cpu().numpy(), ref["dw_out"], "dw_out")


@pytest.mark.parametrize("opt", ["sgd", "adagrad", "adam", "ftrl"])
def test_dense_update(oracle, des, opt):
    import torch
    rng = np.random.default_rng(5)
    n = 10007
    theta = rng.standard_normal(n).astype(np.float32)
    code = {"sgd": 1, "adagrad": 2, "adam": 3, "ftrl": 4}[opt]
    fields = dict(opt_emb=code, lr=0.05, eps=1e-8, beta1=0.9, beta2=0.999, ftrl_alpha=0.1, ftrl_beta=1.0,
                  ftrl_l1=0.02, ftrl_l2=0.1)
    s1, s2 = np.zeros(n, np.float32), np.zeros(n, np.float32)
    th_g, s1_g, s2_g = dev(theta, torch), dev(s1, torch), dev(s2, torch)
    for step in range(1, 4):
        g = (rng.standard_normal(n) * 10.0 ** rng.integers(-6, 1, n)).astype(np.float32)
        oracle.dense_update(theta, g, oracle.Optimizer(**fields, step=step), s1, s2)
        des.dense_update(th_g, dev(g, torch), des.Optimizer(**fields, step=step), s1_g, s2_g)
        torch.cuda.synchronize()
        assert_close(th_g.cpu().numpy(), theta, f"theta step {step}")
        assert_close(s1_g.cpu().numpy(), s1, f"s1 step {step}")
        assert_close(s2_g.cpu().numpy(), s2, f"s2 step {step}")
        # both sides continue from the oracle's state so that one-ulp differences do not compound
        th_g, s1_g, s2_g = dev(theta, torch), dev(s1, torch), dev(s2, torch)


SETTINGS = {
    "sgd": (dict(opt_emb=1, opt_w=1, lr=0.05), dict(opt_emb=1, lr=0.05), (0, 0)),
    "paper": (dict(opt_emb=3, opt_w=4, lr=0.01, eps=1e-7, beta1=0.9, beta2=0.999, ftrl_alpha=0.05, ftrl_beta=1.0,
                   ftrl_l1=1e-4, ftrl_l2=1e-3),
              dict(opt_emb=3, lr=0.002, eps=1e-7, beta1=0.9, beta2=0.999), (2, 2)),
}


@pytest.mark.parametrize("kind,setting,hidden", [("lr", "sgd", (64, 32)), ("fm", "sgd", (64, 32)), ("wd", "sgd", (64, 32)),
                                                 ("deepfm", "sgd", (64, 32)), ("deepfm", "paper", (64, 32)),
                                                 ("deepfm", "sgd", (48,)), ("wd", "paper", (64, 32, 16)),
                                                 ("dcn", "sgd", (64, 32)), ("dcn", "paper", (48,)),
                                                 ("dcn-layer-by-layer", "sgd", (48,))])
def test_training_steps_match_oracle_chain(oracle, des, kind, setting, hidden):
    """Three training steps of the whole model on a shrunken Criteo-shaped workload, library calls
    against the oracle's functions chained in the same order.  Each step is compared from a common
    state: after the comparison the library's weights are overwritten with the oracle's, so the
    test checks every step's arithmetic, not the drift of two fp32 trajectories.  For the same
    reason the optimizer stage of each step is fed the oracle's (fp32-rounded) gradients after the
    library's own have been compared with them: the first Adam / Adagrad step divides by |G| + eps
    and turns a last-bit difference of a near-zero gradient into a visible one."""
    import torch
    from _oracle_model import OracleModel
    from paper_1909_04823_amd.model import Model
    cross_fused = kind != "dcn-layer-by-layer"             # the cross network in one piece, or call by call
    kind = kind.split("-")[0]
    w = synth.workload(1, scale=1 / 16)
    opt_sparse, opt_dense, state_arrays = SETTINGS[setting]
    tower = synth.tower_init(w.seed, w.F, w.D, hidden=hidden)
    if kind == "dcn":
        tower.update(synth.cross_init(w.seed, w.F, w.D, n_cross=3))
    keys0 = synth.preinsert_keys(w)
    vals0 = synth.host_values(w, keys0.shape[0])
    ot = oracle.Table(w.D, w.capacity, seed=w.seed, init_scale=w.init_std)
    ot.insert(keys0, vals0)
    gt = des.Table(w.D, w.capacity, num_shards=w.K, opt=des.OPT_NONE, init_seed=w.seed, init_scale=w.init_std,
                   max_n=1 << 17, state_arrays=state_arrays)
    gt.insert(dev(keys0, torch), dev(vals0, torch))
    om = OracleModel(oracle, ot, w.F, w.K, kind, tower, opt_sparse, opt_dense)
    gm = Model(gt, w.F, kind, tower, w.B, opt_sparse, opt_dense, cross_fused=cross_fused)
    names = [("emb", "emb"), ("w", "w"), ("acc_emb", "acc_emb"), ("acc2_emb", "acc2_emb"), ("acc_w", "acc_w"),
             ("acc2_w", "acc2_w")]
    try:
        for step in range(3):
            print(f"model {kind}/{setting} step {step}", flush=True)
            batch = synth.gen_batch(w, step)
            labels = synth.planted_labels(batch, w.seed)
            c = om.train_step(batch, labels)
            gb = des.Batch.from_numpy(batch)
            dbg = gt.debug_buffers(batch.nnz)
            rows = gm.rows[:batch.nnz]
            gt.find(gb.keys, des.MISS_INSERT, rows)
            gm.forward(gb, rows, dev(labels, torch))
            gm.backward_tower(gb)
            torch.cuda.synchronize()
            assert_equal(rows.cpu().numpy(), c["rows"], "rows")
            assert_close(gm.loss.cpu().numpy(), [c["head"]["loss"]], "loss")
            assert_close(gm.p.cpu().numpy(), c["head"]["p"], "p")
            assert_close(gm.g_logit.cpu().numpy(), c["head"]["g_logit"], "g_logit")
            gm.g_logit.copy_(dev(c["g_logit"], torch))
            if "fm" in gm.parts:
                assert_close(gm.A_sum.cpu().numpy(), c["A_sum"], "A_sum")
                gm.A_sum.copy_(dev(c["A_sum"], torch))
            if gm.dnn:
                assert_close(gm.g_pool.cpu().numpy(), c["g_pool"], "g_pool")
                gm.g_pool.copy_(dev(c["g_pool"], torch))
            for k, g in c["dense_grads"].items():
                assert_close(gm.grads[k].cpu().numpy().reshape(-1), np.asarray(g).reshape(-1), "grad " + k)
                gm.grads[k].copy_(dev(np.asarray(g, np.float32).reshape(gm.grads[k].shape), torch))
            gm.update(gb, rows, dbg=dbg)
            torch.cuda.synchronize()
            assert gt.status() == 0
            U = int(dbg["n_uniq"].item())
            assert_equal(dbg["uniq_rows"][:U].cpu().numpy(), c["merge"]["uniq_rows"], "uniq_rows")
            assert_close(dbg["merged"][:U].cpu().numpy(), c["merge"]["merged"], "merged sparse gradients")
            n = ot.n_rows
            assert gt.size() == n
            for gname, oname in names:
                garr = getattr(gt, gname)
                if garr is not None:
                    assert_close(garr[:n].cpu().numpy(), getattr(ot, oname), f"step {step} {gname}")
                    garr[:n].copy_(torch.from_numpy(np.ascontiguousarray(getattr(ot, oname))))
            for k in om.p:
                if k in gm.params:
                    assert_close(gm.params[k].cpu().numpy(), om.p[k], f"step {step} param {k}")
                    gm.params[k].copy_(torch.from_numpy(om.p[k])); gm.s1[k].copy_(torch.from_numpy(om.s1[k]))
                    gm.s2[k].copy_(torch.from_numpy(om.s2[k]))
    finally:
        gt.close(); ot.close()


@pytest.mark.parametrize("kind", ["deepfm", "dcn"])
def test_model_learns_planted_labels(des, kind):
    """Sixty steps of DeepFM / DCN (Adagrad) on fresh batches whose labels depend on the IDs: predictions are
    made before each batch's update, so they are held-out; over the last ten batches their AUC is well
    above chance and the mean log-loss is below that of a constant predictor at the base rate (0.613)."""
    import torch
    from paper_1909_04823_amd.model import Model, auc
    w = synth.workload(1, scale=1 / 8)
    gt = des.Table(w.D, w.capacity, num_shards=w.K, opt=des.OPT_ADAGRAD, init_seed=w.seed, init_scale=w.init_std,
                   max_n=1 << 18)
    gt.insert(dev(synth.preinsert_keys(w), torch))
    tower = synth.tower_init(1, w.F, w.D, hidden=(64, 32))
    if kind == "dcn":
        tower.update(synth.cross_init(1, w.F, w.D, n_cross=2))
    m = Model(gt, w.F, kind, tower, w.B,
              dict(opt_emb=2, opt_w=2, lr=0.01, eps=1e-8), dict(opt_emb=2, lr=0.005, eps=1e-8))
    losses, aucs = [], []
    try:
        for step in range(60):
            batch = synth.gen_batch(w, step)
            labels = synth.planted_labels(batch, w.seed, strength=4.0)
            loss = m.train_step(des.Batch.from_numpy(batch), dev(labels, torch), insert=False)   # unseen IDs are skipped
            losses.append(float(loss.item()))
            aucs.append(auc(labels, m.p.cpu().numpy()))
        print(kind, "loss", np.round(losses[::10], 4), "auc", np.round(aucs[::10], 3), "last ten: loss",
              round(float(np.mean(losses[-10:])), 4), "auc", round(float(np.mean(aucs[-10:])), 4), flush=True)
        assert gt.status() == 0 and all(np.isfinite(losses))
        assert np.mean(aucs[-10:]) > 0.6, aucs
        assert np.mean(losses[-10:]) < 0.60, losses
    finally:
        gt.close()
